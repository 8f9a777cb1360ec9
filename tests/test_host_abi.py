"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and rejects bad configurations before any
device call."""
import ctypes
import os
import re

import pytest

from paper_2209_12769_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "disco.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dc_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert {"dc_contract_graphs", "dc_gnn_forward", "dc_eval_candidates", "dc_create", "dc_destroy"} <= set(names)
    lib = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n


def test_binding_has_the_same_names():
    for n in _declared_symbols():
        assert hasattr(B, n), n


def test_bad_configurations_are_rejected_on_the_host():
    ok = dict(F=32, H=128, L=3, dtype=B.DC_BF16, max_cand=8, max_base_nodes=1000, max_base_edges=2000,
              max_nodes=0, max_edges=0)
    for patch, want in [(dict(F=0), B.DC_ERR_INVALID_ARG), (dict(L=0), B.DC_ERR_INVALID_ARG),
                        (dict(dtype=5), B.DC_ERR_INVALID_ARG), (dict(max_cand=-1), B.DC_ERR_INVALID_ARG),
                        (dict(F=24), B.DC_ERR_UNSUPPORTED), (dict(H=48), B.DC_ERR_UNSUPPORTED),
                        (dict(H=1024), B.DC_ERR_UNSUPPORTED), (dict(max_base_nodes=3_000_000_000), B.DC_ERR_UNSUPPORTED)]:
        cfg = B.DcConfig(**{**ok, **patch})
        st, h = B.dc_create(cfg)
        assert st == want and not h, (patch, st)
        assert B.dc_workspace_bytes(cfg) == 0


def test_workspace_size_grows_with_capacity():
    a = B.dc_workspace_bytes(B.DcConfig(32, 128, 3, B.DC_BF16, 8, 1000, 2000, 0, 0))
    b = B.dc_workspace_bytes(B.DcConfig(32, 128, 3, B.DC_BF16, 8, 2000, 4000, 0, 0))
    c = B.dc_workspace_bytes(B.DcConfig(32, 128, 3, B.DC_BF16, 8, 2000, 4000, 500, 900))
    assert 0 < a < b and c < b
    # at least the four activation-sized buffers of the contracted capacity
    assert a >= 4 * 1000 * 128 * 2


def test_null_context_is_an_error_not_a_crash():
    lib = B.lib()
    assert lib.dc_destroy(None) == B.DC_ERR_INVALID_ARG
    assert lib.dc_check(None, None) == B.DC_ERR_INVALID_ARG
    assert lib.dc_eval_candidates(None, 1, None, None, None, None, None) == B.DC_ERR_INVALID_ARG
    assert B.dc_last_error(None) == "null context"
