"""The C++ oracle under the address and undefined-behaviour sanitizers (host build only): every entry
point runs on small inputs of every kind in a child process whose oracle library is the sanitized
build; any out-of-bounds access, use after free, signed overflow or misaligned access aborts the child."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

SCRIPT = r"""
import numpy as np
from oracle import oracle as orc
from paper_2209_12769_amd import workloads as wl
assert orc._SO.endswith("libdc_oracle_san.so")
for name, n in (("cfg1", 3), ("cfg2", 4), ("cfg3", 2)):
    w = wl.make(name, n)
    for bf16 in (False, True):
        b = orc.contract(w, bf16)
        p = orc.gnn_forward(b, w.model, w.weights, bf16)
        assert np.isfinite(p).all()
    t, x = wl.profile_of(w)
    c = orc.cost(w, t, x, 0.02, 0.01)
    assert c.shape == (n,)
wa = wl.with_attention(wl.make("cfg2", 3), 4)
assert np.isfinite(orc.evaluate(wa)).all()
# arbitrary labels: cyclic quotients, long lists, one group, empty batch
g = wl.random_dag(5, 120, 0.08, 16)
labs = np.concatenate([wl.random_labels(6, g.n, 7, C=2), wl.random_labels(7, g.n, 60, C=2),
                       np.zeros((1, g.n), np.int32), np.arange(g.n, dtype=np.int32)[None]])
w = wl.custom("san", wl.ModelSpec(16, 32, 2, "f32"), [g], [labs], seed=2)
b = orc.contract(w)
assert b.node_off[5] - b.node_off[4] == 1
orc.gnn_forward(b, w.model, w.weights)
t = np.full(b.ntot, 0.5, np.float32); x = np.full(b.ntot, -1.0, np.float32)
orc.simulate(b, t, x, 0.1, 0.2)
assert orc.evaluate(w.subset([])).size == 0
assert orc.evaluate_parallel(w, False, 3).shape == (6,)
print("sanitized oracle run complete")
"""


def test_oracle_runs_clean_under_asan_and_ubsan():
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], stdout=subprocess.PIPE, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("no address-sanitizer runtime on this host")
    env = dict(os.environ)
    env["DC_ORACLE_SANITIZE"] = "1"
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # the interpreter itself leaks by design and is not instrumented: report errors of the oracle only
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["PYTHONPATH"] = ROOT
    res = subprocess.run([sys.executable, "-c", SCRIPT], cwd=ROOT, env=env, stdout=subprocess.PIPE,
                         stderr=subprocess.STDOUT, text=True, timeout=600)
    assert res.returncode == 0 and "sanitized oracle run complete" in res.stdout, res.stdout[-4000:]
