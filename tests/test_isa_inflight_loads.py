"""Host-side guard for the bulk layer kernel (no GPU): its data-moving waves wait by hand for loads the
compiler does not track, so no compiler-generated instruction may touch a load's destination registers
before the wait that covers it.  The ISA listing of every instantiation is checked for that, and the
checker itself is checked on two hand-made listings."""
import os
import shutil
import textwrap

import pytest

from paper_2209_12769_amd import isa_check


def _listing(tmp_path, body):
    p = tmp_path / "k.s"
    p.write_text("_Z6kernelv:\n" + textwrap.dedent(body) + ".Lfunc_end0:\n")
    return str(p)


def test_checker_flags_a_copy_of_a_register_whose_load_is_in_flight(tmp_path):
    bad = _listing(tmp_path, """\
        \t;;#ASMSTART
        \tglobal_load_dwordx4 v[8:11], v[0:1], off
        \t;;#ASMEND
        \tv_mov_b32_e32 v20, v9
        \ts_waitcnt vmcnt(0)
        """)
    assert len(isa_check.check(bad, r'^_Z6kernelv:')) == 1
    good = _listing(tmp_path, """\
        \t;;#ASMSTART
        \tglobal_load_dwordx4 v[8:11], v[0:1], off
        \t;;#ASMEND
        \t;;#ASMSTART
        \tglobal_load_dwordx4 v[12:15], v[2:3], off
        \t;;#ASMEND
        \ts_waitcnt vmcnt(1)
        \tv_mov_b32_e32 v20, v9
        \ts_waitcnt vmcnt(0)
        \tv_mov_b32_e32 v21, v13
        """)
    assert isa_check.check(good, r'^_Z6kernelv:') == []
    reused = _listing(tmp_path, """\
        \t;;#ASMSTART
        \tglobal_load_dwordx4 v[8:11], v[0:1], off
        \t;;#ASMEND
        \tv_add_u32_e32 v9, 1, v30
        """)
    assert len(isa_check.check(reused, r'^_Z6kernelv:')) == 1


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_no_instruction_touches_a_load_in_flight_in_the_layer_kernels():
    res = isa_check.check_layer256()
    assert len(res) >= 8                      # input widths 256 / 64: gather with 3 and 1 slots, plain product, one-slot DMA
    for kernel, hazards in res.items():
        assert hazards == [], (kernel, hazards[:3])
