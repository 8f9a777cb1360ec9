"""Host-side guard for the bulk layer kernels (no GPU): they wait by hand for loads the compiler does not
track.  Today those are direct copies into LDS without destination registers; should a register
destination come back, no compiler-generated instruction may touch it before the wait that covers the
load.  The ISA listing of every instantiation is checked for that, and the checker itself is checked on
hand-made listings, one of them with a load kept in flight across a loop's back edge."""
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


def test_checker_carries_loads_in_flight_across_a_back_edge(tmp_path):
    # the load is issued at the bottom of the loop and its register is copied at the top of the next
    # round, before any wait: only visible if what is pending at the branch reaches the loop's head
    loop = _listing(tmp_path, """\
        \ts_mov_b32 s0, 0
        .LBB0_1:
        \tv_mov_b32_e32 v20, v9
        \ts_waitcnt vmcnt(0)
        \t;;#ASMSTART
        \tglobal_load_dwordx4 v[8:11], v[0:1], off
        \t;;#ASMEND
        \ts_cbranch_scc1 .LBB0_1
        """)
    assert len(isa_check.check(loop, r'^_Z6kernelv:')) == 1


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_no_instruction_touches_a_load_in_flight_in_the_layer_kernels():
    res = isa_check.check_layer256()
    assert len(res) >= 4                      # input widths 256 / 64: the plain product and the message-passing layer
    for kernel, hazards in res.items():
        assert hazards == [], (kernel, hazards[:3])
