"""The address emulator behind the build-time check of the hand-scheduled kernels (paper_2504_20039_amd/isa_emu.py), on small
hand-written instruction sequences whose results are worked out by hand."""
import numpy as np
import pytest

from paper_2504_20039_amd.isa_emu import Emu, Poison


def run(text, kernarg=b"\0" * 64, wg=3, tid_base=64):
    seen = []
    e = Emu(text.strip().splitlines(), kernarg, wg, tid_base, lambda emu, op, o, t: seen.append((op, t)))
    e.run()
    return e, seen


def test_scalar_arithmetic_carries_and_selects():
    e, _ = run("""
        s_mov_b32 s4, 0xfffffff0
        s_add_u32 s5, s4, 0x20
        s_addc_u32 s6, 0, 0
        s_mul_i32 s7, s2, 100
        s_cmp_lt_i32 s7, 301
        s_cselect_b32 s8, 11, 22
        s_lshl_b64 s[10:11], s[4:5], 4
        s_addk_i32 s7, 0xff00
        s_min_i32 s9, s7, -1
        s_endpgm
    """)
    assert e.s["s5"] == 0x10 and e.s["s6"] == 1                 # the carry of the 32-bit addition
    assert e.s["s8"] == 11                                        # 3 * 100 < 301
    assert e.get64("s[10:11]") == ((0xfffffff0 | (0x10 << 32)) << 4) & (2**64 - 1)
    assert e.s["s7"] == 300 - 256 and e.s["s9"] == 0xFFFFFFFF   # a signed 16-bit constant; the signed minimum


def test_a_counted_loop_and_lane_arithmetic():
    e, seen = run("""
        s_mov_b32 s4, 0
        v_mbcnt_lo_u32_b32 v1, -1, 0
        v_mbcnt_hi_u32_b32 v1, -1, v1
        v_lshrrev_b32_e32 v2, 3, v0
        v_mov_b32_e32 v3, 0
    .LBB0_1:
        v_mad_u32_u24 v3, v2, 3, v3
        s_add_i32 s4, s4, 1
        s_cmp_lg_u32 s4, 5
        s_waitcnt vmcnt(2)
        s_cbranch_scc1 .LBB0_1
        v_readlane_b32 s6, v3, 63
        v_writelane_b32 v4, s6, 2
        v_readfirstlane_b32 s7, v1
        s_endpgm
    """)
    assert np.array_equal(e.v[1], np.arange(64))                  # the lane index
    assert np.array_equal(e.v[3], 15 * ((np.arange(64) + 64) >> 3))
    assert e.s["s6"] == 15 * 15 and e.v[4][2] == 225 and e.s["s7"] == 0
    assert sum(op == "s_waitcnt" for op, _ in seen) == 5


def test_loaded_data_is_unknown_and_a_branch_on_it_stops_the_run():
    text = """
        buffer_load_dword v5, v0, s[8:11], 0 offen
        v_readfirstlane_b32 s4, v5
        s_cmp_eq_u32 s4, 0
        s_cbranch_scc1 .LBB0_2
    .LBB0_2:
        s_endpgm
    """
    with pytest.raises(Poison):
        run(text)


def test_an_instruction_it_does_not_know_raises():
    with pytest.raises(RuntimeError):
        run("s_sendmsg sendmsg(MSG_INTERRUPT)\ns_endpgm")
