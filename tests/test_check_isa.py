"""The build-time model of the vector-memory counter: planted hazards are found, waits of
the right depth clear them, and the shipped kernels that count their own waits are clean."""
import os

import pytest

from paper_2603_10026_amd import build as B
from paper_2603_10026_amd import check_isa as C

HEAD = "kern:\n"
TAIL = "\ts_endpgm\n.Lfunc_end0:\n"


def hazards(body):
    n, hz = C.check_text(HEAD + body + TAIL)
    assert n == 1
    return hz


def test_register_read_before_its_wait_is_reported():
    body = ("\tglobal_load_dwordx4 v[4:7], v1, s[2:3] offset:16\n"
            "\tv_add_f32_e32 v9, v5, v5\n"
            "\ts_waitcnt vmcnt(0)\n")
    hz = hazards(body)
    assert len(hz) == 1 and "v5" in hz[0]


def test_wait_of_the_right_depth_clears_the_oldest_load_only():
    body = ("\tglobal_load_dwordx4 v[4:7], v1, s[2:3]\n"
            "\tglobal_load_dwordx4 v[8:11], v1, s[2:3] offset:16\n"
            "\tglobal_load_lds_dwordx4 v[2:3], off\n"
            "\ts_waitcnt vmcnt(2) lgkmcnt(0)\n"
            "\tv_mov_b32_e32 v20, v4\n")
    assert hazards(body) == []
    assert len(hazards(body + "\tv_mov_b32_e32 v21, v8\n")) == 1
    assert hazards(body + "\ts_waitcnt vmcnt(1)\n\tv_mov_b32_e32 v21, v8\n") == []


def test_copy_at_a_loop_back_edge_is_reported_on_the_second_trip():
    # the load issued late in the body is waited for at the top of the next trip, but a
    # register copy sits between the load and the branch
    body = (".LBB0_1:\n"
            "\ts_waitcnt vmcnt(0)\n"
            "\tv_add_f32_e32 v9, v4, v4\n"
            "\tglobal_load_dwordx4 v[12:15], v1, s[2:3]\n"
            "\tv_mov_b64_e32 v[4:5], v[12:13]\n"
            "\ts_cbranch_scc1 .LBB0_1\n")
    hz = hazards(body)
    assert len(hz) == 1 and "v_mov_b64" in hz[0]
    clean = body.replace("\tv_mov_b64_e32 v[4:5], v[12:13]\n", "")
    assert hazards(clean) == []
    # a read at the top of the loop, ahead of the wait, is only reachable round the back edge
    late = body.replace("\tv_mov_b64_e32 v[4:5], v[12:13]\n", "").replace(
        ".LBB0_1:\n", ".LBB0_1:\n\tv_mul_f32_e32 v30, v13, v13\n")
    hz = hazards(late)
    assert len(hz) == 1 and "second trip" in hz[0]


def test_direct_to_lds_loads_and_stores_count_but_own_no_registers():
    body = ("\tglobal_load_lds_dwordx4 v[2:3], off\n"
            "\tglobal_store_dwordx4 v1, v[4:7], s[2:3]\n"
            "\tv_mov_b32_e32 v2, 0\n"
            "\tv_mov_b32_e32 v4, 0\n")
    assert hazards(body) == []


def test_lds_reads_waited_by_count_and_scalar_loads_in_between():
    body = ("\tds_read_b128 v[4:7], v1\n"
            "\tds_read_b64_tr_b16 v[8:9], v1 offset:64\n"
            "\ts_waitcnt lgkmcnt(1)\n"
            "\tv_mov_b32_e32 v20, v5\n")
    assert hazards(body) == []
    assert len(hazards(body + "\tv_mov_b32_e32 v21, v9\n")) == 1
    # a scalar load shares the counter and may return first: the partial wait proves nothing
    mixed = body.replace("\ts_waitcnt", "\ts_load_dwordx2 s[4:5], s[0:1], 0x0\n\ts_waitcnt")
    hz = hazards(mixed)
    assert any("partial wait" in h for h in hz)
    # the vector-memory queue is left alone by an LDS wait
    both = "\tglobal_load_dwordx4 v[30:33], v1, s[2:3]\n" + body + "\tv_mov_b32_e32 v22, v30\n"
    assert len(hazards(both)) == 1
    n, only_lgkm = C.check_text(HEAD + both + TAIL, counters=("lgkm",))
    assert only_lgkm == []


def test_dot_result_needs_three_wait_states_before_another_kind_of_reader():
    dot = "\tv_dot2c_f32_bf16 v180, v20, v20\n"
    # a copy one instruction later reads the old value
    hz = hazards(dot + "\ts_addc_u32 s11, s11, s9\n\tv_mov_b32_e32 v193, v180\n")
    assert len(hz) == 1 and "v180" in hz[0] and "wait states" in hz[0]
    # three other instructions, or a nop that stands for them, are enough
    assert hazards(dot + "\ts_add_u32 s0, s0, s1\n" * 3 + "\tv_mov_b32_e32 v193, v180\n") == []
    assert hazards(dot + "\ts_nop 2\n\tv_mov_b32_e32 v193, v180\n") == []
    assert len(hazards(dot + "\ts_nop 1\n\tv_mov_b32_e32 v193, v180\n")) == 1
    # the next dot instruction may accumulate into the same register right away
    assert hazards(dot + "\tv_dot2c_f32_bf16 v180, v21, v21\n\ts_nop 3\n\tv_mov_b32_e32 v1, v180\n") == []
    # other registers are free to be read
    assert hazards(dot + "\tv_mov_b32_e32 v193, v181\n") == []


def test_scalar_register_from_a_lane_read_needs_five_wait_states_before_vector_memory():
    rd = "\tv_readfirstlane_b32 s7, v193\n\tv_readfirstlane_b32 s6, v192\n"
    ld = "\tglobal_load_lds_dwordx4 v200, s[6:7]\n\ts_waitcnt vmcnt(0)\n"
    hz = hazards(rd + "\ts_mov_b32 m0, s34\n\ts_nop 0\n" + ld)
    assert len(hz) == 1 and "s7" in hz[0] and "wait states" in hz[0]
    assert hazards(rd + "\ts_mov_b32 m0, s34\n\ts_nop 4\n" + ld) == []
    assert hazards(rd + "\ts_add_u32 s0, s0, s1\n" * 5 + ld) == []
    # a scalar consumer is interlocked
    assert hazards(rd + "\ts_mov_b32 m0, s6\n\ts_nop 0\n\tglobal_load_lds_dwordx4 v200, s[10:11]\n\ts_waitcnt vmcnt(0)\n") == []


def test_spill_inside_a_loop_is_reported_where_waits_are_counted_by_hand():
    body = (".LBB0_1:\n"
            "\tscratch_load_dword v9, off, off offset:4\n"
            "\ts_waitcnt vmcnt(0)\n"
            "\tv_add_u32_e32 v1, v1, v9\n"
            "\ts_cbranch_scc1 .LBB0_1\n")
    hz = hazards(body)
    assert len(hz) == 1 and "spill inside a loop" in hz[0]
    # outside a loop a spill is only slow
    assert hazards("\tscratch_load_dword v9, off, off offset:4\n\ts_waitcnt vmcnt(0)\n") == []
    # and a source whose waits are all the compiler's is not held to this
    n, hz = C.check_text(HEAD + body + TAIL, counters=())
    assert n == 1 and hz == []


def test_sources_with_hand_counted_loads_are_found_and_clean():
    checked = {s: C.hand_counted(os.path.join(B.CSRC, s)) for s in B.SOURCES}
    checked = {s: c for s, c in checked.items() if c}
    assert checked["rmsnorm_gemm.hip"] == ("vm", "lgkm") and checked["fp8_quant_gemm.hip"] == ("vm", "lgkm")
    assert checked["attention_bf16.hip"] == ("lgkm",)
    try:
        cc = B.hipcc()
    except RuntimeError:
        pytest.skip("hipcc not found")
    for s in checked:
        n, hz = C.check_source(os.path.join(B.CSRC, s), cc, B.HIPCC_FLAGS)
        assert n >= 1 and hz == [], (s, hz[:5])
