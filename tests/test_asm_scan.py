"""The build's path-following check of hand-issued loads (paper_2412_14590_amd/asm_scan.py) on small
hand-written listings: it must accept a ring of loads that is awaited before use on every path, and report
a register copied or reused while its load may still be in flight - along a fall-through path, around a
loop's back edge, and when a later wait is too weak to cover the load."""
import pytest

from paper_2412_14590_amd import asm_scan

HEAD = "\t.type\tk,@function\nk:\n"
LOAD = "\t;;#ASMSTART\n\tglobal_load_dwordx4 v[{0}:{1}], v0, s[0:1] offset:0\n\t;;#ASMEND\n"
WAIT = "\t;;#ASMSTART\n\ts_waitcnt vmcnt({0})\n\t;;#ASMEND\n"
TAIL = "\ts_endpgm\n.Lfunc_end0:\n"


def scan(body):
    asm_scan.check_hand_issued_loads(HEAD + body + TAIL, "listing")


def test_a_load_awaited_before_its_use_passes():
    scan(LOAD.format(4, 7) + WAIT.format(0) + "\tv_add_u32_e32 v8, v4, v5\n")


def test_a_use_before_the_wait_is_reported():
    with pytest.raises(RuntimeError, match="v_add_u32_e32 v8, v4, v5"):
        scan(LOAD.format(4, 7) + "\tv_add_u32_e32 v8, v4, v5\n" + WAIT.format(0))


def test_an_older_load_is_retired_by_a_wait_that_leaves_the_younger_one_in_flight():
    # two loads; vmcnt(1) retires the first only
    body = LOAD.format(4, 7) + LOAD.format(8, 11) + WAIT.format(1)
    scan(body + "\tv_mov_b32_e32 v12, v4\n" + WAIT.format(0) + "\tv_mov_b32_e32 v13, v8\n")
    with pytest.raises(RuntimeError, match="v_mov_b32_e32 v13, v8"):
        scan(body + "\tv_mov_b32_e32 v12, v4\n\tv_mov_b32_e32 v13, v8\n" + WAIT.format(0))


def test_a_copy_at_a_loop_latch_of_a_register_requested_in_the_loop_is_reported():
    # the ring pattern that went wrong in a nested loop: request ahead inside the loop, copy at the latch,
    # wait at the top of the next iteration
    loop = (".LBB0_1:\n" + WAIT.format(0) + "\tv_add_u32_e32 v20, v4, v4\n" + LOAD.format(8, 11) +
            "\tv_mov_b64_e32 v[4:5], v[8:9]\n\tv_mov_b64_e32 v[6:7], v[10:11]\n"
            "\ts_add_i32 s2, s2, 1\n\ts_cmp_lt_i32 s2, s3\n\ts_cbranch_scc1 .LBB0_1\n")
    with pytest.raises(RuntimeError, match=r"v_mov_b64_e32 v\[4:5\], v\[8:9\]"):
        scan(LOAD.format(4, 7) + loop)


def test_the_same_ring_with_fixed_registers_passes():
    # two slots that keep their registers: request into one, wait for and use the other, alternating
    loop = (".LBB0_1:\n" + LOAD.format(8, 11) + WAIT.format(1) + "\tv_add_u32_e32 v20, v4, v5\n" +
            LOAD.format(4, 7) + WAIT.format(1) + "\tv_add_u32_e32 v20, v8, v9\n"
            "\ts_add_i32 s2, s2, 1\n\ts_cmp_lt_i32 s2, s3\n\ts_cbranch_scc1 .LBB0_1\n")
    scan(LOAD.format(4, 7) + loop + WAIT.format(0) + "\tv_mov_b32_e32 v30, v4\n")


def test_a_wait_skipped_on_one_path_is_reported():
    body = (LOAD.format(4, 7) + "\ts_cbranch_scc1 .LBB0_2\n" + WAIT.format(0) + ".LBB0_2:\n\tv_mov_b32_e32 v9, v4\n")
    with pytest.raises(RuntimeError, match="v_mov_b32_e32 v9, v4"):
        scan(body)


def test_loads_of_the_compiler_count_as_younger_and_stores_do_not():
    own = "\tglobal_load_dword v30, v[0:1], off\n"
    scan(LOAD.format(4, 7) + own + WAIT.format(1) + "\tv_mov_b32_e32 v9, v4\n")
    store = "\tglobal_store_dword v[0:1], v30, off\n"
    with pytest.raises(RuntimeError, match="v_mov_b32_e32 v9, v4"):
        scan(LOAD.format(4, 7) + store + WAIT.format(1) + "\tv_mov_b32_e32 v9, v4\n")
