"""Host-side check of the tiled kernels' machine code (no GPU needed: hipcc cross-compiles).

The tiled decode-GEMM waits by hand for loads it issues from inline assembly; this test compiles
it and verifies that the compiler left the in-flight registers alone (see check_tile_isa.py in
this folder for the reasoning)."""
import shutil

import pytest

import check_tile_isa


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not installed")
def test_tile_kernel_in_flight_registers(tmp_path):
    asm = tmp_path / "tile_gemm.s"
    check_tile_isa.compile_to_asm(str(asm))
    n_loops, n_exits, problems = check_tile_isa.check(asm.read_text())
    assert not problems, problems[:5]
    # every instantiation of the kernel holds the K loops its template arguments imply, and every
    # loop and every loop exit was checked
    per_kernel = check_tile_isa.loops_by_kernel(asm.read_text())
    # 2 stages x (packed and persistent packed, each with either form of H; shared; unmerged and persistent unmerged)
    assert len(per_kernel) >= 14, sorted(per_kernel)
    for name, n in per_kernel.items():
        assert n == check_tile_isa.expected_loops(name), (name, n)
    assert n_loops == sum(per_kernel.values()) and n_exits == n_loops, (n_loops, n_exits)


def test_checker_flags_a_planted_copy():
    """The checker itself: a copy of a register that an asm load has just written is reported."""
    body = ["\tv_mfma_f32_16x16x32_bf16 v[0:3], v[4:7], v[8:11], v[0:3]"] * 8
    text = "\n".join([".LBB0_1:                                ; =>This Inner Loop Header: Depth=1"] + body + [
        "\t;;#ASMSTART", "\tglobal_load_dwordx4 v[20:23], v1, s[2:3]", "\t;;#ASMEND",
        "\ts_barrier", "\tv_mov_b32_e32 v30, v21", "\ts_barrier",
        "\ts_cbranch_scc1 .LBB0_1"])
    n_loops, _, problems = check_tile_isa.check(text)
    assert n_loops == 1 and len(problems) == 1 and "v_mov_b32" in problems[0]
    clean = text.replace("v_mov_b32_e32 v30, v21", "v_mov_b32_e32 v30, v31")
    assert check_tile_isa.check(clean)[2] == []


def test_checker_flags_scratch_in_a_loop():
    """A spill reload inside a K loop is a load that the hand-written waits do not count."""
    body = ["\tv_mfma_f32_16x16x32_bf16 v[0:3], v[4:7], v[8:11], v[0:3]"] * 8
    text = "\n".join([".LBB0_1:                                ; =>This Inner Loop Header: Depth=1"] + body + [
        "\t;;#ASMSTART", "\tglobal_load_dwordx4 v[20:23], v1, s[2:3]", "\t;;#ASMEND",
        "\ts_barrier", "\tscratch_load_dword v30, off, off", "\ts_barrier",
        "\ts_cbranch_scc1 .LBB0_1"])
    problems = check_tile_isa.check(text)[2]
    assert len(problems) == 1 and "scratch" in problems[0]


def test_checker_follows_the_waits():
    """A register is in flight from its load to the wait that covers it: a read after `vmcnt(0)` is
    fine, a read after a wait that still allows the load to be out is reported, and so is a read at
    the top of the loop of what the previous trip left in flight."""
    hdr = ".LBB0_1:                                ; =>This Inner Loop Header: Depth=1"
    mfma = ["\tv_mfma_f32_16x16x32_bf16 v[0:3], v[4:7], v[8:11], v[0:3]"] * 4
    load = ["\t;;#ASMSTART", "\tglobal_load_dwordx4 v[20:23], v1, s[2:3]", "\t;;#ASMEND"]
    lds_load = ["\t;;#ASMSTART", "\tglobal_load_lds_dwordx4 v1, s[2:3]", "\t;;#ASMEND"]
    def prog(wait, use_at_top=False):
        top = ["\tv_mov_b32_e32 v30, v21"] if use_at_top else []
        return "\n".join([hdr] + top + mfma + load + lds_load + ["\ts_barrier"] +
                         ["\t;;#ASMSTART", "\ts_waitcnt vmcnt(%d)" % wait, "\t;;#ASMEND"] +
                         ([] if use_at_top else ["\tv_mov_b32_e32 v30, v21"]) + mfma + ["\ts_barrier", "\ts_cbranch_scc1 .LBB0_1"])
    assert check_tile_isa.check(prog(1))[2] == []            # one load may be out: the younger one, into LDS
    bad = check_tile_isa.check(prog(2))[2]                    # two may be out: v[20:23] may still be in flight
    assert len(bad) == 1 and "v_mov_b32" in bad[0]
    assert check_tile_isa.check(prog(0))[2] == []
    bad = check_tile_isa.check(prog(2, use_at_top=True))[2]   # left in flight by the previous trip
    assert len(bad) == 1 and "v_mov_b32" in bad[0]
    assert check_tile_isa.check(prog(1, use_at_top=True))[2] == []


def test_checker_accepts_only_dead_lane_reads():
    """A lane-0 read of an in-flight register into a scalar register is how the compiler
    materialises an undefined value; it is accepted only if that scalar is overwritten before it is
    read on every path (here: the loop continues and redefines it, or the exit path ends)."""
    body = ["\tv_mfma_f32_16x16x32_bf16 v[0:3], v[4:7], v[8:11], v[0:3]"] * 8
    def prog(after_exit):
        return "\n".join([".LBB0_1:                                ; =>This Inner Loop Header: Depth=1", "\ts_add_i32 s9, s8, 2"] + body + [
            "\t;;#ASMSTART", "\tglobal_load_dwordx4 v[20:23], v1, s[2:3]", "\t;;#ASMEND",
            "\ts_barrier", "\ts_barrier",
            "\ts_mov_b64 s[4:5], -1", "\ts_cmp_ge_i32 s9, s10",
            "\tv_readfirstlane_b32 s9, v20",
            "\ts_cbranch_scc0 .LBB0_1",                    # continue: s9 is redefined at the top
            "\ts_andn2_b64 vcc, exec, s[4:5]", "\ts_mov_b32 s8, s9",
            "\ts_cbranch_vccnz .LBB0_1",                   # not taken: vcc is zero on this path
            ".LBB0_2:"] + after_exit + ["\ts_endpgm"])
    assert check_tile_isa.check(prog([]))[2] == []
    # a vector compare in its 64-bit encoding overwrites its scalar destination: still dead
    assert check_tile_isa.check(prog(["\tv_cmp_gt_f32_e64 s[8:9], |v1|, s6"]))[2] == []
    bad = check_tile_isa.check(prog(["\ts_add_i32 s11, s9, 1"]))[2]          # the value is used
    assert bad and all("v_readfirstlane" in b for b in bad)

