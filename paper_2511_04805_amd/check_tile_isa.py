"""Static check of the tiled kernels' machine code.

The tiled decode-GEMM issues its weight loads from inline assembly and waits for them two K steps
later, by hand.  Between the load and that wait the destination registers are "in flight": the
hardware may write them at any time, and the compiler does not know it.  The kernel is written so
that the compiler has no reason to touch those registers in between (the refill is an in/out
operand of registers whose old contents are dead), but nothing in the language guarantees it: a
copy, a spill or a re-use of such a register would read stale data or, worse, let the late load
overwrite an unrelated value such as an address.

This module compiles `csrc/tile_gemm.hip` to gfx950 assembly and verifies, for every K loop, that
no instruction after an inline-asm `global_load_dwordx4` names one of its destination registers
before the loop wraps around, that every loop exit waits for all loads before any vector
instruction, and that nothing spills.  Run it after any change to the kernel or the compiler:

    python -m paper_2511_04805_amd.check_tile_isa
"""
import os
import re
import subprocess
import sys
import tempfile

_HERE = os.path.dirname(os.path.abspath(__file__))
_REG = re.compile(r"v\[(\d+):(\d+)\]|\bv(\d+)\b")


def compile_to_asm(out_path):
    from .build import FLAGS as HIPCC_FLAGS  # the flags the library is built with
    cmd = ["hipcc"] + HIPCC_FLAGS + ["-S", "--cuda-device-only", "-o", out_path,
                                     os.path.join(_HERE, "csrc", "tile_gemm.hip")]
    subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.PIPE)


def _regs(text):
    out = set()
    for m in _REG.finditer(text):
        if m.group(1):
            out.update(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


def check(asm_text):
    """Returns (number of K loops checked, number of loop exits checked, list of problems)."""
    lines = asm_text.split("\n")
    problems = []
    for l in lines:
        m = re.search(r"\.vgpr_spill_count:\s+(\d+)", l)
        if m and int(m.group(1)):
            problems.append("register spills: %s" % l.strip())
    labels = {}
    for i, l in enumerate(lines):
        m = re.match(r"^(\.LBB\d+_\d+):", l)
        if m:
            labels[m.group(1)] = i
    n_loops = 0
    for i, l in enumerate(lines):
        m = re.match(r"\s+s_cbranch_\w+\s+(\.LBB\d+_\d+)", l)
        if not m or labels.get(m.group(1), i) >= i:
            continue
        start = labels[m.group(1)]
        body = lines[start:i]
        if (sum("v_mfma" in b for b in body) < 8 or not any("global_load_dwordx4" in b for b in body)
                or sum("s_barrier" in b for b in body) != 2 or any("global_store" in b for b in body)):
            continue                                          # not a K loop (two steps per trip)
        n_loops += 1
        inflight = set()
        in_asm = False
        for k, b in enumerate(body):
            if "ASMSTART" in b:
                in_asm = True
                continue
            if "ASMEND" in b:
                in_asm = False
                continue
            t = b.split(";")[0]
            if not t.strip() or t.strip().startswith("."):
                continue
            is_load = in_asm and "global_load_dwordx4" in t
            hit = _regs(t) & inflight
            if hit and not is_load:
                problems.append("line %d touches in-flight v%s: %s" % (start + k + 1, sorted(hit)[:4], t.strip()))
            if is_load:
                m2 = re.search(r"global_load_dwordx4\s+v\[(\d+):(\d+)\]", t)
                inflight.update(range(int(m2.group(1)), int(m2.group(2)) + 1))
    # loop exits: the hand-written "wait for everything" must be the first thing in its block
    n_exits = 0
    for i, l in enumerate(lines):
        if "s_waitcnt vmcnt(0)" in l and "ASMSTART" in lines[i - 1]:
            j = i - 2
            seg = []
            while j > 0 and not lines[j].startswith(".LBB") and not re.search(r"s_c?branch|s_barrier", lines[j]):
                t = lines[j].strip()
                if t and not t.startswith(";"):
                    seg.append(t)
                j -= 1
            if "s_barrier" in lines[j]:
                continue                                      # the prologue's waits, not a loop exit
            n_exits += 1
            vec = [x for x in seg if re.match(r"(v_|global_|ds_|scratch_|buffer_|flat_)", x)]
            if vec:
                problems.append("line %d: vector instructions before the final wait: %s" % (i + 1, vec[:3]))
    return n_loops, n_exits, problems


def main():
    with tempfile.TemporaryDirectory() as d:
        path = os.path.join(d, "tile_gemm.s")
        compile_to_asm(path)
        n_loops, n_exits, problems = check(open(path).read())
    for p in problems[:20]:
        print(p)
    print("K loops checked: %d, loop exits checked: %d, problems: %d" % (n_loops, n_exits, len(problems)))
    return 1 if problems or n_loops == 0 or n_exits == 0 else 0


if __name__ == "__main__":
    sys.exit(main())
