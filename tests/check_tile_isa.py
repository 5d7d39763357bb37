"""Static check of the tiled kernels' machine code.

The tiled decode-GEMM issues its weight loads from inline assembly and waits for them two K steps
later, by hand.  Between the load and that wait the destination registers are "in flight": the
hardware may write them at any time, and the compiler does not know it.  The kernel is written so
that the compiler has no reason to touch those registers in between (the refill is an in/out
operand of registers whose old contents are dead), but nothing in the language guarantees it: a
copy, a spill or a re-use of such a register would read stale data or, worse, let the late load
overwrite an unrelated value such as an address.

This module compiles `csrc/tile_gemm.hip` to gfx950 assembly and verifies, for every K loop, that
no instruction names a destination register of an inline-asm `global_load_dwordx4` between the
load and the hand-written wait that covers it, across the loop's back edge too (one exception: a lane-0 read into a scalar register that is
overwritten before it is read on every path, which is how the compiler materialises an undefined
value), that every loop exit waits for all loads before any vector instruction, that nothing
spills, and that no K loop touches scratch memory (a reload there would be a load the waits do not
count).  A developer tool that lives with its test (test_tile_isa.py), not in the product
package.  Run it after any change to the kernel or the compiler:

    python tests/check_tile_isa.py
"""
import os
import re
import subprocess
import sys
import tempfile

_ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if _ROOT not in sys.path:
    sys.path.insert(0, _ROOT)
_CSRC = os.path.join(_ROOT, "paper_2511_04805_amd", "csrc")
_REG = re.compile(r"v\[(\d+):(\d+)\]|\bv(\d+)\b")


def compile_to_asm(out_path):
    from paper_2511_04805_amd.build import FLAGS as HIPCC_FLAGS  # the flags the library is built with
    cmd = ["hipcc"] + HIPCC_FLAGS + ["-S", "--cuda-device-only", "-o", out_path,
                                     os.path.join(_CSRC, "tile_gemm.hip")]
    subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.PIPE)


def _regs(text):
    out = set()
    for m in _REG.finditer(text):
        if m.group(1):
            out.update(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


_SREG = re.compile(r"s\[(\d+):(\d+)\]|\bs(\d+)\b")


def _sregs(text):
    out = set()
    for m in _SREG.finditer(text):
        if m.group(1):
            out.update(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


def _scalar_dead(lines, labels, i, reg, seen, budget, ones=frozenset(), vcc_zero=False):
    """True if scalar register `reg` is overwritten before it is read on every feasible path from
    line i (a plain copy into another scalar register is followed: the copy must be dead too).
    `ones`: scalar registers known to hold all ones on the current straight-line path, which is
    how the compiler flags "this is the exit path": vcc = exec & ~ones is then zero and a branch
    on vcc non-zero is not taken."""
    ones = set(ones)
    while i < len(lines):
        budget[0] -= 1
        if budget[0] <= 0:
            return False
        t = lines[i].split(";")[0].strip()
        i += 1
        if not t or (t.startswith(".") and not t.endswith(":")):
            continue
        if t.endswith(":"):                      # a join point: forget what was known
            ones.clear()
            vcc_zero = False
            continue
        parts = t.replace(",", " ").split()
        op, ops = parts[0], parts[1:]
        if op == "s_endpgm":
            return True
        if op in ("s_setpc_b64", "s_swappc_b64"):
            return False
        if re.match(r"(s_cbranch_\w+|s_branch)$", op):
            if op == "s_cbranch_vccnz" and vcc_zero:
                continue                          # not taken
            tgt = labels.get(ops[0])
            if tgt is None:
                return False
            key = (tgt, reg)
            if key not in seen:
                seen.add(key)
                if not _scalar_dead(lines, labels, tgt, reg, seen, budget):
                    return False
            if op == "s_branch" or (op == "s_cbranch_vccz" and vcc_zero):
                return True
            continue
        # (a vector compare in its 64-bit encoding names its scalar destination first; the 32-bit
        # encoding writes vcc implicitly)
        writes_first = (re.match(r"v_cmp_\w+_e64$", op) is not None or
                        not re.match(r"(s_cmp|s_bitcmp|s_waitcnt|s_nop|s_barrier|s_sleep|s_setprio|v_cmp|v_cmpx|global_|ds_|buffer_|scratch_|flat_)", op))
        read_text = " ".join(ops[1:]) if (writes_first and ops) else " ".join(ops)
        if reg in _sregs(read_text):
            if op == "s_mov_b32" and len(ops) == 2 and _sregs(ops[1]) == {reg} and len(_sregs(ops[0])) == 1:
                if not _scalar_dead(lines, labels, i, next(iter(_sregs(ops[0]))), seen, budget, frozenset(ones), vcc_zero):
                    return False
                continue
            return False
        if op == "s_andn2_b64" and len(ops) == 3 and ops[0] == "vcc" and ops[1] == "exec" and _sregs(ops[2]) and _sregs(ops[2]) <= ones:
            vcc_zero = True
        elif writes_first and ops and ops[0] == "vcc" or (op.startswith("v_cmp") and not op.endswith("_e64")):
            vcc_zero = False
        if writes_first and ops:
            w = _sregs(ops[0])
            if op == "s_mov_b64" and len(ops) == 2 and ops[1] == "-1":
                ones |= w
            else:
                ones -= w
            if reg in w:
                return True
    return False


def _known_ones(lines, i):
    """Scalar registers set to all ones by an s_mov_b64 in the straight-line code just above line i
    and not written since."""
    ones, written = set(), set()
    j = i - 1
    while j >= 0:
        t = lines[j].split(";")[0].strip()
        j -= 1
        if not t:
            continue
        if t.endswith(":") or re.match(r"s_c?branch", t):
            break
        parts = t.replace(",", " ").split()
        if parts[0].startswith(("s_cmp", "s_bitcmp", "s_waitcnt", "s_nop", "v_cmp", "global_", "ds_")) or len(parts) < 2:
            continue
        w = _sregs(parts[1])
        if parts[0] == "s_mov_b64" and len(parts) == 3 and parts[2] == "-1":
            ones |= (w - written)
        written |= w
    return frozenset(ones)


def _k_loops(lines, labels):
    """(first line, line of the last backward branch) of every K loop.  A loop is a header label (the
    compiler marks it) with the blocks it notes as belonging to that header; its extent in the text
    runs from the first of these that a backward branch names to the last such branch (the
    compiler may rotate a loop, or place its exit blocks in front of the header).  K loops are those
    whose extent holds matrix instructions, inline-asm weight loads, two or four barriers (two or
    four K steps per trip) and no store."""
    header_of = {}
    for name, at in labels.items():
        if _is_loop_header(lines, at):
            header_of[name] = name
        else:
            m = re.search(r"in Loop: Header=(BB\d+_\d+)", lines[at])
            if m:
                header_of[name] = ".L" + m.group(1)
    extent = {}
    for i, l in enumerate(lines):
        m = re.match(r"\s+s_(?:cbranch_\w+|branch)\s+(\.LBB\d+_\d+)", l)   # (the back edge may be an unconditional branch to a latch block placed in front of the header)
        if not m or labels.get(m.group(1), i) >= i or m.group(1) not in header_of:
            continue
        h = header_of[m.group(1)]
        lo, hi = extent.get(h, (labels[m.group(1)], i))
        extent[h] = (min(lo, labels[m.group(1)]), max(hi, i))
    for start, i in sorted(extent.values()):
        body = lines[start:i]
        if (sum("v_mfma" in b for b in body) < 2 or not any("global_load_dwordx4" in b for b in body)
                or sum("s_barrier" in b for b in body) not in (2, 4) or any("global_store" in b for b in body)):
            continue
        yield start, i


def _is_loop_header(lines, at):
    """The compiler's own note on a label: a loop header (the note may follow on the next comment
    line, after the parent loop's), as opposed to a block that merely belongs to a loop."""
    j = at
    while j < len(lines) and (j == at or lines[j].strip().startswith(";")):
        if re.search(r"=>\s*This (Inner )?Loop Header", lines[j]):
            return True
        j += 1
    return False


def _labels(lines):
    labels = {}
    for i, l in enumerate(lines):
        m = re.match(r"^(\.LBB\d+_\d+):", l)
        if m:
            labels[m.group(1)] = i
    return labels


def loops_by_kernel(asm_text):
    """{mangled kernel name: number of K loops found in it}, for every tile_kernel in the text."""
    lines = asm_text.split("\n")
    starts = [(i, m.group(1)) for i, l in enumerate(lines) for m in [re.match(r"^(_Z\w*tile_kernel\w*):", l)] if m]
    out = {name: 0 for _, name in starts}
    for start, _ in _k_loops(lines, _labels(lines)):
        owner = [name for i, name in starts if i <= start]
        if owner:
            out[owner[-1]] += 1
    return out


def expected_loops(mangled):
    """K loops a tile_kernel<STAGE, DENSE, ALLTOK, PERSIST, HALF> instantiation must contain, from its
    template arguments: one per (expert position, number of token-fragment pairs 1..9) and one more
    per (position, 5..9 pairs the last fragment of which is padding); dense weights have one
    position only; kernels of packed pairs also hold the 3 sizes of the tile that covers both
    experts of a pair."""
    m = re.search(r"tile_kernelILi(\d)ELb(\d)ELb(\d)ELb(\d)ELb(\d)E", mangled)
    assert m, mangled
    dense = m.group(2) == "1"
    return 9 + 5 if dense else 2 * (9 + 5) + 3


def check(asm_text):
    """Returns (number of K loops checked, number of loop exits checked, list of problems)."""
    lines = asm_text.split("\n")
    problems = []
    for l in lines:
        m = re.search(r"\.vgpr_spill_count:\s+(\d+)", l)
        if m and int(m.group(1)):
            problems.append("register spills: %s" % l.strip())
    labels = _labels(lines)
    n_loops = 0
    for start, i in _k_loops(lines, labels):
        body = lines[start:i]
        n_loops += 1
        # A spill inside a K loop would not only be slow: its reload is a load that the hand-written
        # waits do not count, so every wait after it would let one more weight load stay out.
        for k, b in enumerate(body):
            if re.match(r"\s*scratch_", b):
                problems.append("line %d: scratch access inside a K loop: %s" % (start + k + 1, b.strip()))
        # Loads complete in issue order and the waits name how many of the youngest may still be
        # out: keep the queue of outstanding loads (destination registers of the inline-asm weight
        # loads; nothing for a load into LDS) and drop from its old end at every wait.  Three trips
        # through the body (which may be rotated), so that what the end of a trip leaves in flight
        # meets the start of the next in the steady state.
        outstanding = []
        seen = set()
        for trip in range(3):
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
                mw = re.search(r"s_waitcnt.*vmcnt\((\d+)\)", t)
                if mw:
                    del outstanding[:max(0, len(outstanding) - int(mw.group(1)))]
                    continue
                is_load = in_asm and re.search(r"global_load_dwordx4\s+v", t) is not None
                inflight = set().union(*outstanding) if outstanding else set()
                hit = _regs(t) & inflight
                if hit and not is_load and (k, tuple(sorted(hit))) not in seen:
                    seen.add((k, tuple(sorted(hit))))
                    # The compiler materialises an undefined scalar (a loop-carried value on an exit
                    # path) by reading lane 0 of any vector register.  Reading an in-flight register
                    # does not disturb the load; it is accepted only if the scalar is provably dead.
                    mrf = re.match(r"\s*v_readfirstlane_b32\s+s(\d+),\s*v\d+\s*$", t)
                    if not (mrf and _scalar_dead(lines, labels, start + k + 1, int(mrf.group(1)), set(), [60000],
                                                 _known_ones(lines, start + k))):
                        problems.append("line %d touches in-flight v%s: %s" % (start + k + 1, sorted(hit)[:4], t.strip()))
                if is_load:
                    m2 = re.search(r"global_load_dwordx4\s+v\[(\d+):(\d+)\]", t)
                    outstanding.append(set(range(int(m2.group(1)), int(m2.group(2)) + 1)))
                elif re.search(r"\b(global|buffer|flat|scratch)_load", t):
                    outstanding.append(set())                 # into LDS, or the compiler's own: counted, not tracked
    # loop exits: the hand-written "wait for everything" must be the first thing in its block
    n_exits = 0
    for i, l in enumerate(lines):
        if "s_waitcnt vmcnt(0)" in l and "end of K loop" in l and "ASMSTART" in lines[i - 1]:   # the kernel marks this wait with a comment
            j = i - 2
            seg = []
            while j > 0 and not lines[j].startswith(".LBB") and not re.search(r"s_c?branch|s_barrier", lines[j]):
                t = lines[j].strip()
                if t and not t.startswith(";"):
                    seg.append(t)
                j -= 1
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
