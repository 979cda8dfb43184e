"""Static check of compiled gfx950 assembly: results of hand-written MFMAs are not touched too early.

Some kernels issue `v_mfma_*` through inline assembly so that the accumulator lands in ordinary
registers.  The compiler's hazard recogniser does not look inside inline assembly, so nothing
stops it from scheduling, right behind such an MFMA, an instruction that reads or overwrites the
registers the MFMA is still going to write (a register-allocator copy is enough).  On this
hardware that is silent data corruption, not an error.  The kernels place explicit waits; this
script proves, on the assembly the build actually produced, that they suffice.

For every MFMA between `;;#ASMSTART` and `;;#ASMEND` whose destination is a VGPR range it walks
forward through the listing in its printed order, and additionally along every branch that is taken while
the result is not yet safe (a loop's back-edge, a forward branch that skips the wait), counting wait
states (one per instruction, N + 1 for `s_nop N`), and reports any non-MFMA
instruction that names a register of that range, and any MFMA that takes it as an A or B operand,
before `need` wait states have passed.  A following MFMA that accumulates into exactly the same
range is the hardware-interlocked case and is allowed.

The 8-pass 32x32x16 MFMA needs 11 wait states before a VALU read of its result and the 16-pass
32x32x64 e4m3 MFMA 19; the compiler leaves 12 (20) or more in the code it schedules itself, and those
are the defaults here.
"""
import re
import sys

_REG_RANGE = re.compile(r"\bv\[(\d+):(\d+)\]")
_REG_ONE = re.compile(r"\bv(\d+)\b")


def _vgprs(text):
    out = set()
    for m in _REG_RANGE.finditer(text):
        out.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in _REG_ONE.finditer(text):
        out.add(int(m.group(1)))
    return out


def _parse(raw):
    """(op, args, wait states) of an instruction line, or None for anything else."""
    text = raw.split(";")[0].strip()
    if not text or text.startswith(".") or text.endswith(":"):
        return None
    op = text.split()[0]
    args = text[len(op):]
    return text, op, args, (int(args.strip()) + 1 if op == "s_nop" else 1)


def _walk(lines, labels, func, start, pending, track_new, need, need_16_pass, horizon, problems, depth):
    """Walks `lines` (of one function) from index `start` in listing order.  `pending` holds [registers,
    wait states so far, wait states required] of hand-written MFMAs whose results are not yet safe.  With
    track_new the walk covers the function and registers every hand-written MFMA it meets; without, it
    only follows the entries it was given until they are safe.  A branch taken with entries still pending
    is followed to its target with a copy of them (the listing order alone would miss the reader at a loop
    head behind a back-edge, or behind a forward branch that skips the wait)."""
    in_asm = False
    for idx in range(start, len(lines)):
        ln, raw = lines[idx]
        stripped = raw.strip()
        if stripped.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if stripped.startswith(";;#ASMEND"):
            in_asm = False
            continue
        parsed = _parse(raw)
        if parsed is None:
            continue
        text, op, args, states = parsed
        if op.startswith("v_mfma"):
            parts = [a.strip() for a in args.split(",")]
            dst, ab = _vgprs(parts[0]), _vgprs(parts[1]) | _vgprs(parts[2])
            src_c = _vgprs(parts[3]) if len(parts) > 3 else set()
            for regs, waited, req in pending:
                if regs & ab and waited < req:
                    problems.append((func, ln, text, waited))
                if regs & src_c and regs != src_c and waited < req:
                    problems.append((func, ln, text, waited))
            pending = [[regs, waited + states, req] for regs, waited, req in pending]
            if track_new and in_asm and dst:
                pending = [p for p in pending if p[0] != dst]
                pending.append([dst, 0, need_16_pass if "f8f6f4" in op else need])
        else:
            touched = _vgprs(args)
            for regs, waited, req in pending:
                if regs & touched and waited < req:
                    problems.append((func, ln, text, waited))
            pending = [[regs, waited + states, req] for regs, waited, req in pending]
            if op.startswith("s_cbranch") or op == "s_branch":
                unsafe = [list(p) for p in pending if p[1] < p[2]]
                target = labels.get(args.strip())
                if unsafe and target is not None and depth < 4:
                    _walk(lines, labels, func, target, unsafe, False, need, need_16_pass, horizon, problems, depth + 1)
                if op == "s_branch" and not track_new:
                    return  # an unconditional branch: the followed entries continue at the target only
        pending = [p for p in pending if p[1] < horizon]
        if not track_new and all(p[1] >= p[2] for p in pending):
            return


def check(asm_text, need=12, need_16_pass=20, horizon=64):
    """Returns a list of (function, line number within the function, instruction, wait states so far)."""
    problems = []
    funcs, cur = [], None
    for raw in asm_text.split("\n"):
        m = re.match(r"^(_Z\w+):", raw)
        if m:
            cur = (m.group(1), [], {})
            funcs.append(cur)
            continue
        if cur is None:
            continue
        name, lines, labels = cur
        lab = re.match(r"^(\.\w+):", raw)
        if lab:
            labels[lab.group(1)] = len(lines)
        lines.append((len(lines) + 1, raw))
    for name, lines, labels in funcs:
        _walk(lines, labels, name, 0, [], True, need, need_16_pass, horizon, problems, 0)
    return sorted(set(problems), key=problems.index)


def main(argv):
    bad = 0
    for path in argv[1:]:
        for func, ln, text, waited in check(open(path).read()):
            print(f"{path}: {func} +{ln}: `{text}` only {waited} wait states after the MFMA that writes its registers")
            bad += 1
    return 1 if bad else 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
