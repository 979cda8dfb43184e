"""Static check of compiled gfx950 assembly: results of hand-written MFMAs are not touched too early.

Some kernels issue `v_mfma_*` through inline assembly so that the accumulator lands in ordinary
registers.  The compiler's hazard recogniser does not look inside inline assembly, so nothing
stops it from scheduling, right behind such an MFMA, an instruction that reads or overwrites the
registers the MFMA is still going to write (a register-allocator copy is enough).  On this
hardware that is silent data corruption, not an error.  The kernels place explicit waits; this
script proves, on the assembly the build actually produced, that they suffice.

For every MFMA between `;;#ASMSTART` and `;;#ASMEND` whose destination is a VGPR range it walks
forward through the listing (straight-line: labels and branches are ignored, which over-approximates)
counting wait states (one per instruction, N + 1 for `s_nop N`) and reports any non-MFMA
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


def check(asm_text, need=12, need_16_pass=20, horizon=64):
    """Returns a list of (function, line number within the function, instruction, wait states so far)."""
    problems = []
    func, in_asm, pending, ln = None, False, [], 0
    for raw in asm_text.split("\n"):
        m = re.match(r"^(_Z\w+):", raw)
        if m:
            func, in_asm, pending, ln = m.group(1), False, [], 0
            continue
        if func is None:
            continue
        ln += 1
        stripped = raw.strip()
        if stripped.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if stripped.startswith(";;#ASMEND"):
            in_asm = False
            continue
        text = raw.split(";")[0].strip()
        if not text or text.startswith(".") or text.endswith(":"):
            continue
        op = text.split()[0]
        args = text[len(op):]
        states = int(args.strip()) + 1 if op == "s_nop" else 1
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
            if in_asm and dst:
                pending = [p for p in pending if p[0] != dst]
                pending.append([dst, 0, need_16_pass if "f8f6f4" in op else need])
        else:
            touched = _vgprs(args)
            for regs, waited, req in pending:
                if regs & touched and waited < req:
                    problems.append((func, ln, text, waited))
            pending = [[regs, waited + states, req] for regs, waited, req in pending]
        pending = [p for p in pending if p[1] < horizon]
    return problems


def main(argv):
    bad = 0
    for path in argv[1:]:
        for func, ln, text, waited in check(open(path).read()):
            print(f"{path}: {func} +{ln}: `{text}` only {waited} wait states after the MFMA that writes its registers")
            bad += 1
    return 1 if bad else 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
