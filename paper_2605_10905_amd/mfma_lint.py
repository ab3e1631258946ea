"""Build-time check of hand-written MFMA instructions in the generated gfx950 assembly.

The compiler inserts the wait states the hardware needs between a matrix instruction and a vector
instruction that touches its result, but only for matrix instructions it issued itself: the ones
written as inline assembly are opaque to it.  This scans the assembly of a translation unit and
reports every instruction outside an assembly statement that reads or writes a vector register
within WAIT_STATES instructions of an inline-assembly MFMA that wrote it (each instruction counts
one wait state, s_nop N counts N + 1).  In-place accumulation by a later assembly MFMA is allowed.
"""
import re
import sys

WAIT_STATES = 11  # an 8-pass MFMA result read or overwritten by a vector instruction

_RANGE = re.compile(r"\bv\[(\d+):(\d+)\]")
_SINGLE = re.compile(r"\bv(\d+)\b")


def _vregs(text):
    regs = set()
    for lo, hi in _RANGE.findall(text):
        regs.update(range(int(lo), int(hi) + 1))
    for r in _SINGLE.findall(_RANGE.sub(" ", text)):
        regs.add(int(r))
    return regs


def lint(asm_text):
    """Returns a list of (line number, line, registers) violations."""
    pending = {}  # register -> wait states still needed
    in_asm = False
    bad = []
    for n, raw in enumerate(asm_text.split("\n"), 1):
        line = raw.strip()
        if line.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if line.startswith(";;#ASMEND"):
            in_asm = False
            continue
        code = line.split(";")[0].strip()
        if not code or code.endswith(":") or code.startswith("."):
            if code.endswith(":") and code.startswith("_Z"):
                pending = {}  # a new function
            continue
        parts = code.split(None, 1)
        mnem, ops = parts[0], (parts[1] if len(parts) > 1 else "")
        if in_asm and mnem.startswith("v_mfma"):
            fields = [f.strip() for f in ops.split(",")]
            dst = _vregs(fields[0])
            hit = _vregs(",".join(fields[1:3])) & set(pending)
            if hit:
                bad.append((n, raw, sorted(hit)))
            if len(fields) > 3 and _vregs(fields[3]) not in (set(), dst):
                bad.append((n, raw, sorted(_vregs(fields[3]))))  # accumulates into other registers than it reads
            for r in list(pending):
                pending[r] -= 1
            for r in dst:
                pending[r] = WAIT_STATES
        else:
            hit = _vregs(ops) & set(pending)
            if hit and not mnem.startswith("s_"):
                bad.append((n, raw, sorted(hit)))
            dec = int(ops.strip(), 0) + 1 if mnem == "s_nop" else 1
            for r in list(pending):
                pending[r] -= dec
        pending = {r: w for r, w in pending.items() if w > 0}
    return bad


def main(argv):
    bad = []
    for path in argv[1:]:
        with open(path) as f:
            for n, raw, regs in lint(f.read()):
                bad.append(f"{path}:{n}: {raw.strip()}   <- touches v{regs} too soon after an inline MFMA")
    for b in bad:
        print(b)
    return 1 if bad else 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
