"""Static check of the generated gfx950 code for hazards the compiler cannot see.

The decode kernels issue their MFMAs from inline assembly, so the compiler's hazard
recognizer does not know that the registers they write are not readable for a
number of wait states (12 after an 8-pass MFMA for a vector-ALU read, 20 after a
16-pass one, more for a memory instruction).  Our own code supplies the `s_nop`s where it reads results;
this check guards against compiler-inserted code (register moves, spills) that
touches an MFMA destination too early.  It walks each decode kernel's
instruction stream in program order, conservatively assuming fall-through, and
fails the build if a non-MFMA instruction names a register of an MFMA
destination fewer than `MIN_STATES` wait states after that MFMA.
"""
import re
import sys

VALU_STATES = 12  # vector-ALU read of an 8-pass MFMA result
MEM_STATES = 19   # memory / LDS / export instruction reading it
MIN_STATES = VALU_STATES
EXTRA_16_PASS = 8  # a 16-pass MFMA (the 32x32x64 8-bit one) needs this many more of each
_MEM_PREFIXES = ("scratch_", "global_", "buffer_", "flat_", "ds_")

_REG_RANGE = re.compile(r"\b([av])\[(\d+):(\d+)\]")
_REG_ONE = re.compile(r"\b([av])(\d+)\b")


def _regs(text):
    out = set()
    for k, lo, hi in _REG_RANGE.findall(text):
        out.update((k, i) for i in range(int(lo), int(hi) + 1))
    for k, i in _REG_ONE.findall(_REG_RANGE.sub(" ", text)):
        out.add((k, int(i)))
    return out


def check(asm_text, kernel_filter="decode_kernel"):
    """Returns a list of violation strings (empty = fine)."""
    problems = []
    # 1. no register spill traffic inside a basic block that runs part of the MFMA stream: a
    #    spill reload waits on the vector-memory counter and would drain the tile prefetch.
    block, name, in_k = [], None, False
    for raw in asm_text.splitlines() + ["end:"]:
        line = raw.split(";")[0].strip()
        if line.endswith(":"):
            # (a spill access behind a block's last MFMAs, e.g. after the final PV, is harmless)
            first = next((i for i, l in enumerate(block) if l.startswith("scratch_")), None)
            if in_k and first is not None and sum(l.startswith("v_mfma") for l in block[first:]) >= 8:
                problems.append(f"register spill traffic in front of MFMAs in block {name}")
            if not line.startswith("."):
                in_k = kernel_filter in line
            block, name = [], line
        elif line:
            block.append(line)
    # 2. MFMA results read too early
    in_kernel = False
    pending = {}  # register -> wait states elapsed since the MFMA that writes it
    extra = {}    # register -> additional wait states its MFMA needs (16-pass)
    for lineno, raw in enumerate(asm_text.splitlines(), 1):
        line = raw.split(";")[0].strip()
        if not line:
            continue
        if line.endswith(":") and not line.startswith("."):
            in_kernel = kernel_filter in line
            pending = {}
            continue
        if not in_kernel or line.startswith(".") or line.endswith(":"):
            continue
        op, _, rest = line.partition(" ")
        if op.startswith("v_mfma"):
            operands = [x.strip() for x in rest.split(",")]
            dst = _regs(operands[0])
            srcs = _regs(",".join(operands[1:3]))  # A and B must be readable; C may chain
            for r in srcs:
                if r in pending and pending[r] < MIN_STATES + extra.get(r, 0):
                    problems.append(f"line {lineno}: MFMA reads {r} {pending[r]} states after an MFMA wrote it: {line}")
            for r in list(pending):
                pending[r] += 1
            for r in dst:
                pending[r] = 0
                extra[r] = EXTRA_16_PASS if "32x32x64" in op else 0
            continue
        states = 1
        if op == "s_nop":
            states = int(rest.strip()) + 1
        else:
            need = MEM_STATES if op.startswith(_MEM_PREFIXES) else VALU_STATES
            operands = rest.split(",")
            writes_first = (op.startswith("v_") and not op.startswith("v_cmp")) or "_load" in op or \
                op.startswith("ds_read") or op.startswith("ds_bpermute")
            read_text = ",".join(operands[1:]) if writes_first else rest
            for r in sorted(_regs(read_text)):
                if r in pending and pending[r] < need + extra.get(r, 0):
                    problems.append(f"line {lineno}: {pending[r]} wait states after MFMA write of "
                                    f"{r[0]}{r[1]}: {line}")
            if writes_first:  # overwritten: later uses no longer see the MFMA's result
                for r in sorted(_regs(operands[0])):
                    if r in pending:
                        if pending[r] < VALU_STATES + extra.get(r, 0):
                            problems.append(f"line {lineno}: overwrite {pending[r]} wait states after MFMA "
                                            f"write of {r[0]}{r[1]}: {line}")
                        del pending[r]
        for r in list(pending):
            pending[r] += states
            if pending[r] >= 64:
                del pending[r]
        if op in ("s_endpgm",):
            in_kernel = False
    return problems


if __name__ == "__main__":
    probs = check(open(sys.argv[1]).read())
    print("\n".join(probs[:40]) or "ok")
    sys.exit(1 if probs else 0)
