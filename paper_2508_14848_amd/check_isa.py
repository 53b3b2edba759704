"""Build-time check of the 128 x 128 GEMM kernels' machine code (gfx950 assembly from hipcc -S).

The FP32 matrix instructions of the FP64 / FP32 product loops are written as inline assembly with
their accumulators as in/out operands, so that a run of them updates its accumulators in place.
The compiler does not see an inline-assembly instruction's latencies: should the register
allocator move such an accumulator to another register in the middle of a run (it may, under
register pressure), the copy would sit next to matrix instructions without the wait states the
hardware asks for, and read or overwrite a value in flight.  Nothing in the source can forbid
that, so the build looks: in every basic block that holds such matrix instructions, no other
instruction between the first and the last of them may name one of their accumulator registers.
"""
import re
import sys

_REG = re.compile(r"\b([va])\[(\d+):(\d+)\]|\b([va])(\d+)\b")


def _regs(text):
    out = set()
    for m in _REG.finditer(text):
        if m.group(1):
            out.update((m.group(1), r) for r in range(int(m.group(2)), int(m.group(3)) + 1))
        else:
            out.add((m.group(4), int(m.group(5))))
    return out


def violations(asm_path, mnemonic="v_mfma_f32_16x16x4_f32"):
    """Returns (basic blocks with such matrix instructions, offending instructions)."""
    blocks, block = [], []
    for raw in open(asm_path):
        line = raw.split(";")[0].strip()
        if not line or (line.startswith(".") and not line.endswith(":")):
            continue
        if line.endswith(":") or line.startswith("s_cbranch") or line.startswith("s_branch") or line.startswith("s_endpgm"):
            blocks.append(block)
            block = []
            continue
        block.append(line)
    blocks.append(block)
    n, bad = 0, []
    for block in blocks:
        acc = set()
        for line in block:
            if line.startswith(mnemonic):
                acc |= _regs(line.split(None, 1)[1].split(",")[0])        # the destination, which is also the addend
        if not acc:
            continue
        n += 1
        runs = [k for k, line in enumerate(block) if line.startswith(mnemonic)]
        for line in block[runs[0]:runs[-1]]:                             # what lies between the first and the last of them
            if not line.startswith("v_mfma") and _regs(line) & acc:
                bad.append(line)
    return n, bad


if __name__ == "__main__":
    for path in sys.argv[1:]:
        n, bad = violations(path)
        print(path, "blocks:", n, "violations:", len(bad))
        for line in bad[:10]:
            print("   ", line)
        if bad:
            sys.exit(1)
