"""Build-time check of the hand-issued MFMA instructions in the attention kernel.

The compiler does not know that an inline-asm statement is a matrix instruction, so it inserts none of the wait states
the hardware needs between a vector instruction that writes a register and a matrix instruction that reads it, nor
between a matrix instruction and a vector instruction that reads its result.  The kernel is written so that neither
happens (operands resident long before use, results consumed a whole pipeline step later); this script reads the
generated assembly and fails the build if the compiler placed a copy next to one of those instructions after all.
"""
from __future__ import annotations

import re
import sys

OPERAND_GAP = 2     # instructions (wait states) between a vector write of an operand register and the matrix instruction reading it
RESULT_GAP = 12     # instructions between the matrix instruction and a vector read of its result

_REG = re.compile(r"\b([va])(?:\[(\d+):(\d+)\]|(\d+))")


def _regs(text: str):
    out = set()
    for m in _REG.finditer(text):
        lo = int(m.group(2) if m.group(2) is not None else m.group(4))
        hi = int(m.group(3) if m.group(3) is not None else m.group(4))
        out.update((m.group(1), r) for r in range(lo, hi + 1))
    return out


def _instructions(lines):
    """(line number, mnemonic, operand list, inside an inline-asm block) for every instruction line."""
    in_asm = False
    for no, ln in enumerate(lines, 1):
        t = ln.strip()
        if t.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if t.startswith(";;#ASMEND"):
            in_asm = False
            continue
        if not t or t.startswith((";", ".", "//")) or t.endswith(":"):
            continue
        t = t.split(";")[0].strip()
        if not t:
            continue
        parts = t.split(None, 1)
        ops = [o.strip() for o in parts[1].split(",")] if len(parts) > 1 else []
        if parts[0] == "s_nop" and ops:                      # s_nop N idles for N + 1 wait states
            for _ in range(int(ops[0], 0)):
                yield no, "s_nop", ["0"], in_asm
        yield no, parts[0], ops, in_asm


def check(asm_path: str, kernel_prefix: str = "_ZN2vl16attn_mfma_kernel") -> list[str]:
    problems = []
    lines = open(asm_path).read().splitlines()
    start = None
    for i, ln in enumerate(lines):
        if ln.startswith(kernel_prefix) and ln.rstrip().split(";")[0].strip().endswith(":"):
            start = i
        elif start is not None and "s_endpgm" in ln:
            ins = list(_instructions(lines[start:i + 1]))
            name = lines[start].split(":")[0]
            for k, (no, mn, ops, in_asm) in enumerate(ins):
                if not (in_asm and mn.startswith("v_mfma")):
                    continue
                reads = _regs(",".join(ops[1:]))
                writes = _regs(ops[0])
                for no2, mn2, ops2, asm2 in ins[max(0, k - OPERAND_GAP):k]:
                    # a vector-ALU instruction (not a load: those are ordered by s_waitcnt, which the compiler does place)
                    if mn2.startswith("v_") and not mn2.startswith("v_mfma") and ops2 and (_regs(ops2[0]) & reads):
                        problems.append(f"{name}: line {start + no2}: {mn2} {ops2[0]} writes an operand of the hand-issued "
                                        f"{mn} at line {start + no}, fewer than {OPERAND_GAP} instructions before it")
                for no2, mn2, ops2, asm2 in ins[k + 1:k + 1 + RESULT_GAP]:
                    # reading the result, or overwriting it, before the matrix instruction has delivered it
                    if mn2.startswith("v_") and not mn2.startswith("v_mfma") and ops2 and (_regs(",".join(ops2)) & writes):
                        problems.append(f"{name}: line {start + no2}: {mn2} touches the result of the hand-issued {mn} at line "
                                        f"{start + no} too early")
            start = None
    return problems


if __name__ == "__main__":
    bad = check(sys.argv[1])
    for b in bad:
        print(b)
    sys.exit(1 if bad else 0)
