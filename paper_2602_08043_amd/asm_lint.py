"""Hazard check of the generated gfx950 assembly of the kernels that issue MFMAs and global -> LDS loads from
inline assembly (csrc/gemm16_fast.h).  The compiler pads pipeline hazards only for instructions it knows; an
assembly statement is opaque to it.  This pass reads the device assembly of a translation unit and fails the
build when

  * a global_load_lds reads a scalar register that a vector instruction (v_readfirstlane, v_readlane, a compare
    or a carry-out) wrote within the five preceding instructions,
  * a global_load_lds directly follows the s_mov that sets M0,
  * a v_mfma from inline assembly reads a vector register that a vector ALU instruction wrote within the four
    preceding instructions.
"""
from __future__ import annotations

import re
import sys

_REG = re.compile(r"([sv])(?:\[(\d+):(\d+)\]|(\d+))")


def _regs(tok: str, kind: str) -> set[int]:
    out: set[int] = set()
    for m in _REG.finditer(tok):
        if m.group(1) != kind:
            continue
        if m.group(4) is not None:
            out.add(int(m.group(4)))
        else:
            out.update(range(int(m.group(2)), int(m.group(3)) + 1))
    return out


def _instructions(body: str):
    """(mnemonic, operands, in_inline_asm) of every instruction line, in order."""
    in_asm = False
    for line in body.split("\n"):
        t = line.strip()
        if t.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if t.startswith(";;#ASMEND"):
            in_asm = False
            continue
        if not t or t.startswith(";") or t.startswith(".") or t.endswith(":"):
            continue
        t = t.split(";")[0].strip()
        parts = t.split(None, 1)
        ops = [o.strip() for o in parts[1].split(",")] if len(parts) > 1 else []
        yield parts[0], ops, in_asm


def _window(ins, i, states):
    """The instructions in front of instruction i that are fewer than `states` wait states away, nearest first,
    as (distance in wait states, (mnemonic, operands)); an s_nop N is N + 1 wait states."""
    d = 0
    j = i - 1
    while j >= 0 and d < states:
        pm, pops, _ = ins[j]
        d += (int(pops[0], 0) + 1) if pm == "s_nop" and pops else 1
        if d <= states and pm != "s_nop":
            yield d, (pm, pops)
        j -= 1


def lint(asm_text: str, kernel_pattern: str = r"gemm16_fast_kernel") -> list[str]:
    problems = []
    for m in re.finditer(r"^(_Z\w+):.*?s_endpgm", asm_text, re.S | re.M):
        name = m.group(1)
        if not re.search(kernel_pattern, name):
            continue
        ins = list(_instructions(m.group(0)))
        for i, (mn, ops, in_asm) in enumerate(ins):
            if mn.startswith("global_load") and in_asm:
                sregs = set()
                for tok in ops[1:]:
                    sregs |= _regs(tok, "s")
                for d, (pm, pops) in _window(ins, i, 5):
                    if d == 1 and pm == "s_mov_b32" and pops and pops[0] == "m0":
                        problems.append(f"{name}: global_load_lds directly behind s_mov m0 (instruction {i})")
                    if pm.startswith("v_") and not pm.startswith("v_mfma"):
                        written = set()
                        for tok in pops[:2]:
                            written |= _regs(tok, "s")
                        if written & sregs:
                            problems.append(f"{name}: global_load_lds reads s{sorted(written & sregs)} written by {pm} "
                                            f"{d} wait state(s) earlier (instruction {i})")
            if mn.startswith("v_mfma") and in_asm and len(ops) >= 3:
                vregs = _regs(ops[1], "v") | _regs(ops[2], "v")
                for d, (pm, pops) in _window(ins, i, 4):
                    if pm.startswith("v_") and not pm.startswith("v_mfma") and pops:
                        if _regs(pops[0], "v") & vregs:
                            problems.append(f"{name}: v_mfma reads v{sorted(_regs(pops[0], 'v') & vregs)} written by "
                                            f"{pm} {d} wait state(s) earlier (instruction {i})")
    return problems


if __name__ == "__main__":
    bad = []
    for path in sys.argv[1:]:
        bad += lint(open(path).read())
    for b in bad:
        print(b)
    sys.exit(1 if bad else 0)
