"""Build-time check of the generated gfx950 code of the kernels that pin matrix-core instructions.

The 256-row attention kernel issues its matrix-core instructions as inline assembly (so that it can
choose, per instruction, which operands live in accumulation registers).  The compiler inserts the
wait states that the hardware needs between a vector-ALU instruction that writes a register and a
matrix-core instruction that reads it (two) only for instructions it selects itself, not around
inline assembly.  The kernel is written so that no such pair arises (operands that the compiler
might move into place are declared read-write, guarded forms carry their own s_nop); this scan of
the generated code is what checks it on every build: a pinned matrix-core instruction must not read
a register written by one of the two instructions issued before it.
"""
from __future__ import annotations

import re

_RANGE = re.compile(r"([va])\[(\d+):(\d+)\]$")
_SINGLE = re.compile(r"([va])(\d+)$")
_NOT_VALU = ("s_", "ds_", "global_", "buffer_", "flat_", "scratch_")


def _regs(token: str) -> set:
    token = token.strip()
    m = _RANGE.match(token)
    if m:
        return {(m.group(1), i) for i in range(int(m.group(2)), int(m.group(3)) + 1)}
    m = _SINGLE.match(token)
    if m:
        return {(m.group(1), int(m.group(2)))}
    return set()


def pinned_mfma_hazards(isa_text: str):
    """Returns (number of pinned matrix-core instructions, list of (line number, instruction,
    line number of the writer, writer)) for one generated .s file."""
    lines = isa_text.splitlines()
    code = [(i, l.strip()) for i, l in enumerate(lines)
            if l.strip() and not l.strip().startswith((";", ".", "//")) and not l.strip().endswith(":")]
    found, pinned = [], 0
    for k, (i, ins) in enumerate(code):
        if not ins.startswith("v_mfma") or i == 0 or "#ASMSTART" not in lines[i - 1]:
            continue
        pinned += 1
        operands = ins.split(None, 1)[1].split(",")
        sources = set().union(*[_regs(t) for t in operands[1:]])
        for back in (1, 2):
            if k - back < 0:
                break
            pi, prev = code[k - back]
            if prev.startswith("s_nop"):
                break  # the guarded forms: s_nop 1 = two wait states
            if prev.startswith(_NOT_VALU) or " " not in prev:
                continue
            dest = prev.split(None, 1)[1].split(",")[0]
            if _regs(dest) & sources:
                found.append((i + 1, ins, pi + 1, prev))
    return pinned, found


def spill_counts(isa_text: str) -> dict:
    """Kernel symbol -> vector-register spill count, from the metadata at the end of a .s file."""
    out, name = {}, None
    for line in isa_text.splitlines():
        t = line.strip()
        if t.startswith(".name:") and t.split(":", 1)[1].strip().startswith("_Z"):
            name = t.split(":", 1)[1].strip()
        elif t.startswith(".vgpr_spill_count:") and name is not None:
            out[name] = int(t.split(":", 1)[1])
            name = None
    return out
