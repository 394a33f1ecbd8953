"""Static check of the generated gfx950 assembly of the prefill kernel.

The steady-state loop of the bf16 prefill kernel issues its score MFMAs as inline assembly
without wait states in front of them ("unguarded"). That is only valid if no vector-ALU
instruction writes one of the MFMA's source registers within the two instructions before it
(an MFMA reading a freshly written vector register needs two wait states and the hardware
does not interlock). The compiler cannot see the MFMA inside the assembly statement, so this
script verifies the property on the code it actually produced; the build fails otherwise.
"""
from __future__ import annotations

import re

_REG = re.compile(r"\b([va])(?:\[(\d+):(\d+)\]|(\d+))")
WAIT_STATES = 2


def _regs(operand: str) -> set[tuple[str, int]]:
    out = set()
    for m in _REG.finditer(operand):
        bank = m.group(1)
        if m.group(2) is not None:
            lo, hi = int(m.group(2)), int(m.group(3))
        else:
            lo = hi = int(m.group(4))
        out.update((bank, i) for i in range(lo, hi + 1))
    return out


def _is_instruction(line: str) -> bool:
    """Instructions and labels (a label ends the straight-line code the check can follow)."""
    t = line.split(";")[0].strip()
    if not t or t.startswith("//"):
        return False
    if t.endswith(":"):
        return True
    return not t.startswith(".")


def _wait_states(instr: str) -> int:
    m = re.match(r"s_nop\s+(\d+)", instr)
    return int(m.group(1)) + 1 if m else 1


def find_violations(asm_text: str) -> list[str]:
    """Return a description of every unguarded MFMA whose sources are written too late."""
    lines = asm_text.splitlines()
    instrs = [(n, l.strip()) for n, l in enumerate(lines, 1) if _is_instruction(l)]
    bad = []
    seen = 0
    for idx, (n, ins) in enumerate(instrs):
        if not (ins.startswith("v_mfma") and "unguarded" in ins):
            continue
        seen += 1
        ops = ins.split(";")[0].split(None, 1)[1].split(",")
        srcs = set().union(*(_regs(o) for o in ops[1:]))
        budget, j = WAIT_STATES, idx - 1
        while budget > 0 and j >= 0:
            pn, prev = instrs[j]
            if prev.split(";")[0].strip().endswith(":"):
                bad.append("line %d: MFMA within %d instructions of the branch target at line %d"
                           % (n, WAIT_STATES, pn))
                break
            if prev.startswith("v_") and not prev.startswith("v_mfma"):
                dst = _regs(prev.split(None, 1)[1].split(",")[0]) if " " in prev else set()
                if dst & srcs:
                    bad.append("line %d: '%s' writes a source of the MFMA at line %d" % (pn, prev, n))
            budget -= _wait_states(prev)
            j -= 1
    if seen == 0:
        bad.append("no unguarded MFMA found: the marker comment is missing from the assembly")
    return bad


def find_m0_uses_outside_inline_asm(asm_text: str) -> list[str]:
    """The tile loads set M0 without restoring it, which is only valid while nothing the
    compiler itself emits reads or writes M0: report every M0 reference outside the
    hand-written assembly statements."""
    bad, inside = [], False
    for n, line in enumerate(asm_text.splitlines(), 1):
        t = line.strip()
        if t.startswith(";;#ASMSTART"):
            inside = True
        elif t.startswith(";;#ASMEND"):
            inside = False
        elif not inside and _is_instruction(line) and re.search(r"\bm0\b", t.split(";")[0]):
            bad.append("line %d: compiler-generated use of M0: '%s'" % (n, t))
    return bad


def check_file(path: str) -> None:
    with open(path) as f:
        text = f.read()
    bad = find_violations(text) + find_m0_uses_outside_inline_asm(text)
    if bad:
        raise RuntimeError("MFMA source hazard in %s:\n  %s" % (path, "\n  ".join(bad[:20])))
