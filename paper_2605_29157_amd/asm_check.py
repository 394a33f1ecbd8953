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


MFMA_RESULT_WAIT_STATES = 12  # an 8-pass MFMA result may be read by the vector ALU after 11
MFMA_PASSES = 8               # v_mfma_f32_32x32x16_bf16: the pipe accepts the next one 8 states later


def find_early_reads_of_asm_mfma_results(asm_text: str) -> list[str]:
    """An MFMA written as inline assembly is invisible to the compiler, which therefore adds no
    wait states between it and the first instruction that reads its result. The kernels place
    that first read well behind the MFMA (other MFMAs and vector work in between). Verify it on
    the generated code: between an assembly MFMA and the first non-MFMA instruction that reads
    one of its destination registers there must be MFMA_RESULT_WAIT_STATES wait states -- one
    per instruction (s_nop n: n + 1), MFMA_PASSES per further MFMA, which the matrix pipe only
    accepts once the previous one is through. (A later MFMA that reads the block as its
    accumulator input is the normal dependent chain.) This also catches register-allocator
    copies or spills of a freshly written block."""
    instrs = []  # (line number, text, inside inline assembly)
    inside = False
    for n, line in enumerate(asm_text.splitlines(), 1):
        t = line.strip()
        if t.startswith(";;#ASMSTART"):
            inside = True
            continue
        if t.startswith(";;#ASMEND"):
            inside = False
            continue
        if _is_instruction(line):
            instrs.append((n, t.split(";")[0].strip(), inside))
    bad = []
    for i, (n, ins, inside) in enumerate(instrs):
        if not (inside and ins.startswith("v_mfma")):
            continue
        dst = _regs(ins.split(None, 1)[1].split(",")[0])
        states = 0
        for pn, nxt, _ in instrs[i + 1:]:
            if states >= MFMA_RESULT_WAIT_STATES or nxt.endswith(":") or nxt.startswith("s_endpgm"):
                break
            if nxt.startswith("v_mfma"):
                states += MFMA_PASSES
                continue
            parts = nxt.split(None, 1)
            if len(parts) == 2:
                ops = parts[1].split(",")
                # stores and LDS writes read every operand; everything else writes its first
                stores = ("ds_write", "global_store", "scratch_store", "buffer_store")
                reads = ops if parts[0].startswith(stores) else ops[1:]
                if any(_regs(o) & dst for o in reads):
                    bad.append("line %d: '%s' reads the result of the assembly MFMA at line %d after "
                               "only %d wait states" % (pn, nxt, n, states))
                    break
            states += _wait_states(nxt)
    return bad


DOT_RESULT_WAIT_STATES = 3  # a dot-product result may be read by a different instruction after 3


def find_early_reads_of_asm_dot_results(asm_text: str) -> list[str]:
    """The packed dot products (v_dot2c_f32_bf16) are written as inline assembly, so the compiler
    does not know that their result needs DOT_RESULT_WAIT_STATES wait states before any other
    vector instruction may read it (the next dot product of the same accumulation chain, which
    takes it as its addend, is exempt). Verify that on the generated code."""
    instrs = []
    inside = False
    for n, line in enumerate(asm_text.splitlines(), 1):
        t = line.strip()
        if t.startswith(";;#ASMSTART"):
            inside = True
        elif t.startswith(";;#ASMEND"):
            inside = False
        elif _is_instruction(line):
            instrs.append((n, t.split(";")[0].strip(), inside))
    bad = []
    for i, (n, ins, inside) in enumerate(instrs):
        if not (inside and ins.startswith("v_dot2c")):
            continue
        ops = ins.split(None, 1)[1].split(",")
        dst = _regs(ops[0])
        states = 0
        for pn, nxt, _ in instrs[i + 1:]:
            if states >= DOT_RESULT_WAIT_STATES or nxt.endswith(":") or nxt.startswith("s_endpgm"):
                break
            parts = nxt.split(None, 1)
            if len(parts) == 2 and not parts[0].startswith("s_"):
                nops = parts[1].split(",")
                if parts[0].startswith("v_dot2c") and _regs(nops[0]) == dst and not any(_regs(o) & dst for o in nops[1:]):
                    break  # the chain goes on: its end is checked from there
                if any(_regs(o) & dst for o in nops):
                    bad.append("line %d: '%s' touches the result of the assembly dot product at line %d after "
                               "only %d wait states" % (pn, nxt, n, states))
                    break
            states += _wait_states(nxt)
    return bad


def find_foreign_uses_of_asm_loaded_registers(asm_text: str) -> list[str]:
    """Registers that inline-assembly global loads write may hold data that is still on its way;
    only the inline assembly that waits for it (s_waitcnt) may touch them. Between the first such
    load and the last inline-assembly LDS store of a kernel, report every compiler-generated
    instruction that names one of those registers (a copy or a spill there would move stale data)."""
    bad: list[str] = []
    for kernel in re.split(r"\n(?=[A-Za-z_][\w$.]*:\s)", asm_text):
        lines = kernel.split("\n")
        in_app, loaded, first, last = False, set(), None, None
        marks = []
        for n, line in enumerate(lines):
            s = line.strip()
            if s.startswith(";;#ASMSTART"):
                in_app = True
            elif s.startswith(";;#ASMEND"):
                in_app = False
            marks.append(in_app)
            if in_app and s.startswith("global_load_dwordx4"):
                loaded |= _regs(s.split()[1].rstrip(","))
                first = n if first is None else first
            if in_app and s.startswith("ds_write_b128") and loaded:
                last = n
        if not loaded or first is None or last is None:
            continue
        for n in range(first, last + 1):
            s = lines[n].strip()
            if marks[n] or not _is_instruction(lines[n]):
                continue
            ops = s.split(None, 1)
            used = set()
            if len(ops) > 1:
                for operand in ops[1].split(","):
                    used |= _regs(operand.strip())
            hit = used & loaded
            if hit:
                bad.append("line %d: %s  (touches %s)" % (n + 1, s, sorted(hit)[:4]))
    return bad


def check_file(path: str) -> None:
    with open(path) as f:
        text = f.read()
    bad = (find_violations(text) + find_m0_uses_outside_inline_asm(text)
           + find_early_reads_of_asm_mfma_results(text) + find_early_reads_of_asm_dot_results(text))
    if bad:
        raise RuntimeError("MFMA source hazard in %s:\n  %s" % (path, "\n  ".join(bad[:20])))
