"""Checks the wait states around hand-placed matrix instructions in a kernel's gfx950 assembly.

The attention kernel for head size 256 issues its matrix instructions from inline assembly (so that
it, not the compiler, decides which results live in vector and which in accumulator registers).
The compiler does not look inside inline assembly, so it inserts none of the idle issue slots
("wait states") the hardware needs between a matrix instruction and a dependent access; the kernel
places them itself.  Register allocation can still put a copy next to a matrix instruction that the
source does not show, so the build verifies the finished assembly with this module and fails if a
distance is too short.

Rules checked (wait states = instructions issued in between, `s_nop N` counting N + 1):
  * a register written by a 32x32x16 matrix instruction (8 passes) may be touched by a vector,
    LDS or memory instruction, or read as an A or B operand, 12 wait states later; read as a
    different-but-overlapping C operand 10 later; the identical C operand (accumulation) may
    follow at once (two matrix results that overlap need nothing: the matrix pipe completes in
    order, and the compiler's own code for the builtin form places them back to back);
  * for a 4x4x4 matrix instruction (2 passes) the distances are 5 and 4, and the next
    accumulation into the identical registers needs 2;
  * a matrix instruction may read a register 2 wait states after a vector instruction wrote it.

The scan is linear over the function.  At each branch the instructions at the target are scanned
as well with the state at the branch, 24 wait states deep in total and through up to three further
branches; after an unconditional branch or the end of the program the state is dropped.
"""
from __future__ import annotations

import re
from typing import Dict, List, Tuple

_REG = re.compile(r"\b([va])(?:\[(\d+):(\d+)\]|(\d+)\b)")
_LABEL = re.compile(r"^(\.LBB\d+_\d+):")
LOOKAHEAD = 24
MAX_BRANCH_DEPTH = 4


def _regs(text: str) -> set:
    out = set()
    for m in _REG.finditer(text):
        if m.group(4) is not None:
            out.add((m.group(1), int(m.group(4))))
        else:
            out.update((m.group(1), r) for r in range(int(m.group(2)), int(m.group(3)) + 1))
    return out


def kernels(asm: str, contains: str) -> List[str]:
    """Symbols of the functions in `asm` whose (mangled) name contains `contains`."""
    return [m.group(1) for m in re.finditer(r"^(\w+):\s*;\s*@", asm, re.M) if contains in m.group(1)]


def check_kernel(asm: str, symbol: str) -> List[str]:
    """Returns one line per place in function `symbol` where a rule above is broken."""
    src = asm.split("\n")
    start = next(i for i, l in enumerate(src) if l.startswith(symbol + ":"))
    end = next(i for i in range(start, len(src)) if src[i].startswith(".Lfunc_end"))
    labels = {m.group(1): i for i in range(start, end) for m in [_LABEL.match(src[i])] if m}
    found = set()

    def scan(i: int, pending: List[Tuple], written: Dict, state: int, depth: int, first: int) -> None:
        nested = depth > 0
        while i < end:
            line = src[i].split(";")[0].strip()
            i += 1
            if not line or line.endswith(":") or line.startswith("."):
                continue
            if nested and state - first > LOOKAHEAD:
                return
            op, _, args = line.partition(" ")
            args = args.strip()
            if op == "s_nop":
                state += int(args) + 1
                continue
            if op == "s_branch" or op.startswith("s_cbranch"):
                if depth < MAX_BRANCH_DEPTH and args in labels:
                    scan(labels[args], list(pending), dict(written), state + 1, depth + 1, first if nested else state + 1)
                state += 1
                if op == "s_branch":
                    if nested:
                        return
                    pending.clear()
                    written.clear()
                continue
            if op == "s_endpgm":
                if nested:
                    return
                pending.clear()
                written.clear()
                continue
            toks = [t.strip() for t in args.split(",")]
            if op.startswith("v_mfma"):
                dst, a, b = _regs(toks[0]), _regs(toks[1]), _regs(toks[2])
                c = _regs(toks[3]) if len(toks) > 3 else set()
                for regs, need, need_c, at, ln, text in pending:
                    d = state - at - 1
                    where = "line %d `%s` after line %d `%s`: %d wait states" % (i, line, ln, text, d)
                    if (a | b) & regs and d < need:
                        found.add("A/B operand read, %s, %d needed" % (where, need))
                    if c & regs and c != regs and d < need_c:
                        found.add("overlapping C operand, %s, %d needed" % (where, need_c))
                    if c == regs and "4x4x4" in text and d < 2:
                        found.add("4x4x4 accumulation, %s, 2 needed" % where)
                for r in a | b | c:
                    if r in written and state - written[r][0] - 1 < 2:
                        found.add("matrix read after vector write, line %d `%s` after line %d `%s`: %d wait states, 2 needed"
                                  % (i, line, written[r][1], written[r][2], state - written[r][0] - 1))
                        break
                need, need_c = (5, 4) if "4x4x4" in op else (12, 10)
                pending[:] = [p for p in pending if state - p[3] - 1 < p[1] and p[0] != dst]
                pending.append((dst, need, need_c, state, i, line))
                state += 1
                continue
            used = _regs(args)
            for regs, need, _, at, ln, text in pending:
                d = state - at - 1
                if used & regs and d < need:
                    found.add("access to a matrix result, line %d `%s` after line %d `%s`: %d wait states, %d needed"
                              % (i, line, ln, text, d, need))
            if op.startswith("v_") and toks:
                for r in _regs(toks[0]):
                    written[r] = (state, i, line)
                if "swap" in op and len(toks) > 1:      # the half-wave swap writes both operands
                    for r in _regs(toks[1]):
                        written[r] = (state, i, line)
            state += 1
            pending[:] = [p for p in pending if state - p[3] - 1 < p[1]]
            for r in [r for r, w in written.items() if state - w[0] >= 4]:
                del written[r]

    scan(start + 1, [], {}, 0, 0, 0)
    return sorted(found)
