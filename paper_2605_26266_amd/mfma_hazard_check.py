"""Static check of the wait states around matrix instructions whose operands the compiler does not guard.

The per-token attention kernel writes its score MFMAs as inline assembly with a vector-register tuple as C and D.
The compiler treats such a statement as opaque and inserts no wait states for it, so the kernel source places them
(`s_nop`) and this module checks the assembly the compiler produced from it.  The build runs it on every compile of
that kernel and fails when a rule is broken; it reads text only and needs no GPU.

Rules, as the compiler applies them to MFMAs it schedules itself on gfx950 (a wait state is one issued
instruction; `s_nop N` counts N + 1):

  after   an MFMA with a vector-register destination v[a:b], any instruction other than an MFMA that reads or
          writes one of v[a:b] comes at least AFTER_MFMA wait states later (a dependent MFMA may follow at once:
          the matrix pipe interlocks on its own results);
  before  a vector instruction that writes a register an MFMA reads as A, B or scale operand comes at least
          BEFORE_MFMA wait states earlier.

A window that reaches a branch or the end of the program before it closes cannot be followed by a linear scan and is
reported as a problem of its own ("open"): the kernel source closes every window inside its basic block.
"""
from __future__ import annotations

import re
import sys
from typing import List, Tuple

AFTER_MFMA = 12     # 8-pass MFMA (32x32 results) -> first vector read or overwrite of its destination
BEFORE_MFMA = 2     # vector write of an operand -> the MFMA that reads it

_LABEL = re.compile(r"^[_A-Za-z0-9.$]+:")
_RANGE = re.compile(r"\bv\[(\d+):(\d+)\]")
_SINGLE = re.compile(r"\bv(\d+)\b")
_CONTROL = ("s_cbranch", "s_branch", "s_endpgm", "s_setpc")


def _instructions(text: str) -> List[Tuple[str, str]]:
    out = []
    for raw in text.split("\n"):
        line = raw.strip()
        if not line or line.startswith((";", "//")):
            continue
        if _LABEL.match(line):
            out.append(("label", line))
            continue
        if line.startswith("."):
            continue
        out.append(("ins", line.split(";")[0].strip()))
    return out


def _vregs(token: str) -> set:
    regs = set()
    for m in _RANGE.finditer(token):
        regs |= set(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in _SINGLE.finditer(token):
        regs.add(int(m.group(1)))
    return regs


def _split(ins: str) -> Tuple[str, List[str]]:
    parts = ins.split(None, 1)
    if len(parts) < 2:
        return parts[0], []
    return parts[0], re.split(r",\s*(?![^\[]*\])", parts[1])


def _states(op: str, operands: List[str]) -> int:
    return int(operands[0], 0) + 1 if op == "s_nop" else 1


def check(text: str) -> Tuple[int, List[str]]:
    """Return (number of MFMAs seen, list of problems) for one assembly listing."""
    ins = _instructions(text)
    problems: List[str] = []
    n_mfma = 0
    for idx, (kind, line) in enumerate(ins):
        if kind != "ins":
            continue
        op, operands = _split(line)
        if not op.startswith("v_mfma"):
            continue
        n_mfma += 1
        if operands and operands[0].startswith("v"):
            dst = _vregs(operands[0])
            states, j = 0, idx + 1
            while states < AFTER_MFMA:
                if j >= len(ins):
                    problems.append("open window after '%s': end of listing" % line)
                    break
                kind2, line2 = ins[j]
                j += 1
                if kind2 == "label":
                    continue
                op2, operands2 = _split(line2)
                if op2.startswith(_CONTROL):
                    problems.append("open window after '%s': reaches '%s' after %d wait states" % (line, line2, states))
                    break
                if not op2.startswith("v_mfma") and not op2.startswith("s_"):
                    touched = set()
                    for o in operands2:
                        touched |= _vregs(o)
                    if touched & dst:
                        problems.append("'%s' touches the result of '%s' after %d wait states (%d needed)"
                                        % (line2, line, states, AFTER_MFMA))
                        break
                states += _states(op2, operands2)
        src = set()
        for o in operands[1:3] + operands[4:6]:
            src |= _vregs(o.split(" ")[0])
        states, j = 0, idx - 1
        while states < BEFORE_MFMA and j >= 0:
            kind2, line2 = ins[j]
            j -= 1
            if kind2 == "label":
                break       # a jump target: what runs before it is not this listing's previous line
            op2, operands2 = _split(line2)
            if op2 == "s_nop":
                states += _states(op2, operands2)
                continue
            if (op2.startswith("v_") and not op2.startswith(("v_mfma", "v_cmp")) and operands2
                    and _vregs(operands2[0]) & src):
                problems.append("'%s' writes an operand of '%s' %d wait states earlier (%d needed)"
                                % (line2, line, states, BEFORE_MFMA))
                break
            states += 1
    return n_mfma, problems


def check_file(path: str) -> Tuple[int, List[str]]:
    with open(path) as f:
        return check(f.read())


if __name__ == "__main__":
    count, found = check_file(sys.argv[1])
    for p in found:
        print(p)
    print("checked %d MFMAs; %d problems" % (count, len(found)))
    sys.exit(1 if found else 0)
