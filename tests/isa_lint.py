"""A check of the compiled gfx950 assembly of this library's own kernels: results of matrix
instructions that were written as assembly statements are not read too early.

The compiler inserts the wait states a matrix instruction's readers need only for instructions
it selected itself; an assembly statement is opaque to it.  The kernels that issue
v_mfma_f32_32x32x16_bf16 from assembly statements (csrc/vfm_common.h: mfma32_v, mfma32_acc)
therefore keep this rule by construction: any instruction that touches the destination tuple of
such an MFMA is either the next accumulation into that same tuple, or lies at least two matrix
instructions (or 16 issue slots of other instructions and s_nop states) downstream.  The
instruction occupies the matrix pipe for 8 passes, and a wavefront issues in order, so two further
MFMAs put 16 passes between writer and reader.

This module parses the assembly text hipcc emits with -S and walks every path from each such
MFMA (fall-through, branch targets) until the rule is met or broken.
"""
from __future__ import annotations

import re
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

MFMA_PASSES = 8          # v_mfma_f32_32x32x16_bf16 on gfx950
NEEDED = 2 * MFMA_PASSES

_REG = re.compile(r"(?<![\w.])([va])(?:\[(\d+):(\d+)\]|(\d+)\b)")
_LABEL = re.compile(r"^([.\w$]+):")


@dataclass
class Inst:
    line: int
    text: str
    mnemonic: str
    regs: List[Tuple[str, int, int]]          # every vector/accumulator register operand: (file, lo, hi)
    from_asm: bool
    target: Optional[str] = None              # branch target label


@dataclass
class Program:
    insts: List[Inst] = field(default_factory=list)
    labels: Dict[str, int] = field(default_factory=dict)     # label -> index of the next instruction


def parse(text: str) -> Program:
    prog = Program()
    in_asm = False
    for n, raw in enumerate(text.splitlines(), 1):
        s = raw.strip()
        if s.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if s.startswith(";;#ASMEND"):
            in_asm = False
            continue
        m = _LABEL.match(s)
        if m and not in_asm:
            prog.labels[m.group(1)] = len(prog.insts)
            continue
        s = s.split(";", 1)[0].strip()
        if not s or s.startswith("."):
            continue
        parts = s.split(None, 1)
        mnem = parts[0]
        if not re.match(r"^(v_|s_|ds_|global_|buffer_|flat_|scratch_)", mnem):
            continue
        ops = parts[1] if len(parts) > 1 else ""
        regs = []
        for f, lo, hi, single in _REG.findall(ops):
            regs.append((f, int(lo), int(hi)) if single == "" else (f, int(single), int(single)))
        inst = Inst(n, s, mnem, regs, in_asm)
        if mnem.startswith("s_cbranch") or mnem == "s_branch":
            inst.target = ops.strip()
        prog.insts.append(inst)
    return prog


def _overlaps(a, b) -> bool:
    return a[0] == b[0] and a[1] <= b[2] and b[1] <= a[2]


def _mfma_operands(inst: Inst):
    """The four operands of an MFMA (destination, A, B, C) as register ranges; None for a constant."""
    out = []
    for o in inst.text.split(None, 1)[1].split(",")[:4]:
        m = _REG.search(o)
        if not m:
            out.append(None)
            continue
        f, lo, hi, single = m.groups()
        out.append((f, int(lo), int(hi)) if single is None else (f, int(single), int(single)))
    return out + [None] * (4 - len(out))


def _states(inst: Inst) -> int:
    if inst.mnemonic == "s_nop":
        return int(inst.text.split()[1], 0) + 1
    return 1


def check(text: str, max_steps: int = 400) -> List[str]:
    """Returns one message per assembly-statement MFMA whose destination is touched too early."""
    prog = parse(text)
    bad = []
    for i, w in enumerate(prog.insts):
        if not (w.from_asm and w.mnemonic.startswith("v_mfma")):
            continue
        dest = _mfma_operands(w)[0]
        if dest is None:
            bad.append(f"line {w.line}: cannot read the destination of '{w.text}'")
            continue
        # depth-first over paths; a state is (index, distance so far)
        best: Dict[int, int] = {}
        stack = [(i + 1, 0)]
        steps = 0
        while stack:
            pos, dist = stack.pop()
            while True:
                steps += 1
                if steps > max_steps * 8:
                    bad.append(f"line {w.line}: path search from '{w.text}' did not end")
                    stack.clear()
                    break
                if dist >= NEEDED or pos >= len(prog.insts):
                    break
                if best.get(pos, -1) >= 0 and best[pos] <= dist:
                    break                      # been here at no greater distance
                best[pos] = dist
                r = prog.insts[pos]
                if r.mnemonic == "s_endpgm":
                    break
                if r.mnemonic in ("s_setpc_b64", "s_swappc_b64"):
                    bad.append(f"line {w.line}: indirect jump at line {r.line} after '{w.text}'")
                    break
                if any(_overlaps(dest, x) for x in r.regs):
                    chained = False
                    if r.mnemonic.startswith("v_mfma"):
                        d2, a2, b2, c2 = _mfma_operands(r)
                        chained = (d2 == dest and c2 == dest
                                   and not any(x is not None and _overlaps(dest, x) for x in (a2, b2)))
                    if not chained:
                        bad.append(f"line {r.line}: '{r.text}' touches {dest[0]}[{dest[1]}:{dest[2]}] only {dist} "
                                   f"issue states after the assembly MFMA at line {w.line}")
                    break
                dist += MFMA_PASSES if r.mnemonic.startswith("v_mfma") else _states(r)
                if r.target is not None:
                    tgt = prog.labels.get(r.target)
                    if tgt is None:
                        bad.append(f"line {r.line}: unknown branch target {r.target}")
                        break
                    if r.mnemonic == "s_branch":
                        pos = tgt
                        continue
                    stack.append((tgt, dist))
                pos += 1
    return bad
