"""Static check of the compiled GPU code for the kernels that request loads with inline assembly.

A register that an inline-asm `global_load_dwordx4` writes is "pending" from that instruction until an
inline-asm `s_waitcnt` that names it (the kernels list the registers in a comment on the wait).  The
compiler does not know that such a register is filled later, so nothing it generates, whether a move,
a spill or an ordinary use, may touch a pending register on any path.  This walks the control-flow
graph of the assembly text and reports every such instruction.
"""
from __future__ import annotations

import re
from typing import Dict, List, Tuple


def _regs(text: str) -> set:
    regs = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]", text):
        regs.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in re.finditer(r"\bv(\d+)\b", text):
        regs.add(int(m.group(1)))
    return regs


def kernels(asm_text: str) -> Dict[str, str]:
    parts = re.split(r"\n(_Z[\w]+):\s*;?[^\n]*\n", asm_text)
    return {parts[i]: parts[i + 1].split(".section")[0] for i in range(1, len(parts), 2)}


def check_kernel(body: str) -> Tuple[int, int, List[Tuple[int, str, List[int]]]]:
    """Returns (instructions, async loads found, violations)."""
    ins: List[Tuple[str, bool]] = []
    labels: Dict[str, int] = {}
    in_asm = False
    for line in body.split("\n"):
        t = line.strip()
        if t.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if t.startswith(";;#ASMEND"):
            in_asm = False
            continue
        m = re.match(r"^(\.LBB\d+_\d+):", t)
        if m:
            labels[m.group(1)] = len(ins)
            continue
        if not t or t.startswith(";") or t.startswith("."):
            continue
        ins.append((t, in_asm))
    n = len(ins)
    succ: List[List[int]] = [[] for _ in range(n)]
    for k, (t, _) in enumerate(ins):
        op = t.split()[0]
        if op == "s_endpgm":
            continue
        if op == "s_branch":
            succ[k].append(labels[t.split()[1]])
            continue
        if op.startswith("s_cbranch"):
            succ[k].append(labels[t.split()[1]])
        if k + 1 < n:
            succ[k].append(k + 1)
    state: List = [None] * n
    state[0] = frozenset()
    work = [0]
    viol: Dict[int, Tuple[str, List[int]]] = {}
    loads = 0
    seen_load = set()
    while work:
        k = work.pop()
        pend = set(state[k])
        t, a = ins[k]
        if a and t.startswith("global_load_dwordx4"):
            m = re.match(r"global_load_dwordx4 v\[(\d+):(\d+)\]", t)
            pend.update(range(int(m.group(1)), int(m.group(2)) + 1))
            if k not in seen_load:
                seen_load.add(k)
                loads += 1
        elif a and t.startswith("s_waitcnt vmcnt") and ";" in t:
            pend -= _regs(t.split(";", 1)[1])
        elif not a:
            hit = _regs(t.split(";")[0]) & pend
            if hit:
                viol[k] = (t, sorted(hit)[:4])
        out = frozenset(pend)
        for j in succ[k]:
            new = out if state[j] is None else (state[j] | out)
            if new != state[j]:
                state[j] = new
                work.append(j)
    return n, loads, [(k, viol[k][0], viol[k][1]) for k in sorted(viol)]
