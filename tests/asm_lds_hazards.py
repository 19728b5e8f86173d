"""Static check of generated gfx950 assembly: no instruction may touch the destination registers of an LDS read
before an `s_waitcnt lgkmcnt(n)` has retired that read.

The K-major path of the GEMM kernel issues its LDS fragment reads from inline assembly and places the waits by hand,
so the compiler's own bookkeeping does not cover them; the source ties every result to its wait, and this checker
looks at what the compiler made of it.  It walks the control-flow graph of every kernel in a `.s` file with the
queue of outstanding LDS operations and reports every instruction that reads or writes a vector register an
outstanding LDS read will still deliver into.  LDS operations complete in issue order, so after a wait for lgkmcnt(n)
at most the n youngest of them are outstanding.  Scalar and flat loads share the counter and complete in any order:
whatever of them is outstanding only takes room away from LDS operations among the n, so leaving them out of the
model is the worst case for the LDS reads and keeps the check sound.
"""
from __future__ import annotations

import re
from typing import Dict, List, Optional, Tuple

_REG_RANGE = re.compile(r"\bv\[(\d+):(\d+)\]")
_REG_ONE = re.compile(r"\bv(\d+)\b")
_LABEL = re.compile(r"^([.\w$]+):")
_LGKM = re.compile(r"lgkmcnt\((\d+)\)")
_FAR = re.compile(r"\((\.LBB\w+)-\.Lpost_getpc\d+\)")


def _vregs(text: str) -> set:
    regs = set()
    for a, b in _REG_RANGE.findall(text):
        regs.update(range(int(a), int(b) + 1))
    for a in _REG_ONE.findall(_REG_RANGE.sub(" ", text)):
        regs.add(int(a))
    return regs


class Insn:
    __slots__ = ("line", "op", "args", "text")

    def __init__(self, line: int, text: str):
        self.line = line
        self.text = text
        parts = text.split(None, 1)
        self.op = parts[0]
        self.args = parts[1] if len(parts) > 1 else ""


def split_kernels(asm: str) -> Dict[str, List[Tuple[int, str]]]:
    """name -> [(line number, text)] (instructions and local labels) for every function of the file."""
    kernels, cur, name = {}, None, None
    for no, raw in enumerate(asm.splitlines(), 1):
        line = raw.split(";", 1)[0].strip()
        if not line:
            continue
        m = _LABEL.match(line)
        if m and not m.group(1).startswith("."):
            name, cur = m.group(1), []           # a function's own label
            continue
        if cur is None:
            continue
        if line.startswith(".Lfunc_end"):
            kernels[name] = cur
            cur = None
            continue
        if line.startswith("."):
            if m:
                cur.append((no, line))           # local label
            continue                             # directive
        cur.append((no, line))
    return kernels


def check_kernel(lines: List[Tuple[int, str]], max_states: int = 200000) -> List[str]:
    """Violations found in one kernel (empty list = none)."""
    insns: List[Insn] = []
    labels: Dict[str, int] = {}
    for no, text in lines:
        m = _LABEL.match(text)
        if m:
            labels[m.group(1)] = len(insns)
            continue
        insns.append(Insn(no, text))

    def far_target(i: int) -> Optional[int]:
        for j in range(i - 1, max(i - 8, -1), -1):
            m = _FAR.search(insns[j].text)
            if m:
                return labels.get(m.group(1))
        return None

    label_pcs = set(labels.values())
    violations: List[str] = []
    seen = set()
    # queue entries: the vector registers an outstanding LDS read delivers into, () for an LDS operation without a result
    work: List[Tuple[int, tuple]] = [(0, ())]
    states = 0
    while work:
        pc, pending = work.pop()
        queue = list(pending)
        while pc < len(insns):
            ins = insns[pc]
            key = None
            if pc in label_pcs:
                key = (pc, tuple(queue))
                if key in seen:
                    break
                seen.add(key)
                states += 1
                if states > max_states:
                    return violations + ["state limit reached: the walk did not finish"]
            op = ins.op
            if op == "s_waitcnt":
                m = _LGKM.search(ins.args)
                if m:
                    keep = int(m.group(1))
                    while len(queue) > keep:
                        queue.pop(0)
                pc += 1
                continue
            outstanding = set()
            for q in queue:
                if q:
                    outstanding.update(q)
            if outstanding:
                # an LDS read's own destination is not a use: LDS results land in issue order, also onto each other
                used = ins.args.split(",", 1)[1] if op.startswith("ds_read") and "," in ins.args else ins.args
                touched = _vregs(used) & outstanding
                if touched:
                    violations.append(f"line {ins.line}: `{ins.text}` touches v{sorted(touched)} before the LDS read into it is waited for")
            if op.startswith("ds_"):
                dest: Tuple[int, ...] = ()
                if op.startswith("ds_read") or op.startswith("ds_load") or "_rtn" in op or op.startswith("ds_bpermute") or op.startswith("ds_permute") or op.startswith("ds_swizzle"):
                    first = ins.args.split(",", 1)[0]
                    dest = tuple(sorted(_vregs(first)))
                queue.append(dest)
                pc += 1
                continue
            if op == "s_endpgm":
                break
            if op == "s_branch":
                tgt = labels.get(ins.args.strip())
                if tgt is None:
                    violations.append(f"line {ins.line}: unknown branch target {ins.args}")
                    break
                pc = tgt
                continue
            if op.startswith("s_cbranch"):
                tgt = labels.get(ins.args.strip())
                if tgt is None:
                    violations.append(f"line {ins.line}: unknown branch target {ins.args}")
                    break
                work.append((tgt, tuple(queue)))
                pc += 1
                continue
            if op == "s_setpc_b64":
                tgt = far_target(pc)
                if tgt is None:
                    violations.append(f"line {ins.line}: indirect jump with no recognisable target")
                    break
                pc = tgt
                continue
            pc += 1
    return violations


def check_file_text(asm: str) -> Dict[str, List[str]]:
    return {name: check_kernel(lines) for name, lines in split_kernels(asm).items()}


def check_file(path: str) -> Dict[str, List[str]]:
    with open(path) as f:
        return check_file_text(f.read())
