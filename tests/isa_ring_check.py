"""Static check of the compiled load rings (host-side test tooling, no GPU).

The pipelined product kernels issue their global loads from inline assembly and wait for them
with explicit `s_waitcnt vmcnt(n)`.  The compiler takes the destination registers of such a
load as defined at once, so nothing but the source's own structure keeps it from scheduling an
instruction that reads (or re-uses) such a register before the wait that covers it.  This
module walks the compiler's assembly output for gfx950 and proves, per kernel, that it did not:

* the control-flow graph of a kernel is rebuilt from labels and branches;
* along every path the vector-memory operations in flight are followed as a queue (they
  complete in issue order; `s_waitcnt vmcnt(n)` retires all but the newest n);
* an instruction that names a VGPR which an inline-assembly load still in flight will write
  is a violation.

A kernel's set of reachable queues is finite because the rings are periodic.
"""
from __future__ import annotations

import re
from dataclasses import dataclass, field

_VREG = re.compile(r"\bv(\d+)\b|\bv\[(\d+):(\d+)\]")
_VMCNT = re.compile(r"vmcnt\((\d+)\)")
_LABEL = re.compile(r"^([.\w$]+):")
_VMEM = re.compile(r"^(global_|buffer_|scratch_|flat_)(load|store|atomic)")


def _vregs(text: str) -> set:
    out = set()
    for m in _VREG.finditer(text):
        if m.group(1) is not None:
            out.add(int(m.group(1)))
        else:
            out.update(range(int(m.group(2)), int(m.group(3)) + 1))
    return out


@dataclass
class Ins:
    text: str
    line: int
    in_asm: bool


@dataclass
class Block:
    name: str
    ins: list = field(default_factory=list)
    succ: list = field(default_factory=list)


def split_kernels(asm_text: str) -> dict:
    """name -> list of (line number, text) of the kernel's body."""
    kernels, cur, name = {}, None, None
    for no, raw in enumerate(asm_text.splitlines(), 1):
        if cur is None:
            m = re.match(r"^(_Z\w+):\s*(;.*)?$", raw)
            if m:
                name, cur = m.group(1), []
            continue
        if raw.startswith(".Lfunc_end"):
            kernels[name] = cur
            cur = None
            continue
        cur.append((no, raw))
    return kernels


def build_cfg(body) -> list:
    blocks = [Block("entry")]
    in_asm = False
    for no, raw in body:
        s = raw.strip()
        if s.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if s.startswith(";;#ASMEND"):
            in_asm = False
            continue
        m = _LABEL.match(s)
        if m and not in_asm:
            blocks.append(Block(m.group(1)))
            continue
        s = s.split(";")[0].strip()
        if not s or s.startswith("."):
            continue
        blocks[-1].ins.append(Ins(s, no, in_asm))
        if not in_asm and s.split()[0].startswith(("s_cbranch", "s_branch", "s_endpgm")):
            blocks.append(Block(f"after.{no}"))      # a branch ends its block
    index = {b.name: i for i, b in enumerate(blocks)}
    for i, b in enumerate(blocks):
        fall = True
        for ins in b.ins:
            op = ins.text.split()[0]
            if op.startswith("s_cbranch"):
                b.succ.append(index[ins.text.split()[-1]])
            elif op == "s_branch":
                b.succ.append(index[ins.text.split()[-1]])
                fall = False
            elif op == "s_endpgm":
                fall = False
        if fall and i + 1 < len(blocks):
            b.succ.append(i + 1)
    return blocks


def check_kernel(body, max_states: int = 4096) -> list:
    """Violations as (line, instruction, register set); empty = the ring is respected."""
    blocks = build_cfg(body)
    seen = [set() for _ in blocks]
    work = [(0, ())]
    violations = {}
    n_states = 0
    while work:
        bi, q = work.pop()
        if q in seen[bi]:
            continue
        seen[bi].add(q)
        n_states += 1
        if n_states > max_states:
            raise RuntimeError("state space of the ring did not close")
        q = list(q)
        for ins in blocks[bi].ins:
            op = ins.text.split()[0]
            if op == "s_waitcnt":
                m = _VMCNT.search(ins.text)
                if m:
                    keep = int(m.group(1))
                    if len(q) > keep:
                        q = q[len(q) - keep:] if keep else []
                continue
            regs = _vregs(ins.text)
            pending = set().union(*q) if q else set()
            bad = regs & pending
            if bad:
                violations[ins.line] = (ins.line, ins.text, tuple(sorted(bad)))
            if _VMEM.match(op):
                dest = frozenset()
                if ins.in_asm and "load" in op and "_lds_" not in op:
                    dest = frozenset(_vregs(ins.text.split(",")[0]))
                q.append(dest)
        if not any(q):
            q = []                                   # nothing tracked in flight: the count is irrelevant
        for s in blocks[bi].succ:
            work.append((s, tuple(q)))
    return sorted(violations.values())


def kernels_with_asm_loads(asm_text: str) -> dict:
    out = {}
    for name, body in split_kernels(asm_text).items():
        in_asm = False
        for _, raw in body:
            s = raw.strip()
            if s.startswith(";;#ASMSTART"):
                in_asm = True
            elif s.startswith(";;#ASMEND"):
                in_asm = False
            elif in_asm and re.match(r"(global|buffer)_load_dword", s):
                out[name] = body
                break
    return out
