"""Static check of the ring prefill kernels' gfx950 assembly.

The unit loop of csrc/prefill_bf16_ring.hip issues its LDS reads (and one scalar load) as inline
assembly that the compiler does not track, and waits for them by count.  The compiler believes such a
value is there as soon as the instruction has been issued, so nothing but the kernel's own waits keeps
it from touching the destination registers too early: a copy, a spill, or -- once the value is dead in
its eyes -- a reuse of the registers for something else while the read is still in flight, which
then lands on top of the new contents.  This module replays every kernel's instruction stream with a
model of the LDS counter (operations of a wave complete in order; s_waitcnt lgkmcnt(N) returns when
at most N are outstanding; scalar loads return out of order and are only known to be back after
lgkmcnt(0)) and reports every instruction that reads or writes a register while a load into it may
still be in flight.  Loops are replayed a second time from their head with the state of the back edge.
"""
from __future__ import annotations

import re
from typing import List, Tuple

_REG = re.compile(r"\b([vsa])(\d+)\b|\b([vsa])\[(\d+):(\d+)\]")


def _regs(text: str):
    out = set()
    for m in _REG.finditer(text):
        if m.group(1):
            out.add((m.group(1), int(m.group(2))))
        else:
            out.update((m.group(3), i) for i in range(int(m.group(4)), int(m.group(5)) + 1))
    return out


def kernels(asm_text: str):
    """Yields (name, [instruction lines]) for every kernel body in an assembly file."""
    name, body = None, []
    for line in asm_text.splitlines():
        m = re.match(r"^(_Z\w+):", line)
        if m:
            name, body = m.group(1), []
            continue
        if name is None:
            continue
        s = line.strip()
        if s.startswith(".Lfunc_end"):
            if any("s_endpgm" in b for b in body):
                yield name, body
            name = None
            continue
        if not s or s.startswith(";") and "ASM" not in s or s.startswith(".") and not s.startswith(".LBB"):
            continue
        body.append(s.split(";")[0].strip() if not s.startswith(";;#ASM") else s)


def lint(body: List[str]) -> List[Tuple[int, str, str]]:
    """Returns (line index, instruction, reason) for every hazard found in one kernel body."""
    problems = []
    labels = {l[:-1]: i for i, l in enumerate(body) if l.startswith(".LBB") and l.endswith(":")}
    replayed = set()

    def run(lo, hi, fifo, smem):
        i = lo
        while i < hi:
            ins = body[i]
            i += 1
            if not ins or ins.startswith(";;#ASM") or ins.endswith(":"):
                continue
            op = ins.split()[0]
            if op == "s_waitcnt":
                m = re.search(r"lgkmcnt\((\d+)\)", ins)
                if m:
                    n = int(m.group(1))
                    while len(fifo) > n:
                        fifo.pop(0)
                    if n == 0:
                        smem.clear()
                continue
            touched = _regs(ins.split(None, 1)[1] if " " in ins else "")
            for dest in list(fifo) + list(smem):
                if dest and touched & dest:
                    # the issuing instruction itself is handled below; anything else is a hazard
                    problems.append((i - 1, ins, "touches %s while a load into it may be in flight" % sorted(touched & dest)[:4]))
                    break
            if op.startswith("ds_read") or op.startswith("ds_load"):
                fifo.append(frozenset(_regs(ins.split(None, 1)[1].split(",")[0])))
            elif op.startswith("ds_write") or op.startswith("ds_store"):
                fifo.append(frozenset())
            elif op.startswith("s_load") or op.startswith("s_buffer_load"):
                smem.append(frozenset(_regs(ins.split(None, 1)[1].split(",")[0])))
            elif op in ("s_branch",) or op.startswith("s_cbranch"):
                tgt = ins.split()[-1]
                if tgt in labels and labels[tgt] < i and (tgt, i) not in replayed:
                    replayed.add((tgt, i))
                    run(labels[tgt], i, list(fifo), list(smem))  # one more trip round the loop with this state
        return fifo, smem

    run(0, len(body), [], [])
    return problems
