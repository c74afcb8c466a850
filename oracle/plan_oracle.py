"""CPU oracle for the static buffer plan of a flat launch list.  TEST INFRASTRUCTURE ONLY.

Only the tests may import this module; the product never does and this module
imports nothing from the product.

What it computes (Sec. "Phase 4: IR Analysis & Optimization"):

* the live interval [s_i, e_i] of every virtual register of a flat instruction
  list -- s_i the index of the instruction that writes it, e_i the index of the
  last instruction that reads it (Eq. "liveness") -- and the dead-after map
  that lists, per instruction index, the registers whose last use is there;
* the linear-scan assignment of N virtual registers to M physical buffer slots
  (Alg. "Linear-Scan Buffer Allocation"): intervals are visited by ascending
  start; before each one, every active interval that ended strictly before its
  start gives its buffer back to the free pool; the interval takes a buffer
  from the pool if one is there, else a new buffer;
* the buffer reduction ratio rho_buf = 1 - M/N (Eq. "buf_reduction").

The paper's slots have no byte size.  `workspace_plan` is the one extension
used to turn slots into byte offsets of one workspace: registers are grouped
by their byte size (registers that live within one instruction only, such as
scratch areas, form a single group sized to the largest of them), each group
is assigned by its own linear scan, and the groups are laid out one after the
other (so a buffer never has to hold a register larger than its group's).

Readings where the paper leaves the choice open:
* a register that no instruction writes (a scratch area an instruction uses
  for itself) starts at its first mention; a register nobody reads ends where
  it starts;
* intervals with equal start are visited by ascending register number;
* the algorithm box only says that a buffer is popped from the free pool: the
  lowest-numbered free buffer is taken;
* new buffers are numbered 0, 1, 2, ... in the order they are created.

`linear_scan` is written from that statement directly (for every interval, look
at all intervals visited before it), with no active list and no pool, so that
a reader can check it by eye and so that it shares no structure with the
heap-based sweep of the library.

Pins (tests/test_plan_oracle_pins.py): hand-worked programs (a chain, a
diamond, a fan-out, the choice among several free buffers); on random programs no two registers that share a buffer
have intersecting closed intervals and M equals the largest number of
intervals alive at one index (greedy colouring by start is optimal on interval
graphs), both checked by brute force over all pairs / indices; every register
appears in the dead-after map exactly once, at its end; a planted mistake in the
expiry test (<= for <) is caught by the interference check.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

Instr = Tuple[int, Sequence[int]]          # (output_reg or -1, input_regs)
Interval = Optional[Tuple[int, int]]       # None: the register is never mentioned


def live_intervals(program: Sequence[Instr], n_regs: int) -> List[Interval]:
    """Eq. "liveness": start = index of the write, end = index of the last read."""
    start: List[Optional[int]] = [None] * n_regs
    end: List[Optional[int]] = [None] * n_regs
    for j, (out, ins) in enumerate(program):
        mentioned = list(ins) + ([out] if out >= 0 else [])
        for r in mentioned:
            if start[r] is None:
                start[r] = j
            end[r] = j
    return [None if start[r] is None else (start[r], end[r]) for r in range(n_regs)]


def dead_after(intervals: Sequence[Interval]) -> Dict[int, List[int]]:
    """Instruction index -> registers whose last use is that instruction (ascending)."""
    out: Dict[int, List[int]] = {}
    for r, iv in enumerate(intervals):
        if iv is not None:
            out.setdefault(iv[1], []).append(r)
    return out


def linear_scan(intervals: Sequence[Interval]) -> Tuple[List[int], int]:
    """Alg. "Linear-Scan Buffer Allocation", written as what it assigns rather than how: the
    intervals are visited by ascending start; a buffer is taken while an already visited
    interval that has not ended strictly before this start holds it; the interval gets the
    lowest-numbered buffer nobody holds (a free one if there is one, otherwise the next new
    number).  Returns (buffer of each register, M); registers without an interval get -1."""
    order = sorted((r for r, iv in enumerate(intervals) if iv is not None),
                   key=lambda r: (intervals[r][0], r))
    reg_to_buf = [-1] * len(intervals)
    visited: List[int] = []
    for r in order:
        s, _ = intervals[r]
        held = {reg_to_buf[j] for j in visited if not intervals[j][1] < s}
        b = 0
        while b in held:
            b += 1
        reg_to_buf[r] = b
        visited.append(r)
    n_bufs = 1 + max(reg_to_buf) if order else 0
    return reg_to_buf, n_bufs


def buffer_reduction(n_bufs: int, n_regs: int) -> float:
    """Eq. "buf_reduction"."""
    return 1.0 - n_bufs / n_regs


def workspace_plan(intervals: Sequence[Interval], nbytes: Sequence[int],
                   align: int = 256) -> Tuple[List[int], int, int]:
    """Byte offset of every register inside one workspace, the workspace size and the
    number of buffers.  Registers of equal byte size form a group, except that all registers
    living within a single instruction (start == end: scratch areas, results nobody reads)
    form one group of their own whose buffers span the largest of them.  Each group gets its
    own linear scan; groups follow each other in the order of their first register."""
    groups: Dict[object, List[int]] = {}
    for r, iv in enumerate(intervals):
        if iv is not None:
            key = "single" if iv[0] == iv[1] else nbytes[r]
            groups.setdefault(key, []).append(r)
    offset = [-1] * len(intervals)
    base, total_bufs = 0, 0
    for _, regs in groups.items():             # dicts keep insertion order
        sub = [intervals[r] for r in regs]
        buf, m = linear_scan(sub)
        size = max(nbytes[r] for r in regs)
        stride = (size + align - 1) // align * align
        for r, b in zip(regs, buf):
            offset[r] = base + b * stride
        base += m * stride
        total_bufs += m
    return offset, base, total_bufs
