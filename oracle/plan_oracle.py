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
* the free pool is first in, first out, and buffers released in one step enter
  it in the order their intervals were activated;
* new buffers are numbered 0, 1, 2, ... in the order they are created.

Pins (tests/test_plan_oracle_pins.py): hand-worked programs (a chain, a
diamond, a fan-out); on random programs no two registers that share a buffer
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
    """Alg. "Linear-Scan Buffer Allocation".  Returns (buffer of each register, M);
    registers without an interval get buffer -1."""
    order = sorted((r for r, iv in enumerate(intervals) if iv is not None),
                   key=lambda r: (intervals[r][0], r))
    reg_to_buf = [-1] * len(intervals)
    active: List[Tuple[int, int]] = []     # (end, buffer), in activation order
    free_pool: List[int] = []
    n_bufs = 0
    for r in order:
        s, e = intervals[r]
        keep = []
        for (e_j, b_j) in active:
            if e_j < s:
                free_pool.append(b_j)
            else:
                keep.append((e_j, b_j))
        active = keep
        if free_pool:
            b = free_pool.pop(0)
        else:
            b = n_bufs
            n_bufs += 1
        reg_to_buf[r] = b
        active.append((e, b))
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


# ---------------------------------------------------------------------------------------
# The launch list of the decoder stack, written from the list of steps of one layer
# (first norm, QKV projection, rotary embedding of q and of k, fused attention, output
# projection with the residual add, second norm, MLP up with its activation, MLP down
# with the residual add), in the register form of Alg. "FX -> NPUIR Lowering": one output
# register per instruction, numbered in program order.  Tensors the caller owns (input,
# output, KV cache, weights) are constants, not registers.

OPS = {"embed": 0, "norm": 1, "gemm_qkv": 2, "rope_q": 3, "rope_k": 4, "attn": 5,
       "gemm_res": 6, "gemm_act": 7, "gemm": 8}


def decoder_program(n_layers: int, tokens: bool, rope_separate: bool, norm2_separate: bool,
                    norm1_separate: bool = True):
    """Returns (program, kinds): program = [(op, output_reg, input_regs)], kinds[r] names what
    register r holds ('h', 'y', 'q', 'o', 'u', 'ws_qkv', 'ws_o', 'ws_up', 'ws_down',
    'ws_attn', 'ws_head').

    Every projection and the attention carry a scratch register (its byte size may be zero).
    `rope_separate` = q and k are rotated by launches of their own; `norm2_separate` = the
    second norm is a launch of its own (else the output projection produces it as a second
    result next to the new residual stream; an instruction has one output register, so the
    normalised rows are listed among that instruction's inputs and start living there).
    `norm1_separate` = every layer starts with a norm launch of its own and the stack ends
    with one (else only the first layer does: the MLP down projection of a layer produces, as a
    second result, the rows that the next layer's first norm - after the last layer: the final
    norm - would; with no LM head those last rows are the caller's output and take no register,
    and the last residual stream, which nobody reads, is added in place).
    Registers are numbered in the order they are created: per instruction its output, then
    its second result, then its scratch area.
    With `tokens` the program starts with the embedding gather and ends with the tied
    LM head; otherwise the hidden states come from the caller and the final norm writes the
    caller's output.
    """
    program, kinds = [], []

    def new(kind):
        kinds.append(kind)
        return len(kinds) - 1

    def emit(op, out, ins):
        program.append((OPS[op], out, list(ins)))

    def scratch(kind):
        return [new(kind)]

    h = -1                                   # -1: the caller's input tensor
    if tokens:
        h = new("h")
        emit("embed", h, [])
    y_next = None
    for layer in range(n_layers):
        res = [h] if h >= 0 else []
        if norm1_separate or layer == 0:
            y = new("y")
            emit("norm", y, res)
        else:
            y = y_next
        q = new("q")
        emit("gemm_qkv", q, [y] + scratch("ws_qkv"))
        if rope_separate:
            emit("rope_q", -1, [q])
            emit("rope_k", -1, [])
        o = new("o")
        emit("attn", o, [q] + scratch("ws_attn"))
        h_mid = new("h")
        if norm2_separate:
            emit("gemm_res", h_mid, [o] + res + scratch("ws_o"))
            y2 = new("y")
            emit("norm", y2, [h_mid])
        else:
            y2 = new("y")
            emit("gemm_res", h_mid, [o] + res + [y2] + scratch("ws_o"))
        u = new("u")
        emit("gemm_act", u, [y2] + scratch("ws_up"))
        if norm1_separate:
            h_out = new("h")
            emit("gemm_res", h_out, [u, h_mid] + scratch("ws_down"))
        elif layer == n_layers - 1 and not tokens:
            # nobody reads the last residual stream: it is added in place, no new register
            h_out = -1
            emit("gemm_res", -1, [u, h_mid] + scratch("ws_down"))
        else:
            h_out = new("h")
            y_next = new("y")
            emit("gemm_res", h_out, [u, h_mid, y_next] + scratch("ws_down"))
        h = h_out
    if tokens:
        if norm1_separate:
            yf = new("y")
            emit("norm", yf, [h])
        else:
            yf = y_next
        emit("gemm", -1, [yf] + scratch("ws_head"))
    elif norm1_separate:
        emit("norm", -1, [h])
    return program, kinds
