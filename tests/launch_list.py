"""Expected launch list of a decoder stack, in register form: a TEST FIXTURE.

Written from the list of steps of one layer (first norm, QKV projection, rotary embedding of q
and of k, fused attention, output projection with the residual add, second norm, MLP up with its
activation, MLP down with the residual add), in the register form of Alg. "FX -> NPUIR Lowering":
one output register per instruction, numbered in program order; tensors the caller owns (input,
output, KV cache, weights) are constants, not registers.

This is not part of the oracle: the paper defines no decoder launch list, so comparing the
library's lowering with this generator is a regression check of the lowering (pinned itself by the
hand-written lists in tests/test_plan_host.py), not parity with the paper.  Which steps a launch
absorbs is passed in by the caller, case by case.
"""
from __future__ import annotations

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
