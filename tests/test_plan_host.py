"""Host logic of the static buffer plan, through the C ABI, against the plan oracle: exact
integer equality on random programs, and on the launch lists of compiled decoder stacks (the
oracle plans the very program the library reports).  The lowering itself -- which launches a
decoder stack becomes -- is not a paper object: it is checked against lists written out by hand
below and, for more shapes, against the generator in tests/launch_list.py, as a regression
check.  No GPU: the plan functions are host code, and compiling a model launches nothing (the
weight pointers below are made-up aligned addresses that are never dereferenced).

Sec. "Phase 4: IR Analysis & Optimization" (Eq. "liveness", Alg. "Linear-Scan Buffer
Allocation"), Alg. "FX -> NPUIR Lowering".
"""
import ctypes as C
import random

import pytest

from oracle import plan_oracle as P
from paper_2604_16498_amd import binding as B
from launch_list import OPS, decoder_program
from test_plan_oracle_pins import max_alive, random_program


def to_lists(iv):
    return [(-1 if x is None else x[0]) for x in iv], [(-1 if x is None else x[1]) for x in iv]


@pytest.mark.parametrize("seed", range(30))
def test_plan_functions_match_the_oracle_on_random_programs(seed):
    rng = random.Random(300 + seed)
    prog, n = random_program(rng, rng.randint(1, 80), fan_in=rng.randint(1, 5))
    n += rng.randint(0, 2)                     # trailing registers nobody mentions
    iv = P.live_intervals(prog, n)
    start, end = B.forge_plan_liveness([o for o, _ in prog], [i for _, i in prog], n)
    assert (start, end) == to_lists(iv)
    assert B.forge_plan_dead_after(end, len(prog)) == P.dead_after(iv)
    buf, m = B.forge_plan_linear_scan(start, end)
    assert (buf, m) == P.linear_scan(iv)
    sizes = [rng.choice([0, 100, 256, 4096, 5000, 1 << 20]) for _ in range(n)]
    off, total, nb = B.forge_plan_workspace(start, end, sizes)
    assert (off, total, nb) == P.workspace_plan(iv, sizes)


def test_hand_worked_chain_through_the_abi():
    n = 7
    start, end = B.forge_plan_liveness(list(range(n)), [[]] + [[j - 1] for j in range(1, n)], n)
    assert start == list(range(n)) and end == [j + 1 for j in range(n - 1)] + [n - 1]
    buf, m = B.forge_plan_linear_scan(start, end)
    assert m == 2 and buf == [j % 2 for j in range(n)]


def test_empty_program():
    assert B.forge_plan_liveness([], [], 0) == ([], [])
    assert B.forge_plan_linear_scan([], []) == ([], 0)
    assert B.forge_plan_workspace([], [], []) == ([], 0, 0)
    start, end = B.forge_plan_liveness([], [], 3)
    assert start == [-1] * 3 and end == [-1] * 3
    assert B.forge_plan_workspace(start, end, [8, 8, 8]) == ([-1] * 3, 0, 0)


def test_malformed_programs_are_rejected():
    l = B.lib()
    ints = lambda v: (C.c_int * max(1, len(v)))(*v)
    s, e = ints([0, 0]), ints([0, 0])
    # register out of range, as output and as input
    assert l.forge_plan_liveness(1, ints([5]), ints([0, 0]), ints([]), 2, s, e) == 1
    assert l.forge_plan_liveness(1, ints([0]), ints([0, 1]), ints([2]), 2, s, e) == 1
    # in_begin not starting at zero / decreasing
    assert l.forge_plan_liveness(1, ints([0]), ints([1, 1]), ints([0]), 2, s, e) == 1
    assert l.forge_plan_liveness(2, ints([0, 1]), ints([0, 1, 0]), ints([0]), 2, s, e) == 1
    # NULL outputs
    assert l.forge_plan_liveness(1, ints([0]), ints([0, 0]), ints([]), 2, None, e) == 1
    # an interval that ends before it starts, or starts at -1 but has an end
    m = C.c_int(0)
    assert l.forge_plan_linear_scan(1, ints([3]), ints([2]), ints([0]), C.byref(m)) == 1
    assert l.forge_plan_linear_scan(1, ints([-1]), ints([2]), ints([0]), C.byref(m)) == 1
    with pytest.raises(B.ForgeError):
        B.forge_plan_dead_after([4], 2)


# ------------------------------------------------------------------ compiled decoder stacks

class Shape:
    def __init__(self, **kw):
        self.__dict__.update(kw)


def fake_model(shape, n_layers, tokens, dt, vocab=1000, n_pos=512, w8=False):
    """Descriptors whose pointers are distinct aligned made-up addresses."""
    addr = [0x10000]

    def ptr():
        addr[0] += 0x1000
        return addr[0]

    layers = []
    for _ in range(n_layers):
        d = B.BlockDesc()
        d.d_model, d.q_heads, d.kv_heads, d.head_dim, d.d_ff = (shape.d_model, shape.q_heads, shape.kv_heads,
                                                                shape.head_dim, shape.d_ff)
        d.norm, d.eps, d.mlp_act = B.NORM[shape.norm], 1e-5, B.ACT[shape.mlp_act]
        d.use_rope, d.rope_base, d.dt = int(shape.use_rope), 10000.0, dt
        for name in ("norm1_g", "w_qkv", "w_o", "norm2_g", "w_up", "w_down") + (
                ("s_qkv", "s_o", "s_up", "s_down") if w8 else ()):
            setattr(d, name, ptr())
        layers.append(d)
    m = B.ModelDesc()
    arr = (B.BlockDesc * n_layers)(*layers)
    m._layer_array = arr
    m.n_layers, m.layers = n_layers, C.cast(arr, C.POINTER(B.BlockDesc))
    m.vocab, m.n_pos, m.logits_ld = (vocab, n_pos, 0) if tokens else (0, 0, 0)
    m.wte, m.wpe = (ptr(), ptr()) if tokens else (None, None)
    m.normf_g, m.normf_b = ptr(), None
    return m


GPT = Shape(d_model=256, q_heads=4, kv_heads=4, head_dim=64, d_ff=1024, norm="layernorm",
            mlp_act="gelu_tanh", use_rope=False)
LLAMA = Shape(d_model=512, q_heads=4, kv_heads=2, head_dim=128, d_ff=1408, norm="rmsnorm",
              mlp_act="swiglu", use_rope=True)

# Which steps a launch absorbs, listed by hand per case (not computed by the library's rule):
# `rope` = q and k are rotated by launches of their own, `norm2` / `norm1` = the second / every
# first norm is a launch of its own.  A bf16 step of at most 64 rows folds all three into the
# reduce steps of its projections; a bf16 prompt rotates in the epilogue of its QKV projection
# (not on int8 weights) and keeps the norms apart; fp32 keeps everything apart.
CASES = [
    # name, shape, layers, tokens, dtype, batch, q_len, pos0, kv_cap, rope, norm2, norm1
    ("gpt_prefill_bf16", GPT, 3, True, B.FORGE_BF16, 2, 128, 0, 128, False, True, True),
    ("gpt_prefill_f32", GPT, 2, True, B.FORGE_F32, 1, 128, 0, 128, False, True, True),
    ("llama_prefill_bf16", LLAMA, 4, False, B.FORGE_BF16, 1, 256, 0, 256, False, True, True),
    ("llama_decode_bf16", LLAMA, 4, False, B.FORGE_BF16, 8, 1, 300, 301, False, False, False),
    ("llama_decode_f32", LLAMA, 2, False, B.FORGE_F32, 8, 1, 40, 64, True, True, True),
    ("gpt_decode_bf16", GPT, 12, True, B.FORGE_BF16, 4, 1, 100, 128, False, False, False),
    ("llama_decode_int8", LLAMA, 3, False, B.FORGE_BF16, 16, 1, 300, 320, False, False, False),
    # (an int8 prompt runs the bf16 kernels on a bf16 copy of each weight: the projection rotates)
    ("llama_prefill_int8", LLAMA, 2, False, B.FORGE_BF16, 1, 96, 0, 96, False, True, True),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_compiled_program_and_its_plan(case):
    name, shape, L, tokens, dt, batch, q_len, pos0, kv_cap, rope, norm2, norm1 = case
    w8 = name.endswith("int8")
    model = fake_model(shape, L, tokens, dt, w8=w8)
    cm = B.CompiledModel(model, batch, q_len, pos0, kv_cap)
    ops, out_reg, ins, reg_bytes, reg_offset = cm.program()
    ni, nr, _, nb = cm.counts()

    # the lowering (regression check against the fixture generator)
    prog, kinds = decoder_program(L, tokens, rope_separate=rope, norm2_separate=norm2, norm1_separate=norm1)
    assert (ni, nr) == (len(prog), len(kinds))
    assert ops == [p[0] for p in prog]
    assert out_reg == [p[1] for p in prog]
    assert ins == [p[2] for p in prog]

    # byte sizes of the tensor registers, from the shapes
    T = batch * q_len
    es = 2 if dt == B.FORGE_BF16 else 4
    want = {"h": T * shape.d_model * es, "y": T * shape.d_model * es,
            "q": T * shape.q_heads * shape.head_dim * es, "o": T * shape.q_heads * shape.head_dim * es,
            "u": T * shape.d_ff * es}
    for r, k in enumerate(kinds):
        if k in want:
            assert reg_bytes[r] == want[k], (r, k)
    # the scratch registers' sizes are the library's own business: they are an INPUT of the plan
    # below; here only that each is what the public size query of that launch reports
    act = B.ACT[shape.mlp_act]
    nqkv = (shape.q_heads + 2 * shape.kv_heads) * shape.head_dim
    hd = shape.q_heads * shape.head_dim
    l = B.lib()
    gws = (lambda M, N, K, a, _dt: l.forge_gemm_w8_workspace_bytes(M, N, K, a)) if w8 else l.forge_gemm_workspace_bytes
    # (a bf16 prompt that rotates in its QKV epilogue keeps a cos / sin table there instead:
    # one fp32 pair per row of the prompt and rotation pair)
    # (behind the bf16 copy of the weight when the weight is int8)
    rope_table = shape.use_rope and dt == B.FORGE_BF16 and q_len > 1 and T > 64
    w_copy = (nqkv * shape.d_model * 2 + 255) // 256 * 256 if w8 else 0
    def tail_ws(N, K):
        """A projection whose output is not a plain matrix (head split, or a row norm behind it):
        where the plain one of its shape is finished inside the GEMM (public query 0 for a decode
        step), this one keeps the single fp32 plane that its reduce step reads."""
        b = gws(T, N, K, 0, dt)
        return T * N * 4 if b == 0 and T <= 64 and dt == B.FORGE_BF16 and not w8 else b
    scratch = {"ws_qkv": w_copy + q_len * shape.head_dim * 4 if rope_table else tail_ws(nqkv, shape.d_model),
               "ws_o": tail_ws(shape.d_model, hd),
               "ws_up": gws(T, shape.d_ff, shape.d_model, act, dt),
               "ws_down": tail_ws(shape.d_model, shape.d_ff),
               "ws_attn": l.forge_attn_fused_workspace_bytes(batch, shape.q_heads, shape.kv_heads, q_len,
                                                             pos0 + q_len, shape.head_dim, dt),
               "ws_head": l.forge_gemm_workspace_bytes(T, 1000, shape.d_model, 0, dt)}
    for r, k in enumerate(kinds):
        if k in scratch:
            assert reg_bytes[r] == scratch[k], (r, k)

    # the plan (oracle parity): liveness and byte plan of the program the library reports, with
    # the sizes it reports, computed by the oracle
    iv = P.live_intervals(list(zip(out_reg, ins)), nr)
    off, total, bufs = P.workspace_plan(iv, reg_bytes)
    assert reg_offset == off
    assert cm.workspace_bytes() == total
    assert nb == bufs
    # fewer buffers than registers
    assert nb < nr
    cm.close()


def _names(prog):
    return [(OPS[op], out, ins) for op, out, ins in prog]


# One Llama-shaped decode step of two layers, eight rows, bf16, written out by hand from the
# layer's steps.  Registers are numbered as they appear: per instruction its output, then its
# second result, then its scratch area.  At this size the reduce step of the QKV projection
# rotates q and k, the one of the output projection also writes the second norm's rows (y2, a
# second result: listed among the inputs), and the one of the MLP down projection writes the NEXT
# layer's first-norm rows; the last layer's down projection writes the caller's output (the final
# norm) and adds the residual stream in place, so it has no output register.
LLAMA_DECODE_2L = [
    ("norm", 0, []),                      # y = Norm1(x), x is the caller's
    ("gemm_qkv", 1, [0, 2]),              # q (k, v go to the cache), scratch 2
    ("attn", 3, [1, 4]),                  # o, scratch 4
    ("gemm_res", 5, [3, 6, 7]),           # h = x + o Wo^T; second result y2 = 6; scratch 7
    ("gemm_act", 8, [6, 9]),              # u = act(y2 Wup^T), scratch 9
    ("gemm_res", 10, [8, 5, 11, 12]),     # h' = h + u Wdown^T; next layer's rows 11; scratch 12
    ("gemm_qkv", 13, [11, 14]),
    ("attn", 15, [13, 16]),
    ("gemm_res", 17, [15, 10, 18, 19]),
    ("gemm_act", 20, [18, 21]),
    ("gemm_res", -1, [20, 17, 22]),       # in place; the caller's output takes the final norm
]

# One GPT-shaped layer with token input and the tied head, a 256-row prompt: every step is a
# launch of its own (no rotary embedding in this family).
GPT_PREFILL_1L = [
    ("embed", 0, []),
    ("norm", 1, [0]),
    ("gemm_qkv", 2, [1, 3]),
    ("attn", 4, [2, 5]),
    ("gemm_res", 6, [4, 0, 7]),
    ("norm", 8, [6]),
    ("gemm_act", 9, [8, 10]),
    ("gemm_res", 11, [9, 6, 12]),
    ("norm", 13, [11]),
    ("gemm", -1, [13, 14]),
]


@pytest.mark.parametrize("hand,shape,L,tokens,batch,q_len,pos0,kv_cap,flags", [
    (LLAMA_DECODE_2L, LLAMA, 2, False, 8, 1, 300, 301, (False, False, False)),
    (GPT_PREFILL_1L, GPT, 1, True, 2, 128, 0, 128, (False, True, True)),
], ids=["llama_decode_2L", "gpt_prefill_1L"])
def test_lowering_against_hand_written_lists(hand, shape, L, tokens, batch, q_len, pos0, kv_cap, flags):
    cm = B.CompiledModel(fake_model(shape, L, tokens, B.FORGE_BF16), batch, q_len, pos0, kv_cap)
    ops, out_reg, ins, _, _ = cm.program()
    cm.close()
    assert list(zip(ops, out_reg, ins)) == _names(hand)
    # the fixture generator used for the other shapes writes the same list
    prog, _ = decoder_program(L, tokens, *flags)
    assert [tuple(p) for p in prog] == _names(hand)


# ------------------------------------------------------------------ the fixture generator itself

@pytest.mark.parametrize("tokens,rope,norm2", [(True, False, True), (False, True, True), (False, False, False)])
def test_decoder_program_shape(tokens, rope, norm2):
    L = 3
    prog, kinds = decoder_program(L, tokens, rope, norm2)
    per_layer = 6 + (2 if rope else 0) + (1 if norm2 else 0)
    assert len(prog) == L * per_layer + (3 if tokens else 1)
    # every register is written or first mentioned before any later use, numbering is dense
    iv = P.live_intervals([(o, i) for _, o, i in prog], len(kinds))
    assert all(x is not None for x in iv)
    starts = [s for s, _ in iv]
    assert starts == sorted(starts)
    # scratch areas live inside one instruction only
    assert all(iv[r][0] == iv[r][1] for r, k in enumerate(kinds) if k.startswith("ws_"))
    buf, m = P.linear_scan(iv)
    n = len(kinds)
    assert 0.0 < P.buffer_reduction(m, n) < 1.0
    assert m == max_alive(iv)


def test_decoder_program_buffer_count_does_not_grow_with_depth():
    counts = []
    for L in (1, 2, 12, 32):
        prog, kinds = decoder_program(L, True, False, True)
        iv = P.live_intervals([(o, i) for _, o, i in prog], len(kinds))
        counts.append(P.linear_scan(iv)[1])
    assert counts[1] == counts[2] == counts[3]
    assert counts[0] <= counts[1]


def test_buffer_count_is_independent_of_depth_and_reduction_grows():
    rho = []
    for L in (2, 8, 32):
        cm = B.CompiledModel(fake_model(GPT, L, True, B.FORGE_BF16), 2, 128, 0, 128)
        ni, nr, _, nb = cm.counts()
        rho.append((nb, 1 - nb / nr))
        cm.close()
    assert rho[0][0] == rho[1][0] == rho[2][0]
    assert rho[0][1] < rho[1][1] < rho[2][1]


def test_compile_rejects_bad_arguments():
    l = B.lib()
    model = fake_model(GPT, 2, True, B.FORGE_BF16)
    h = C.c_void_p(None)
    assert l.forge_compile_model(C.byref(model), 0, 128, 0, 128, C.byref(h)) == 1
    assert l.forge_compile_model(C.byref(model), 1, 128, 8, 128, C.byref(h)) == 1      # past the cache
    assert l.forge_compile_model(C.byref(model), 1, 128, 0, 1024, None) == 1
    assert l.forge_compile_model(C.byref(model), 1, 600, 0, 1024, C.byref(h)) == 1     # past n_pos = 512
    assert l.forge_compile_model(C.byref(model), 1, 2, 2**31 - 1, 1024, C.byref(h)) == 1  # pos0 + q_len wraps
    assert l.forge_compile_model(C.byref(model), 70000, 1, 0, 128, C.byref(h)) == 2       # batch past a grid dimension
    assert l.forge_compile_model(C.byref(model), 40000, 512, 0, 512, C.byref(h)) == 2     # more than 2^24 rows
    assert not h.value
    assert l.forge_compiled_run(None, None) == 1
    cm = B.CompiledModel(model, 1, 128, 0, 128)
    assert l.forge_compiled_run(cm._h, None) == 1                                        # not bound yet
    good = C.c_void_p(0x100000)
    assert l.forge_compiled_bind(cm._h, good, good, good, good, good, 0, good) == 3      # workspace too small
    assert l.forge_compiled_bind(cm._h, good, good, good, good, good, 1 << 40, None) == 1  # NULL stream
    cm.close()
