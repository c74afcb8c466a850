"""GPU parity: each C-ABI operator against the fp64 oracle on the same seeded inputs.
Sizes span several tiles and a ragged tail; the tolerance is the one stated for the path
(fp32: max-abs 1e-4; bf16: l2 error <= 2e-2 of the l2 norm and, per element,
|got - ref| <= 2e-2 |ref| + 2e-2 rms(ref); see util.py)."""
import math

import numpy as np
import pytest
import torch

from oracle import forge_oracle as O
from paper_2604_16498_amd import inputs as I
from util import check, dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def F():
    from paper_2604_16498_amd import binding
    binding.lib()
    return binding


def tdtype(bf16):
    return torch.bfloat16 if bf16 else torch.float32


# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
@pytest.mark.parametrize("kind", ["layernorm", "rmsnorm"])
@pytest.mark.parametrize("rows,d", [(128, 768), (64, 4096), (37, 2048), (5, 8), (3, 16384),
                                    (1000, 1032), (9, 520), (8192, 768), (13, 3000), (6, 5000), (1100, 1288), (2048, 2048)])
def test_residual_norm(F, bf16, kind, rows, d):
    x = I.normal(60, 0, "x", (rows, d), 1.5, mean=0.3, bf16=bf16)
    dl = I.normal(60, 0, "delta", (rows, d), 0.7, bf16=bf16)
    g = I.normal(60, 0, "norm1_g", (d,), 0.2, mean=1.0, bf16=bf16)
    b = I.normal(60, 0, "norm1_b", (d,), 0.2, bf16=bf16)
    for use_delta in (True, False):
        h_ref, y_ref = O.residual_norm(x, dl if use_delta else None, g, b, 1e-5, kind)
        tx, tg, tb = dev(x, bf16), dev(g, bf16), dev(b, bf16)
        td = dev(dl, bf16) if use_delta else None
        th = torch.empty_like(tx) if use_delta else None
        ty = torch.empty_like(tx)
        F.forge_residual_norm(tx, td, tg, tb, th, ty, 1e-5, kind)
        torch.cuda.synchronize()
        check(ty, y_ref, bf16, "y")
        if use_delta:
            check(th, h_ref, bf16, "h")


# ---------------------------------------------------------------------------------------------
GEMM_SHAPES = [(128, 2304, 768), (100, 200, 72), (1, 8, 8), (300, 515, 264), (257, 1001, 64),
               (64, 768, 3072), (513, 384, 136), (64, 4096, 512), (33, 130, 1032), (2, 1536, 4096)]


@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
@pytest.mark.parametrize("act", ["none", "gelu_tanh", "gelu_erf", "relu", "silu", "swiglu"])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_bias_act(F, bf16, act, M, N, K):
    wn = 2 * N if act == "swiglu" else N
    x = I.normal(61, 0, "x", (M, K), 1.0, bf16=bf16)
    w = I.normal(61, 0, "w_up", (wn, K), 1.0 / math.sqrt(K), bf16=bf16)
    b = I.normal(61, 0, "b_up", (wn,), 0.5, bf16=bf16)
    r = I.normal(61, 0, "residual", (M, N), 1.0, bf16=bf16)
    tx, tw, tb, tr = (dev(a, bf16) for a in (x, w, b, r))
    for use_b, use_r in ((True, True), (False, False)):
        ref = O.gemm_bias_act(x, w, b if use_b else None, r if use_r else None, act)
        ty = torch.empty(M, N, dtype=tdtype(bf16), device="cuda")
        ws = F.workspace(F.forge_gemm_workspace_bytes(M, N, K, act, tdtype(bf16)))
        F.forge_gemm_bias_gelu(tx, tw, tb if use_b else None, tr if use_r else None, ty, act, ws)
        torch.cuda.synchronize()
        check(ty, ref, bf16, "gemm %s" % act)


@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
@pytest.mark.parametrize("M,N,K", [(40, 136, 64), (200, 515, 72)])
def test_gated_weight_with_alternating_rows(F, bf16, M, N, K):
    """A gated weight stored (gate 0, up 0, gate 1, up 1, ...) is re-laid once into gate rows, then
    up rows (bit-exact row permutation, weights and bias), and the SwiGLU GEMM on it matches the
    oracle on the blocked weight."""
    w = I.normal(67, 0, "w_up", (2 * N, K), 1.0 / math.sqrt(K), bf16=bf16)     # blocked: gate rows, up rows
    b = I.normal(67, 0, "b_up", (2 * N,), 0.5, bf16=bf16)
    x = I.normal(67, 0, "x", (M, K), 1.0, bf16=bf16)
    wi = np.empty_like(w); wi[0::2] = w[:N]; wi[1::2] = w[N:]                      # what a caller holds
    bi = np.empty_like(b); bi[0::2] = b[:N]; bi[1::2] = b[N:]
    tw = F.forge_deinterleave_gated_rows(dev(wi, bf16))
    tb = F.forge_deinterleave_gated_rows(dev(bi, bf16))
    torch.cuda.synchronize()
    assert np.array_equal(host(tw), w.astype(np.float64)) and np.array_equal(host(tb), b.astype(np.float64))
    q = torch.arange(2 * 7 * 5, dtype=torch.int8, device="cuda").reshape(14, 5)    # odd row size: byte copies
    got = F.forge_deinterleave_gated_rows(q).cpu().numpy()
    assert np.array_equal(got, np.concatenate([q.cpu().numpy()[0::2], q.cpu().numpy()[1::2]]))
    ty = torch.empty(M, N, dtype=tdtype(bf16), device="cuda")
    ws = F.workspace(F.forge_gemm_workspace_bytes(M, N, K, "swiglu", tdtype(bf16)))
    F.forge_gemm_bias_gelu(dev(x, bf16), tw, tb, None, ty, "swiglu", ws)
    torch.cuda.synchronize()
    check(ty, O.gemm_bias_act(x, w, b, None, "swiglu"), bf16, "swiglu on a re-laid weight")


@pytest.mark.parametrize("epi", ["bias+residual", "bias", "residual", "none"])
@pytest.mark.parametrize("M,N,K,ld", [(300, 1001, 128, 1008), (257, 515, 64, 520), (130, 50257, 64, 50264)])
def test_gemm_padded_row_stride(F, M, N, K, ld, epi):
    """Odd N with a padded, 16-byte aligned row stride takes the persistent kernel with or
    without a bias / residual (the ragged last 8-column chunk of a row takes its bias element by
    element and its residual from inside the padded stride); the padding stays untouched."""
    x = I.normal(67, 0, "x", (M, K), 1.0, bf16=True)
    w = I.normal(67, 0, "w_up", (N, K), 0.1, bf16=True)
    b = I.normal(67, 0, "b_up", (N,), 0.5, bf16=True) if "bias" in epi else None
    r = I.normal(67, 0, "residual", (M, ld), 1.0, bf16=True) if "residual" in epi else None
    ref = O.gemm_bias_act(x, w, b, None if r is None else r[:, :N], "gelu_tanh")
    ty = torch.full((M, ld), 7.0, dtype=torch.bfloat16, device="cuda")
    assert "pers" in F.forge_gemm_variant(M, N, K, "gelu_tanh", torch.bfloat16, ldy=ld)
    F.forge_gemm_bias_gelu(dev(x, True), dev(w, True), dev(b, True), dev(r, True), ty, "gelu_tanh", n=N)
    torch.cuda.synchronize()
    check(ty[:, :N], ref, True, "padded-stride gemm, %s" % epi)
    assert torch.all(ty[:, N:] == 7.0)


@pytest.mark.parametrize("M,N,K,act,use_b,use_r,ld", [
    (5137, 1832, 128, "none", True, True, 0),        # 128-tiles: 615 > resident blocks, K shorter than the store window
    (5137, 1832, 640, "gelu_tanh", True, False, 0),  # parked rows drain inside the next k loop
    (5137, 1825, 640, "none", False, False, 1832),   # ragged last column chunk, padded row stride
    (5200, 1792, 192, "none", False, True, 0),       # residual only
    (5893, 5896, 192, "none", True, True, 0),        # 256-tiles: 576 > resident blocks, ragged edges
    (5893, 5891, 64, "relu", False, False, 5896),    # 256-tiles, odd N
    (5893, 5891, 128, "gelu_tanh", True, True, 5896),  # 256-tiles, odd N, bias and residual on the ragged chunk
    (5137, 1825, 640, "none", True, True, 1832),     # 128-tiles, odd N, bias and residual
    (5893, 2824, 128, "swiglu", True, False, 0),     # gated 256 x 128 output tiles
])
def test_gemm_many_tiles_per_block(F, M, N, K, act, use_b, use_r, ld):
    """More tiles than resident blocks: every persistent block walks over several tiles, edge
    tiles included, so the cross-tile prefetch and the deferred row stores are exercised."""
    wn = 2 * N if act == "swiglu" else N
    ldy = ld or N
    x = I.normal(68, 0, "x", (M, K), 1.0, bf16=True)
    w = I.normal(68, 0, "w_up", (wn, K), 1.0 / math.sqrt(K), bf16=True)
    b = I.normal(68, 0, "b_up", (wn,), 0.5, bf16=True) if use_b else None
    r = I.normal(68, 0, "residual", (M, ldy), 1.0, bf16=True) if use_r else None
    ref = O.gemm_bias_act(x, w, b, None if r is None else r[:, :N], act)
    assert "pers" in F.forge_gemm_variant(M, N, K, act, torch.bfloat16, ldy=ldy)
    ty = torch.full((M, ldy), 7.0, dtype=torch.bfloat16, device="cuda")
    F.forge_gemm_bias_gelu(dev(x, True), dev(w, True), None if b is None else dev(b, True),
                           None if r is None else dev(r, True), ty, act, n=N)
    torch.cuda.synchronize()
    check(ty[:, :N], ref, True, "persistent gemm %s" % act)
    assert torch.all(ty[:, N:] == 7.0)
    again = torch.full((M, ldy), 7.0, dtype=torch.bfloat16, device="cuda")
    F.forge_gemm_bias_gelu(dev(x, True), dev(w, True), None if b is None else dev(b, True),
                           None if r is None else dev(r, True), again, act, n=N)
    torch.cuda.synchronize()
    assert torch.equal(again, ty)


@pytest.mark.parametrize("M,N,K,act,use_b,use_r,ld", [
    (64, 24576, 256, "none", True, True, 0),           # 192 blocks of 128 weight rows: the smallest fused case
    (64, 24576, 192, "gelu_tanh", True, False, 0),
    (33, 24578, 128, "silu", False, True, 24584),      # ragged last chunk, padded row stride, fewer than 64 rows
    (1, 30000, 64, "relu", True, False, 0),            # a single row, a single slab
    (64, 12288, 256, "swiglu", True, False, 0),        # gated: 64 gate rows + their 64 up rows per block
    (40, 12296, 128, "swiglu", False, False, 0),       # gated, outputs not a multiple of 64
    (17, 50257, 128, "none", False, False, 50264),     # an LM head at decode size
    (64, 24576, 128, "gelu_erf", True, True, 0),
    # a short reduction (K < 1024) is one k range whatever the number of weight rows
    (8, 3072, 768, "gelu_tanh", True, False, 0),       # the GPT-2-small MLP up projection of a decode step
    (64, 1001, 512, "none", True, True, 1008),
    (1, 8, 64, "silu", False, False, 0),
    (5, 704, 960, "swiglu", True, False, 0),
])
def test_gemm_decode_sized_finishes_in_the_gemm(F, M, N, K, act, use_b, use_r, ld):
    """At most 64 rows against enough weight rows for one k range of 128-row blocks to cover the
    chip, or a reduction short enough to be one k range anyway: the weight-streaming kernel applies
    bias, activation and residual itself (no partial planes, no reduce launch) and needs no
    workspace."""
    wn = 2 * N if act == "swiglu" else N
    ldy = ld or N
    x = I.normal(69, 0, "x", (M, K), 1.0, bf16=True)
    w = I.normal(69, 0, "w_up", (wn, K), 1.0 / math.sqrt(K), bf16=True)
    b = I.normal(69, 0, "b_up", (wn,), 0.5, bf16=True) if use_b else None
    r = I.normal(69, 0, "residual", (M, ldy), 1.0, bf16=True) if use_r else None
    ref = O.gemm_bias_act(x, w, b, None if r is None else r[:, :N], act)
    assert F.forge_gemm_variant(M, N, K, act, torch.bfloat16, ldy=ldy) == "gemm_bf16_wstream_fused<128>"
    assert F.forge_gemm_workspace_bytes(M, N, K, act, torch.bfloat16) == 0
    ty = torch.full((M, ldy), 7.0, dtype=torch.bfloat16, device="cuda")
    args = (dev(x, True), dev(w, True), None if b is None else dev(b, True), None if r is None else dev(r, True))
    F.forge_gemm_bias_gelu(*args, ty, act, None, n=N)
    torch.cuda.synchronize()
    check(ty[:, :N], ref, True, "fused decode gemm %s" % act)
    assert torch.all(ty[:, N:] == 7.0)
    again = torch.full((M, ldy), 7.0, dtype=torch.bfloat16, device="cuda")
    F.forge_gemm_bias_gelu(*args, again, act, None, n=N)
    torch.cuda.synchronize()
    assert torch.equal(again, ty)


@pytest.mark.parametrize("M,N,K,act", [
    (128, 512, 2048, "none"), (130, 520, 4096, "gelu_tanh"), (257, 256, 14336, "none"),
    (100, 384, 2048, "swiglu"), (512, 128, 8192, "silu"),
])
def test_gemm_few_tiles_long_k(F, M, N, K, act):
    """A prompt-sized M against a long reduction: few output tiles, so the k loop is split over
    the chip when the caller provides the workspace; without it the same problem runs unsplit."""
    wn = 2 * N if act == "swiglu" else N
    x = I.normal(69, 0, "x", (M, K), 1.0, bf16=True)
    w = I.normal(69, 0, "w_up", (wn, K), 1.0 / math.sqrt(K), bf16=True)
    b = I.normal(69, 0, "b_up", (wn,), 0.5, bf16=True)
    r = I.normal(69, 0, "residual", (M, N), 1.0, bf16=True)
    ref = O.gemm_bias_act(x, w, b, r, act)
    need = F.forge_gemm_workspace_bytes(M, N, K, act, torch.bfloat16)
    assert need > 0
    tx, tw, tb, tr = (dev(a, True) for a in (x, w, b, r))
    y1 = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    F.forge_gemm_bias_gelu(tx, tw, tb, tr, y1, act, F.workspace(need))
    y2 = torch.empty_like(y1)
    F.forge_gemm_bias_gelu(tx, tw, tb, tr, y2, act)          # no workspace: unsplit
    torch.cuda.synchronize()
    check(y1, ref, True, "split-k gemm %s" % act)
    check(y2, ref, True, "unsplit gemm %s" % act)
    y3 = torch.empty_like(y1)
    F.forge_gemm_bias_gelu(tx, tw, tb, tr, y3, act, F.workspace(need))
    torch.cuda.synchronize()
    assert torch.equal(y1, y3)


def _random_gemm_cases():
    rng = np.random.default_rng(20260416)
    cases = []
    for _ in range(36):
        M = int(rng.choice([1, 7, 63, 64, 65, 127, 128, 129, 200, 255, 256, 257, 511, 640, 1000, 2049]))
        N = int(rng.choice([8, 40, 64, 120, 128, 136, 248, 256, 264, 392, 513, 1000, 1031, 2056]))
        K = int(rng.choice([8, 64, 72, 128, 192, 200, 512, 1024, 1088, 2048]))
        act = str(rng.choice(["none", "gelu_tanh", "gelu_erf", "relu", "silu", "swiglu"]))
        cases.append((M, N, K, act, bool(rng.integers(2)), bool(rng.integers(2)), bool(rng.integers(2))))
    return cases


@pytest.mark.parametrize("M,N,K,act,use_b,use_r,pad", _random_gemm_cases())
def test_gemm_random_shapes(F, M, N, K, act, use_b, use_r, pad):
    """Seeded sweep over shapes around the tile, slab and alignment boundaries of every GEMM
    variant (decode-sized, tile kernels with and without k split, generic fallback), with and
    without bias / residual / padded output rows, workspace always provided."""
    wn = 2 * N if act == "swiglu" else N
    ldy = (N + 15) // 8 * 8 if pad else N
    x = I.normal(79, 0, "x", (M, K), 1.0, bf16=True)
    w = I.normal(79, 0, "w_up", (wn, K), 1.0 / math.sqrt(K), bf16=True)
    b = I.normal(79, 0, "b_up", (wn,), 0.5, bf16=True) if use_b else None
    r = I.normal(79, 0, "residual", (M, ldy), 1.0, bf16=True) if use_r else None
    ref = O.gemm_bias_act(x, w, b, None if r is None else r[:, :N], act)
    ty = torch.full((M, ldy), 7.0, dtype=torch.bfloat16, device="cuda")
    ws = F.workspace(max(256, F.forge_gemm_workspace_bytes(M, N, K, act, torch.bfloat16)))
    F.forge_gemm_bias_gelu(dev(x, True), dev(w, True), None if b is None else dev(b, True),
                           None if r is None else dev(r, True), ty, act, ws, n=N)
    torch.cuda.synchronize()
    check(ty[:, :N], ref, True, "gemm %s %dx%dx%d via %s" % (act, M, N, K, F.forge_gemm_variant(M, N, K, act, torch.bfloat16, ldy=ldy)))
    assert torch.all(ty[:, N:] == 7.0)


def test_gemm_residual_in_place(F):
    M, N, K = 200, 256, 128
    x = I.normal(62, 0, "x", (M, K), 1.0, bf16=True)
    w = I.normal(62, 0, "w_o", (N, K), 0.1, bf16=True)
    r = I.normal(62, 0, "residual", (M, N), 1.0, bf16=True)
    ref = O.gemm_bias_act(x, w, None, r, "none")
    ty = dev(r, True)
    F.forge_gemm_bias_gelu(dev(x, True), dev(w, True), None, ty, ty, "none")
    torch.cuda.synchronize()
    check(ty, ref, True, "in-place residual")


# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("B,Hq,Hkv,Sq,Skv,dh,mb,mh", [
    (2, 4, 2, 100, 100, 64, True, True),      # mask per batch and head
    (3, 4, 4, 128, 128, 128, True, False),    # padded sequences: per batch, all heads
    (1, 8, 2, 300, 333, 128, False, False),   # one plane for everything, odd kv_len
    (2, 4, 1, 1, 200, 64, True, True),        # single query row
    (1, 2, 2, 520, 520, 64, False, True),     # several query blocks
])
def test_attn_fused_masked(F, bf16, causal, B, Hq, Hkv, Sq, Skv, dh, mb, mh):
    """Additive mask on the scaled scores: random finite values plus -inf on a padded tail of
    keys (different per sequence when the mask has a batch axis)."""
    q = I.normal(66, 0, "q", (B, Hq, Sq, dh), 1.0, bf16=bf16)
    k = I.normal(66, 0, "k_cache", (B, Hkv, Skv, dh), 1.0, bf16=bf16)
    v = I.normal(66, 0, "v_cache", (B, Hkv, Skv, dh), 1.0, bf16=bf16)
    mask = I.normal(66, 0, "misc", (B if mb else 1, Hq if mh else 1, Sq, Skv), 1.5).astype(np.float32)
    for b in range(mask.shape[0]):
        pad = (7 * (b + 1)) % max(1, min(Skv - Sq if causal else Skv, 40))     # keep key 0 for every row
        if pad and not (causal and Skv - pad < Sq):
            mask[b, :, :, Skv - pad:] = -np.inf
    scale = 1 / math.sqrt(dh)
    ref = O.attention(q, k, v, scale, causal, mask)
    out = torch.empty(B, Sq, Hq * dh, dtype=tdtype(bf16), device="cuda")
    F.forge_attn_fused_masked(dev(q, bf16), dev(k, bf16), dev(v, bf16), torch.from_numpy(mask).cuda(), out,
                              scale=scale, causal=causal)
    torch.cuda.synchronize()
    check(out, ref, bf16, "masked attention")


# ---------------------------------------------------------------------------------------------
ATTN_SHAPES = [  # B, Hq, Hkv, Sq, Skv, cap, dh
    (1, 12, 12, 128, 128, 128, 64),
    (2, 8, 2, 100, 100, 100, 128),
    (2, 4, 4, 1, 300, 320, 64),
    (1, 4, 2, 70, 200, 256, 128),
    (1, 2, 1, 333, 333, 333, 64),
    (3, 8, 2, 1, 1, 8, 128),
    (1, 2, 2, 257, 257, 257, 128),
    (1, 4, 2, 1000, 1000, 1000, 128),
    (2, 3, 3, 700, 700, 704, 64),
    (1, 2, 1, 130, 900, 900, 128),
    (2, 8, 2, 1, 2049, 2112, 128),
    (1, 8, 4, 1, 700, 704, 64),
    (1, 6, 2, 1, 300, 300, 128),
    (2, 4, 4, 1, 257, 257, 128),
    # decode with many (sequence, KV head) pairs: one block walks the whole cache, no combine
    (66, 8, 8, 1, 777, 800, 64),
    (130, 8, 4, 1, 45, 64, 128),
    # ... and with about one pair per CU: two row ranges
    (33, 32, 8, 1, 1000, 1000, 128),
    # decode with 3, 5, 6, 7, 8 and 16 query heads per KV head (16: two blocks of 8 per KV head)
    (2, 64, 8, 1, 513, 520, 128),
    (70, 16, 2, 1, 300, 300, 64),
    (2, 10, 2, 1, 900, 900, 64),
    (1, 12, 2, 1, 1500, 1504, 128),
    (3, 7, 1, 1, 260, 264, 64),
    (1, 32, 2, 1, 400, 400, 128),
    # larger groups in several blocks per KV head: 32 = 4 x 8 (one KV head), 12 = 2 x 6, 24 = 3 x 8,
    # 9 = 3 x 3, with and without row ranges; 11 has no such split (vector-ALU path)
    (3, 32, 1, 1, 1100, 1104, 128),
    (40, 32, 1, 1, 300, 320, 64),
    (2, 24, 2, 1, 700, 704, 64),
    (70, 24, 1, 1, 200, 200, 128),
    (2, 9, 1, 1, 530, 536, 128),
    (2, 11, 1, 1, 140, 144, 64),
]


@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("B,Hq,Hkv,Sq,Skv,cap,dh", ATTN_SHAPES)
def test_attn_fused(F, bf16, causal, B, Hq, Hkv, Sq, Skv, cap, dh):
    q = I.normal(63, 0, "q", (B, Hq, Sq, dh), 1.0, bf16=bf16)
    k = I.normal(63, 0, "k", (B, Hkv, cap, dh), 1.0, bf16=bf16)
    v = I.normal(63, 0, "v", (B, Hkv, cap, dh), 1.0, bf16=bf16)
    scale = 1.0 / math.sqrt(dh)
    ref = O.attention(q, k[:, :, :Skv], v[:, :, :Skv], scale, causal)
    tq, tk, tv = dev(q, bf16), dev(k, bf16), dev(v, bf16)
    out = torch.empty(B, Sq, Hq * dh, dtype=tdtype(bf16), device="cuda")
    ws = F.workspace(F.forge_attn_fused_workspace_bytes(B, Hq, Hkv, Sq, Skv, dh, tdtype(bf16)))
    F.forge_attn_fused(tq, tk, tv, out, kv_len=Skv, scale=scale, causal=causal, workspace=ws)
    torch.cuda.synchronize()
    check(out, ref, bf16, "attention")


def _random_attn_cases():
    rng = np.random.default_rng(16498)
    cases = []
    for _ in range(28):          # prompts: query and key counts around the 32-query / 64-key / 256-query boundaries
        B = int(rng.integers(1, 4)); Hkv = int(rng.choice([1, 2, 3])); G = int(rng.choice([1, 1, 2, 3, 4, 8]))
        Sq = int(rng.choice([2, 31, 33, 64, 65, 127, 129, 255, 256, 257, 300, 511, 513, 700, 1025]))
        Skv = Sq + int(rng.choice([0, 0, 0, 1, 63, 64, 100, 300]))
        cases.append((B, Hkv * G, Hkv, Sq, Skv, Skv + int(rng.choice([0, 8, 40])), int(rng.choice([64, 128])),
                      bool(rng.integers(2))))
    for _ in range(28):          # one query per sequence: every group size, caches around the 128 / 256-row range sizes
        B = int(rng.choice([1, 2, 3, 8, 33, 70])); Hkv = int(rng.choice([1, 2, 4])); G = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 12, 16, 24, 32]))
        Skv = int(rng.choice([1, 2, 16, 17, 127, 128, 129, 255, 256, 257, 511, 512, 513, 1000, 1500]))
        cases.append((B, Hkv * G, Hkv, 1, Skv, Skv + int(rng.choice([0, 8, 64])), int(rng.choice([64, 128])), True))
    return cases


@pytest.mark.parametrize("B,Hq,Hkv,Sq,Skv,cap,dh,causal", _random_attn_cases())
def test_attn_random_shapes(F, B, Hq, Hkv, Sq, Skv, cap, dh, causal):
    """Seeded sweep over bf16 attention shapes: prompts with and without a longer key range, and
    single queries over caches of every group size (grouped, multi-query, several blocks per KV
    head), each against the oracle on the same inputs."""
    q = I.normal(67, 0, "q", (B, Hq, Sq, dh), 1.0, bf16=True)
    k = I.normal(67, 0, "k_cache", (B, Hkv, cap, dh), 1.0, bf16=True)
    v = I.normal(67, 0, "v_cache", (B, Hkv, cap, dh), 1.0, bf16=True)
    scale = 1.0 / math.sqrt(dh)
    ref = O.attention(q, k[:, :, :Skv], v[:, :, :Skv], scale, causal)
    out = torch.empty(B, Sq, Hq * dh, dtype=torch.bfloat16, device="cuda")
    ws = F.workspace(F.forge_attn_fused_workspace_bytes(B, Hq, Hkv, Sq, Skv, dh, torch.bfloat16))
    F.forge_attn_fused(dev(q, True), dev(k, True), dev(v, True), out, kv_len=Skv, scale=scale, causal=causal, workspace=ws)
    torch.cuda.synchronize()
    check(out, ref, True, "attention B%d Hq%d Hkv%d Sq%d Skv%d dh%d causal%d" % (B, Hq, Hkv, Sq, Skv, dh, causal))


def test_attn_sharp_softmax(F):
    """Large score spread: one key dominates each row, the online rescaling must not lose it."""
    B, H, S, dh = 1, 2, 200, 64
    q = I.normal(64, 0, "q", (B, H, S, dh), 6.0, bf16=True)
    k = I.normal(64, 0, "k", (B, H, S, dh), 6.0, bf16=True)
    v = I.normal(64, 0, "v", (B, H, S, dh), 1.0, bf16=True)
    ref = O.attention(q, k, v, 0.125, True)
    out = torch.empty(B, S, H * dh, dtype=torch.bfloat16, device="cuda")
    F.forge_attn_fused(dev(q, True), dev(k, True), dev(v, True), out, scale=0.125)
    torch.cuda.synchronize()
    check(out, ref, True, "sharp attention")


# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
@pytest.mark.parametrize("dh", [64, 128])
def test_rope(F, bf16, dh):
    B, H, cap, row0, n_rows, pos0 = 2, 3, 50, 7, 40, 2040
    x = I.normal(65, 0, "q", (B, H, cap, dh), 1.0, bf16=bf16)
    ref = x.astype(np.float64).copy()
    ref[:, :, row0:row0 + n_rows] = O.rope(x[:, :, row0:row0 + n_rows], np.arange(pos0, pos0 + n_rows), 500000.0)
    tx = dev(x, bf16)
    F.forge_rope(tx, n_rows=n_rows, row0=row0, pos0=pos0, base=500000.0)
    torch.cuda.synchronize()
    check(tx, ref, bf16, "rope")
    assert np.array_equal(host(tx)[:, :, :row0], x[:, :, :row0].astype(np.float64))


@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
def test_embed(F, bf16):
    B, S, d, V, P = 3, 17, 264, 1001, 40
    wte = I.normal(66, 0, "wte", (V, d), 0.02, bf16=bf16)
    wpe = I.normal(66, 0, "wpe", (P, d), 0.02, bf16=bf16)
    ids = I.token_ids(66, B, S, V)
    ref = O.embed(ids, wte, wpe, pos0=5)
    h = torch.empty(B, S, d, dtype=tdtype(bf16), device="cuda")
    F.forge_embed(torch.from_numpy(ids).cuda(), dev(wte, bf16), dev(wpe, bf16), h, pos0=5)
    torch.cuda.synchronize()
    check(h, ref, bf16, "embed")
