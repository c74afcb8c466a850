"""GPU parity of the weight-only int8 path (Sec. "Precision Strategy for Llama-3.1-8B": symmetric
int8 weights, 16-bit activations) against the fp64 oracle.

* the quantisation kernel must reproduce the oracle's integers and scales bit for bit (both take
  the rounding decision in fp32);
* the quantised GEMM and the quantised decoder layer are compared, at the bf16 tolerance of the
  other GEMM / layer tests, with the oracle's plain linear on the DEQUANTISED weight q * scale:
  the same integers go to both sides (they come from the oracle's quantiser, never from the GPU).
"""
import math

import numpy as np
import pytest
import torch

from oracle import forge_oracle as O
from paper_2604_16498_amd import inputs as I
from util import check, dev, dev_dict, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def F():
    from paper_2604_16498_amd import binding
    binding.lib()
    return binding


def q_dev(q, s):
    return torch.from_numpy(q).cuda(), torch.from_numpy(s).cuda()


@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
@pytest.mark.parametrize("N,K", [(1, 8), (7, 100), (33, 256), (64, 1000), (130, 4096)])
def test_quantize_int8_bit_exact(F, bf16, N, K):
    w = I.normal(91, 0, "w_up", (N, K), 0.02, bf16=bf16)
    if N > 2:
        w[1] = 0.0                                  # a row of zeros: scale 1, q 0
        w[2, : min(K, 8)] = np.float32(0.5) * np.arange(1, min(K, 8) + 1, dtype=np.float32)   # exact ties when ...
        w[2, min(K, 8) - 1] = 127.0                 # ... the row maximum makes the scale exactly 1
    q_ref, s_ref = O.quantize_int8(w)
    tq, ts = F.forge_quantize_int8(dev(w, bf16))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(ts.cpu().numpy(), s_ref)
    np.testing.assert_array_equal(tq.cpu().numpy(), q_ref)


W8_SHAPES = [(1, 128, 128), (7, 520, 128), (16, 1000, 512), (33, 136, 1024), (64, 4096, 512),
             (64, 768, 3072), (48, 257, 384), (2, 1536, 4096), (130, 392, 256), (200, 264, 128),
             # prompts: the weight is written out as bf16 once, the bf16 kernels apply the row scale
             (600, 1032, 256), (300, 1001, 128), (4096, 4096, 128), (1100, 520, 2048)]


@pytest.mark.parametrize("act", ["none", "gelu_tanh", "silu", "swiglu"])
@pytest.mark.parametrize("M,N,K", W8_SHAPES)
def test_gemm_w8(F, act, M, N, K):
    wn = 2 * N if act == "swiglu" else N
    x = I.normal(92, 0, "x", (M, K), 1.0, bf16=True)
    w = I.normal(92, 0, "w_up", (wn, K), 1.0 / math.sqrt(K), bf16=True)
    b = I.normal(92, 0, "b_up", (wn,), 0.5, bf16=True)
    r = I.normal(92, 0, "residual", (M, N), 1.0, bf16=True)
    q, s = O.quantize_int8(w)
    wd = O.dequantize_int8(q, s)
    tq, ts = q_dev(q, s)
    tx, tb, tr = dev(x, True), dev(b, True), dev(r, True)
    ws = F.workspace(F.forge_gemm_w8_workspace_bytes(M, N, K, act))
    for use_b, use_r in ((True, True), (False, False)):
        ref = O.gemm_bias_act(x, wd, b if use_b else None, r if use_r else None, act)
        ty = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
        F.forge_gemm_w8(tx, tq, ts, tb if use_b else None, tr if use_r else None, ty, act, ws)
        torch.cuda.synchronize()
        check(ty, ref, True, "w8 gemm %s" % act)
    again = torch.empty_like(ty)
    F.forge_gemm_w8(tx, tq, ts, None, None, again, act, ws)
    torch.cuda.synchronize()
    assert torch.equal(again, ty)


def test_gemm_w8_extreme_rows(F):
    """Rows whose scale differs by orders of magnitude and a row of zeros: the scale is applied
    per output column after the reduction."""
    M, N, K = 9, 128, 256
    x = I.normal(93, 0, "x", (M, K), 1.0, bf16=True)
    w = I.normal(93, 0, "w_up", (N, K), 1.0, bf16=True)
    w *= (2.0 ** ((np.arange(N) % 24) - 12)).astype(np.float32)[:, None]      # powers of two: still bf16 values
    w[5] = 0.0
    q, s = O.quantize_int8(w)
    ref = O.gemm_bias_act(x, O.dequantize_int8(q, s), None, None, "none")
    tq, ts = q_dev(q, s)
    ty = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    F.forge_gemm_w8(dev(x, True), tq, ts, None, None, ty, "none", F.workspace(F.forge_gemm_w8_workspace_bytes(M, N, K, "none")))
    torch.cuda.synchronize()
    got = host(ty)
    assert np.all(got[:, 5] == 0.0)
    # columns differ by 2^24 in magnitude: compare column by column
    for n in range(N):
        if n != 5:
            check(ty[:, n], ref[:, n], True, "w8 column %d" % n)


def test_gemm_w8_rejects(F):
    x = torch.zeros(4, 72, dtype=torch.bfloat16, device="cuda")
    q = torch.zeros(64, 72, dtype=torch.int8, device="cuda")
    s = torch.ones(64, dtype=torch.float32, device="cuda")
    y = torch.empty(4, 64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(F.ForgeError) as e:                       # K not a multiple of 128
        F.forge_gemm_w8(x, q, s, None, None, y, "none", F.workspace(1 << 20))
    assert e.value.status == 2
    x = torch.zeros(4, 128, dtype=torch.bfloat16, device="cuda")
    q = torch.zeros(64, 128, dtype=torch.int8, device="cuda")
    with pytest.raises(F.ForgeError) as e:                       # workspace too small
        F.forge_gemm_w8(x, q, s, None, None, y, "none", F.workspace(256))
    assert e.value.status == 3


# ------------------------------------------------------------------ decoder layer on int8 weights

LLAMA = I.BlockShape(512, 8, 2, 64, 768, norm="rmsnorm", mlp_act="swiglu", use_rope=True,
                     rope_base=500000.0, has_bias=False)
GPT = I.BlockShape(256, 4, 4, 64, 1024)
NAMES = (("w_qkv", "s_qkv"), ("w_o", "s_o"), ("w_up", "s_up"), ("w_down", "s_down"))


def quantised_weights(w):
    """(oracle-side weights with every projection replaced by its dequantised form, GPU-side dict
    with int8 weights and scales)."""
    wo, wg = dict(w), {}
    for k, v in w.items():
        wg[k] = None if v is None else dev(v, True)
    for wn, sn in NAMES:
        q, s = O.quantize_int8(w[wn])
        wo[wn] = O.dequantize_int8(q, s)
        wg[wn], wg[sn] = q_dev(q, s)
    return wo, wg


@pytest.mark.parametrize("sh,B,S,pos0", [(LLAMA, 8, 1, 70), (LLAMA, 1, 130, 0), (GPT, 4, 1, 33), (GPT, 2, 40, 0)],
                         ids=["llama_decode", "llama_prefill", "gpt_decode", "gpt_prefill"])
def test_block_w8(F, sh, B, S, pos0):
    cap = 200
    w = I.block_weights(sh, 94, 0, bf16=True, random_affine=True, weight_std=0.05)
    wo, wg = quantised_weights(w)
    x = I.normal(94, 0, "x", (B, S, sh.d_model), 1.0, bf16=True)
    kc = I.normal(94, 0, "k_cache", (B, sh.kv_heads, cap, sh.head_dim), 1.0, bf16=True)
    vc = I.normal(94, 0, "v_cache", (B, sh.kv_heads, cap, sh.head_dim), 1.0, bf16=True)
    kr, vr = kc.astype(np.float64), vc.astype(np.float64)
    ref = O.decoder_block(sh, wo, x, kr, vr, pos0=pos0)
    desc = F.make_block_desc(sh, wg)
    tx, tk, tv = dev(x, True), dev(kc, True), dev(vc, True)
    out = torch.empty_like(tx)
    ws = F.workspace(F.forge_decoder_block_workspace_bytes(desc, B, S, cap))
    F.forge_decoder_block(desc, tx, out, tk, tv, pos0, ws)
    torch.cuda.synchronize()
    check(tk[:, :, :pos0 + S], kr[:, :, :pos0 + S], True, "k cache")
    check(tv[:, :, :pos0 + S], vr[:, :, :pos0 + S], True, "v cache")
    check(out, ref, True, "w8 decoder layer", chain=True)


def test_block_w8_rejects_partial_scales_and_fp32(F):
    sh = GPT
    w = I.block_weights(sh, 95, 0, bf16=True)
    _, wg = quantised_weights(w)
    wg["s_o"] = None
    desc = F.make_block_desc(sh, wg)
    assert F.forge_decoder_block_workspace_bytes(desc, 1, 8, 8) == 0       # invalid descriptor
    x = torch.zeros(1, 8, sh.d_model, dtype=torch.bfloat16, device="cuda")
    kc = torch.zeros(1, sh.kv_heads, 8, sh.head_dim, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(F.ForgeError) as e:
        F.forge_decoder_block(desc, x, torch.empty_like(x), kc, kc.clone(), 0, F.workspace(1 << 20))
    assert e.value.status == 1


def test_compiled_model_on_int8_weights(F):
    """A decode step of a two-layer int8 stack through the compiled launcher equals the plain
    launch list bit for bit (same kernels, the scratch areas at their planned places)."""
    sh, L, B, cap, pos0 = LLAMA, 2, 8, 96, 70
    gpu_layers = []
    for l in range(L):
        _, wg = quantised_weights(I.block_weights(sh, 96, l, bf16=True, random_affine=True, weight_std=0.05))
        gpu_layers.append(wg)
    wl = I.scaled(I.WORKLOADS[4], block=sh, layers=L, batch=B, seq=1)
    tm = dev_dict(I.model_weights(wl, random_affine=True), True)
    model = F.make_model_desc([F.make_block_desc(sh, w) for w in gpu_layers], tm)
    x = dev(I.normal(96, 0, "x", (B, 1, sh.d_model), 1.0, bf16=True), True)
    k_init = dev(I.normal(96, 0, "k_cache", (L, B, sh.kv_heads, cap, sh.head_dim), 1.0, bf16=True), True)
    v_init = dev(I.normal(96, 0, "v_cache", (L, B, sh.kv_heads, cap, sh.head_dim), 1.0, bf16=True), True)
    plain = torch.empty(B, 1, sh.d_model, dtype=torch.bfloat16, device="cuda")
    kc0, vc0 = k_init.clone(), v_init.clone()
    F.forge_model_forward(model, x, plain, kc0, vc0, pos0, F.workspace(F.forge_model_workspace_bytes(model, B, 1, cap)))
    torch.cuda.synchronize()
    cm = F.CompiledModel(model, B, 1, pos0, cap)
    out = torch.zeros_like(plain)
    kc, vc = k_init.clone(), v_init.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    cm.bind(x, out, kc, vc, F.workspace(cm.workspace_bytes()), side)
    for _ in range(2):
        out.zero_(); kc.copy_(k_init); vc.copy_(v_init)
        torch.cuda.synchronize()
        cm.run(side)
        side.synchronize()
        assert torch.equal(out, plain) and torch.equal(kc, kc0) and torch.equal(vc, vc0)
    cm.close()
