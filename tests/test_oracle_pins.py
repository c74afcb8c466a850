"""Pins of the CPU oracle against things other than itself.

The paper prints no worked numeric example of the fused operators, so the oracle
is pinned by (1) invariants and closed forms that the definitions fix,
(2) special cases that reduce to a torch CPU fp64 library routine (the fused
attention module of Sec. "Pass 4: Attention Fusion" *is* a call to the library's
scaled-dot-product attention), and (3) a second evaluation written from scratch
in pure Python scalar loops in *fused* order (online softmax, bias/activation/
residual applied on the accumulator), which must agree with the unfused oracle
to rounding -- the paper's own fidelity claim (Sec. "Numerical Fidelity").
"""
import cmath
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import forge_oracle as O
from paper_2604_16498_amd import inputs as I

RNG = np.random.default_rng(20260416)


def rnd(*shape, std=1.0):
    return RNG.standard_normal(shape) * std


# ---------------------------------------------------------------------------
# softmax / attention
# ---------------------------------------------------------------------------


def test_probs_rows_sum_to_one_and_mask():
    q, k = rnd(2, 4, 7, 8), rnd(2, 2, 11, 8)
    P = O.attention_probs(q, k, 0.3, causal=True)
    assert P.shape == (2, 4, 7, 11)
    assert np.all(P >= 0)
    assert np.abs(P.sum(-1) - 1).max() < 1e-14
    off = 11 - 7
    for i in range(7):
        assert np.all(P[..., i, i + off + 1:] == 0.0)
        assert np.all(P[..., i, :i + off + 1] > 0.0)
    Pn = O.attention_probs(q, k, 0.3, causal=False)
    assert np.all(Pn > 0) and np.abs(Pn.sum(-1) - 1).max() < 1e-14


def test_single_key_returns_v0():
    q, k, v = rnd(1, 2, 1, 4), rnd(1, 2, 1, 4), rnd(1, 2, 1, 4)
    o = O.attention(q, k, v, 0.5, causal=True)
    assert np.array_equal(o.reshape(2, 4), v.reshape(2, 4))


def test_zero_query_gives_running_mean():
    B, H, S, dh = 1, 2, 9, 4
    k, v = rnd(B, H, S, dh), rnd(B, H, S, dh)
    q = np.zeros((B, H, S, dh))
    P = O.attention_probs(q, k, 1.0, causal=True)
    for i in range(S):
        assert np.allclose(P[0, :, i, :i + 1], 1.0 / (i + 1), atol=1e-15)
    o = O.attention(q, k, v, 1.0, causal=True)             # [B,S,H*dh]
    for h in range(H):
        run = np.cumsum(v[0, h], axis=0) / np.arange(1, S + 1)[:, None]
        assert np.allclose(o[0, :, h * dh:(h + 1) * dh], run, atol=1e-14)


def test_dominant_key_selects_its_value():
    S, dh = 6, 4
    k = np.zeros((1, 1, S, dh)); k[0, 0, 2, 0] = 1.0
    q = np.zeros((1, 1, S, dh)); q[0, 0, :, 0] = 200.0
    v = rnd(1, 1, S, dh)
    o = O.attention(q, k, v, 1.0, causal=True)
    for i in range(2, S):
        assert np.allclose(o[0, i], v[0, 0, 2], atol=1e-12)


def test_scale_is_applied_before_softmax():
    # two keys, scores s0, s1 -> p0 = 1 / (1 + exp(scale*(s1 - s0)))
    q = np.array([[[[0.0, 0.0], [1.0, 2.0]]]])
    k = np.array([[[[0.5, -1.0], [2.0, 0.25]]]])
    v = np.array([[[[1.0, 0.0], [0.0, 1.0]]]])
    scale = 0.37
    s0 = 1.0 * 0.5 + 2.0 * -1.0
    s1 = 1.0 * 2.0 + 2.0 * 0.25
    p0 = 1.0 / (1.0 + math.exp(scale * (s1 - s0)))
    o = O.attention(q, k, v, scale, causal=True)
    assert np.allclose(o[0, 1], [p0, 1 - p0], atol=1e-15)
    assert np.allclose(o[0, 0], [1.0, 0.0])


def test_causality_later_tokens_do_not_matter():
    B, H, S, dh = 1, 2, 10, 4
    q, k, v = rnd(B, H, S, dh), rnd(B, H, S, dh), rnd(B, H, S, dh)
    o1 = O.attention(q, k, v, 0.5, True)
    t = 6
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    q2[:, :, t + 1:] += 3.0; k2[:, :, t + 1:] -= 5.0; v2[:, :, t + 1:] *= -7.0
    o2 = O.attention(q2, k2, v2, 0.5, True)
    assert np.array_equal(o1[:, :t + 1], o2[:, :t + 1])
    assert not np.allclose(o1[:, t + 1:], o2[:, t + 1:])


def test_head_and_batch_permutation_equivariance():
    B, H, S, dh = 3, 4, 5, 4
    q, k, v = rnd(B, H, S, dh), rnd(B, H, S, dh), rnd(B, H, S, dh)
    o = O.attention(q, k, v, 0.5, True).reshape(B, S, H, dh)
    pb, ph = [2, 0, 1], [3, 1, 0, 2]
    o2 = O.attention(q[pb][:, ph], k[pb][:, ph], v[pb][:, ph], 0.5, True).reshape(B, S, H, dh)
    assert np.array_equal(o2, o[pb][:, :, ph])


def test_gqa_equals_mha_on_replicated_kv():
    B, Hq, Hkv, S, dh = 2, 8, 2, 6, 4
    q, k, v = rnd(B, Hq, S, dh), rnd(B, Hkv, S, dh), rnd(B, Hkv, S, dh)
    o = O.attention(q, k, v, 0.5, True)
    g = Hq // Hkv
    k_rep = np.stack([k[:, h // g] for h in range(Hq)], axis=1)   # heads 0..3 -> kv 0, 4..7 -> kv 1
    v_rep = np.stack([v[:, h // g] for h in range(Hq)], axis=1)
    o_rep = O.attention(q, k_rep, v_rep, 0.5, True)
    assert np.array_equal(o, o_rep)


@pytest.mark.parametrize("Hq,Hkv,Sq,Skv", [(4, 4, 9, 9), (8, 2, 5, 12), (4, 1, 1, 17)])
def test_attention_vs_library_sdpa(Hq, Hkv, Sq, Skv):
    B, dh = 2, 8
    q, k, v = rnd(B, Hq, Sq, dh), rnd(B, Hkv, Skv, dh), rnd(B, Hkv, Skv, dh)
    scale = 1 / math.sqrt(dh)
    o = O.attention(q, k, v, scale, True)
    tq, tk, tv = (torch.from_numpy(a) for a in (q, k, v))
    # bottom-right aligned causal mask written as a boolean matrix
    mask = torch.tril(torch.ones(Sq, Skv, dtype=torch.bool), diagonal=Skv - Sq)
    ref = F.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=scale, enable_gqa=True)
    ref = ref.permute(0, 2, 1, 3).reshape(B, Sq, Hq * dh).numpy()
    assert np.abs(o - ref).max() < 1e-13
    if Sq == Skv:
        ref2 = F.scaled_dot_product_attention(tq, tk, tv, is_causal=True, enable_gqa=True)
        assert np.abs(o - ref2.permute(0, 2, 1, 3).reshape(B, Sq, Hq * dh).numpy()).max() < 1e-13


# ---------------------------------------------------------------------------
# RoPE
# ---------------------------------------------------------------------------


def test_rope_identity_norm_and_relative_shift():
    S, dh = 7, 8
    x, y = rnd(2, 3, S, dh), rnd(2, 3, S, dh)
    assert np.array_equal(O.rope(x, np.zeros(S, int), 500000.0), x)
    pos = np.arange(S) + 11
    rx = O.rope(x, pos, 500000.0)
    half = dh // 2
    # each (i, i+half) pair is rotated: pair norms are preserved
    assert np.allclose(rx[..., :half] ** 2 + rx[..., half:] ** 2,
                       x[..., :half] ** 2 + x[..., half:] ** 2, atol=1e-13)
    # q_m . k_n depends on m - n only
    s1 = np.einsum("bhid,bhjd->bhij", O.rope(x, pos, 1e4), O.rope(y, pos, 1e4))
    s2 = np.einsum("bhid,bhjd->bhij", O.rope(x, pos + 1000, 1e4), O.rope(y, pos + 1000, 1e4))
    assert np.allclose(s1, s2, atol=1e-10)


def test_rope_vs_complex_rotation():
    S, dh, base = 5, 6, 500000.0
    x = rnd(S, dh)
    pos = np.array([0, 1, 2, 100, 2048])
    r = O.rope(x, pos, base)
    half = dh // 2
    for s in range(S):
        for i in range(half):
            z = complex(x[s, i], x[s, i + half]) * cmath.exp(1j * pos[s] * base ** (-2.0 * i / dh))
            assert abs(r[s, i] - z.real) < 1e-12 and abs(r[s, i + half] - z.imag) < 1e-12


def test_rope_known_quarter_turn():
    # dh = 2: theta_0 = 1; position pi/2 is not an integer, so use the angle sum:
    # rotating (1, 0) by p radians gives (cos p, sin p)
    r = O.rope(np.array([[1.0, 0.0]] * 3), np.array([1, 2, 3]), 10000.0)
    assert np.allclose(r[:, 0], np.cos([1, 2, 3])) and np.allclose(r[:, 1], np.sin([1, 2, 3]))


def test_rope_convention_vs_llama_reference_routines():
    """The pairing (i, i + dh/2), the sign of the rotation and theta_i = base^(-2i/dh) are the
    convention of the Llama family.  The rotary-embedding module and `apply_rotary_pos_emb` of the
    `transformers` package (a library, nothing of ours) apply it to the same q and k; the module
    keeps its inverse frequencies in fp32, hence 1e-5 and not 1e-13 - an interleaved pairing, a
    flipped sign or a different exponent is off by O(1).  Where the package is missing this pin is
    skipped; the convention stays pinned by the complex-rotation and quarter-turn tests above."""
    tf = pytest.importorskip("transformers")
    from transformers.models.llama.modeling_llama import LlamaRotaryEmbedding, apply_rotary_pos_emb
    dh, H, base = 16, 2, 500000.0
    cfg = tf.LlamaConfig(hidden_size=H * dh, num_attention_heads=H, num_key_value_heads=H, rope_theta=base,
                         max_position_embeddings=4096, num_hidden_layers=1, intermediate_size=8, vocab_size=8)
    rot = LlamaRotaryEmbedding(config=cfg)
    pos = np.array([0, 1, 2, 5, 9, 33, 63, 2048])
    q, k = rnd(1, H, len(pos), dh), rnd(1, H, len(pos), dh)
    tq, tk = torch.from_numpy(q), torch.from_numpy(k)
    cos, sin = rot(tq, torch.from_numpy(pos)[None, :])
    q_lib, k_lib = apply_rotary_pos_emb(tq, tk, cos.double(), sin.double())
    # position 2048 times an fp32 frequency: the angle itself carries ~1e-4 of rounding
    tol = np.where(pos[:, None] > 100, 2e-3, 1e-5)
    assert np.all(np.abs(q_lib.numpy() - O.rope(q, pos, base)) < tol)
    assert np.all(np.abs(k_lib.numpy() - O.rope(k, pos, base)) < tol)
    # the check has teeth: the interleaved pairing (2i, 2i+1) of the same angles is far away
    half = dh // 2
    perm = np.concatenate([np.arange(0, dh, 2), np.arange(1, dh, 2)])
    inter = np.empty_like(q)
    inter[..., perm] = O.rope(q[..., perm], pos, base)
    assert np.abs(inter[:, :, 1:] - q_lib.numpy()[:, :, 1:]).max() > 0.1


# ---------------------------------------------------------------------------
# norms
# ---------------------------------------------------------------------------


def test_layer_norm_moments_and_invariance():
    x = rnd(5, 64) * 3 + 2
    eps = 1e-5
    y = O.layer_norm(x, None, None, eps)
    assert np.abs(y.mean(-1)).max() < 1e-14
    var = x.var(-1)
    assert np.allclose(y.var(-1), var / (var + eps), rtol=1e-13)
    y2 = O.layer_norm(4.0 * x + 9.0, None, None, 0.0)
    assert np.allclose(y2, O.layer_norm(x, None, None, 0.0), atol=1e-12)
    g, b = rnd(64), rnd(64)
    assert np.allclose(O.layer_norm(x, g, b, eps), y * g + b, atol=1e-14)
    ref = F.layer_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), torch.from_numpy(b), eps).numpy()
    assert np.abs(O.layer_norm(x, g, b, eps) - ref).max() < 1e-13


def test_layer_norm_two_point_closed_form():
    # d = 2: x = (a, b) -> mean (a+b)/2, var ((a-b)/2)^2 -> y = +-1 / sqrt(1 + eps/var)
    y = O.layer_norm(np.array([[3.0, 1.0]]), None, None, 0.25)
    assert np.allclose(y, [[1 / math.sqrt(1.25), -1 / math.sqrt(1.25)]])


def test_rms_norm_moments_and_invariance():
    x = rnd(5, 64) * 3 + 2
    eps = 1e-5
    y = O.rms_norm(x, None, eps)
    ms = (x ** 2).mean(-1)
    assert np.allclose((y ** 2).mean(-1), ms / (ms + eps), rtol=1e-13)
    assert np.allclose(O.rms_norm(7.0 * x, None, 0.0), O.rms_norm(x, None, 0.0), atol=1e-13)
    g = rnd(64)
    ref = F.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), eps).numpy()
    assert np.abs(O.rms_norm(x, g, eps) - ref).max() < 1e-13
    # (3, 4): mean square 12.5
    assert np.allclose(O.rms_norm(np.array([[3.0, 4.0]]), np.array([2.0, 1.0]), 0.0),
                       [[6 / math.sqrt(12.5), 4 / math.sqrt(12.5)]])


def test_residual_norm_pair():
    x, dlt, g, b = rnd(4, 16), rnd(4, 16), rnd(16), rnd(16)
    h, y = O.residual_norm(x, dlt, g, b, 1e-5, "layernorm")
    assert np.array_equal(h, x + dlt)
    assert np.array_equal(y, O.layer_norm(x + dlt, g, b, 1e-5))
    h2, y2 = O.residual_norm(x, None, g, None, 1e-5, "rmsnorm")
    assert np.array_equal(h2, x) and np.array_equal(y2, O.rms_norm(x, g, 1e-5))


# ---------------------------------------------------------------------------
# activations
# ---------------------------------------------------------------------------


def test_gelu_and_silu_closed_forms():
    x = np.linspace(-8, 8, 2001)
    g = O.gelu_tanh(x)
    assert np.allclose(g - O.gelu_tanh(-x), x, atol=1e-14)       # odd part is x/2
    assert O.gelu_tanh(np.array([0.0]))[0] == 0.0
    assert abs(O.gelu_tanh(np.array([30.0]))[0] - 30.0) < 1e-12 and abs(O.gelu_tanh(np.array([-30.0]))[0]) < 1e-12
    ref = F.gelu(torch.from_numpy(x), approximate="tanh").numpy()
    assert np.abs(g - ref).max() < 1e-14
    # it is the tanh form, not the erf form: they differ by a few 1e-4, never by more than 1e-3
    erf = F.gelu(torch.from_numpy(x)).numpy()
    assert 1e-4 < np.abs(g - erf).max() < 1e-3
    # scalar evaluation through the logistic form of tanh: tanh(u) = 2*sigmoid(2u) - 1
    for xv in (-2.5, -0.3, 0.7, 1.0, 3.1):
        u = math.sqrt(2 / math.pi) * (xv + 0.044715 * xv ** 3)
        assert abs(O.gelu_tanh(np.array([xv]))[0] - xv / (1 + math.exp(-2 * u))) < 1e-14
    # the exact (erf) form: library routine, scalar evaluation, odd part, and Phi as a distribution
    ge = O.gelu_erf(x)
    assert np.abs(ge - erf).max() < 1e-14
    assert np.allclose(ge - O.gelu_erf(-x), x, atol=1e-14)
    for xv in (-2.5, -0.3, 0.7, 1.0, 3.1):
        assert abs(O.gelu_erf(np.array([xv]))[0] - 0.5 * xv * (1 + math.erf(xv / math.sqrt(2)))) < 1e-15
    assert abs(O.gelu_erf(np.array([1.0]))[0] - 0.8413447460685429) < 1e-15   # Phi(1)
    s = O.silu(x)
    assert np.allclose(s - O.silu(-x), x, atol=1e-14)
    assert np.abs(s - F.silu(torch.from_numpy(x)).numpy()).max() < 1e-14
    assert abs(O.silu(np.array([1.0]))[0] - 1 / (1 + math.exp(-1))) < 1e-15
    assert np.array_equal(O.relu(np.array([-1.0, 0.0, 2.0])), [0.0, 0.0, 2.0])


# ---------------------------------------------------------------------------
# linear + epilogues
# ---------------------------------------------------------------------------


def py_linear(x, w, b):
    M, K, N = len(x), len(x[0]), len(w)
    return [[sum(x[m][k] * w[n][k] for k in range(K)) + (b[n] if b is not None else 0.0)
             for n in range(N)] for m in range(M)]


def test_linear_brute_force_and_identity():
    x, w, b = rnd(5, 7), rnd(3, 7), rnd(3)
    z = O.linear(x, w, b)
    assert z.shape == (5, 3)
    assert np.abs(z - np.array(py_linear(x.tolist(), w.tolist(), b.tolist()))).max() < 1e-13
    assert np.array_equal(O.linear(x, np.eye(7), None), x)
    bb = rnd(7)
    assert np.allclose(O.linear(x, np.eye(7), bb), x + bb)
    ref = F.linear(torch.from_numpy(x), torch.from_numpy(w), torch.from_numpy(b)).numpy()
    assert np.abs(z - ref).max() < 1e-13


@pytest.mark.parametrize("act", ["none", "gelu_tanh", "gelu_erf", "relu", "silu", "swiglu"])
def test_gemm_bias_act_order(act):
    M, K, N = 4, 6, 8
    x, w, b = rnd(M, K), rnd(N, K), rnd(N)
    nout = N // 2 if act == "swiglu" else N
    res = rnd(M, nout)
    y = O.gemm_bias_act(x, w, b, res, act)
    z = py_linear(x.tolist(), w.tolist(), b.tolist())

    def sig(t):
        return 1 / (1 + math.exp(-t))
    for m in range(M):
        for n in range(nout):
            if act == "none":
                e = z[m][n]
            elif act == "relu":
                e = max(z[m][n], 0.0)
            elif act == "silu":
                e = z[m][n] * sig(z[m][n])
            elif act == "gelu_tanh":
                t = z[m][n]
                e = 0.5 * t * (1 + math.tanh(math.sqrt(2 / math.pi) * (t + 0.044715 * t ** 3)))
            elif act == "gelu_erf":
                e = 0.5 * z[m][n] * (1 + math.erf(z[m][n] / math.sqrt(2)))
            else:
                gate, up = z[m][n], z[m][n + nout]      # gate rows first, up rows after
                e = gate * sig(gate) * up
            assert abs(y[m, n] - (e + res[m, n])) < 1e-13


# ---------------------------------------------------------------------------
# whole block: independent pure-Python evaluation in fused order
# ---------------------------------------------------------------------------


def py_block_fused(sh, w, x, kc=None, vc=None, pos0=0):
    """Scalar-loop decoder layer for one sequence, written in the order a fused
    implementation evaluates it: online softmax over keys one at a time, bias /
    activation / residual applied to the finished dot product."""
    S, d = len(x), sh.d_model
    Hq, Hkv, dh, Fm = sh.q_heads, sh.kv_heads, sh.head_dim, sh.d_ff
    half = dh // 2

    def norm(row, g, b):
        if sh.norm == "layernorm":
            mu = sum(row) / d
            var = sum((t - mu) ** 2 for t in row) / d
            r = 1 / math.sqrt(var + sh.eps)
            return [(row[i] - mu) * r * g[i] + (b[i] if b is not None else 0.0) for i in range(d)]
        ms = sum(t * t for t in row) / d
        r = 1 / math.sqrt(ms + sh.eps)
        return [row[i] * r * g[i] for i in range(d)]

    def dot(a, b_):
        return sum(p * q for p, q in zip(a, b_))

    def rot(vec, p):
        if not sh.use_rope:
            return vec
        out = list(vec)
        for i in range(half):
            a = p * sh.rope_base ** (-2.0 * i / dh)
            out[i] = vec[i] * math.cos(a) - vec[i + half] * math.sin(a)
            out[i + half] = vec[i + half] * math.cos(a) + vec[i] * math.sin(a)
        return out

    K = [[None] * (pos0 + S) for _ in range(Hkv)]
    V = [[None] * (pos0 + S) for _ in range(Hkv)]
    for g in range(Hkv):
        for p in range(pos0):
            K[g][p], V[g][p] = list(kc[g][p]), list(vc[g][p])
    Q = [[None] * S for _ in range(Hq)]
    for t in range(S):
        y = norm(x[t], w["norm1_g"], w["norm1_b"])
        z = [dot(y, w["w_qkv"][n]) + (w["b_qkv"][n] if w["b_qkv"] is not None else 0.0)
             for n in range((Hq + 2 * Hkv) * dh)]
        for h in range(Hq):
            Q[h][t] = rot(z[h * dh:(h + 1) * dh], pos0 + t)
        for g in range(Hkv):
            K[g][pos0 + t] = rot(z[(Hq + g) * dh:(Hq + g + 1) * dh], pos0 + t)
            V[g][pos0 + t] = z[(Hq + Hkv + g) * dh:(Hq + Hkv + g + 1) * dh]
    out = []
    scale = 1 / math.sqrt(dh)
    for t in range(S):
        o = []
        for h in range(Hq):
            g = h // (Hq // Hkv)
            m, l, acc = -math.inf, 0.0, [0.0] * dh
            for j in range(pos0 + t + 1):
                s = dot(Q[h][t], K[g][j]) * scale
                m_new = max(m, s)
                c = math.exp(m - m_new) if m != -math.inf else 0.0
                p = math.exp(s - m_new)
                l = l * c + p
                acc = [a * c + p * vv for a, vv in zip(acc, V[g][j])]
                m = m_new
            o += [a / l for a in acc]
        h1 = [dot(o, w["w_o"][n]) + (w["b_o"][n] if w["b_o"] is not None else 0.0) + x[t][n]
              for n in range(d)]
        mrow = norm(h1, w["norm2_g"], w["norm2_b"])
        if sh.mlp_act == "swiglu":
            u = []
            for n in range(Fm):
                gate = dot(mrow, w["w_up"][n])
                up = dot(mrow, w["w_up"][Fm + n])
                u.append(gate / (1 + math.exp(-gate)) * up)
        else:
            u = []
            for n in range(Fm):
                t_ = dot(mrow, w["w_up"][n]) + (w["b_up"][n] if w["b_up"] is not None else 0.0)
                u.append(0.5 * t_ * (1 + math.tanh(math.sqrt(2 / math.pi) * (t_ + 0.044715 * t_ ** 3))))
        out.append([dot(u, w["w_down"][n]) + (w["b_down"][n] if w["b_down"] is not None else 0.0) + h1[n]
                    for n in range(d)])
    return out, K, V


def tolist_w(w):
    return {k: (None if a is None else a.astype(np.float64).tolist()) for k, a in w.items()}


GPT_TINY = I.BlockShape(8, 2, 2, 4, 16)
LLAMA_TINY = I.BlockShape(16, 4, 2, 4, 12, norm="rmsnorm", mlp_act="swiglu", use_rope=True,
                          rope_base=500000.0, has_bias=False)


@pytest.mark.parametrize("sh", [GPT_TINY, LLAMA_TINY], ids=["gpt", "llama"])
def test_block_fused_order_equals_unfused(sh):
    S = 5
    w = I.block_weights(sh, 90, 0, bf16=False, bias_std=0.5, random_affine=True, weight_std=0.4)
    x = I.normal(90, 0, "x", (2, S, sh.d_model))
    got = O.decoder_block(sh, w, x)
    wl = tolist_w(w)
    for b in range(2):
        ref, _, _ = py_block_fused(sh, wl, x[b].astype(np.float64).tolist())
        assert np.abs(got[b] - np.array(ref)).max() < 1e-12


@pytest.mark.parametrize("sh", [GPT_TINY, LLAMA_TINY], ids=["gpt", "llama"])
def test_block_with_cache_and_decode_equals_prefill_row(sh):
    S = 6
    w = I.block_weights(sh, 91, 0, bf16=False, bias_std=0.5, random_affine=True, weight_std=0.4)
    x = I.normal(91, 0, "x", (1, S + 1, sh.d_model)).astype(np.float64)
    full = O.decoder_block(sh, w, x)                                  # prefill of S+1 tokens
    cap = 9
    kc = np.zeros((1, sh.kv_heads, cap, sh.head_dim)); vc = np.zeros_like(kc)
    pre = O.decoder_block(sh, w, x[:, :S], kc, vc, pos0=0)            # prefill of S tokens, fills cache
    assert np.abs(pre - full[:, :S]).max() < 1e-13
    assert np.all(kc[:, :, S:] == 0)
    dec = O.decoder_block(sh, w, x[:, S:S + 1], kc, vc, pos0=S)       # one decode step
    assert np.abs(dec[:, 0] - full[:, S]).max() < 1e-13
    assert np.any(kc[:, :, S] != 0) and np.all(kc[:, :, S + 1:] == 0)
    # the pure-Python fused-order evaluation of the same decode step
    kc2 = np.zeros_like(kc); vc2 = np.zeros_like(vc)
    O.decoder_block(sh, w, x[:, :S], kc2, vc2, pos0=0)
    ref, K, V = py_block_fused(sh, tolist_w(w), x[0, S:S + 1].tolist(),
                               kc2[0].tolist(), vc2[0].tolist(), pos0=S)
    assert np.abs(dec[0] - np.array(ref)).max() < 1e-12
    assert np.abs(kc[0, :, S] - np.array([K[g][S] for g in range(sh.kv_heads)])).max() < 1e-13


def test_block_zero_projections_is_identity():
    sh = GPT_TINY
    w = I.block_weights(sh, 92, 0, bf16=False, bias_std=0.0)
    w["w_o"] = np.zeros_like(w["w_o"]); w["w_down"] = np.zeros_like(w["w_down"])
    x = I.normal(92, 0, "x", (2, 4, sh.d_model))
    assert np.array_equal(O.decoder_block(sh, w, x), x.astype(np.float64))


def test_block_query_rows_equal_full_rows():
    sh = LLAMA_TINY
    w = I.block_weights(sh, 93, 0, bf16=False)
    x = I.normal(93, 0, "x", (2, 9, sh.d_model))
    full = O.decoder_block(sh, w, x)
    rows = [0, 3, 8]
    part = O.decoder_block(sh, w, x, query_rows=rows)
    assert np.abs(part - full[:, rows]).max() < 1e-13


def test_block_vs_library_composition():
    """Same layer composed from torch CPU fp64 library routines (GPT flavour)."""
    sh = I.BlockShape(32, 4, 4, 8, 64)
    w = I.block_weights(sh, 94, 0, bf16=False, bias_std=0.3, random_affine=True, weight_std=0.2)
    x = I.normal(94, 0, "x", (2, 11, 32))
    got = O.decoder_block(sh, w, x)
    t = {k: torch.from_numpy(v.astype(np.float64)) for k, v in w.items()}
    xt = torch.from_numpy(x.astype(np.float64))
    y = F.layer_norm(xt, (32,), t["norm1_g"], t["norm1_b"], sh.eps)
    q, k, v = F.linear(y, t["w_qkv"], t["b_qkv"]).split(32, dim=-1)
    hd = lambda a: a.reshape(2, 11, 4, 8).transpose(1, 2)
    o = F.scaled_dot_product_attention(hd(q), hd(k), hd(v), is_causal=True).transpose(1, 2).reshape(2, 11, 32)
    h = xt + F.linear(o, t["w_o"], t["b_o"])
    m = F.layer_norm(h, (32,), t["norm2_g"], t["norm2_b"], sh.eps)
    ref = h + F.linear(F.gelu(F.linear(m, t["w_up"], t["b_up"]), approximate="tanh"), t["w_down"], t["b_down"])
    assert np.abs(got - ref.numpy()).max() < 1e-12


# ---------------------------------------------------------------------------
# model wrapper
# ---------------------------------------------------------------------------


def test_gpt_forward_tied_head_and_embedding():
    sh = GPT_TINY
    wl = I.scaled(I.WORKLOADS[2], block=sh, layers=2, vocab=19, n_pos=7, batch=2, seq=5)
    mw = I.model_weights(wl, random_affine=True)
    layers = [I.block_weights(sh, 95, l, bf16=False, random_affine=True) for l in range(2)]
    ids = I.token_ids(95, 2, 5, 19)
    logits = O.gpt_forward(sh, layers, mw, ids=ids)
    assert logits.shape == (2, 5, 19)
    h = O.embed(ids, mw["wte"], mw["wpe"])
    for b in range(2):
        for s in range(5):
            assert np.array_equal(h[b, s], mw["wte"][ids[b, s]].astype(np.float64) + mw["wpe"][s])
    for w in layers:
        h = O.decoder_block(sh, w, h)
    y = O.layer_norm(h, mw["normf_g"], mw["normf_b"], sh.eps)
    assert np.array_equal(O.gpt_forward(sh, layers, mw, ids=ids, return_hidden=True), y)
    # the head is the token table: logit of token v is the dot product with its embedding row
    for vtok in (0, 7, 18):
        assert np.allclose(logits[..., vtok], y @ mw["wte"][vtok].astype(np.float64), atol=1e-14)


# ---------------------------------------------------------------------------
# the input module's storage conversions (used by both sides)
# ---------------------------------------------------------------------------


def test_bf16_conversion_matches_torch():
    a = (RNG.standard_normal(10000) * 10.0 ** RNG.integers(-6, 6, 10000)).astype(np.float32)
    a[:4] = [0.0, -0.0, np.float32(1.00390625), np.float32(1.01171875)]   # ties: to even
    bits = I.f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16)
    assert np.array_equal(bits, ref.view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(I.bf16_bits_to_f32(bits), ref.float().numpy())
    assert np.array_equal(I.bf16_round(I.bf16_round(a)), I.bf16_round(a))


def test_generators_are_reproducible_and_distinct():
    a = I.normal(2, 3, "w_qkv", (4, 5), 0.02)
    assert np.array_equal(a, I.normal(2, 3, "w_qkv", (4, 5), 0.02))
    assert not np.array_equal(a, I.normal(2, 4, "w_qkv", (4, 5), 0.02))
    assert not np.array_equal(a, I.normal(2, 3, "w_o", (4, 5), 0.02))
    big = I.normal(2, 0, "w_up", (3072, 768), 0.02)
    assert abs(big.std() - 0.02) < 2e-4 and abs(big.mean()) < 1e-4
    ids = I.token_ids(2, 8, 1024, 50257)
    assert ids.min() >= 0 and ids.max() < 50257 and ids.dtype == np.int32


# ---------------------------------------------------------------------------
# the optional additive mask of the attention chain
# ---------------------------------------------------------------------------


def test_attention_additive_mask():
    B, Hq, Hkv, Sq, Skv, dh = 2, 4, 2, 5, 7, 8
    q, k, v = rnd(B, Hq, Sq, dh), rnd(B, Hkv, Skv, dh), rnd(B, Hkv, Skv, dh)
    scale = 1 / math.sqrt(dh)
    base = O.attention(q, k, v, scale, False)
    # a zero mask, and a mask that is constant along the keys, change nothing
    assert np.array_equal(O.attention(q, k, v, scale, False, np.zeros((1, 1, Sq, Skv))), base)
    shift = rnd(B, Hq, Sq, 1) * np.ones((1, 1, 1, Skv))
    assert np.abs(O.attention(q, k, v, scale, False, shift) - base).max() < 1e-13
    # -inf above the (bottom-right aligned) diagonal is the causal flag
    i = np.arange(Sq)[:, None]; j = np.arange(Skv)[None, :]
    tri = np.where(j > i + (Skv - Sq), -np.inf, 0.0)[None, None]
    assert np.abs(O.attention(q, k, v, scale, False, tri) - O.attention(q, k, v, scale, True)).max() < 1e-14
    # -inf on the last keys of one sequence (padding) is attention over the shorter sequence
    pad = np.zeros((B, 1, Sq, Skv)); pad[1, :, :, 4:] = -np.inf
    got = O.attention(q, k, v, scale, False, pad)
    assert np.abs(got[0] - base[0]).max() < 1e-14
    assert np.abs(got[1:] - O.attention(q[1:], k[1:, :, :4], v[1:, :, :4], scale, False)).max() < 1e-13
    # a finite random mask, per batch and head, against the library routine the paper's fused op calls
    m = rnd(B, Hq, Sq, Skv)
    kk = np.repeat(k, Hq // Hkv, axis=1); vv = np.repeat(v, Hq // Hkv, axis=1)
    ref = F.scaled_dot_product_attention(torch.from_numpy(q), torch.from_numpy(kk), torch.from_numpy(vv),
                                         attn_mask=torch.from_numpy(m), scale=scale)
    ref = ref.permute(0, 2, 1, 3).reshape(B, Sq, Hq * dh).numpy()
    assert np.abs(O.attention(q, k, v, scale, False, m) - ref).max() < 1e-13
    # two keys, closed form: p_0 = sigmoid((s_0 + m_0) - (s_1 + m_1))
    q1, k1, v1 = rnd(1, 1, 1, dh), rnd(1, 1, 2, dh), rnd(1, 1, 2, dh)
    m1 = np.array([[[[0.3, -1.1]]]])
    s0, s1 = (q1[0, 0, 0] @ k1[0, 0, 0]) * scale + 0.3, (q1[0, 0, 0] @ k1[0, 0, 1]) * scale - 1.1
    p0 = 1 / (1 + math.exp(s1 - s0))
    assert np.abs(O.attention(q1, k1, v1, scale, False, m1)[0, 0] - (p0 * v1[0, 0, 0] + (1 - p0) * v1[0, 0, 1])).max() < 1e-14


# ---------------------------------------------------------------------------------------------
# symmetric per-channel int8 weights (Sec. "Precision Strategy for Llama-3.1-8B")

def test_int8_quantisation_error_is_at_most_half_a_step():
    rng = np.random.default_rng(8)
    w = (rng.standard_normal((37, 200)) * 0.02).astype(np.float32)
    q, s = O.quantize_int8(w)
    assert q.dtype == np.int8 and s.dtype == np.float32 and s.shape == (37,)
    assert q.min() >= -127 and q.max() <= 127
    # every row uses the full range: its largest magnitude maps to +-127
    assert np.all(np.max(np.abs(q.astype(np.int32)), axis=1) == 127)
    err = np.abs(O.dequantize_int8(q, s) - w.astype(np.float64))
    assert np.all(err <= 0.5 * s[:, None].astype(np.float64) * (1 + 1e-6))
    np.testing.assert_allclose(s, np.max(np.abs(w), axis=1) / 127.0, rtol=1e-7)


def test_int8_weights_on_the_grid_come_back_exactly():
    rng = np.random.default_rng(9)
    q0 = rng.integers(-127, 128, size=(16, 64)).astype(np.int8)
    q0[:, 0] = 127                                   # the row maximum defines the scale
    s0 = (2.0 ** rng.integers(-12, -4, size=16)).astype(np.float32)     # powers of two: exact products
    w = q0.astype(np.float32) * s0[:, None]
    q, s = O.quantize_int8(w)
    np.testing.assert_array_equal(q, q0)
    np.testing.assert_array_equal(s, s0)
    # idempotent: quantising the dequantised weight changes nothing
    q2, s2 = O.quantize_int8(O.dequantize_int8(q, s).astype(np.float32))
    np.testing.assert_array_equal(q2, q); np.testing.assert_array_equal(s2, s)


def test_int8_sign_symmetry_zero_rows_and_ties():
    rng = np.random.default_rng(10)
    w = (rng.standard_normal((5, 33))).astype(np.float32)
    w[2] = 0.0
    q, s = O.quantize_int8(w)
    qn, sn = O.quantize_int8(-w)
    np.testing.assert_array_equal(qn, -q); np.testing.assert_array_equal(sn, s)
    assert np.all(q[2] == 0) and s[2] == 1.0
    # ties go to the even integer: with scale 1 (row maximum 127) the values k + 0.5 are exact ties
    t = np.array([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5]], dtype=np.float32)
    q, s = O.quantize_int8(t)
    assert s[0] == 1.0
    np.testing.assert_array_equal(q[0], [127, 0, 2, 2, 0, -2, -2, 126])


def test_int8_matches_plain_python_loops():
    import struct
    rng = np.random.default_rng(11)
    w = (rng.standard_normal((4, 9)) * 0.3).astype(np.float32)
    q, s = O.quantize_int8(w)

    def f32(v):                         # round a Python float to fp32
        return struct.unpack("f", struct.pack("f", v))[0]

    for n in range(4):
        amax = max(abs(float(v)) for v in w[n])
        sc = f32(amax / 127.0)
        assert sc == float(s[n])
        for k in range(9):
            r = f32(float(w[n, k]) / sc)
            assert int(q[n, k]) == max(-127, min(127, round(r)))      # Python's round: ties to even


def test_int8_linear_is_linear_on_the_dequantised_weight_and_close_to_the_original():
    rng = np.random.default_rng(12)
    w = (rng.standard_normal((24, 512)) * 0.02).astype(np.float32)
    x = rng.standard_normal((6, 512)).astype(np.float32)
    q, s = O.quantize_int8(w)
    z8 = O.linear(x, O.dequantize_int8(q, s))
    # factoring the scale out of the sum is the same thing: s[n] * sum_k x q
    z8b = (x.astype(np.float64) @ q.astype(np.float64).T) * s.astype(np.float64)[None, :]
    np.testing.assert_allclose(z8, z8b, rtol=1e-12, atol=1e-12)
    # quantisation noise: uniform in +-s/2 per weight => rms error of a dot product ~ |x| s / sqrt(12)
    z = O.linear(x, w)
    bound = np.linalg.norm(x, axis=1)[:, None] * s[None, :] / np.sqrt(12.0)
    assert np.sqrt(np.mean(((z8 - z) / bound) ** 2)) < 1.3
    assert np.max(np.abs(z8 - z) / bound) < 5.0
