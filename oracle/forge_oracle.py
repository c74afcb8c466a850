"""CPU oracle for the fused decoder-block forward.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import
this module.  The product path (the HIP library and its binding) never does, and
this module imports nothing from the product.

What it computes: the *unfused* chain of operators that the paper's attention
fusion pass and operator fusion pass start from, evaluated in fp64 with the
N x N score matrix S and probability matrix P written out in memory, exactly as
the pre-fusion graph does (Sec. "Pass 4: Attention Fusion", the attention chain
equation  Q.K^T -> scale -> [mask] -> softmax -> .V  and the SDPA equation
softmax(Q.K^T / sqrt(d_k)).V ; Sec. "Pass 5: Operator Fusion", whose fused op is
matmul, then bias add, then the activation, with the weight stored
[out_features, in_features], and whose fourth pattern is a residual add after a
matmul).  Fusion preserves the result up to floating-point rounding
(Sec. "Numerical Fidelity"), so the plain definition *is* the expected value of
every fused kernel.

There is no blocking, no online softmax and no fused epilogue here.  numpy's
fp64 ``@`` serves as the matrix product; everything else is elementwise numpy.
All inputs are upcast to fp64 on entry and nothing is rounded in between.

Operators the paper names but never defines (LayerNorm, RMSNorm, the GELU form,
RoPE, grouped-query attention, SwiGLU, a KV cache) follow the standard
definitions stated in each docstring.

Pins (tests/test_oracle_pins.py): softmax rows sum to one; causality; uniform
attention closed form; GQA == MHA on replicated K/V; RoPE norm / relative-shift
invariance; LayerNorm / RMSNorm moments; GELU / SiLU closed forms and odd-part
identities; identity-weight and zero-weight special cases; pure-Python brute
force of every operator and of a whole block on tiny shapes, written in fused
(online-softmax, epilogue) order; decode step == last row of a longer prefill;
torch CPU fp64 library routines as special cases.
Weight-only int8: quantize_int8 / dequantize_int8 (pins: half-step error bound, grid
weights returned exactly, sign symmetry, idempotence, pure-Python loops); a quantised linear is
`linear` on the dequantised weight.
The two conventions the paper leaves open are pinned by library routines: the GQA
grouping order (contiguous groups) by torch's grouped-query scaled_dot_product_attention,
the RoPE pairing (rotate-half), sign and frequencies by the Llama rotary-embedding
routines of the `transformers` package (to the fp32 precision of that module's angles).
"""
from __future__ import annotations

import math

import numpy as np

__all__ = [
    "layer_norm", "rms_norm", "residual_norm", "linear", "gelu_tanh", "gelu_erf", "silu", "relu",
    "gemm_bias_act", "rope", "attention_probs", "attention", "embed", "lm_head",
    "decoder_block", "gpt_forward",
]


def _f64(a):
    return None if a is None else np.asarray(a, dtype=np.float64)


# ----------------------------------------------------------------------------
# normalisation (named in Sec. "Precision Strategy for Llama-3.1-8B" and
# Sec. "Contributions" only; standard definitions)
# ----------------------------------------------------------------------------


def layer_norm(x, gamma, beta, eps):
    """y = (x - mean) / sqrt(var + eps) * gamma + beta over the last axis.

    var is the biased variance (divide by d); eps sits inside the square root.
    """
    x = _f64(x)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    y = (x - mu) / np.sqrt(var + eps)
    if gamma is not None:
        y = y * _f64(gamma)
    if beta is not None:
        y = y + _f64(beta)
    return y


def rms_norm(x, g, eps):
    """y = x / sqrt(mean(x^2) + eps) * g over the last axis (gain is g, not 1+g)."""
    x = _f64(x)
    ms = (x ** 2).mean(axis=-1, keepdims=True)
    y = x / np.sqrt(ms + eps)
    if g is not None:
        y = y * _f64(g)
    return y


def residual_norm(x, delta, gamma, beta, eps, kind):
    """(h, y) with h = x + delta (delta may be None) and y = Norm(h).

    The add-then-normalise pair around each projection of a pre-norm block; the
    add is the paper's fourth fusion pattern (a residual add following a matmul,
    Sec. "Pass 5: Operator Fusion") carried into the norm that consumes it.
    """
    h = _f64(x) if delta is None else _f64(x) + _f64(delta)
    if kind == "layernorm":
        y = layer_norm(h, gamma, beta, eps)
    elif kind == "rmsnorm":
        y = rms_norm(h, gamma, eps)
    else:
        raise ValueError(kind)
    return h, y


# ----------------------------------------------------------------------------
# linear + activation (Sec. "Pass 5: Operator Fusion")
# ----------------------------------------------------------------------------


def linear(x, w, b=None):
    """z[t, n] = sum_k x[t, k] w[n, k] + b[n]; w is [out_features, in_features]."""
    z = _f64(x) @ _f64(w).T
    if b is not None:
        z = z + _f64(b)
    return z


def quantize_int8(w):
    """Symmetric int8 weights, one scale per output channel (Sec. "Precision Strategy for
    Llama-3.1-8B": symmetric int8 weight quantisation with 16-bit activations; the paper gives no
    granularity or rounding, so: per row of the [out, in] weight, no zero point, range -127..127).

    The integer decision is taken in fp32, the precision the kernel takes it in:
    scale[n] = max_k |w[n, k]| / 127 and q[n, k] = rint(w[n, k] / scale[n]) (ties to even), both
    as IEEE fp32 divisions.  A row of zeros gets scale 1 and q = 0.  Returns (q int8, scale fp32).
    """
    w32 = np.asarray(w, dtype=np.float32)
    amax = np.max(np.abs(w32), axis=1)
    scale = np.where(amax > 0, amax / np.float32(127.0), np.float32(1.0)).astype(np.float32)
    q = np.rint(w32 / scale[:, None])
    q = np.clip(q, -127, 127).astype(np.int8)
    return q, scale


def dequantize_int8(q, scale):
    """The weight the quantised linear multiplies by: q[n, k] * scale[n], in fp64."""
    return q.astype(np.float64) * scale.astype(np.float64)[:, None]


def gelu_tanh(x):
    """0.5 x (1 + tanh( sqrt(2/pi) (x + 0.044715 x^3) ))."""
    x = _f64(x)
    return 0.5 * x * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))


def gelu_erf(x):
    """0.5 x (1 + erf(x / sqrt 2)): the exact form (the tanh form is the reading taken for the
    paper's "GELU"; this one is offered as the other fusion variant)."""
    x = _f64(x)
    try:
        from scipy.special import erf
    except ImportError:            # the standard library's erf, element by element: slower, same values
        erf = np.vectorize(math.erf, otypes=[np.float64])
    return 0.5 * x * (1.0 + erf(x / math.sqrt(2.0)))


def silu(x):
    """x / (1 + exp(-x))."""
    x = _f64(x)
    return x / (1.0 + np.exp(-x))


def relu(x):
    return np.maximum(_f64(x), 0.0)


def gemm_bias_act(x, w, bias=None, residual=None, act="none"):
    """act(x w^T + bias) (+ residual): matmul, then bias, then activation, then the add.

    act: "none" | "gelu_tanh" | "gelu_erf" | "relu" | "silu" | "swiglu".
    "swiglu": w is [2F, K], rows 0..F-1 are the gate projection and rows F..2F-1
    the up projection; the result is silu(gate) * up, shape [..., F].
    """
    z = linear(x, w, bias)
    if act == "none":
        y = z
    elif act == "gelu_tanh":
        y = gelu_tanh(z)
    elif act == "gelu_erf":
        y = gelu_erf(z)
    elif act == "relu":
        y = relu(z)
    elif act == "silu":
        y = silu(z)
    elif act == "swiglu":
        f = z.shape[-1] // 2
        y = silu(z[..., :f]) * z[..., f:]
    else:
        raise ValueError(act)
    if residual is not None:
        y = y + _f64(residual)
    return y


# ----------------------------------------------------------------------------
# rotary position embedding (named in Sec. "Pass 3: Constant Folding" only)
# ----------------------------------------------------------------------------


def rope(x, positions, base):
    """Rotate-half RoPE on the last axis of x[..., S, dh] at integer positions[S].

    theta_i = base^(-2i/dh), i in [0, dh/2); the pair is (i, i + dh/2):
      x'_i        = x_i cos(p theta_i) - x_{i+dh/2} sin(p theta_i)
      x'_{i+dh/2} = x_{i+dh/2} cos(p theta_i) + x_i sin(p theta_i)
    """
    x = _f64(x)
    dh = x.shape[-1]
    half = dh // 2
    i = np.arange(half, dtype=np.float64)
    theta = float(base) ** (-2.0 * i / dh)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * theta[None, :]   # [S, half]
    c, s = np.cos(ang), np.sin(ang)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


# ----------------------------------------------------------------------------
# attention (Sec. "Pass 4: Attention Fusion")
# ----------------------------------------------------------------------------


def attention_probs(q, k, scale, causal, mask=None):
    """P[b, h, i, j]: the probability matrix of the unfused chain, written out.

    q [B, Hq, Sq, dh]; k [B, Hkv, Skv, dh] un-transposed, as the fused op takes it.
    S = scale * q k^T;  the optional mask node of the chain (Sec. "Pass 4: Attention Fusion")
    adds mask[b or 0, h or 0, i, j] (finite or -inf) to S;  if causal, S_ij = -inf for
    j > i + (Skv - Sq);  row softmax with the row maximum subtracted.  Query head h reads kv head
    h // (Hq / Hkv).  Every row must keep at least one key.
    """
    q, k = _f64(q), _f64(k)
    B, Hq, Sq, dh = q.shape
    _, Hkv, Skv, _ = k.shape
    group = Hq // Hkv
    P = np.empty((B, Hq, Sq, Skv), dtype=np.float64)
    for b in range(B):
        for h in range(Hq):
            S = (q[b, h] @ k[b, h // group].T) * scale
            if mask is not None:
                mk = _f64(mask)
                S = S + mk[b if mk.shape[0] > 1 else 0, h if mk.shape[1] > 1 else 0]
            if causal:
                i = np.arange(Sq)[:, None]
                j = np.arange(Skv)[None, :]
                S = np.where(j > i + (Skv - Sq), -np.inf, S)
            S = S - S.max(axis=-1, keepdims=True)
            E = np.exp(S)
            P[b, h] = E / E.sum(axis=-1, keepdims=True)
    return P


def attention(q, k, v, scale, causal, mask=None):
    """out[B, Sq, Hq*dh] = softmax(mask(scale q k^T)) v, heads concatenated per token.
    mask: optional additive [B or 1, Hq or 1, Sq, Skv]."""
    q, v = _f64(q), _f64(v)
    B, Hq, Sq, dh = q.shape
    Hkv = v.shape[1]
    group = Hq // Hkv
    out = np.empty((B, Sq, Hq * dh), dtype=np.float64)
    for b in range(B):
        # one batch element at a time keeps the written-out P at Hq*Sq*Skv doubles
        mb = None if mask is None else (mask[b:b + 1] if np.shape(mask)[0] > 1 else mask)
        P = attention_probs(q[b:b + 1], _f64(k)[b:b + 1], scale, causal, mb)[0]
        for h in range(Hq):
            out[b, :, h * dh:(h + 1) * dh] = P[h] @ v[b, h // group]
    return out


# ----------------------------------------------------------------------------
# model pieces
# ----------------------------------------------------------------------------


def embed(ids, wte, wpe, pos0=0):
    """h0[b, s] = wte[ids[b, s]] + wpe[pos0 + s]."""
    ids = np.asarray(ids)
    S = ids.shape[1]
    return _f64(wte)[ids] + _f64(wpe)[pos0:pos0 + S][None, :, :]


def lm_head(y, wte):
    """logits = y wte^T with the token table itself (tied weights, Sec. "Tied Weight Resolution")."""
    return _f64(y) @ _f64(wte).T


def decoder_block(shape, w, x, k_cache=None, v_cache=None, pos0=0, query_rows=None):
    """One pre-norm decoder layer.  Returns the new residual stream.

    shape: attributes d_model, q_heads, kv_heads, head_dim, d_ff, norm, eps,
           mlp_act ("gelu_tanh" | "swiglu"), use_rope, rope_base.
    w:     dict norm1_g, norm1_b, w_qkv, b_qkv, w_o, b_o, norm2_g, norm2_b, w_up,
           b_up, w_down, b_down (biases / shifts may be None).
    x:     [B, q_len, d] residual stream.
    k_cache, v_cache: optional fp64 arrays [B, Hkv, cap, dh], updated IN PLACE at
           positions pos0 .. pos0+q_len-1; attention then runs over positions
           0 .. pos0+q_len-1.  Without caches pos0 must be 0.
    query_rows: optional list of row indices; K and V are still produced for all
           rows, the rest of the layer is evaluated for these rows only and the
           result is [B, len(query_rows), d].

    Steps: norm1 -> QKV linear -> split heads -> RoPE on q, k -> cache write ->
    causal attention -> out projection + residual -> norm2 -> up projection +
    activation -> down projection + residual.
    """
    x = _f64(x)
    B, S, d = x.shape
    Hq, Hkv, dh = shape.q_heads, shape.kv_heads, shape.head_dim
    scale = 1.0 / math.sqrt(dh)

    _, y = residual_norm(x, None, w["norm1_g"], w.get("norm1_b"), shape.eps, shape.norm)
    qkv = linear(y, w["w_qkv"], w.get("b_qkv"))                       # [B, S, (Hq+2Hkv) dh]
    q = qkv[..., :Hq * dh].reshape(B, S, Hq, dh).transpose(0, 2, 1, 3)
    k = qkv[..., Hq * dh:(Hq + Hkv) * dh].reshape(B, S, Hkv, dh).transpose(0, 2, 1, 3)
    v = qkv[..., (Hq + Hkv) * dh:].reshape(B, S, Hkv, dh).transpose(0, 2, 1, 3)
    if shape.use_rope:
        pos = np.arange(pos0, pos0 + S)
        q = rope(q, pos, shape.rope_base)
        k = rope(k, pos, shape.rope_base)
    if k_cache is not None:
        k_cache[:, :, pos0:pos0 + S, :] = k
        v_cache[:, :, pos0:pos0 + S, :] = v
        k_all = k_cache[:, :, :pos0 + S, :]
        v_all = v_cache[:, :, :pos0 + S, :]
    else:
        if pos0 != 0:
            raise ValueError("pos0 != 0 needs caches")
        k_all, v_all = k, v

    if query_rows is None:
        o = attention(q, k_all, v_all, scale, causal=True)           # [B, S, Hq*dh]
        h = x
    else:
        rows = list(query_rows)
        o = np.empty((B, len(rows), Hq * dh), dtype=np.float64)
        for n, r in enumerate(rows):
            # one query at absolute position pos0+r sees keys 0 .. pos0+r
            o[:, n:n + 1, :] = attention(q[:, :, r:r + 1, :], k_all[:, :, :pos0 + r + 1, :],
                                         v_all[:, :, :pos0 + r + 1, :], scale, causal=True)
        h = x[:, rows, :]

    h = gemm_bias_act(o, w["w_o"], w.get("b_o"), residual=h, act="none")
    _, m = residual_norm(h, None, w["norm2_g"], w.get("norm2_b"), shape.eps, shape.norm)
    u = gemm_bias_act(m, w["w_up"], w.get("b_up"), act=shape.mlp_act)
    return gemm_bias_act(u, w["w_down"], w.get("b_down"), residual=h, act="none")


def gpt_forward(shape, layer_weights, model_w, ids=None, x=None, return_hidden=False):
    """Embedding (or a given hidden state) -> L decoder layers -> final norm -> tied LM head.

    model_w: dict wte, wpe (only with ids), normf_g, normf_b.
    Returns logits [B, S, V]; with return_hidden (or no token table) the final
    normed hidden state [B, S, d].
    """
    if x is None:
        h = embed(ids, model_w["wte"], model_w["wpe"])
    else:
        h = _f64(x)
    for w in layer_weights:
        h = decoder_block(shape, w, h)
    _, y = residual_norm(h, None, model_w["normf_g"], model_w.get("normf_b"), shape.eps, shape.norm)
    if return_hidden or model_w.get("wte") is None:
        return y
    return lm_head(y, model_w["wte"])
