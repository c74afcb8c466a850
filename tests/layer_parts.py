"""One decoder layer taken apart: every operator of the layer launched on its own through the C
ABI, each compared with the oracle's operator fed the GPU's OWN input of that operator.

This separates the two things a whole-layer comparison mixes: whether each kernel is right (one
rounding against an fp64 result on identical inputs: the strict bound) and how the roundings of
the ~10 bf16 stores between the kernels add up along the layer.  The last operator's output must
equal forge_decoder_block's bit for bit (same kernels, same order), so the parts ARE the layer.
Test helper: no arithmetic of the method here, only launches, data movement and comparisons.
"""
import numpy as np
import torch

from oracle import forge_oracle as O
from util import check, host, strict_err


def layer_by_parts(F, sh, w, tw, tx, block_out, seq, rows, what, block_k=None):
    """Prefill (position 0) of tx [B, S, d] (bf16, GPU) through the layer's operators.
    w / tw: the layer's weights on the host / the GPU.  The oracle checks sequence `seq`, rows
    `rows` (a list, or None for all).  block_k: the K cache forge_decoder_block wrote.
    Returns {stage: (strict elementwise error, l2 error)}.

    A bf16 layer with rotary embedding rotates q and k inside its QKV projection, before the one
    rounding; taken apart, the projection rounds and forge_rope rounds again.  There the layer's
    own K rows are checked against the oracle's projection + rotation of the same input (one
    rounding: the strict bound), and the last operator's output is compared with the layer's
    within the bf16 bound instead of bit for bit."""
    B, S, d = tx.shape
    Hq, Hkv, dh = sh.q_heads, sh.kv_heads, sh.head_dim
    T, hd, nqkv = B * S, Hq * dh, (Hq + 2 * Hkv) * dh
    bf = torch.bfloat16
    new = lambda *shape: torch.empty(*shape, dtype=bf, device="cuda")
    R = list(range(S)) if rows is None else list(rows)
    errs = {}

    failures = []

    def stage(name, got, ref):
        errs[name] = strict_err(host(got).reshape(np.shape(ref)), ref)
        try:                       # every stage is reported before the first failure is raised
            check(got, ref, True, "%s: %s" % (what, name))
        except AssertionError as e:
            failures.append(str(e))

    x2 = tx.reshape(T, d)
    # 1. first norm
    y = new(T, d)
    F.forge_residual_norm(x2, None, tw["norm1_g"], tw.get("norm1_b"), None, y, sh.eps, sh.norm)
    torch.cuda.synchronize()
    stage("norm1", y.view(B, S, d)[seq, R],
          O.residual_norm(host(tx[seq, R]), None, w["norm1_g"], w.get("norm1_b"), sh.eps, sh.norm)[1])
    # 2. QKV projection (plain output; the layer's own launch scatters the same values head-major)
    qkv = new(T, nqkv)
    F.forge_gemm_bias_gelu(y, tw["w_qkv"], tw.get("b_qkv"), None, qkv, "none")
    torch.cuda.synchronize()
    stage("qkv", qkv.view(B, S, nqkv)[seq, R], O.linear(host(y.view(B, S, d)[seq, R]), w["w_qkv"], w.get("b_qkv")))
    heads = lambda t, n: t.reshape(B, S, n, dh).permute(0, 2, 1, 3).contiguous()
    q = heads(qkv[:, :hd], Hq)
    k = heads(qkv[:, hd:hd + Hkv * dh], Hkv)
    v = heads(qkv[:, hd + Hkv * dh:], Hkv)
    # 3. rotary embedding
    if sh.use_rope:
        q0, k0 = host(q[seq][:, R]), host(k[seq][:, R])
        F.forge_rope(q, base=sh.rope_base)
        F.forge_rope(k, base=sh.rope_base)
        torch.cuda.synchronize()
        stage("rope q", q[seq][:, R], O.rope(q0, np.asarray(R), sh.rope_base))
        stage("rope k", k[seq][:, R], O.rope(k0, np.asarray(R), sh.rope_base))
        if block_k is not None:
            k64 = O.linear(host(y.view(B, S, d)[seq, R]), w["w_qkv"], w.get("b_qkv"))[:, hd:hd + Hkv * dh]
            k64 = k64.reshape(len(R), Hkv, dh).transpose(1, 0, 2)
            stage("qkv + rope in one kernel (the layer's K rows)", block_k[seq][:, R], O.rope(k64, np.asarray(R), sh.rope_base))
    # 4. fused attention
    o = new(B, S, hd)
    F.forge_attn_fused(q, k, v, o, causal=True)
    torch.cuda.synchronize()
    hq, hk, hv = host(q[seq:seq + 1]), host(k[seq:seq + 1]), host(v[seq:seq + 1])
    if rows is None:
        ref_o = O.attention(hq, hk, hv, dh ** -0.5, True)[0]
    else:
        ref_o = np.concatenate([O.attention(hq[:, :, r:r + 1], hk[:, :, :r + 1], hv[:, :, :r + 1], dh ** -0.5, True)[0]
                                for r in R])
    stage("attention", o[seq, R], ref_o)
    # 5. output projection + residual
    h1 = new(T, d)
    F.forge_gemm_bias_gelu(o.view(T, hd), tw["w_o"], tw.get("b_o"), x2, h1, "none")
    torch.cuda.synchronize()
    stage("out proj + residual", h1.view(B, S, d)[seq, R],
          O.gemm_bias_act(host(o[seq, R]), w["w_o"], w.get("b_o"), residual=host(tx[seq, R])))
    # 6. second norm
    m = new(T, d)
    F.forge_residual_norm(h1, None, tw["norm2_g"], tw.get("norm2_b"), None, m, sh.eps, sh.norm)
    torch.cuda.synchronize()
    stage("norm2", m.view(B, S, d)[seq, R],
          O.residual_norm(host(h1.view(B, S, d)[seq, R]), None, w["norm2_g"], w.get("norm2_b"), sh.eps, sh.norm)[1])
    # 7. MLP up + activation
    u = new(T, sh.d_ff)
    F.forge_gemm_bias_gelu(m, tw["w_up"], tw.get("b_up"), None, u, sh.mlp_act)
    torch.cuda.synchronize()
    stage("mlp up + act", u.view(B, S, sh.d_ff)[seq, R],
          O.gemm_bias_act(host(m.view(B, S, d)[seq, R]), w["w_up"], w.get("b_up"), act=sh.mlp_act))
    # 8. MLP down + residual
    h2 = new(T, d)
    F.forge_gemm_bias_gelu(u, tw["w_down"], tw.get("b_down"), h1, h2, "none")
    torch.cuda.synchronize()
    stage("mlp down + residual", h2.view(B, S, d)[seq, R],
          O.gemm_bias_act(host(u.view(B, S, sh.d_ff)[seq, R]), w["w_down"], w.get("b_down"),
                          residual=host(h1.view(B, S, d)[seq, R])))
    assert not failures, "; ".join(failures)
    if sh.use_rope:
        check(h2.view(B, S, d)[seq, R], host(block_out[seq, R]), True, "%s: operators one by one vs the layer" % what)
    else:
        assert torch.equal(h2.view(B, S, d), block_out), "%s: the operators one by one differ from forge_decoder_block" % what
    print("%s, kernel by kernel on identical inputs (strict elementwise / l2): %s" %
          (what, ", ".join("%s %.2e / %.2e" % (n, e[0], e[1]) for n, e in errs.items())))
    return errs
