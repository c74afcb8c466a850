"""Helpers shared by the GPU parity tests (no arithmetic of the method here)."""
import numpy as np
import torch

FP32_MAX_ABS = 1e-4     # fp32 paths: max-abs error against the fp64 oracle

# bf16 paths, "2e-2 relative".  Read as a tensor-level relative error, ||g - r||_2 <= 2e-2 ||r||_2,
# plus an elementwise allclose-style bound |g - r| <= 2e-2 |r| + ATOL * rms(r) that catches
# localised damage (a wrong tile is off by O(rms), 25x above it).
#  - single kernel, identical inputs on both sides: ATOL = 2e-2 (one rounding: errors ~3e-3)
#  - a chain of kernels (decoder layer / model): every bf16 store between kernels adds a
#    relative rounding error of 2^-9/sqrt(3) = 0.11% rms; a layer has ~10 such stores, giving a
#    per-element sigma of 0.4-0.5% of rms (measured l2: 0.37% GPT-2 shape, 0.48% 8B shape).  The
#    largest of 1e6..2e7 elements sits at 5-6 sigma for Gaussian errors and further out for the
#    silu(gate)*up products, i.e. 2-3% of rms for a CORRECT pipeline, so ATOL = 4e-2 there.
BF16_REL = 2e-2
BF16_ATOL_OP = 2e-2
BF16_ATOL_CHAIN = 4e-2


def dev(a, bf16):
    """numpy fp32 array (bf16-representable when bf16) -> GPU tensor of the storage type."""
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a))
    if t.dtype == torch.float32 and bf16:
        t = t.to(torch.bfloat16)          # exact: the values already fit
    return t.cuda()


def dev_dict(w, bf16):
    return {k: dev(v, bf16) for k, v in w.items()}


def host(t):
    """GPU tensor -> numpy fp64."""
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel_err(got, ref, atol=BF16_ATOL_OP):
    """(max over elements of |g-r| / (2e-2 |r| + atol rms(r)) * 2e-2, relative l2 error).

    The first number is the elementwise error in units where 2e-2 is the bound."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    rms = np.sqrt(np.mean(ref ** 2)) + 1e-30
    e = np.abs(got - ref) / (BF16_REL * np.abs(ref) + atol * rms) * BF16_REL
    l2 = np.linalg.norm(got - ref) / (np.linalg.norm(ref) + 1e-30)
    return float(e.max()), float(l2)


def check(got_t, ref, bf16, what="", chain=False):
    got = host(got_t).reshape(np.asarray(ref).shape)
    assert np.isfinite(got).all(), "%s: non-finite output" % what
    if bf16:
        mx, l2 = rel_err(got, ref, BF16_ATOL_CHAIN if chain else BF16_ATOL_OP)
        assert mx <= BF16_REL and l2 <= BF16_REL, \
            "%s: bf16 elementwise %.3e / l2 %.3e exceed %.1e" % (what, mx, l2, BF16_REL)
        return l2
    err = float(np.abs(got - ref).max())
    assert err <= FP32_MAX_ABS, "%s: fp32 max-abs err %.3e > %.1e" % (what, err, FP32_MAX_ABS)
    return err
