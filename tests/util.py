"""Helpers shared by the GPU parity tests (no arithmetic of the method here)."""
import numpy as np
import torch

FP32_MAX_ABS = 1e-4     # fp32 paths: max-abs error against the fp64 oracle

# bf16 paths, "2e-2 relative".  Read per element as |g - r| <= 2e-2 max(|r|, rms(r)) -- the error
# relative to the element, with the tensor's rms as the floor below which "relative" stops
# meaning anything -- together with the tensor-level ||g - r||_2 <= 2e-2 ||r||_2.  This STRICT
# bound binds wherever both sides start from identical inputs: one kernel, or one decoder layer
# fed the GPU's own layer input.  Every check prints its error in units of that bound.
#
# Drift through a stack of L layers (tokens in, logits out) is reported, not held to the strict
# bound: every bf16 store between kernels adds a relative rounding error of 2^-9/sqrt(3) = 0.11%
# rms and a layer has ~10 of them, so the per-element sigma grows with depth.  Those tests gate
# the l2 error at 2e-2 and the elementwise allclose-style bound |g - r| <= 2e-2 |r| + 4e-2 rms(r),
# which still catches localised damage (a wrong tile is off by O(rms), 25x above it).
BF16_REL = 2e-2
BF16_ATOL_DRIFT = 4e-2


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


def strict_err(got, ref):
    """(max over elements of |g-r| / max(|r|, rms(r)), relative l2 error)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    rms = np.sqrt(np.mean(ref ** 2)) + 1e-30
    e = np.abs(got - ref) / np.maximum(np.abs(ref), rms)
    l2 = np.linalg.norm(got - ref) / (np.linalg.norm(ref) + 1e-30)
    return float(e.max()), float(l2)


def drift_err(got, ref):
    """(max over elements of |g-r| / (2e-2 |r| + 4e-2 rms(r)) * 2e-2, relative l2 error): the
    elementwise error of a multi-layer result in units where 2e-2 is the bound."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    rms = np.sqrt(np.mean(ref ** 2)) + 1e-30
    e = np.abs(got - ref) / (BF16_REL * np.abs(ref) + BF16_ATOL_DRIFT * rms) * BF16_REL
    l2 = np.linalg.norm(got - ref) / (np.linalg.norm(ref) + 1e-30)
    return float(e.max()), float(l2)


def check(got_t, ref, bf16, what="", chain=False):
    """One kernel, or (chain=True) one decoder layer, against the oracle on identical inputs:
    the strict bound.  Returns the elementwise error (bf16: in units where 2e-2 is the bound)."""
    got = host(got_t).reshape(np.asarray(ref).shape)
    assert np.isfinite(got).all(), "%s: non-finite output" % what
    if bf16:
        mx, l2 = strict_err(got, ref)
        print("%s: bf16 strict elementwise %.3e (bound %.1e), l2 %.3e" % (what, mx, BF16_REL, l2))
        assert mx <= BF16_REL and l2 <= BF16_REL, \
            "%s: bf16 strict elementwise %.3e / l2 %.3e exceed %.1e" % (what, mx, l2, BF16_REL)
        return mx
    err = float(np.abs(got - ref).max())
    assert err <= FP32_MAX_ABS, "%s: fp32 max-abs err %.3e > %.1e" % (what, err, FP32_MAX_ABS)
    return err


def check_drift(got_t, ref, what=""):
    """A bf16 result that went through several layers since the two sides last agreed: the
    strict metric is printed, the drift bound is gated.  Returns (strict, l2)."""
    got = (host(got_t) if hasattr(got_t, "detach") else np.asarray(got_t, np.float64)).reshape(np.asarray(ref).shape)
    assert np.isfinite(got).all(), "%s: non-finite output" % what
    strict, l2 = strict_err(got, ref)
    mx, _ = drift_err(got, ref)
    print("%s: bf16 drift: strict elementwise %.3e, drift-bound units %.3e, l2 %.3e" % (what, strict, mx, l2))
    assert mx <= BF16_REL and l2 <= BF16_REL, \
        "%s: bf16 drift elementwise %.3e / l2 %.3e exceed %.1e" % (what, mx, l2, BF16_REL)
    return strict, l2
