"""Helpers shared by the GPU parity tests (no arithmetic of the method here)."""
import numpy as np
import torch

FP32_MAX_ABS = 1e-4     # fp32 paths: max-abs error against the fp64 oracle
BF16_REL = 2e-2         # bf16 paths: |g - r| / max(|r|, rms(r)) per element


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


def rel_err(got, ref):
    """Per-element error relative to max(|ref|, rms(ref)); returns (max, l2 ratio)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    rms = np.sqrt(np.mean(ref ** 2)) + 1e-30
    e = np.abs(got - ref) / np.maximum(np.abs(ref), rms)
    l2 = np.linalg.norm(got - ref) / (np.linalg.norm(ref) + 1e-30)
    return float(e.max()), float(l2)


def check(got_t, ref, bf16, what=""):
    got = host(got_t).reshape(np.asarray(ref).shape)
    assert np.isfinite(got).all(), "%s: non-finite output" % what
    if bf16:
        mx, l2 = rel_err(got, ref)
        assert mx <= BF16_REL, "%s: bf16 rel err %.3e (l2 %.3e) > %.1e" % (what, mx, l2, BF16_REL)
        return mx
    err = float(np.abs(got - ref).max())
    assert err <= FP32_MAX_ABS, "%s: fp32 max-abs err %.3e > %.1e" % (what, err, FP32_MAX_ABS)
    return err
