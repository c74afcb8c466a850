"""The allocation-free decode attention (the library's own fixed scratch array instead of a caller
workspace) against forge_attn_fused on the same inputs: same kernels, same order, so the outputs
must be bit-identical, and both within the bf16 bound of the fp64 oracle.  Two calls in a row
share the array, the second with a smaller input."""
import numpy as np
import pytest
import torch

from oracle import forge_oracle as O
from paper_2604_16498_amd import inputs as I
from util import check, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def F():
    from paper_2604_16498_amd import binding
    binding.lib()
    return binding


def _case(F, seed, B, Hq, Hkv, dh, kv_len, cap):
    q = I.normal(seed, 0, "q", (B, Hq, 1, dh), 1.0, bf16=True)
    k = I.normal(seed, 0, "k_cache", (B, Hkv, cap, dh), 1.0, bf16=True)
    v = I.normal(seed, 0, "v_cache", (B, Hkv, cap, dh), 1.0, bf16=True)
    tq, tk, tv = dev(q, True), dev(k, True), dev(v, True)
    need = F.forge_attn_fused_workspace_bytes(B, Hq, Hkv, 1, kv_len, dh, torch.bfloat16)
    assert 0 < need <= F.forge_attn_decode_static_max_bytes(), "the case must use the scratch array"
    ws = F.workspace(need)
    want = torch.empty(B, 1, Hq * dh, dtype=torch.bfloat16, device="cuda")
    F.forge_attn_fused(tq, tk, tv, want, kv_len, causal=True, workspace=ws)
    got = torch.full_like(want, 7.0)
    F.forge_attn_decode_static(tq, tk, tv, got, kv_len)
    torch.cuda.synchronize()
    assert torch.equal(got, want), "static-scratch call differs from the workspace call"
    check(got, O.attention(q, k[:, :, :kv_len], v[:, :, :kv_len], dh ** -0.5, True), True,
          "static-scratch decode attention B=%d kv_len=%d" % (B, kv_len))


def test_two_calls_in_a_row_share_the_scratch(F):
    _case(F, 91, 4, 32, 8, 128, 2049, 2100)      # 32 pairs -> 16 ranges of partials
    _case(F, 92, 2, 8, 2, 64, 700, 704)          # smaller: 4 pairs -> 2 ranges, over the stale partials


def test_too_large_for_the_fixed_array_is_rejected(F):
    # 2 sequences x 128 query heads x 32 ranges x 130 floats = 4.3 MB: more than the 4 MB array
    B, Hq, Hkv, dh, kv_len = 2, 128, 2, 128, 64 * 128
    assert F.forge_attn_fused_workspace_bytes(B, Hq, Hkv, 1, kv_len, dh, torch.bfloat16) > F.forge_attn_decode_static_max_bytes()
    q = torch.zeros(B, Hq, 1, dh, dtype=torch.bfloat16, device="cuda")
    k = torch.zeros(B, Hkv, kv_len, dh, dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(B, 1, Hq * dh, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(F.ForgeError) as e:
        F.forge_attn_decode_static(q, k, k, out, kv_len)
    assert e.value.status == 3
