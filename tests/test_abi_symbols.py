"""The C-ABI library loads, exports every function include/forge.h declares, and rejects bad
arguments on the host before any launch (so these calls are safe without a GPU)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "forge.h")
LIB = os.path.join(ROOT, "paper_2604_16498_amd", "libforge.so")


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(forge_[a-z_0-9]+)\s*\(", src)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2604_16498_amd import build
        build.build(verbose=False)
    return C.CDLL(LIB)


def test_header_declares_the_four_named_calls():
    names = declared_functions()
    for n in ("forge_attn_fused", "forge_gemm_bias_gelu", "forge_residual_norm", "forge_decoder_block"):
        assert n in names


def test_every_declared_symbol_is_exported_and_bound(lib):
    from paper_2604_16498_amd import binding
    names = declared_functions()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), "library does not export %s" % n
        assert n in binding.SIGNATURES, "binding has no signature for %s" % n
    assert sorted(binding.SIGNATURES) == names


def test_status_strings(lib):
    lib.forge_status_string.restype = C.c_char_p
    got = [lib.forge_status_string(i).decode() for i in range(5)]
    assert got == ["FORGE_OK", "FORGE_ERR_INVALID_ARG", "FORGE_ERR_UNSUPPORTED",
                   "FORGE_ERR_WORKSPACE", "FORGE_ERR_HIP"]


def test_argument_errors_are_caught_on_the_host():
    from paper_2604_16498_amd import binding as B
    l = B.lib()
    vp = C.c_void_p
    good = vp(0x1000)            # aligned, never dereferenced: every call below fails its checks first
    odd = vp(0x1004)
    # NULL / misaligned pointers
    assert l.forge_residual_norm(None, None, good, None, None, good, 4, 64, 1e-5, 0, 0, None) == 1
    assert l.forge_residual_norm(odd, None, good, None, None, good, 4, 64, 1e-5, 0, 0, None) == 1
    # unsupported width, bad sizes
    assert l.forge_residual_norm(good, None, good, None, None, vp(0x2000), 4, 60, 1e-5, 0, 0, None) == 2
    assert l.forge_residual_norm(good, None, good, None, None, vp(0x2000), 0, 64, 1e-5, 0, 0, None) == 1
    # gemm: K not a multiple of 8 for bf16; y aliasing x
    assert l.forge_gemm_bias_gelu(good, vp(0x2000), None, None, vp(0x3000), 4, 4, 12, 0, 0, 1, None, 0, None) == 2
    assert l.forge_gemm_bias_gelu(good, vp(0x2000), None, None, good, 4, 4, 16, 0, 0, 1, None, 0, None) == 1
    assert l.forge_gemm_bias_gelu(good, vp(0x2000), None, None, vp(0x3000), 4, 4, 16, 0, 9, 1, None, 0, None) == 1
    assert l.forge_gemm_bias_gelu(good, vp(0x2000), None, None, vp(0x3000), 4, 4, 16, 3, 0, 1, None, 0, None) == 1   # ldy < N
    # attention: head dim, head ratio, causal with kv_len < q_len
    a = (good, vp(0x2000), vp(0x3000), vp(0x4000))
    assert l.forge_attn_fused(*a, 1, 4, 4, 8, 8, 32, 4 * 8 * 32, 8 * 32, 0.1, 1, 1, None, 0, None) == 2
    assert l.forge_attn_fused(*a, 1, 4, 3, 8, 8, 64, 3 * 8 * 64, 8 * 64, 0.1, 1, 1, None, 0, None) == 1
    assert l.forge_attn_fused(*a, 1, 4, 4, 8, 4, 64, 4 * 4 * 64, 4 * 64, 0.1, 1, 1, None, 0, None) == 1
    # size limits: batch or heads past a grid dimension, too many rows, too many GEMM outputs
    assert l.forge_attn_fused(*a, 65536, 4, 4, 8, 8, 64, 4 * 8 * 64, 8 * 64, 0.1, 1, 1, None, 0, None) == 2
    assert l.forge_attn_fused(*a, 1, 65536, 65536, 8, 8, 64, 65536 * 8 * 64, 8 * 64, 0.1, 1, 1, None, 0, None) == 2
    assert l.forge_attn_fused(*a, 4096, 4, 4, 8192, 8192, 64, 4 * 8192 * 64, 8192 * 64, 0.1, 1, 1, None, 0, None) == 2
    assert l.forge_attn_fused_workspace_bytes(65536, 4, 4, 1, 8, 64, 1) == 0
    assert l.forge_gemm_bias_gelu(good, vp(0x2000), None, None, vp(0x3000), (1 << 24) + 1, 8, 16, 0, 0, 1, None, 0, None) == 2
    assert l.forge_gemm_bias_gelu(good, vp(0x2000), None, None, vp(0x3000), 1 << 20, 1 << 20, 16, 0, 0, 1, None, 0, None) == 2
    assert l.forge_gemm_workspace_bytes(1 << 20, 1 << 20, 16, 0, 1) == 0
    # positions: pos0 + seq must not wrap around
    assert l.forge_embed(good, vp(0x2000), vp(0x3000), vp(0x4000), 1, 2, 64, 100, 512, 2**31 - 1, 1, None) == 1
    assert l.forge_embed(good, vp(0x2000), vp(0x3000), vp(0x4000), 1, 8, 64, 100, 512, 505, 1, None) == 1
    # row re-layout: NULL, overlapping ranges, no rows
    assert l.forge_deinterleave_gated_rows(None, good, 4, 16, None) == 1
    assert l.forge_deinterleave_gated_rows(good, vp(0x1000 + 64), 4, 16, None) == 1      # 128-byte ranges overlap
    assert l.forge_deinterleave_gated_rows(good, vp(0x2000), 0, 16, None) == 1
    # block: NULL descriptor; workspace size of an invalid descriptor is 0
    assert l.forge_decoder_block(None, good, good, good, good, 1, 1, 0, 1, good, 0, None) == 1
    d = B.BlockDesc()
    assert l.forge_decoder_block_workspace_bytes(C.byref(d), 1, 1, 1) == 0


def test_attention_scale_must_be_positive_and_finite():
    from paper_2604_16498_amd import binding as B
    l = B.lib()
    vp = C.c_void_p
    a = (vp(0x1000), vp(0x2000), vp(0x3000), vp(0x4000))
    mask = C.cast(vp(0x5000), C.POINTER(C.c_float))
    pos = C.cast(vp(0x6000), C.POINTER(C.c_int32))
    for bad in (0.0, -0.125, float("inf"), float("nan")):
        assert l.forge_attn_fused(*a, 1, 4, 4, 8, 8, 64, 4 * 8 * 64, 8 * 64, bad, 1, 1, None, 0, None) == 1
        assert l.forge_attn_fused(*a, 1, 4, 4, 8, 8, 64, 4 * 8 * 64, 8 * 64, bad, 1, 0, None, 0, None) == 1
        assert l.forge_attn_fused_masked(a[0], a[1], a[2], mask, a[3], 1, 4, 4, 8, 8, 64, 4 * 8 * 64, 8 * 64,
                                         0, 0, bad, 0, 1, None) == 1
        assert l.forge_attn_decode_varlen(*a, pos, 1, 4, 4, 7, 64, 4 * 8 * 64, 8 * 64, bad, 1, None, 0, None) == 1


def test_decode_attention_scratch_is_monotone_in_the_cache_length():
    """A generation loop asks once, for the capacity of its cache, and then attends over every
    shorter length: the size for a longer cache must never be smaller, and the layer's and
    the model's workspace (sized for kv_cap) must cover the attention call at every step."""
    from paper_2604_16498_amd import binding as B
    l = B.lib()
    for batch, hq, hkv, dh in [(8, 32, 8, 128), (4, 12, 12, 64), (2, 12, 12, 64), (1, 32, 8, 128),
                               (3, 16, 4, 128), (16, 8, 8, 64), (64, 32, 8, 128),
                               # groups of 16 and 32 query heads (several blocks per KV head), 11 (none)
                               (2, 32, 2, 128), (3, 32, 1, 64), (2, 11, 1, 64)]:
        prev = 0
        for kv_len in list(range(1, 700)) + list(range(700, 9000, 37)):
            need = l.forge_attn_fused_workspace_bytes(batch, hq, hkv, 1, kv_len, dh, B.FORGE_BF16)
            assert need >= prev, (batch, hq, hkv, dh, kv_len, need, prev)
            prev = need
        # never more than one partial (dh + 2 floats) per query head and split, 64 splits at most
        assert prev <= batch * hq * 64 * (dh + 2) * 4
    # the two cases that used to shrink with the length
    a = l.forge_attn_fused_workspace_bytes(8, 32, 8, 1, 769, 128, B.FORGE_BF16)
    b = l.forge_attn_fused_workspace_bytes(8, 32, 8, 1, 2049, 128, B.FORGE_BF16)
    assert 0 < a <= b


def test_gemm_variant_names_the_kernel_that_runs():
    """The diagnostic applies the launcher's own rule: unaligned output rows (an odd dense N) and
    a reduction that is not a whole number of 64-element slabs go to the generic kernel, a
    decode-sized problem to the weight-streaming one, everything else to the persistent one."""
    import torch
    from paper_2604_16498_amd import binding as F
    v = lambda M, N, K, act="none", ldy=0: F.forge_gemm_variant(M, N, K, act, torch.bfloat16, ldy=ldy)
    assert v(300, 1001, 128) == "gemm_bf16_generic<128,128,2,2>"            # rows of 2002 bytes
    assert v(300, 1001, 128, ldy=1008) == "gemm_bf16_pers<128,128,2,4>"
    assert v(300, 1000, 72) == "gemm_bf16_generic<128,128,2,2>"             # K % 64 != 0
    assert v(8192, 3072, 768, "gelu_tanh") == "gemm_bf16_pers<128,128,2,4>"
    assert v(8192, 50257, 768, ldy=50264) == "gemm_bf16_pers<256,256,2,4>"
    assert v(4096, 14336, 4096, "swiglu") == "gemm_bf16_pers<256,256,2,4>"
    assert v(4096, 1001, 4096, "swiglu", ldy=1008) == "gemm_bf16_generic<128,128,2,2>"   # gated pairs need N % 8 == 0
    assert v(64, 4096, 4096) == "gemm_bf16_wstream+splitk"
    assert v(64, 4096, 72) == "gemm_bf16_generic<64,64,2,2>+splitk"
    assert F.forge_gemm_variant(128, 768, 768, "none", torch.float32) == "gemm_f32<64,64,2,2>"
