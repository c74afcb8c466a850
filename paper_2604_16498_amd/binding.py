"""ctypes binding of the forge C ABI (include/forge.h).

Argument marshalling only: every function here takes torch tensors that already
live on the GPU, passes their device pointers, sizes and the current HIP stream
to the entry point of the same name, and raises :class:`ForgeError` on a
non-zero status.  No step of the computation runs in Python or in torch ops.
The shared library must exist (``python -m paper_2604_16498_amd.build``); there
is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libforge.so")

FORGE_F32, FORGE_BF16 = 0, 1
ACT = {"none": 0, "gelu_tanh": 1, "relu": 2, "silu": 3, "swiglu": 4, "gelu_erf": 5}
NORM = {"layernorm": 0, "rmsnorm": 1}


class ForgeError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s" % (where, status_string(status)))


class BlockDesc(C.Structure):
    _fields_ = [
        ("d_model", C.c_int), ("q_heads", C.c_int), ("kv_heads", C.c_int), ("head_dim", C.c_int),
        ("d_ff", C.c_int), ("norm", C.c_int), ("eps", C.c_float), ("mlp_act", C.c_int),
        ("use_rope", C.c_int), ("rope_base", C.c_float), ("dt", C.c_int),
        ("norm1_g", C.c_void_p), ("norm1_b", C.c_void_p), ("w_qkv", C.c_void_p), ("b_qkv", C.c_void_p),
        ("w_o", C.c_void_p), ("b_o", C.c_void_p), ("norm2_g", C.c_void_p), ("norm2_b", C.c_void_p),
        ("w_up", C.c_void_p), ("b_up", C.c_void_p), ("w_down", C.c_void_p), ("b_down", C.c_void_p),
        ("s_qkv", C.c_void_p), ("s_o", C.c_void_p), ("s_up", C.c_void_p), ("s_down", C.c_void_p),
    ]


class ModelDesc(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int), ("vocab", C.c_int), ("n_pos", C.c_int), ("logits_ld", C.c_int),
        ("layers", C.POINTER(BlockDesc)),
        ("wte", C.c_void_p), ("wpe", C.c_void_p), ("normf_g", C.c_void_p), ("normf_b", C.c_void_p),
    ]


_lib = None

_vp, _i, _f, _sz, _i64 = C.c_void_p, C.c_int, C.c_float, C.c_size_t, C.c_int64
_ip, _szp = C.POINTER(C.c_int), C.POINTER(C.c_size_t)

# name -> (restype, argtypes); the single list of what include/forge.h declares
SIGNATURES = {
    "forge_status_string": (C.c_char_p, [_i]),
    "forge_version": (_i, []),
    "forge_attn_fused_workspace_bytes": (_sz, [_i, _i, _i, _i, _i, _i, _i]),
    "forge_attn_fused": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i64, _i64, _f, _i, _i, _vp, _sz, _vp]),
    "forge_attn_fused_masked": (_i, [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i64, _i64, _i64, _i64, _f, _i,
                                     _i, _vp]),
    "forge_gemm_workspace_bytes": (_sz, [_i, _i, _i, _i, _i]),
    "forge_gemm_variant": (C.c_char_p, [_i, _i, _i, _i, _i, _i]),
    "forge_gemm_bias_gelu": (_i, [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _vp, _sz, _vp]),
    "forge_quantize_int8": (_i, [_vp, _vp, _vp, _i, _i, _i, _vp]),
    "forge_deinterleave_gated_rows": (_i, [_vp, _vp, _i, C.c_size_t, _vp]),
    "forge_gemm_w8_workspace_bytes": (_sz, [_i, _i, _i, _i]),
    "forge_gemm_w8": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _vp, _sz, _vp]),
    "forge_residual_norm": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _f, _i, _i, _vp]),
    "forge_rope": (_i, [_vp, _i, _i, _i, _i, _i64, _i64, _i, _i, _f, _i, _vp]),
    "forge_embed": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i, _vp]),
    "forge_decoder_block_workspace_bytes": (_sz, [C.POINTER(BlockDesc), _i, _i, _i]),
    "forge_decoder_block": (_i, [C.POINTER(BlockDesc), _vp, _vp, _vp, _vp, _i, _i, _i, _i, _vp, _sz, _vp]),
    "forge_model_workspace_bytes": (_sz, [C.POINTER(ModelDesc), _i, _i, _i]),
    "forge_model_forward": (_i, [C.POINTER(ModelDesc), _vp, _vp, _vp, _vp, _i, _i, _i, _i, _vp, _sz, _vp]),
    "forge_attn_decode_varlen": (_i, [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i64, _i64, _f, _i, _vp, _sz, _vp]),
    "forge_trace_start": (_i, [_i, _vp]),
    "forge_trace_stop": (_i, [_ip, _ip, C.POINTER(C.c_float), _i]),
    "forge_attn_decode_static_max_bytes": (_sz, []),
    "forge_attn_decode_static": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i64, _i64, _f, _vp]),
    "forge_decoder_block_decode": (_i, [C.POINTER(BlockDesc), _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _vp, _sz, _vp]),
    "forge_model_decode": (_i, [C.POINTER(ModelDesc), _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _vp, _sz, _vp]),
    "forge_compiled_bind_decode": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "forge_plan_liveness": (_i, [_i, _ip, _ip, _ip, _i, _ip, _ip]),
    "forge_plan_dead_after": (_i, [_i, _ip, _i, _ip, _ip]),
    "forge_plan_linear_scan": (_i, [_i, _ip, _ip, _ip, _ip]),
    "forge_plan_workspace": (_i, [_i, _ip, _ip, _szp, _szp, _szp, _ip]),
    "forge_compile_model": (_i, [C.POINTER(ModelDesc), _i, _i, _i, _i, C.POINTER(_vp)]),
    "forge_compiled_destroy": (None, [_vp]),
    "forge_compiled_workspace_bytes": (_sz, [_vp]),
    "forge_compiled_counts": (_i, [_vp, _ip, _ip, _ip, _ip]),
    "forge_compiled_program": (_i, [_vp, _ip, _ip, _ip, _ip, _szp, _szp]),
    "forge_compiled_bind": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "forge_compiled_run": (_i, [_vp, _vp]),
}


def lib() -> C.CDLL:
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError("%s is missing: build it with `python -m paper_2604_16498_amd.build`"
                              % _LIB_PATH)
        l = C.CDLL(_LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype = res
            fn.argtypes = args
        _lib = l
    return _lib


def status_string(status: int) -> str:
    return lib().forge_status_string(status).decode()


def _p(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("forge tensors must be contiguous GPU tensors")
    return C.c_void_p(t.data_ptr())


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return FORGE_F32
    if t.dtype == torch.bfloat16:
        return FORGE_BF16
    raise ValueError("unsupported dtype %s" % t.dtype)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ws(t: Optional[torch.Tensor]):
    return (_p(t), 0 if t is None else t.numel() * t.element_size())


def _check(status: int, where: str):
    if status != 0:
        raise ForgeError(status, where)


def workspace(nbytes: int, device="cuda") -> Optional[torch.Tensor]:
    """Device scratch of at least nbytes (None when nothing is needed)."""
    return None if nbytes == 0 else torch.empty(nbytes, dtype=torch.uint8, device=device)


# ---------------------------------------------------------------------------------------------


def forge_attn_fused_workspace_bytes(batch, q_heads, kv_heads, q_len, kv_len, head_dim, dtype) -> int:
    dt = FORGE_BF16 if dtype == torch.bfloat16 else FORGE_F32
    return lib().forge_attn_fused_workspace_bytes(batch, q_heads, kv_heads, q_len, kv_len, head_dim, dt)


def forge_attn_fused(q, k, v, out, kv_len=None, scale=None, causal=True, workspace=None,
                     kv_batch_stride=None, kv_head_stride=None):
    """q [B,Hq,Sq,dh]; k, v [B,Hkv,cap,dh] (cap >= kv_len); out [B,Sq,Hq*dh]."""
    B, Hq, Sq, dh = q.shape
    Hkv, cap = k.shape[1], k.shape[2]
    kv_len = cap if kv_len is None else kv_len
    scale = dh ** -0.5 if scale is None else scale
    hs = cap * dh if kv_head_stride is None else kv_head_stride
    bs = Hkv * hs if kv_batch_stride is None else kv_batch_stride
    wp, wb = _ws(workspace)
    _check(lib().forge_attn_fused(_p(q), _p(k), _p(v), _p(out), B, Hq, Hkv, Sq, kv_len, dh, bs, hs,
                                  scale, int(causal), _dt(q), wp, wb, _stream()), "forge_attn_fused")
    return out


def forge_attn_fused_masked(q, k, v, mask, out, kv_len=None, scale=None, causal=False):
    """As forge_attn_fused, with an additive fp32 mask [B or 1, Hq or 1, Sq, kv_len] on the
    scaled scores (size-1 axes broadcast)."""
    B, Hq, Sq, dh = q.shape
    Hkv, cap = k.shape[1], k.shape[2]
    kv_len = cap if kv_len is None else kv_len
    scale = dh ** -0.5 if scale is None else scale
    hs = cap * dh
    bs = Hkv * hs
    assert mask.dtype == torch.float32 and mask.is_contiguous() and mask.shape[2:] == (Sq, kv_len)
    mhs = 0 if mask.shape[1] == 1 else Sq * kv_len
    mbs = 0 if mask.shape[0] == 1 else mask.shape[1] * Sq * kv_len
    _check(lib().forge_attn_fused_masked(_p(q), _p(k), _p(v), _p(mask), _p(out), B, Hq, Hkv, Sq, kv_len, dh,
                                         bs, hs, mbs, mhs, scale, int(causal), _dt(q), _stream()),
           "forge_attn_fused_masked")
    return out


def forge_gemm_workspace_bytes(M, N, K, act, dtype) -> int:
    dt = FORGE_BF16 if dtype == torch.bfloat16 else FORGE_F32
    return lib().forge_gemm_workspace_bytes(M, N, K, ACT[act], dt)


def forge_gemm_variant(M, N, K, act, dtype, ldy=0) -> str:
    dt = FORGE_BF16 if dtype == torch.bfloat16 else FORGE_F32
    return lib().forge_gemm_variant(M, N, K, ldy, ACT[act], dt).decode()


def forge_gemm_bias_gelu(x, w, bias, residual, y, act="gelu_tanh", workspace=None, n=None):
    """y[M,:N] = act(x[M,K] w[N,K]^T + bias) (+ residual); swiglu: w is [2N,K].
    y (and residual) may be wider than N (row stride y.shape[1]); pass n=N then."""
    M, K = x.shape
    ldy = y.shape[1]
    N = ldy if n is None else n
    wp, wb = _ws(workspace)
    _check(lib().forge_gemm_bias_gelu(_p(x), _p(w), _p(bias), _p(residual), _p(y), M, N, K, ldy,
                                      ACT[act], _dt(x), wp, wb, _stream()), "forge_gemm_bias_gelu")
    return y


def forge_deinterleave_gated_rows(src):
    """src [2N, ...] with alternating gate / up rows -> new tensor, gate rows first."""
    assert src.is_cuda and src.is_contiguous() and src.shape[0] % 2 == 0
    dst = torch.empty_like(src)
    row_bytes = src[0].numel() * src.element_size()
    _check(lib().forge_deinterleave_gated_rows(_p(src), _p(dst), src.shape[0] // 2, row_bytes, _stream()),
           "forge_deinterleave_gated_rows")
    return dst


def forge_quantize_int8(w):
    """w [N,K] (bf16 or fp32, GPU) -> (q int8 [N,K], scale fp32 [N])."""
    N, K = w.shape
    q = torch.empty(N, K, dtype=torch.int8, device=w.device)
    scale = torch.empty(N, dtype=torch.float32, device=w.device)
    _check(lib().forge_quantize_int8(_p(w), _p(q), _p(scale), N, K, _dt(w), _stream()), "forge_quantize_int8")
    return q, scale


def forge_gemm_w8_workspace_bytes(M, N, K, act) -> int:
    return lib().forge_gemm_w8_workspace_bytes(M, N, K, ACT[act])


def forge_gemm_w8(x, wq, wscale, bias, residual, y, act="none", workspace=None, n=None):
    """y[M,:N] = act(x[M,K] (wq * wscale[:,None])^T + bias) (+ residual); x, y bf16, wq int8."""
    M, K = x.shape
    ldy = y.shape[1]
    N = ldy if n is None else n
    wp, wb = _ws(workspace)
    _check(lib().forge_gemm_w8(_p(x), _p(wq), _p(wscale), _p(bias), _p(residual), _p(y), M, N, K, ldy,
                               ACT[act], wp, wb, _stream()), "forge_gemm_w8")
    return y


def forge_residual_norm(x, delta, gamma, beta, h_out, y, eps=1e-5, kind="layernorm"):
    rows, d = x.shape[0] if x.dim() == 2 else x.numel() // x.shape[-1], x.shape[-1]
    _check(lib().forge_residual_norm(_p(x), _p(delta), _p(gamma), _p(beta), _p(h_out), _p(y), rows, d,
                                     eps, NORM[kind], _dt(x), _stream()), "forge_residual_norm")
    return h_out, y


def forge_rope(x, n_rows=None, row0=0, pos0=0, base=10000.0):
    """In place on x [B,H,rows_cap,dh]; rotates rows row0..row0+n_rows-1 at positions pos0.."""
    B, H, cap, dh = x.shape
    n_rows = cap - row0 if n_rows is None else n_rows
    _check(lib().forge_rope(_p(x), B, H, n_rows, dh, H * cap * dh, cap * dh, row0, pos0, base, _dt(x),
                            _stream()), "forge_rope")
    return x


def forge_embed(ids, wte, wpe, h, pos0=0):
    B, S = ids.shape
    _check(lib().forge_embed(_p(ids), _p(wte), _p(wpe), _p(h), B, S, wte.shape[1], wte.shape[0],
                             wpe.shape[0], pos0, _dt(wte), _stream()), "forge_embed")
    return h


def make_block_desc(shape, w: Dict[str, Optional[torch.Tensor]]) -> BlockDesc:
    """shape: object with the BlockShape attributes; w: name -> GPU tensor (or None).
    The returned struct holds raw pointers: keep ``w`` alive while it is in use."""
    d = BlockDesc()
    d.d_model, d.q_heads, d.kv_heads, d.head_dim, d.d_ff = (shape.d_model, shape.q_heads,
                                                            shape.kv_heads, shape.head_dim, shape.d_ff)
    d.norm = NORM[shape.norm]
    d.eps = shape.eps
    d.mlp_act = ACT[shape.mlp_act]
    d.use_rope = int(shape.use_rope)
    d.rope_base = shape.rope_base
    # int8 weights (with "s_*" scale vectors in w): the activation dtype is that of the norm gain
    d.dt = _dt(w["norm1_g"] if w.get("s_qkv") is not None else w["w_qkv"])
    for name in ("norm1_g", "norm1_b", "w_qkv", "b_qkv", "w_o", "b_o", "norm2_g", "norm2_b",
                 "w_up", "b_up", "w_down", "b_down", "s_qkv", "s_o", "s_up", "s_down"):
        t = w.get(name)
        if t is not None and (not t.is_cuda or not t.is_contiguous()):
            raise ValueError("weight %s must be a contiguous GPU tensor" % name)
        setattr(d, name, None if t is None else t.data_ptr())
    return d


def forge_decoder_block_workspace_bytes(desc: BlockDesc, batch, q_len, kv_cap) -> int:
    return lib().forge_decoder_block_workspace_bytes(C.byref(desc), batch, q_len, kv_cap)


def forge_decoder_block(desc: BlockDesc, x_in, x_out, k_cache, v_cache, pos0, workspace):
    """x_in/x_out [B,q_len,d]; caches [B,Hkv,kv_cap,dh]."""
    B, q_len, _ = x_in.shape
    kv_cap = k_cache.shape[2]
    wp, wb = _ws(workspace)
    _check(lib().forge_decoder_block(C.byref(desc), _p(x_in), _p(x_out), _p(k_cache), _p(v_cache), B,
                                     q_len, pos0, kv_cap, wp, wb, _stream()), "forge_decoder_block")
    return x_out


def make_model_desc(layer_descs: Sequence[BlockDesc], mw: Dict[str, Optional[torch.Tensor]],
                    logits_ld: int = 0) -> ModelDesc:
    """mw: wte, wpe (both or neither), normf_g, normf_b.  Keeps the layer array alive on the struct."""
    m = ModelDesc()
    arr = (BlockDesc * len(layer_descs))(*layer_descs)
    m._layer_array = arr            # owner
    m.n_layers = len(layer_descs)
    m.layers = C.cast(arr, C.POINTER(BlockDesc))
    wte, wpe = mw.get("wte"), mw.get("wpe")
    m.vocab = 0 if wte is None else wte.shape[0]
    m.n_pos = 0 if wpe is None else wpe.shape[0]
    m.logits_ld = logits_ld
    for name in ("wte", "wpe", "normf_g", "normf_b"):
        t = mw.get(name)
        setattr(m, name, None if t is None else t.data_ptr())
    return m


def forge_model_workspace_bytes(model: ModelDesc, batch, q_len, kv_cap) -> int:
    return lib().forge_model_workspace_bytes(C.byref(model), batch, q_len, kv_cap)


def forge_model_forward(model: ModelDesc, inp, out, k_cache, v_cache, pos0, workspace):
    """inp: int32 ids [B,q_len] (token model) or hidden state [B,q_len,d]; caches [L,B,Hkv,cap,dh]."""
    B, q_len = inp.shape[0], inp.shape[1]
    kv_cap = k_cache.shape[3]
    wp, wb = _ws(workspace)
    _check(lib().forge_model_forward(C.byref(model), _p(inp), _p(out), _p(k_cache), _p(v_cache), B,
                                     q_len, pos0, kv_cap, wp, wb, _stream()), "forge_model_forward")
    return out


# ---------------------------------------------------------------------------------------------
# Decode step with per-sequence positions (seq_pos: int32 GPU tensor [B]).


def forge_attn_decode_varlen(q, k, v, out, seq_pos, max_pos, scale=None, workspace=None):
    """q [B,Hq,1,dh]; k, v [B,Hkv,cap,dh]; out [B,1,Hq*dh]; sequence b attends rows [0, seq_pos[b]]."""
    B, Hq, _, dh = q.shape
    Hkv, cap = k.shape[1], k.shape[2]
    scale = dh ** -0.5 if scale is None else scale
    wp, wb = _ws(workspace)
    assert seq_pos.dtype == torch.int32 and seq_pos.numel() == B
    _check(lib().forge_attn_decode_varlen(_p(q), _p(k), _p(v), _p(out), _p(seq_pos), B, Hq, Hkv, max_pos, dh,
                                          Hkv * cap * dh, cap * dh, scale, _dt(q), wp, wb, _stream()),
           "forge_attn_decode_varlen")
    return out


OP_NAMES = ["embed", "norm", "gemm_qkv", "rope_q", "rope_k", "attn", "gemm_res", "gemm_act", "gemm"]


def forge_trace_start(capacity: int):
    _check(lib().forge_trace_start(capacity, _stream()), "forge_trace_start")


def forge_trace_stop(capacity: int):
    """-> [(operator name, milliseconds)] of the launch lists run since forge_trace_start."""
    n = C.c_int(0)
    ops = (C.c_int * capacity)()
    ms = (C.c_float * capacity)()
    _check(lib().forge_trace_stop(C.byref(n), ops, ms, capacity), "forge_trace_stop")
    return [(OP_NAMES[ops[i]], float(ms[i])) for i in range(min(n.value, capacity))]


def forge_attn_decode_static_max_bytes() -> int:
    return int(lib().forge_attn_decode_static_max_bytes())


def forge_attn_decode_static(q, k, v, out, kv_len=None, scale=None):
    """forge_attn_fused for q_len 1 (bf16, causal) with the library's own fixed scratch: no workspace.
    q [B,Hq,1,dh]; k, v [B,Hkv,cap,dh]; out [B,1,Hq*dh]."""
    B, Hq, Sq, dh = q.shape
    assert Sq == 1 and q.dtype == torch.bfloat16
    Hkv, cap = k.shape[1], k.shape[2]
    kv_len = cap if kv_len is None else kv_len
    scale = dh ** -0.5 if scale is None else scale
    _check(lib().forge_attn_decode_static(_p(q), _p(k), _p(v), _p(out), B, Hq, Hkv, kv_len, dh,
                                          Hkv * cap * dh, cap * dh, scale, _stream()),
           "forge_attn_decode_static")
    return out


def forge_decoder_block_decode(desc: BlockDesc, x_in, x_out, k_cache, v_cache, seq_pos, max_pos, workspace):
    B = x_in.shape[0]
    kv_cap = k_cache.shape[2]
    wp, wb = _ws(workspace)
    assert seq_pos.dtype == torch.int32 and seq_pos.numel() == B
    _check(lib().forge_decoder_block_decode(C.byref(desc), _p(x_in), _p(x_out), _p(k_cache), _p(v_cache),
                                            _p(seq_pos), B, max_pos, kv_cap, wp, wb, _stream()),
           "forge_decoder_block_decode")
    return x_out


def forge_model_decode(model: ModelDesc, inp, out, k_cache, v_cache, seq_pos, max_pos, workspace):
    B = inp.shape[0]
    kv_cap = k_cache.shape[3]
    wp, wb = _ws(workspace)
    assert seq_pos.dtype == torch.int32 and seq_pos.numel() == B
    _check(lib().forge_model_decode(C.byref(model), _p(inp), _p(out), _p(k_cache), _p(v_cache), _p(seq_pos), B,
                                    max_pos, kv_cap, wp, wb, _stream()), "forge_model_decode")
    return out


# ---------------------------------------------------------------------------------------------
# Static buffer plan (host arrays in, host arrays out) and the compiled executor.


def _ints(values):
    return (C.c_int * max(1, len(values)))(*values)


def forge_plan_liveness(out_reg: Sequence[int], in_lists: Sequence[Sequence[int]], n_regs: int):
    """Program = per instruction an output register (-1: none) and the registers it reads.
    Returns (start, end) lists, -1 for registers never mentioned."""
    n = len(out_reg)
    begin, flat = [0], []
    for ins in in_lists:
        flat.extend(ins)
        begin.append(len(flat))
    start, end = _ints([0] * n_regs), _ints([0] * n_regs)
    _check(lib().forge_plan_liveness(n, _ints(out_reg), _ints(begin), _ints(flat), n_regs, start, end),
           "forge_plan_liveness")
    return list(start)[:n_regs], list(end)[:n_regs]


def forge_plan_dead_after(end: Sequence[int], n_instr: int) -> Dict[int, list]:
    live = sum(1 for e in end if e >= 0)
    begin, regs = _ints([0] * (n_instr + 1)), _ints([0] * live)
    _check(lib().forge_plan_dead_after(len(end), _ints(end), n_instr, begin, regs), "forge_plan_dead_after")
    return {j: list(regs[begin[j]:begin[j + 1]]) for j in range(n_instr) if begin[j + 1] > begin[j]}


def forge_plan_linear_scan(start: Sequence[int], end: Sequence[int]):
    n = len(start)
    buf, m = _ints([0] * n), C.c_int(0)
    _check(lib().forge_plan_linear_scan(n, _ints(start), _ints(end), buf, C.byref(m)), "forge_plan_linear_scan")
    return list(buf)[:n], m.value


def forge_plan_workspace(start: Sequence[int], end: Sequence[int], nbytes: Sequence[int]):
    """Returns (offset per register, total bytes, number of buffers); offset -1 where start < 0."""
    n = len(start)
    sizes = (C.c_size_t * max(1, n))(*nbytes)
    off = (C.c_size_t * max(1, n))()
    total, m = C.c_size_t(0), C.c_int(0)
    _check(lib().forge_plan_workspace(n, _ints(start), _ints(end), sizes, off, C.byref(total), C.byref(m)),
           "forge_plan_workspace")
    none = C.c_size_t(-1).value
    return [-1 if o == none else o for o in list(off)[:n]], total.value, m.value


class CompiledModel:
    """Handle of forge_compile_model for one fixed (batch, q_len, pos0, kv_cap).  `bind` records
    the HIP graph on a non-default stream, `run` replays it.  Keeps the descriptor (and through
    it nothing else) alive: the caller keeps the weight tensors alive."""

    def __init__(self, model: ModelDesc, batch: int, q_len: int, pos0: int, kv_cap: int):
        self._h = C.c_void_p(None)
        self._model = model
        _check(lib().forge_compile_model(C.byref(model), batch, q_len, pos0, kv_cap, C.byref(self._h)),
               "forge_compile_model")
        self._bound = None

    def close(self):
        if self._h:
            lib().forge_compiled_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def workspace_bytes(self) -> int:
        return lib().forge_compiled_workspace_bytes(self._h)

    def counts(self):
        """(instructions, registers, register reads, buffers)"""
        a, b, c, d = C.c_int(0), C.c_int(0), C.c_int(0), C.c_int(0)
        _check(lib().forge_compiled_counts(self._h, C.byref(a), C.byref(b), C.byref(c), C.byref(d)),
               "forge_compiled_counts")
        return a.value, b.value, c.value, d.value

    def program(self):
        """(ops, out_reg, in_lists, reg_bytes, reg_offset)"""
        ni, nr, nreads, _ = self.counts()
        op, out, begin, regs = _ints([0] * ni), _ints([0] * ni), _ints([0] * (ni + 1)), _ints([0] * nreads)
        nb, off = (C.c_size_t * max(1, nr))(), (C.c_size_t * max(1, nr))()
        _check(lib().forge_compiled_program(self._h, op, out, begin, regs, nb, off), "forge_compiled_program")
        ins = [list(regs[begin[j]:begin[j + 1]]) for j in range(ni)]
        return list(op)[:ni], list(out)[:ni], ins, list(nb)[:nr], list(off)[:nr]

    def bind(self, inp, out, k_cache, v_cache, workspace, stream: "torch.cuda.Stream"):
        wp, wb = _ws(workspace)
        _check(lib().forge_compiled_bind(self._h, _p(inp), _p(out), _p(k_cache), _p(v_cache), wp, wb,
                                         C.c_void_p(stream.cuda_stream)), "forge_compiled_bind")
        self._bound = (inp, out, k_cache, v_cache, workspace)     # keep the tensors alive
        return self

    def bind_decode(self, inp, out, k_cache, v_cache, seq_pos, workspace, stream: "torch.cuda.Stream"):
        wp, wb = _ws(workspace)
        _check(lib().forge_compiled_bind_decode(self._h, _p(inp), _p(out), _p(k_cache), _p(v_cache), _p(seq_pos),
                                                wp, wb, C.c_void_p(stream.cuda_stream)), "forge_compiled_bind_decode")
        self._bound = (inp, out, k_cache, v_cache, seq_pos, workspace)
        return self

    def run(self, stream: "torch.cuda.Stream"):
        _check(lib().forge_compiled_run(self._h, C.c_void_p(stream.cuda_stream)), "forge_compiled_run")
