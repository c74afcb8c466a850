// Host-side helpers shared by the entry points: argument checks, dtype dispatch of the
// launchers, workspace carving.  Internal to the library.
#pragma once
#include "common.hpp"

namespace forge {

inline size_t esize(forge_dtype dt) { return dt == FORGE_BF16 ? 2 : 4; }
inline bool dtype_ok(forge_dtype dt) { return dt == FORGE_F32 || dt == FORGE_BF16; }
inline bool req(const void* p) { return p != nullptr && aligned16(p); }
inline bool opt(const void* p) { return p == nullptr || aligned16(p); }
// The softmax scale: positive and finite.  The matrix-core kernels take the running maximum of
// the raw scores and apply the scale afterwards, which is the maximum of the scaled scores only
// for a positive factor.
inline bool scale_ok(float scale) { return scale > 0.0f && scale <= 3.0e38f; }

// rows (2r, 2r + 1) of src -> rows (r, pairs + r) of dst (defined with the elementwise kernels)
forge_status launch_deinterleave_rows(const void* src, void* dst, int pairs, size_t row_bytes, hipStream_t s);

// Size limits of one call (beyond them: FORGE_ERR_UNSUPPORTED).  Row counts and element offsets
// are 64-bit inside the kernels; these bounds keep tile counts and thread counts inside 32 bits
// and batch / head counts inside a grid dimension.
constexpr int64_t kMaxRows = 1ll << 24;        // batch * q_len, GEMM rows, GEMM columns
constexpr int64_t kMaxOutputs = 1ll << 36;     // GEMM rows * columns
constexpr int kMaxGridDim = 65535;             // batch, heads
inline bool rows_ok(int batch, int q_len) { return (int64_t)batch * q_len <= kMaxRows; }
inline bool grid_ok(int batch, int heads) { return batch <= kMaxGridDim && heads <= kMaxGridDim; }
inline bool gemm_size_ok(int M, int N) {
  return M <= kMaxRows && N <= kMaxRows && (int64_t)M * N <= kMaxOutputs;
}
// rows [pos0, pos0 + n) lie inside [0, cap), without overflowing the sum
inline bool span_ok(int pos0, int n, int cap) { return pos0 >= 0 && n >= 1 && n <= cap && pos0 <= cap - n; }

// carve 256-byte aligned pieces out of one workspace
struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* b) : base(static_cast<char*>(b)) {}
  void* take(size_t bytes) {
    void* p = base ? base + off : nullptr;
    off += align_up(bytes, 256);
    return p;
  }
};

inline forge_status attn_dispatch(const AttnArgs& a, forge_dtype dt, hipStream_t s) {
  if (dt == FORGE_F32) return launch_attn_f32(a, s);
  if (a.q_len == 1 && a.mask == nullptr) return launch_attn_decode_bf16(a, s);
  return launch_attn_prefill_bf16(a, s);
}

inline size_t attn_ws(int batch, int q_heads, int kv_heads, int q_len, int kv_len, int head_dim,
               forge_dtype dt) {
  if (dt == FORGE_BF16 && q_len == 1)
    return attn_decode_workspace_bytes(batch, q_heads, kv_heads, kv_len, head_dim);
  return 0;
}

// plain: see gemm_bf16_workspace_bytes
inline size_t gemm_ws(int M, int N, int K, forge_act act, forge_dtype dt, bool w8, bool plain = false) {
  if (w8) return gemm_w8_workspace_bytes(M, N, K, act);
  return dt == FORGE_BF16 ? gemm_bf16_workspace_bytes(M, N, K, act, plain) : gemm_f32_workspace_bytes(M, N, K, act);
}

// int8 weights: all four scale vectors given (checked by check_block_desc: all or none)
inline bool block_w8(const forge_block_desc* d) { return d->s_qkv != nullptr; }

inline forge_status gemm_dispatch(const GemmArgs& a, forge_dtype dt, hipStream_t s) {
  return dt == FORGE_BF16 ? launch_gemm_bf16(a, s) : launch_gemm_f32(a, s);
}

inline forge_status check_block_desc(const forge_block_desc* d) {
  if (d == nullptr || !dtype_ok(d->dt)) return FORGE_ERR_INVALID_ARG;
  if (d->d_model < 8 || d->q_heads < 1 || d->kv_heads < 1 || d->d_ff < 8) return FORGE_ERR_INVALID_ARG;
  if (d->q_heads % d->kv_heads != 0) return FORGE_ERR_INVALID_ARG;
  if (d->head_dim != 64 && d->head_dim != 128) return FORGE_ERR_UNSUPPORTED;
  if (d->q_heads > kMaxGridDim || d->d_ff > kMaxRows) return FORGE_ERR_UNSUPPORTED;
  if (d->d_model % 8 != 0 || d->d_ff % 8 != 0 || d->d_model > 16384) return FORGE_ERR_UNSUPPORTED;
  if (d->mlp_act != FORGE_ACT_GELU_TANH && d->mlp_act != FORGE_ACT_SWIGLU &&
      d->mlp_act != FORGE_ACT_RELU && d->mlp_act != FORGE_ACT_SILU && d->mlp_act != FORGE_ACT_GELU_ERF)
    return FORGE_ERR_UNSUPPORTED;
  if (d->norm != FORGE_NORM_LAYERNORM && d->norm != FORGE_NORM_RMSNORM) return FORGE_ERR_INVALID_ARG;
  if (!req(d->norm1_g) || !req(d->w_qkv) || !req(d->w_o) || !req(d->norm2_g) || !req(d->w_up) ||
      !req(d->w_down))
    return FORGE_ERR_INVALID_ARG;
  if (!opt(d->norm1_b) || !opt(d->b_qkv) || !opt(d->b_o) || !opt(d->norm2_b) || !opt(d->b_up) ||
      !opt(d->b_down))
    return FORGE_ERR_INVALID_ARG;
  if (d->use_rope && !(d->rope_base > 1.0f)) return FORGE_ERR_INVALID_ARG;
  const int n_scales = (d->s_qkv != nullptr) + (d->s_o != nullptr) + (d->s_up != nullptr) + (d->s_down != nullptr);
  if (n_scales != 0 && n_scales != 4) return FORGE_ERR_INVALID_ARG;
  if (n_scales == 4) {
    if (!req(d->s_qkv) || !req(d->s_o) || !req(d->s_up) || !req(d->s_down)) return FORGE_ERR_INVALID_ARG;
    // int8 weights go with bf16 activations and whole 128-element slabs of every reduction
    if (d->dt != FORGE_BF16 || d->d_model % 128 != 0 || d->d_ff % 128 != 0 ||
        (d->q_heads * d->head_dim) % 128 != 0)
      return FORGE_ERR_UNSUPPORTED;
  }
  return FORGE_OK;
}

inline forge_status check_model(const forge_model_desc* m) {
  if (m == nullptr || m->n_layers < 1 || m->layers == nullptr) return FORGE_ERR_INVALID_ARG;
  for (int l = 0; l < m->n_layers; ++l) {
    forge_status st = check_block_desc(&m->layers[l]);
    if (st != FORGE_OK) return st;
    const forge_block_desc *a = &m->layers[l], *b = &m->layers[0];
    if (a->d_model != b->d_model || a->dt != b->dt || a->kv_heads != b->kv_heads ||
        a->head_dim != b->head_dim)
      return FORGE_ERR_UNSUPPORTED;
  }
  if (!req(m->normf_g) || !opt(m->normf_b)) return FORGE_ERR_INVALID_ARG;
  if ((m->wte == nullptr) != (m->wpe == nullptr)) return FORGE_ERR_INVALID_ARG;
  if (m->wte != nullptr && (!req(m->wte) || !req(m->wpe) || m->vocab < 1 || m->n_pos < 1))
    return FORGE_ERR_INVALID_ARG;
  if (m->wte != nullptr && m->vocab > kMaxRows) return FORGE_ERR_UNSUPPORTED;
  if (m->logits_ld != 0 && m->logits_ld < m->vocab) return FORGE_ERR_INVALID_ARG;
  return FORGE_OK;
}

}  // namespace forge
