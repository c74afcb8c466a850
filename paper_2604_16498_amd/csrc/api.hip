// C ABI of the forge library: argument checks on the host, then a fixed list of launches on
// the caller's stream.  Nothing here allocates, frees or synchronises.
#include "api_internal.hpp"

using namespace forge;

#include <mutex>
#include <vector>

namespace {

// ---- per-operator timing of the launch lists (forge_trace_*) ---------------------------------
// While a trace is open, the launch lists record one HIP event on their stream after every
// operator (a launch, or a split-K launch pair); the time between two events is that operator's
// duration inside the step, launch gaps included.  The events are created when the trace is
// opened, so the launch lists themselves still allocate nothing.
struct Trace {
  std::mutex mu;
  bool open = false;
  int n = 0;
  std::vector<hipEvent_t> ev;    // ev[0] opens the trace, ev[i + 1] follows operator i
  std::vector<int> op;
};
Trace g_trace;

inline void trace_mark(hipStream_t s, forge_op op) {
  if (!g_trace.open) return;                    // unsynchronised fast path: a trace is opened and
  std::lock_guard<std::mutex> lock(g_trace.mu); // closed by the thread that also launches
  if (!g_trace.open || g_trace.n + 1 >= (int)g_trace.ev.size()) return;
  if (hipEventRecord(g_trace.ev[g_trace.n + 1], s) != hipSuccess) return;
  g_trace.op[g_trace.n++] = (int)op;
}

struct BlockPlan {
  size_t y, q, o, u, attn, gemm, total;
};

BlockPlan plan_block(const forge_block_desc* d, int batch, int q_len, int kv_cap) {
  const size_t es = esize(d->dt);
  const size_t T = (size_t)batch * q_len;
  const int hd = d->q_heads * d->head_dim;
  const int nqkv = (d->q_heads + 2 * d->kv_heads) * d->head_dim;
  BlockPlan p;
  p.y = align_up(T * d->d_model * es, 256);
  p.q = align_up(T * hd * es, 256);
  p.o = align_up(T * hd * es, 256);
  p.u = align_up(T * d->d_ff * es, 256);
  p.attn = align_up(attn_ws(batch, d->q_heads, d->kv_heads, q_len, kv_cap, d->head_dim, d->dt), 256);
  const bool w8 = block_w8(d);
  size_t g = 0;
  for (size_t v : {gemm_qkv_workspace_bytes((int)T, nqkv, d->d_model, d->dt, w8, d->use_rope != 0, q_len, d->head_dim),
                   gemm_ws((int)T, d->d_model, hd, FORGE_ACT_NONE, d->dt, w8),
                   gemm_ws((int)T, d->d_ff, d->d_model, d->mlp_act, d->dt, w8, true),
                   gemm_ws((int)T, d->d_model, d->d_ff, FORGE_ACT_NONE, d->dt, w8)})
    g = v > g ? v : g;
  p.gemm = align_up(g, 256);
  p.total = p.y + p.q + p.o + p.u + p.attn + p.gemm;
  return p;
}

// where a layer keeps its normalised rows: the first piece carved from its workspace
inline void* block_norm_rows(void* workspace) { return workspace; }

// the launch list of one layer; all arguments already validated
// seq_pos (device, [batch], or NULL): per-sequence positions of a decode step (q_len == 1); pos0 is
// then the largest position the caller vouches for
// next_norm / x_normed chain the layers of a decode-sized stack (only where gemm_fuses_tail()
// holds for the model width): the reduce step of the MLP down projection also produces the rows
// the NEXT consumer normalises (next layer's first norm, or the model's final norm) into
// next_norm->y_norm, and a layer called with x_normed finds its first norm already done.
forge_status run_block(const forge_block_desc* d, const void* x_in, void* x_out, void* k_cache,
                       void* v_cache, int batch, int q_len, int pos0, int kv_cap, void* workspace,
                       hipStream_t s, const int* seq_pos = nullptr, const NormTail* next_norm = nullptr,
                       bool x_normed = false) {
  const BlockPlan pl = plan_block(d, batch, q_len, kv_cap);
  Carver cv(workspace);
  void* y = cv.take(pl.y);          // == block_norm_rows(workspace)
  void* q = cv.take(pl.q);
  void* o = cv.take(pl.o);
  void* u = cv.take(pl.u);
  void* aws = cv.take(pl.attn);
  void* gws = cv.take(pl.gemm);
  const int T = batch * q_len;
  const int dm = d->d_model, dh = d->head_dim, hd = d->q_heads * dh;
  const int nqkv = (d->q_heads + 2 * d->kv_heads) * dh;
  const int64_t kv_hs = (int64_t)kv_cap * dh, kv_bs = kv_hs * d->kv_heads;
  forge_status st;

  // 1. first norm (unless the previous layer's last reduce step left it in y)
  if (!x_normed) {
    st = launch_residual_norm(x_in, nullptr, d->norm1_g, d->norm1_b, nullptr, y, T, dm, d->eps, d->norm, d->dt, s);
    if (st != FORGE_OK) return st;
    trace_mark(s, FORGE_OP_NORM);
  }
  // 2. QKV projection, written head-major: q to the workspace, k and v into the cache rows
  // (the projection rotates q and k itself where it can: in the reduce step of a decode-sized one,
  // in the epilogue of a prompt-sized bf16 one)
  const bool rope_in_gemm = d->use_rope && gemm_qkv_fuses_rope(T, nqkv, dm, dh, q_len, d->dt, block_w8(d));
  QkvSplit sp = {q, k_cache, v_cache, d->q_heads, d->kv_heads, dh, q_len, kv_cap, pos0,
                 rope_in_gemm ? 1 : 0, d->rope_base, seq_pos, nullptr};
  GemmArgs g = {y, d->w_qkv, d->b_qkv, nullptr, nullptr, T, nqkv, dm, 0, FORGE_ACT_NONE, &sp, nullptr, gws, pl.gemm, d->s_qkv};
  st = gemm_dispatch(g, d->dt, s);
  if (st != FORGE_OK) return st;
  trace_mark(s, FORGE_OP_GEMM_QKV);
  // 3. rotary embedding of the new q and k rows
  if (d->use_rope && !rope_in_gemm) {
    st = launch_rope(q, batch, d->q_heads, q_len, dh, (int64_t)d->q_heads * q_len * dh,
                     (int64_t)q_len * dh, 0, pos0, d->rope_base, d->dt, s, seq_pos, false);
    if (st != FORGE_OK) return st;
    trace_mark(s, FORGE_OP_ROPE_Q);
    st = launch_rope(k_cache, batch, d->kv_heads, q_len, dh, kv_bs, kv_hs, pos0, pos0, d->rope_base, d->dt, s,
                     seq_pos, true);
    if (st != FORGE_OK) return st;
    trace_mark(s, FORGE_OP_ROPE_K);
  }
  // 4. fused causal attention over cache rows [0, pos0 + q_len)
  AttnArgs at = {q, k_cache, v_cache, o, batch, d->q_heads, d->kv_heads, q_len, pos0 + q_len, dh,
                 kv_bs, kv_hs, 1.0f / sqrtf((float)dh), 1, aws, pl.attn, nullptr, 0, 0, seq_pos};
  st = attn_dispatch(at, d->dt, s);
  if (st != FORGE_OK) return st;
  trace_mark(s, FORGE_OP_ATTN);
  // 5. output projection + bias + residual
  //    (decode-sized: the reduce step of the projection also produces the second norm)
  const bool norm_in_gemm = gemm_fuses_tail(T, dm, d->dt);
  NormTail nt = {d->norm2_g, d->norm2_b, y, d->eps, d->norm};
  g = GemmArgs{o, d->w_o, d->b_o, x_in, x_out, T, dm, hd, 0, FORGE_ACT_NONE, nullptr,
               norm_in_gemm ? &nt : nullptr, gws, pl.gemm, d->s_o};
  st = gemm_dispatch(g, d->dt, s);
  if (st != FORGE_OK) return st;
  trace_mark(s, FORGE_OP_GEMM_RES);
  // 6. second norm
  if (!norm_in_gemm) {
    st = launch_residual_norm(x_out, nullptr, d->norm2_g, d->norm2_b, nullptr, y, T, dm, d->eps, d->norm, d->dt, s);
    if (st != FORGE_OK) return st;
    trace_mark(s, FORGE_OP_NORM);
  }
  // 7. MLP up projection + bias + activation (SwiGLU: gate and up in one pass)
  g = GemmArgs{y, d->w_up, d->b_up, nullptr, u, T, d->d_ff, dm, 0, d->mlp_act, nullptr, nullptr, gws, pl.gemm, d->s_up};
  st = gemm_dispatch(g, d->dt, s);
  if (st != FORGE_OK) return st;
  trace_mark(s, FORGE_OP_GEMM_ACT);
  // 8. MLP down projection + bias + residual
  //    (+ the next consumer's norm of the new residual stream, see above)
  g = GemmArgs{u, d->w_down, d->b_down, x_out, x_out, T, dm, d->d_ff, 0, FORGE_ACT_NONE, nullptr, next_norm, gws, pl.gemm, d->s_down};
  st = gemm_dispatch(g, d->dt, s);
  if (st == FORGE_OK) trace_mark(s, FORGE_OP_GEMM_RES);
  return st;
}

struct ModelPlan {
  size_t h, yf, block, total;
};

ModelPlan plan_model(const forge_model_desc* m, int batch, int q_len, int kv_cap) {
  const forge_block_desc* d0 = &m->layers[0];
  const size_t es = esize(d0->dt);
  const size_t T = (size_t)batch * q_len;
  ModelPlan p;
  p.h = align_up(T * d0->d_model * es, 256);
  p.yf = m->wte != nullptr ? align_up(T * d0->d_model * es, 256) : 0;
  p.block = 0;
  for (int l = 0; l < m->n_layers; ++l) {
    const size_t b = plan_block(&m->layers[l], batch, q_len, kv_cap).total;
    p.block = b > p.block ? b : p.block;
  }
  const size_t head = m->wte != nullptr ? align_up(gemm_ws((int)T, m->vocab, d0->d_model, FORGE_ACT_NONE, d0->dt, false, true), 256) : 0;
  p.block = head > p.block ? head : p.block;
  p.total = p.h + p.yf + p.block;
  return p;
}

}  // namespace

extern "C" {

const char* forge_status_string(forge_status s) {
  switch (s) {
    case FORGE_OK: return "FORGE_OK";
    case FORGE_ERR_INVALID_ARG: return "FORGE_ERR_INVALID_ARG";
    case FORGE_ERR_UNSUPPORTED: return "FORGE_ERR_UNSUPPORTED";
    case FORGE_ERR_WORKSPACE: return "FORGE_ERR_WORKSPACE";
    case FORGE_ERR_HIP: return "FORGE_ERR_HIP";
  }
  return "FORGE_ERR_UNKNOWN";
}

int forge_version(void) { return 100; }

forge_status forge_trace_start(int capacity, void* stream) {
  if (capacity < 1 || capacity > (1 << 20)) return FORGE_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lock(g_trace.mu);
  if (g_trace.open) return FORGE_ERR_INVALID_ARG;
  g_trace.ev.assign(capacity + 1, nullptr);
  g_trace.op.assign(capacity, 0);
  g_trace.n = 0;
  for (hipEvent_t& e : g_trace.ev) {
    if (hipEventCreate(&e) != hipSuccess) {
      for (hipEvent_t& f : g_trace.ev)
        if (f != nullptr) (void)hipEventDestroy(f);
      g_trace.ev.clear();
      return FORGE_ERR_HIP;
    }
  }
  if (hipEventRecord(g_trace.ev[0], static_cast<hipStream_t>(stream)) != hipSuccess) {
    for (hipEvent_t& f : g_trace.ev) (void)hipEventDestroy(f);
    g_trace.ev.clear();
    return FORGE_ERR_HIP;
  }
  g_trace.open = true;
  return FORGE_OK;
}

forge_status forge_trace_stop(int* n_ops, int* ops, float* ms, int capacity) {
  std::lock_guard<std::mutex> lock(g_trace.mu);
  if (!g_trace.open) return FORGE_ERR_INVALID_ARG;
  g_trace.open = false;
  forge_status st = FORGE_OK;
  const int n = g_trace.n;
  if (n_ops != nullptr) *n_ops = n;
  if (n > 0 && hipEventSynchronize(g_trace.ev[n]) != hipSuccess) st = FORGE_ERR_HIP;
  for (int i = 0; i < n && i < capacity && st == FORGE_OK; ++i) {
    if (ops != nullptr) ops[i] = g_trace.op[i];
    if (ms != nullptr && hipEventElapsedTime(&ms[i], g_trace.ev[i], g_trace.ev[i + 1]) != hipSuccess)
      st = FORGE_ERR_HIP;
  }
  for (hipEvent_t& e : g_trace.ev) (void)hipEventDestroy(e);
  g_trace.ev.clear();
  g_trace.op.clear();
  return st;
}

size_t forge_attn_fused_workspace_bytes(int batch, int q_heads, int kv_heads, int q_len, int kv_len,
                                        int head_dim, forge_dtype dt) {
  if (batch < 1 || q_heads < 1 || kv_heads < 1 || q_len < 1 || kv_len < 1) return 0;
  if (!grid_ok(batch, q_heads) || !rows_ok(batch, q_len)) return 0;
  return attn_ws(batch, q_heads, kv_heads, q_len, kv_len, head_dim, dt);
}

forge_status forge_attn_fused(const void* q, const void* k, const void* v, void* out, int batch,
                              int q_heads, int kv_heads, int q_len, int kv_len, int head_dim,
                              int64_t kv_batch_stride, int64_t kv_head_stride, float scale,
                              int causal, forge_dtype dt, void* workspace, size_t workspace_bytes,
                              void* stream) {
  if (!dtype_ok(dt) || !req(q) || !req(k) || !req(v) || !req(out) || !opt(workspace))
    return FORGE_ERR_INVALID_ARG;
  if (batch < 1 || q_heads < 1 || kv_heads < 1 || q_len < 1 || kv_len < 1) return FORGE_ERR_INVALID_ARG;
  if (q_heads % kv_heads != 0 || !scale_ok(scale)) return FORGE_ERR_INVALID_ARG;
  if (causal && kv_len < q_len) return FORGE_ERR_INVALID_ARG;
  if (head_dim != 64 && head_dim != 128) return FORGE_ERR_UNSUPPORTED;
  if (!grid_ok(batch, q_heads) || !rows_ok(batch, q_len)) return FORGE_ERR_UNSUPPORTED;
  if (kv_head_stride < (int64_t)kv_len * head_dim || kv_batch_stride < kv_head_stride * kv_heads)
    return FORGE_ERR_INVALID_ARG;
  if (kv_head_stride % 8 != 0 || kv_batch_stride % 8 != 0) return FORGE_ERR_INVALID_ARG;
  if (out == q || out == k || out == v) return FORGE_ERR_INVALID_ARG;
  const size_t need = attn_ws(batch, q_heads, kv_heads, q_len, kv_len, head_dim, dt);
  if (need > 0 && (workspace == nullptr || workspace_bytes < need)) return FORGE_ERR_WORKSPACE;
  AttnArgs a = {q, k, v, out, batch, q_heads, kv_heads, q_len, kv_len, head_dim,
                kv_batch_stride, kv_head_stride, scale, causal, workspace, workspace_bytes, nullptr, 0, 0};
  return attn_dispatch(a, dt, static_cast<hipStream_t>(stream));
}

forge_status forge_attn_fused_masked(const void* q, const void* k, const void* v, const float* mask,
                                     void* out, int batch, int q_heads, int kv_heads, int q_len,
                                     int kv_len, int head_dim, int64_t kv_batch_stride,
                                     int64_t kv_head_stride, int64_t mask_batch_stride,
                                     int64_t mask_head_stride, float scale, int causal,
                                     forge_dtype dt, void* stream) {
  if (!dtype_ok(dt) || !req(q) || !req(k) || !req(v) || !req(out) || mask == nullptr ||
      (reinterpret_cast<uintptr_t>(mask) & 3u) != 0)
    return FORGE_ERR_INVALID_ARG;
  if (batch < 1 || q_heads < 1 || kv_heads < 1 || q_len < 1 || kv_len < 1) return FORGE_ERR_INVALID_ARG;
  if (q_heads % kv_heads != 0 || !scale_ok(scale)) return FORGE_ERR_INVALID_ARG;
  if (causal && kv_len < q_len) return FORGE_ERR_INVALID_ARG;
  if (head_dim != 64 && head_dim != 128) return FORGE_ERR_UNSUPPORTED;
  if (!grid_ok(batch, q_heads) || !rows_ok(batch, q_len)) return FORGE_ERR_UNSUPPORTED;
  if (kv_head_stride < (int64_t)kv_len * head_dim || kv_batch_stride < kv_head_stride * kv_heads)
    return FORGE_ERR_INVALID_ARG;
  if (kv_head_stride % 8 != 0 || kv_batch_stride % 8 != 0) return FORGE_ERR_INVALID_ARG;
  const int64_t plane = (int64_t)q_len * kv_len;
  if ((mask_head_stride != 0 && mask_head_stride < plane) ||
      (mask_batch_stride != 0 && mask_batch_stride < (mask_head_stride != 0 ? mask_head_stride * q_heads : plane)))
    return FORGE_ERR_INVALID_ARG;
  if (out == q || out == k || out == v) return FORGE_ERR_INVALID_ARG;
  AttnArgs a = {q, k, v, out, batch, q_heads, kv_heads, q_len, kv_len, head_dim,
                kv_batch_stride, kv_head_stride, scale, causal, nullptr, 0,
                mask, mask_batch_stride, mask_head_stride};
  return attn_dispatch(a, dt, static_cast<hipStream_t>(stream));
}

size_t forge_gemm_workspace_bytes(int M, int N, int K, forge_act act, forge_dtype dt) {
  if (M < 1 || N < 1 || K < 1 || !gemm_size_ok(M, N)) return 0;
  return gemm_ws(M, N, K, act, dt, false, true);
}

const char* forge_gemm_variant(int M, int N, int K, int ldy, forge_act act, forge_dtype dt) {
  if (M < 1 || N < 1 || K < 1) return "none";
  return dt == FORGE_BF16 ? gemm_bf16_variant(M, N, K, ldy > 0 ? ldy : N, act) : "gemm_f32<64,64,2,2>";
}

forge_status forge_gemm_bias_gelu(const void* x, const void* w, const void* bias,
                                  const void* residual, void* y, int M, int N, int K, int ldy,
                                  forge_act act, forge_dtype dt, void* workspace,
                                  size_t workspace_bytes, void* stream) {
  if (!dtype_ok(dt) || !req(x) || !req(w) || !req(y) || !opt(bias) || !opt(residual) || !opt(workspace))
    return FORGE_ERR_INVALID_ARG;
  if (M < 1 || N < 1 || K < 1 || ldy < 0 || (ldy > 0 && ldy < N)) return FORGE_ERR_INVALID_ARG;
  if (act < FORGE_ACT_NONE || act > FORGE_ACT_GELU_ERF) return FORGE_ERR_INVALID_ARG;
  if (K % (dt == FORGE_BF16 ? 8 : 4) != 0 || !gemm_size_ok(M, N)) return FORGE_ERR_UNSUPPORTED;
  if (y == x || y == w) return FORGE_ERR_INVALID_ARG;
  // only the decode-sized bf16 problems cannot run without their partial-sum planes
  const size_t need = dt == FORGE_BF16 && M <= 64 ? gemm_ws(M, N, K, act, dt, false, true) : 0;
  if (need > 0 && (workspace == nullptr || workspace_bytes < need)) return FORGE_ERR_WORKSPACE;
  GemmArgs a = {x, w, bias, residual, y, M, N, K, ldy, act, nullptr, nullptr, workspace, workspace_bytes};
  return gemm_dispatch(a, dt, static_cast<hipStream_t>(stream));
}

forge_status forge_deinterleave_gated_rows(const void* src, void* dst, int n_pairs, size_t row_bytes,
                                          void* stream) {
  if (src == nullptr || dst == nullptr || n_pairs < 1 || row_bytes < 1) return FORGE_ERR_INVALID_ARG;
  if (n_pairs > (1 << 30) || row_bytes > ((size_t)1 << 40)) return FORGE_ERR_UNSUPPORTED;
  // out of place: the two 2 * n_pairs * row_bytes ranges must not overlap
  const uintptr_t a = reinterpret_cast<uintptr_t>(src), b = reinterpret_cast<uintptr_t>(dst);
  const size_t total = 2 * (size_t)n_pairs * row_bytes;
  if ((a <= b ? b - a : a - b) < total) return FORGE_ERR_INVALID_ARG;
  return launch_deinterleave_rows(src, dst, n_pairs, row_bytes, static_cast<hipStream_t>(stream));
}

size_t forge_gemm_w8_workspace_bytes(int M, int N, int K, forge_act act) {
  if (M < 1 || N < 1 || K < 1 || !gemm_size_ok(M, N)) return 0;
  return gemm_ws(M, N, K, act, FORGE_BF16, true);
}

forge_status forge_gemm_w8(const void* x, const int8_t* wq, const float* wscale, const void* bias,
                           const void* residual, void* y, int M, int N, int K, int ldy,
                           forge_act act, void* workspace, size_t workspace_bytes, void* stream) {
  if (!req(x) || !req(wq) || !req(wscale) || !req(y) || !opt(bias) || !opt(residual) || !req(workspace))
    return FORGE_ERR_INVALID_ARG;
  if (M < 1 || N < 1 || K < 1 || ldy < 0 || (ldy > 0 && ldy < N)) return FORGE_ERR_INVALID_ARG;
  if (act < FORGE_ACT_NONE || act > FORGE_ACT_GELU_ERF) return FORGE_ERR_INVALID_ARG;
  if (K % 128 != 0 || !gemm_size_ok(M, N)) return FORGE_ERR_UNSUPPORTED;
  if (y == x) return FORGE_ERR_INVALID_ARG;
  if (workspace_bytes < gemm_ws(M, N, K, act, FORGE_BF16, true)) return FORGE_ERR_WORKSPACE;
  GemmArgs a = {x, wq, bias, residual, y, M, N, K, ldy, act, nullptr, nullptr, workspace, workspace_bytes, wscale};
  return gemm_dispatch(a, FORGE_BF16, static_cast<hipStream_t>(stream));
}

forge_status forge_quantize_int8(const void* w, int8_t* q, float* scale, int N, int K, forge_dtype dt,
                                 void* stream) {
  if (!dtype_ok(dt) || !req(w) || q == nullptr || scale == nullptr || (reinterpret_cast<uintptr_t>(scale) & 3u) != 0)
    return FORGE_ERR_INVALID_ARG;
  if (N < 1 || K < 1) return FORGE_ERR_INVALID_ARG;
  return launch_quantize_int8(w, q, scale, N, K, dt, static_cast<hipStream_t>(stream));
}

forge_status forge_residual_norm(const void* x, const void* delta, const void* gamma,
                                 const void* beta, void* h_out, void* y, int rows, int d, float eps,
                                 forge_norm kind, forge_dtype dt, void* stream) {
  if (!dtype_ok(dt) || !req(x) || !req(gamma) || !req(y) || !opt(delta) || !opt(beta) || !opt(h_out))
    return FORGE_ERR_INVALID_ARG;
  if (rows < 1 || d < 1 || !(eps >= 0.f)) return FORGE_ERR_INVALID_ARG;
  if (kind != FORGE_NORM_LAYERNORM && kind != FORGE_NORM_RMSNORM) return FORGE_ERR_INVALID_ARG;
  if (d % 8 != 0 || d > 16384) return FORGE_ERR_UNSUPPORTED;
  if (y == x || (h_out != nullptr && h_out == y)) return FORGE_ERR_INVALID_ARG;
  return launch_residual_norm(x, delta, gamma, beta, h_out, y, rows, d, eps, kind, dt,
                              static_cast<hipStream_t>(stream));
}

forge_status forge_rope(void* x, int batch, int heads, int n_rows, int head_dim,
                        int64_t batch_stride, int64_t head_stride, int row0, int pos0, float base,
                        forge_dtype dt, void* stream) {
  if (!dtype_ok(dt) || !req(x)) return FORGE_ERR_INVALID_ARG;
  if (batch < 1 || heads < 1 || n_rows < 1 || row0 < 0 || pos0 < 0 || !(base > 1.0f))
    return FORGE_ERR_INVALID_ARG;
  if (head_dim < 16 || head_dim % 16 != 0) return FORGE_ERR_UNSUPPORTED;
  if (!rows_ok(batch, n_rows)) return FORGE_ERR_UNSUPPORTED;
  if (head_stride < ((int64_t)row0 + n_rows) * head_dim || batch_stride < head_stride * heads)
    return FORGE_ERR_INVALID_ARG;
  if (head_stride % 8 != 0 || batch_stride % 8 != 0) return FORGE_ERR_INVALID_ARG;
  return launch_rope(x, batch, heads, n_rows, head_dim, batch_stride, head_stride, row0, pos0, base,
                     dt, static_cast<hipStream_t>(stream));
}

forge_status forge_embed(const int32_t* ids, const void* wte, const void* wpe, void* h, int batch,
                         int seq, int d, int vocab, int n_pos, int pos0, forge_dtype dt,
                         void* stream) {
  if (!dtype_ok(dt) || ids == nullptr || !req(wte) || !req(wpe) || !req(h)) return FORGE_ERR_INVALID_ARG;
  if (batch < 1 || d < 1 || vocab < 1 || !span_ok(pos0, seq, n_pos)) return FORGE_ERR_INVALID_ARG;
  if (d % 8 != 0 || !rows_ok(batch, seq)) return FORGE_ERR_UNSUPPORTED;
  return launch_embed(ids, wte, wpe, h, batch, seq, d, vocab, n_pos, pos0, dt,
                      static_cast<hipStream_t>(stream));
}

size_t forge_decoder_block_workspace_bytes(const forge_block_desc* desc, int batch, int q_len,
                                           int kv_cap) {
  if (check_block_desc(desc) != FORGE_OK || batch < 1 || q_len < 1 || kv_cap < q_len) return 0;
  if (!grid_ok(batch, desc->q_heads) || !rows_ok(batch, q_len)) return 0;
  return plan_block(desc, batch, q_len, kv_cap).total;
}

forge_status forge_decoder_block(const forge_block_desc* desc, const void* x_in, void* x_out,
                                 void* k_cache, void* v_cache, int batch, int q_len, int pos0,
                                 int kv_cap, void* workspace, size_t workspace_bytes, void* stream) {
  forge_status st = check_block_desc(desc);
  if (st != FORGE_OK) return st;
  if (!req(x_in) || !req(x_out) || !req(k_cache) || !req(v_cache) || !req(workspace))
    return FORGE_ERR_INVALID_ARG;
  if (batch < 1 || !span_ok(pos0, q_len, kv_cap)) return FORGE_ERR_INVALID_ARG;
  if (!grid_ok(batch, desc->q_heads) || !rows_ok(batch, q_len)) return FORGE_ERR_UNSUPPORTED;
  if (workspace_bytes < plan_block(desc, batch, q_len, kv_cap).total) return FORGE_ERR_WORKSPACE;
  return run_block(desc, x_in, x_out, k_cache, v_cache, batch, q_len, pos0, kv_cap, workspace,
                   static_cast<hipStream_t>(stream));
}

size_t forge_model_workspace_bytes(const forge_model_desc* model, int batch, int q_len, int kv_cap) {
  if (check_model(model) != FORGE_OK || batch < 1 || q_len < 1 || kv_cap < q_len) return 0;
  if (!grid_ok(batch, 1) || !rows_ok(batch, q_len)) return 0;
  return plan_model(model, batch, q_len, kv_cap).total;
}

static forge_status model_forward(const forge_model_desc* model, const void* input, void* output,
                                  void* k_cache, void* v_cache, int batch, int q_len, int pos0,
                                  int kv_cap, void* workspace, size_t workspace_bytes, void* stream,
                                  const int* seq_pos) {
  forge_status st = check_model(model);
  if (st != FORGE_OK) return st;
  if (input == nullptr || !req(output) || !req(k_cache) || !req(v_cache) || !req(workspace))
    return FORGE_ERR_INVALID_ARG;
  if (batch < 1 || !span_ok(pos0, q_len, kv_cap)) return FORGE_ERR_INVALID_ARG;
  const bool tokens = model->wte != nullptr;
  if (tokens && !span_ok(pos0, q_len, model->n_pos)) return FORGE_ERR_INVALID_ARG;
  if (!grid_ok(batch, 1) || !rows_ok(batch, q_len)) return FORGE_ERR_UNSUPPORTED;
  if (!tokens && !aligned16(input)) return FORGE_ERR_INVALID_ARG;
  const ModelPlan pl = plan_model(model, batch, q_len, kv_cap);
  if (workspace_bytes < pl.total) return FORGE_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const forge_block_desc* d0 = &model->layers[0];
  const forge_dtype dt = d0->dt;
  const int T = batch * q_len, dm = d0->d_model;
  Carver cv(workspace);
  void* h = cv.take(pl.h);
  void* yf = tokens ? cv.take(pl.yf) : output;
  void* bws = cv.take(pl.block);
  const size_t layer_kv_bytes = (size_t)batch * d0->kv_heads * kv_cap * d0->head_dim * esize(dt);

  const void* x = input;
  if (tokens) {
    st = launch_embed(static_cast<const int32_t*>(input), model->wte, model->wpe, h, batch, q_len,
                      dm, model->vocab, model->n_pos, pos0, dt, s, seq_pos);
    if (st != FORGE_OK) return st;
    trace_mark(s, FORGE_OP_EMBED);
    x = h;
  }
  // decode-sized steps: every norm after the first rides on the reduce step of the projection
  // before it (one launch less per layer, and the norm sees the fp32 sum before it is rounded)
  const bool chain = gemm_fuses_tail(T, dm, dt);
  for (int l = 0; l < model->n_layers; ++l) {
    NormTail nt;
    if (chain) {
      const forge_block_desc* nx = l + 1 < model->n_layers ? &model->layers[l + 1] : nullptr;
      nt = nx != nullptr ? NormTail{nx->norm1_g, nx->norm1_b, block_norm_rows(bws), nx->eps, nx->norm}
                         : NormTail{model->normf_g, model->normf_b, yf, d0->eps, d0->norm};
    }
    st = run_block(&model->layers[l], x, h, static_cast<char*>(k_cache) + l * layer_kv_bytes,
                   static_cast<char*>(v_cache) + l * layer_kv_bytes, batch, q_len, pos0, kv_cap, bws, s,
                   seq_pos, chain ? &nt : nullptr, chain && l > 0);
    if (st != FORGE_OK) return st;
    x = h;
  }
  if (!chain) {
    st = launch_residual_norm(h, nullptr, model->normf_g, model->normf_b, nullptr, yf, T, dm, d0->eps,
                              d0->norm, dt, s);
    if (st != FORGE_OK) return st;
    trace_mark(s, FORGE_OP_NORM);
  }
  if (!tokens) return FORGE_OK;
  // tied LM head: the token table is the weight of the last projection
  GemmArgs g = {yf, model->wte, nullptr, nullptr, output, T, model->vocab, dm, model->logits_ld, FORGE_ACT_NONE,
                nullptr, nullptr, bws, pl.block};
  st = gemm_dispatch(g, dt, s);
  if (st == FORGE_OK) trace_mark(s, FORGE_OP_GEMM);
  return st;
}

forge_status forge_model_forward(const forge_model_desc* model, const void* input, void* output,
                                 void* k_cache, void* v_cache, int batch, int q_len, int pos0,
                                 int kv_cap, void* workspace, size_t workspace_bytes, void* stream) {
  return model_forward(model, input, output, k_cache, v_cache, batch, q_len, pos0, kv_cap, workspace,
                       workspace_bytes, stream, nullptr);
}

static bool seq_pos_ok(const int32_t* seq_pos) {
  return seq_pos != nullptr && (reinterpret_cast<uintptr_t>(seq_pos) & 3u) == 0;
}

forge_status forge_attn_decode_varlen(const void* q, const void* k, const void* v, void* out,
                                      const int32_t* seq_pos, int batch, int q_heads, int kv_heads,
                                      int max_pos, int head_dim, int64_t kv_batch_stride,
                                      int64_t kv_head_stride, float scale, forge_dtype dt,
                                      void* workspace, size_t workspace_bytes, void* stream) {
  if (!dtype_ok(dt) || !req(q) || !req(k) || !req(v) || !req(out) || !opt(workspace) || !seq_pos_ok(seq_pos))
    return FORGE_ERR_INVALID_ARG;
  if (batch < 1 || q_heads < 1 || kv_heads < 1 || max_pos < 0 || max_pos == INT32_MAX) return FORGE_ERR_INVALID_ARG;
  if (q_heads % kv_heads != 0 || !scale_ok(scale)) return FORGE_ERR_INVALID_ARG;
  if (head_dim != 64 && head_dim != 128) return FORGE_ERR_UNSUPPORTED;
  if (!grid_ok(batch, q_heads)) return FORGE_ERR_UNSUPPORTED;
  const int kv_len = max_pos + 1;
  if (kv_head_stride < (int64_t)kv_len * head_dim || kv_batch_stride < kv_head_stride * kv_heads)
    return FORGE_ERR_INVALID_ARG;
  if (kv_head_stride % 8 != 0 || kv_batch_stride % 8 != 0) return FORGE_ERR_INVALID_ARG;
  if (out == q || out == k || out == v) return FORGE_ERR_INVALID_ARG;
  const size_t need = attn_ws(batch, q_heads, kv_heads, 1, kv_len, head_dim, dt);
  if (need > 0 && (workspace == nullptr || workspace_bytes < need)) return FORGE_ERR_WORKSPACE;
  AttnArgs a = {q, k, v, out, batch, q_heads, kv_heads, 1, kv_len, head_dim,
                kv_batch_stride, kv_head_stride, scale, 1, workspace, workspace_bytes, nullptr, 0, 0, seq_pos};
  return attn_dispatch(a, dt, static_cast<hipStream_t>(stream));
}

forge_status forge_attn_decode_static(const void* q, const void* k, const void* v, void* out, int batch,
                                      int q_heads, int kv_heads, int kv_len, int head_dim,
                                      int64_t kv_batch_stride, int64_t kv_head_stride, float scale,
                                      void* stream) {
  if (!req(q) || !req(k) || !req(v) || !req(out)) return FORGE_ERR_INVALID_ARG;
  if (batch < 1 || q_heads < 1 || kv_heads < 1 || kv_len < 1) return FORGE_ERR_INVALID_ARG;
  if (q_heads % kv_heads != 0 || !scale_ok(scale)) return FORGE_ERR_INVALID_ARG;
  if (head_dim != 64 && head_dim != 128) return FORGE_ERR_UNSUPPORTED;
  if (!grid_ok(batch, q_heads)) return FORGE_ERR_UNSUPPORTED;
  if (kv_head_stride < (int64_t)kv_len * head_dim || kv_batch_stride < kv_head_stride * kv_heads)
    return FORGE_ERR_INVALID_ARG;
  if (kv_head_stride % 8 != 0 || kv_batch_stride % 8 != 0) return FORGE_ERR_INVALID_ARG;
  if (out == q || out == k || out == v) return FORGE_ERR_INVALID_ARG;
  // the partials of this call must fit the fixed array
  if (attn_ws(batch, q_heads, kv_heads, 1, kv_len, head_dim, FORGE_BF16) > attn_decode_static_scratch_bytes())
    return FORGE_ERR_WORKSPACE;
  void* scratch_ptr = nullptr;
  const forge_status st = attn_decode_static_scratch(&scratch_ptr);
  if (st != FORGE_OK) return st;
  AttnArgs a = {q, k, v, out, batch, q_heads, kv_heads, 1, kv_len, head_dim, kv_batch_stride, kv_head_stride,
                scale, 1, scratch_ptr, attn_decode_static_scratch_bytes(), nullptr, 0, 0};
  return attn_dispatch(a, FORGE_BF16, static_cast<hipStream_t>(stream));
}

size_t forge_attn_decode_static_max_bytes(void) { return attn_decode_static_scratch_bytes(); }

forge_status forge_decoder_block_decode(const forge_block_desc* desc, const void* x_in, void* x_out,
                                        void* k_cache, void* v_cache, const int32_t* seq_pos,
                                        int batch, int max_pos, int kv_cap, void* workspace,
                                        size_t workspace_bytes, void* stream) {
  forge_status st = check_block_desc(desc);
  if (st != FORGE_OK) return st;
  if (!req(x_in) || !req(x_out) || !req(k_cache) || !req(v_cache) || !req(workspace) || !seq_pos_ok(seq_pos))
    return FORGE_ERR_INVALID_ARG;
  if (batch < 1 || max_pos < 0 || max_pos >= kv_cap) return FORGE_ERR_INVALID_ARG;
  if (!grid_ok(batch, desc->q_heads)) return FORGE_ERR_UNSUPPORTED;
  if (workspace_bytes < plan_block(desc, batch, 1, kv_cap).total) return FORGE_ERR_WORKSPACE;
  return run_block(desc, x_in, x_out, k_cache, v_cache, batch, 1, max_pos, kv_cap, workspace,
                   static_cast<hipStream_t>(stream), seq_pos);
}

forge_status forge_model_decode(const forge_model_desc* model, const void* input, void* output,
                                void* k_cache, void* v_cache, const int32_t* seq_pos, int batch,
                                int max_pos, int kv_cap, void* workspace, size_t workspace_bytes,
                                void* stream) {
  if (!seq_pos_ok(seq_pos)) return FORGE_ERR_INVALID_ARG;
  return model_forward(model, input, output, k_cache, v_cache, batch, 1, max_pos, kv_cap, workspace,
                       workspace_bytes, stream, seq_pos);
}

}  // extern "C"
