// Fused attention on the vector ALUs (small-shape / full-precision path).  One 64-lane wave owns
// one query row and walks the keys in chunks of 64 with an online softmax: lane j scores key j
// of the chunk, the chunk maximum / sum are wave reductions, and the P.V product is accumulated
// with lane d owning output column d (and d + 64 when dh = 128).  S and P exist only in
// registers.  All arithmetic is fp32; this is the FORGE_F32 attention (operands never rounded)
// and the bf16 path for shapes the matrix-core kernels do not take.
#include "common.hpp"

namespace forge {
namespace {

template <typename T, int DH>
__global__ __launch_bounds__(256) void attn_simple_kernel(
    const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v,
    T* __restrict__ out, int batch, int q_heads, int kv_heads, int q_len, int kv_len,
    int64_t kv_bs, int64_t kv_hs, float scale, int causal, const float* __restrict__ mask,
    int64_t mask_bs, int64_t mask_hs, const int* __restrict__ kv_pos) {
  constexpr int NO = DH / 64;
  __shared__ __attribute__((aligned(16))) float qs[4][DH];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t n_rows = (int64_t)batch * q_heads * q_len;
  const bool active = (int64_t)blockIdx.x * 4 + wave < n_rows;
  // a wave past the end recomputes row 0 and skips the store, so every wave reaches the barrier
  const int64_t row_id = active ? (int64_t)blockIdx.x * 4 + wave : 0;
  const int i = (int)(row_id % q_len);
  const int h = (int)((row_id / q_len) % q_heads);
  const int b = (int)(row_id / ((int64_t)q_len * q_heads));
  const int g = h / (q_heads / kv_heads);
  const T* qrow = q + row_id * DH;
  const T* kb = k + (int64_t)b * kv_bs + (int64_t)g * kv_hs;
  const T* vb = v + (int64_t)b * kv_bs + (int64_t)g * kv_hs;
#pragma unroll
  for (int t = 0; t < NO; ++t) qs[wave][lane + 64 * t] = to_f32<T>(qrow[lane + 64 * t]);
  __syncthreads();

  // per-sequence length (decode step of a generation loop): rows [0, kv_pos[b]] plus the new ones
  if (kv_pos != nullptr) kv_len = min(max(kv_pos[b], 0) + q_len, kv_len);
  const int limit = causal ? i + (kv_len - q_len) + 1 : kv_len;   // keys [0, limit)
  const float* mrow = mask == nullptr ? nullptr : mask + b * mask_bs + h * mask_hs + (int64_t)i * kv_len;
  float m = -1e30f, l = 0.f, acc[NO];      // finite start: a chunk that is masked out entirely stays 0
#pragma unroll
  for (int t = 0; t < NO; ++t) acc[t] = 0.f;

  for (int c0 = 0; c0 < limit; c0 += 64) {
    const int j = c0 + lane;
    float s = -INFINITY;
    if (j < limit) {
      const T* kr = kb + (int64_t)j * DH;
      float d = 0.f;
#pragma unroll
      for (int e = 0; e < DH; e += 8) {
        float kv[8];
        Vec8<T>::load(kr + e, kv);
#pragma unroll
        for (int u = 0; u < 8; ++u) d += kv[u] * qs[wave][e + u];
      }
      s = d * scale;
      if (mrow != nullptr) s += mrow[j];
    }
    const float m_new = fmaxf(m, wave_max(s));
    const float p = __expf(s - m_new);        // exp(-inf) = 0 for lanes past the limit
    const float corr = __expf(m - m_new);     // first chunk: exp(-1e30 - m_new) = 0
    l = l * corr + wave_sum(p);
#pragma unroll
    for (int t = 0; t < NO; ++t) acc[t] *= corr;
    const int nk = min(64, limit - c0);
    for (int jj = 0; jj < nk; ++jj) {
      const float pj = __shfl(p, jj, 64);
      const T* vr = vb + (int64_t)(c0 + jj) * DH;
#pragma unroll
      for (int t = 0; t < NO; ++t) acc[t] += pj * to_f32<T>(vr[lane + 64 * t]);
    }
    m = m_new;
  }
  if (!active) return;
  const float inv = 1.0f / l;
  T* orow = out + ((int64_t)b * q_len + i) * ((int64_t)q_heads * DH) + (int64_t)h * DH;
#pragma unroll
  for (int t = 0; t < NO; ++t) orow[lane + 64 * t] = from_f32<T>(acc[t] * inv);
}

template <typename T>
forge_status launch_t(const AttnArgs& a, hipStream_t s) {
  const int64_t n_rows = (int64_t)a.batch * a.q_heads * a.q_len;
  dim3 grid((unsigned)ceil_div64(n_rows, 4)), block(256);
  if (a.head_dim == 64)
    attn_simple_kernel<T, 64><<<grid, block, 0, s>>>(
        (const T*)a.q, (const T*)a.k, (const T*)a.v, (T*)a.out, a.batch, a.q_heads, a.kv_heads,
        a.q_len, a.kv_len, a.kv_batch_stride, a.kv_head_stride, a.scale, a.causal, a.mask,
        a.mask_batch_stride, a.mask_head_stride, a.kv_pos);
  else if (a.head_dim == 128)
    attn_simple_kernel<T, 128><<<grid, block, 0, s>>>(
        (const T*)a.q, (const T*)a.k, (const T*)a.v, (T*)a.out, a.batch, a.q_heads, a.kv_heads,
        a.q_len, a.kv_len, a.kv_batch_stride, a.kv_head_stride, a.scale, a.causal, a.mask,
        a.mask_batch_stride, a.mask_head_stride, a.kv_pos);
  else
    return FORGE_ERR_UNSUPPORTED;
  return launch_status();
}

}  // namespace

forge_status launch_attn_f32(const AttnArgs& a, hipStream_t s) {
  // a prompt goes to the matrix-core kernel; single queries, masks and per-sequence lengths stay here
  if (a.mask == nullptr && a.kv_pos == nullptr && a.q_len >= 16) return launch_attn_f32_mfma(a, s);
  return launch_t<float>(a, s);
}
forge_status launch_attn_simple_bf16(const AttnArgs& a, hipStream_t s) { return launch_t<bf16>(a, s); }

}  // namespace forge
