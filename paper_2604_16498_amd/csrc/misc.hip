// Rotary position embedding (in place), token + position embedding, the one-time int8
// quantisation of a weight and the one-time re-layout of an interleaved gated weight.  HBM-bound
// elementwise kernels.
#include "api_internal.hpp"

namespace forge {
namespace {

// One thread owns 8 consecutive pair indices i0..i0+7 of one sequence row s of one batch
// element and walks over a GROUP of heads: the angles p * theta_i depend on (s, i) only, so sin/cos
// are evaluated once per thread (in fp64: p * theta reaches thousands of radians, where an fp32
// product alone would already cost 1e-4 of absolute accuracy) and reused for every head of the
// group.  The launcher picks the number of head groups so that short inputs (a decode step has
// one row per sequence) still fill the chip, while long ones amortise the sin/cos over many heads.
template <typename T>
__global__ __launch_bounds__(256) void rope_kernel(T* __restrict__ x, int batch, int heads,
                                                   int n_rows, int head_dim, int64_t batch_stride,
                                                   int64_t head_stride, int row0, int pos0,
                                                   float base, int head_groups,
                                                   const int* __restrict__ pos, int rows_at_pos) {
  const int half = head_dim / 2;
  const int chunks = half / 8;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t total = (int64_t)batch * n_rows * chunks * head_groups;
  if (gid >= total) return;
  const int c = (int)(gid % chunks);
  const int hg = (int)((gid / chunks) % head_groups);
  const int s = (int)((gid / ((int64_t)chunks * head_groups)) % n_rows);
  const int b = (int)(gid / ((int64_t)chunks * head_groups * n_rows));
  const int per = ceil_div(heads, head_groups);
  const int h0 = hg * per, h1 = min(heads, h0 + per);
  const int pb = seq_position(pos, b, pos0);    // position of this sequence's first new row
  const double p = (double)(pb + s);
  const double l2b = log2((double)base);
  float cs[8], sn[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const double theta = exp2(-2.0 * (double)(c * 8 + i) / (double)head_dim * l2b);
    double sv, cv;
    sincos(p * theta, &sv, &cv);
    cs[i] = (float)cv;
    sn[i] = (float)sv;
  }
  T* row = x + (int64_t)b * batch_stride + (int64_t)((rows_at_pos ? pb : row0) + s) * head_dim + c * 8;
  for (int h = h0; h < h1; ++h) {
    T* p1 = row + (int64_t)h * head_stride;
    T* p2 = p1 + half;
    float a[8], d[8], oa[8], od[8];
    Vec8<T>::load(p1, a);
    Vec8<T>::load(p2, d);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      oa[i] = a[i] * cs[i] - d[i] * sn[i];
      od[i] = d[i] * cs[i] + a[i] * sn[i];
    }
    Vec8<T>::store(p1, oa);
    Vec8<T>::store(p2, od);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void embed_kernel(const int32_t* __restrict__ ids,
                                                    const T* __restrict__ wte,
                                                    const T* __restrict__ wpe, T* __restrict__ h,
                                                    int batch, int seq, int d, int vocab, int pos0,
                                                    const int* __restrict__ pos) {
  const int chunks = d / 8;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (int64_t)batch * seq * chunks) return;
  const int c = (int)(gid % chunks);
  const int64_t t = gid / chunks;
  const int s = (int)(t % seq);
  int id = ids[t];
  id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);
  float a[8], p[8];
  Vec8<T>::load(wte + (int64_t)id * d + c * 8, a);
  Vec8<T>::load(wpe + (int64_t)(seq_position(pos, (int)(t / seq), pos0) + s) * d + c * 8, p);
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] += p[i];
  Vec8<T>::store(h + t * d + c * 8, a);
}

// Symmetric int8 quantisation with one scale per weight row (Sec. "Precision Strategy for
// Llama-3.1-8B": symmetric int8 weights, 16-bit activations).  One block per row: the row maximum
// of |w|, scale = max / 127 and q = rint(w / scale), both as correctly rounded fp32 divisions
// (the precision the integer decision is defined in), clipped to [-127, 127].  A row of zeros
// gets scale 1.
template <typename T>
__global__ __launch_bounds__(256) void quantize_int8_kernel(const T* __restrict__ w, int8_t* __restrict__ q,
                                                            float* __restrict__ scale, int K) {
  __shared__ float red[4];
  const int n = blockIdx.x;
  const T* row = w + (int64_t)n * K;
  float amax = 0.f;
  for (int k = threadIdx.x; k < K; k += 256) amax = fmaxf(amax, fabsf((float)row[k]));
  amax = wave_max(amax);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = amax;
  __syncthreads();
  amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  const float sc = amax > 0.f ? __fdiv_rn(amax, 127.0f) : 1.0f;
  if (threadIdx.x == 0) scale[n] = sc;
  int8_t* out = q + (int64_t)n * K;
  for (int k = threadIdx.x; k < K; k += 256) {
    const float r = rintf(__fdiv_rn((float)row[k], sc));
    out[k] = (int8_t)(int)fminf(fmaxf(r, -127.f), 127.f);
  }
}

// Destination row r < pairs takes source row 2r, destination row pairs + r takes source row
// 2r + 1.  One block per destination row; 16-byte copies when rows and pointers allow.
__global__ __launch_bounds__(256) void deinterleave_rows_kernel(const char* __restrict__ src,
                                                                char* __restrict__ dst, int pairs,
                                                                int64_t row_bytes, int vec) {
  const int r = blockIdx.x;
  const int64_t s = r < pairs ? 2 * (int64_t)r : 2 * (int64_t)(r - pairs) + 1;
  const char* a = src + s * row_bytes;
  char* b = dst + (int64_t)r * row_bytes;
  if (vec) {
    for (int64_t i = (int64_t)threadIdx.x * 16; i < row_bytes; i += 256 * 16)
      *reinterpret_cast<u32x4*>(b + i) = *reinterpret_cast<const u32x4*>(a + i);
  } else {
    for (int64_t i = threadIdx.x; i < row_bytes; i += 256) b[i] = a[i];
  }
}

}  // namespace

forge_status launch_deinterleave_rows(const void* src, void* dst, int pairs, size_t row_bytes, hipStream_t s) {
  const int vec = row_bytes % 16 == 0 && aligned16(src) && aligned16(dst);
  deinterleave_rows_kernel<<<2 * (unsigned)pairs, 256, 0, s>>>((const char*)src, (char*)dst, pairs,
                                                               (int64_t)row_bytes, vec);
  return launch_status();
}

forge_status launch_quantize_int8(const void* w, int8_t* q, float* scale, int N, int K, forge_dtype dt,
                                  hipStream_t s) {
  if (dt == FORGE_BF16)
    quantize_int8_kernel<bf16><<<N, 256, 0, s>>>((const bf16*)w, q, scale, K);
  else
    quantize_int8_kernel<float><<<N, 256, 0, s>>>((const float*)w, q, scale, K);
  return launch_status();
}

forge_status launch_rope(void* x, int batch, int heads, int n_rows, int head_dim,
                         int64_t batch_stride, int64_t head_stride, int row0, int pos0, float base,
                         forge_dtype dt, hipStream_t s, const int* pos, bool rows_at_pos) {
  const int64_t base_threads = (int64_t)batch * n_rows * (head_dim / 16);
  // enough head groups to reach ~128k threads, at most one group per head
  int head_groups = (int)ceil_div64(131072, base_threads);
  head_groups = head_groups < 1 ? 1 : (head_groups > heads ? heads : head_groups);
  const int64_t total = base_threads * head_groups;
  dim3 grid((unsigned)ceil_div64(total, 256)), block(256);
  if (dt == FORGE_BF16)
    rope_kernel<bf16><<<grid, block, 0, s>>>((bf16*)x, batch, heads, n_rows, head_dim, batch_stride,
                                             head_stride, row0, pos0, base, head_groups, pos, rows_at_pos ? 1 : 0);
  else
    rope_kernel<float><<<grid, block, 0, s>>>((float*)x, batch, heads, n_rows, head_dim,
                                              batch_stride, head_stride, row0, pos0, base, head_groups, pos,
                                              rows_at_pos ? 1 : 0);
  return launch_status();
}

forge_status launch_embed(const int32_t* ids, const void* wte, const void* wpe, void* h, int batch,
                          int seq, int d, int vocab, int n_pos, int pos0, forge_dtype dt,
                          hipStream_t s, const int* pos) {
  (void)n_pos;
  const int64_t total = (int64_t)batch * seq * (d / 8);
  dim3 grid((unsigned)ceil_div64(total, 256)), block(256);
  if (dt == FORGE_BF16)
    embed_kernel<bf16><<<grid, block, 0, s>>>(ids, (const bf16*)wte, (const bf16*)wpe, (bf16*)h,
                                              batch, seq, d, vocab, pos0, pos);
  else
    embed_kernel<float><<<grid, block, 0, s>>>(ids, (const float*)wte, (const float*)wpe, (float*)h,
                                               batch, seq, d, vocab, pos0, pos);
  return launch_status();
}

}  // namespace forge
