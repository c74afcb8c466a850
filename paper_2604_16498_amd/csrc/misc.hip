// Rotary position embedding (in place) and token + position embedding.  Both are HBM-bound
// elementwise kernels with 128-bit accesses.
#include "common.hpp"

namespace forge {
namespace {

// One thread owns 8 consecutive pair indices i0..i0+7 of one sequence row s of one batch
// element and walks over all heads: the angles p * theta_i depend on (s, i) only, so sin/cos
// are evaluated once (in fp64: p * theta reaches thousands of radians, where an fp32 product
// alone would already cost 1e-4 of absolute accuracy) and reused for every head.
template <typename T>
__global__ __launch_bounds__(256) void rope_kernel(T* __restrict__ x, int batch, int heads,
                                                   int n_rows, int head_dim, int64_t batch_stride,
                                                   int64_t head_stride, int row0, int pos0,
                                                   float base) {
  const int half = head_dim / 2;
  const int chunks = half / 8;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t total = (int64_t)batch * n_rows * chunks;
  if (gid >= total) return;
  const int c = (int)(gid % chunks);
  const int s = (int)((gid / chunks) % n_rows);
  const int b = (int)(gid / ((int64_t)chunks * n_rows));
  const double p = (double)(pos0 + s);
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
  T* row = x + (int64_t)b * batch_stride + (int64_t)(row0 + s) * head_dim + c * 8;
  for (int h = 0; h < heads; ++h) {
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
                                                    int batch, int seq, int d, int vocab, int pos0) {
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
  Vec8<T>::load(wpe + (int64_t)(pos0 + s) * d + c * 8, p);
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] += p[i];
  Vec8<T>::store(h + t * d + c * 8, a);
}

}  // namespace

forge_status launch_rope(void* x, int batch, int heads, int n_rows, int head_dim,
                         int64_t batch_stride, int64_t head_stride, int row0, int pos0, float base,
                         forge_dtype dt, hipStream_t s) {
  const int64_t total = (int64_t)batch * n_rows * (head_dim / 16);
  dim3 grid((unsigned)ceil_div64(total, 256)), block(256);
  if (dt == FORGE_BF16)
    rope_kernel<bf16><<<grid, block, 0, s>>>((bf16*)x, batch, heads, n_rows, head_dim, batch_stride,
                                             head_stride, row0, pos0, base);
  else
    rope_kernel<float><<<grid, block, 0, s>>>((float*)x, batch, heads, n_rows, head_dim,
                                              batch_stride, head_stride, row0, pos0, base);
  return launch_status();
}

forge_status launch_embed(const int32_t* ids, const void* wte, const void* wpe, void* h, int batch,
                          int seq, int d, int vocab, int n_pos, int pos0, forge_dtype dt,
                          hipStream_t s) {
  (void)n_pos;
  const int64_t total = (int64_t)batch * seq * (d / 8);
  dim3 grid((unsigned)ceil_div64(total, 256)), block(256);
  if (dt == FORGE_BF16)
    embed_kernel<bf16><<<grid, block, 0, s>>>(ids, (const bf16*)wte, (const bf16*)wpe, (bf16*)h,
                                              batch, seq, d, vocab, pos0);
  else
    embed_kernel<float><<<grid, block, 0, s>>>(ids, (const float*)wte, (const float*)wpe, (float*)h,
                                               batch, seq, d, vocab, pos0);
  return launch_status();
}

}  // namespace forge
