// bf16 fused attention for one new query per sequence over a KV cache (decode).  HBM-bound:
// every cached K and V row is read exactly once, with 128-bit loads, and nothing else of
// comparable size moves.
//
// Split-KV: block (split, kv head, batch) streams CHUNK consecutive cache rows of ONE kv head
// for all G = Hq/Hkv query heads that share it (grouped-query attention reads the cache once
// per group, not once per query head).  Each of the 4 waves owns 64 rows.  A cache row of dh
// elements is spread over dh/8 lanes (16 B each), so one wave-wide load covers 64/(dh/8) rows;
// a wave issues ALL its K and V loads first (the whole 64-row slice sits in registers) and then
// computes, so a CU always has tens of KB in flight.
//
// Per row group: partial dot products with packed bf16 dot2 (fp32 accumulate), a DPP butterfly
// over the lanes of a row, online softmax in the exp2 domain with LAZY rescaling (the running
// maximum only moves when some row beats it, which becomes rare after the first rows), and the
// P.V accumulation in fp32 with each lane owning 8 output columns for every query head.
// Lane-group, wave and block partials are merged with a fixed-order log-sum-exp combine; the
// block writes (m, l, o) per query head to the workspace and a second kernel merges the splits
// in split order -- no atomics, so the result is bitwise reproducible.
#include "common.hpp"

namespace forge {
namespace {

constexpr int CHUNK = 256;   // cache rows per block
constexpr int WROWS = 64;    // cache rows per wave

struct DecParams {
  const bf16* q;
  const bf16* k;
  const bf16* v;
  float* part;     // [B, Hkv, splits, G, dh + 2]
  int q_heads, kv_heads, kv_len, splits;
  int64_t kv_bs, kv_hs;
  float scale_log2e;
};

template <int CTRL> __device__ inline float dpp_add(float x) {
  const int t = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false);
  return x + __int_as_float(t);
}
// sum over the LPR (8 or 16) consecutive lanes that hold one cache row; all of them get it
template <int LPR> __device__ inline float row_sum(float x) {
  x = dpp_add<0xB1>(x);    // quad_perm [1,0,3,2]
  x = dpp_add<0x4E>(x);    // quad_perm [2,3,0,1]
  x = dpp_add<0x141>(x);   // row_half_mirror
  if (LPR == 16) x = dpp_add<0x140>(x);   // row_mirror
  return x;
}

template <int DH, int G>
__global__ __launch_bounds__(256) void attn_decode_kernel(DecParams p) {
  constexpr int LPR = DH / 8;          // lanes per cache row
  constexpr int RPI = 64 / LPR;        // rows per wave-wide load
  constexpr int STEPS = WROWS / RPI;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int slot = lane / LPR, c = lane % LPR;
  const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;

  const bf16* kb = p.k + (int64_t)b * p.kv_bs + (int64_t)g * p.kv_hs + c * 8;
  const bf16* vb = p.v + (int64_t)b * p.kv_bs + (int64_t)g * p.kv_hs + c * 8;
  const int row0 = split * CHUNK + wave * WROWS + slot;
  const int row_end = min(p.kv_len, (split + 1) * CHUNK);

  // ---- issue every load of this wave's slice -------------------------------------------------
  u32x4 kr[STEPS], vr[STEPS];
#pragma unroll
  for (int s = 0; s < STEPS; ++s) {
    const int row = min(row0 + s * RPI, p.kv_len - 1);   // rows past the end re-read the last row
    kr[s] = *reinterpret_cast<const u32x4*>(kb + (int64_t)row * DH);
    vr[s] = *reinterpret_cast<const u32x4*>(vb + (int64_t)row * DH);
  }
  // the G query rows, 8 elements per lane, kept packed for dot2
  u32x4 qr[G];
#pragma unroll
  for (int h = 0; h < G; ++h)
    qr[h] = *reinterpret_cast<const u32x4*>(p.q + ((int64_t)b * p.q_heads + g * G + h) * DH + c * 8);

  float m[G], l[G], acc[G][8];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    m[h] = -1e30f;
    l[h] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[h][e] = 0.f;
  }
  const float cl = p.scale_log2e;

#pragma unroll
  for (int s = 0; s < STEPS; ++s) {
    const bool valid = row0 + s * RPI < row_end;
    float sc[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      // whole-vector casts, then element pairs by shuffle (never a cast of a single element)
      const bf16x8 k8 = __builtin_bit_cast(bf16x8, kr[s]);
      const bf16x8 q8 = __builtin_bit_cast(bf16x8, qr[h]);
      float d = 0.f;
      d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(k8, k8, 0, 1), __builtin_shufflevector(q8, q8, 0, 1), d, false);
      d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(k8, k8, 2, 3), __builtin_shufflevector(q8, q8, 2, 3), d, false);
      d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(k8, k8, 4, 5), __builtin_shufflevector(q8, q8, 4, 5), d, false);
      d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(k8, k8, 6, 7), __builtin_shufflevector(q8, q8, 6, 7), d, false);
      d = row_sum<LPR>(d) * cl;
      sc[h] = valid ? d : -INFINITY;
    }
    bool grow = false;
#pragma unroll
    for (int h = 0; h < G; ++h) grow |= sc[h] > m[h];
    if (__any(grow)) {   // wave-uniform: some row raised a running maximum
#pragma unroll
      for (int h = 0; h < G; ++h) {
        const float mn = fmaxf(m[h], sc[h]);
        const float alpha = __builtin_amdgcn_exp2f(m[h] - mn);
        m[h] = mn;
        l[h] *= alpha;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[h][e] *= alpha;
      }
    }
    float vf[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) { vf[2 * e] = bf_lo(vr[s][e]); vf[2 * e + 1] = bf_hi(vr[s][e]); }
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const float pr = __builtin_amdgcn_exp2f(sc[h] - m[h]);   // exp2(-inf) = 0 for rows past the end
      l[h] += pr;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[h][e] += pr * vf[e];
    }
  }

  // ---- merge the RPI lane groups of the wave (xor over the lane bits above the row bits) ------
#pragma unroll
  for (int o = LPR; o < 64; o <<= 1) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const float m2 = __shfl_xor(m[h], o, 64), l2 = __shfl_xor(l[h], o, 64);
      const float mn = fmaxf(m[h], m2);
      const float a1 = __builtin_amdgcn_exp2f(m[h] - mn), a2 = __builtin_amdgcn_exp2f(m2 - mn);
      l[h] = l[h] * a1 + l2 * a2;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[h][e] = acc[h][e] * a1 + __shfl_xor(acc[h][e], o, 64) * a2;
      m[h] = mn;
    }
  }
  // ---- merge the 4 waves through LDS, fixed order ------------------------------------------------
  __shared__ float sm[4][G][DH + 2];
  if (slot == 0) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
#pragma unroll
      for (int e = 0; e < 8; ++e) sm[wave][h][c * 8 + e] = acc[h][e];
      if (c == 0) { sm[wave][h][DH] = m[h]; sm[wave][h][DH + 1] = l[h]; }
    }
  }
  __syncthreads();
  float* dst = p.part + ((((int64_t)b * p.kv_heads + g) * p.splits + split) * G) * (DH + 2);
  for (int idx = tid; idx < G * DH; idx += 256) {
    const int h = idx / DH, d = idx % DH;
    float mn = sm[0][h][DH];
#pragma unroll
    for (int w = 1; w < 4; ++w) mn = fmaxf(mn, sm[w][h][DH]);
    float o = 0.f, lt = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float a = __builtin_amdgcn_exp2f(sm[w][h][DH] - mn);
      o += sm[w][h][d] * a;
      lt += sm[w][h][DH + 1] * a;
    }
    dst[h * (DH + 2) + d] = o;
    if (d == 0) { dst[h * (DH + 2) + DH] = mn; dst[h * (DH + 2) + DH + 1] = lt; }
  }
}

// one block per (batch, query head): merge the splits in order and normalise
template <int DH>
__global__ __launch_bounds__(DH) void attn_decode_combine(const float* __restrict__ part,
                                                          bf16* __restrict__ out, int q_heads,
                                                          int kv_heads, int splits) {
  const int h = blockIdx.x, b = blockIdx.y, d = threadIdx.x;
  const int G = q_heads / kv_heads;
  const int g = h / G, hh = h % G;
  const float* src = part + ((((int64_t)b * kv_heads + g) * splits) * G + hh) * (DH + 2);
  const int64_t stride = (int64_t)G * (DH + 2);
  float mn = -1e30f;
  for (int s = 0; s < splits; ++s) mn = fmaxf(mn, src[s * stride + DH]);
  float o = 0.f, lt = 0.f;
  for (int s = 0; s < splits; ++s) {
    const float a = __builtin_amdgcn_exp2f(src[s * stride + DH] - mn);
    o += src[s * stride + d] * a;
    lt += src[s * stride + DH + 1] * a;
  }
  out[((int64_t)b * q_heads + h) * DH + d] = (bf16)(o / lt);
}

template <int DH, int G>
forge_status launch_dg(const AttnArgs& a, hipStream_t s) {
  DecParams p;
  p.q = (const bf16*)a.q;
  p.k = (const bf16*)a.k;
  p.v = (const bf16*)a.v;
  p.part = (float*)a.workspace;
  p.q_heads = a.q_heads;
  p.kv_heads = a.kv_heads;
  p.kv_len = a.kv_len;
  p.splits = ceil_div(a.kv_len, CHUNK);
  p.kv_bs = a.kv_batch_stride;
  p.kv_hs = a.kv_head_stride;
  p.scale_log2e = a.scale * 1.4426950408889634f;
  attn_decode_kernel<DH, G><<<dim3(p.splits, a.kv_heads, a.batch), 256, 0, s>>>(p);
  if (hipGetLastError() != hipSuccess) return FORGE_ERR_HIP;
  attn_decode_combine<DH><<<dim3(a.q_heads, a.batch), DH, 0, s>>>(p.part, (bf16*)a.out, a.q_heads,
                                                                  a.kv_heads, p.splits);
  return launch_status();
}

template <int DH>
forge_status launch_d(const AttnArgs& a, hipStream_t s) {
  switch (a.q_heads / a.kv_heads) {
    case 1: return launch_dg<DH, 1>(a, s);
    case 2: return launch_dg<DH, 2>(a, s);
    case 4: return launch_dg<DH, 4>(a, s);
    default: return launch_attn_simple_bf16(a, s);   // other group sizes: vector-ALU path
  }
}

}  // namespace

size_t attn_decode_workspace_bytes(int batch, int q_heads, int kv_heads, int kv_len, int head_dim) {
  const int splits = ceil_div(kv_len, CHUNK);
  return (size_t)batch * q_heads * splits * (head_dim + 2) * sizeof(float);
}

forge_status launch_attn_decode_bf16(const AttnArgs& a, hipStream_t s) {
  const size_t need = attn_decode_workspace_bytes(a.batch, a.q_heads, a.kv_heads, a.kv_len, a.head_dim);
  if (a.workspace == nullptr || a.workspace_bytes < need) return FORGE_ERR_WORKSPACE;
  if (a.head_dim == 64) return launch_d<64>(a, s);
  if (a.head_dim == 128) return launch_d<128>(a, s);
  return FORGE_ERR_UNSUPPORTED;
}

}  // namespace forge
