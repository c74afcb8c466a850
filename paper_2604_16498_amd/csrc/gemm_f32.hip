// fp32 fused linear:  y = act(x . w^T + bias) (+ residual), true fp32 operands on the fp32
// matrix cores (v_mfma_f32_32x32x2_f32), so the result stays within fp32 rounding of the
// definition (no reduced-precision operand shortcut).
//
// Tiling: a 256-thread block (4 waves as 2 x 2) owns a 64 x 64 tile of y; each wave owns a
// 32 x 32 accumulator.  K is walked in slabs of 32: the x slab [64,32] and the w slab [64,32]
// (both K-contiguous in memory) are copied to LDS with 128-bit accesses, rows padded to 36
// floats so that eight lanes reading the same column chunk of eight consecutive rows hit
// disjoint banks.  The MFMA contracts two k per issue (lanes 0-31 supply one, lanes 32-63 the
// other); lanes 0-31 walk k = 0..15 of the slab and lanes 32-63 walk k = 16..31, so every
// lane reads four consecutive floats per 128-bit LDS read.  The slabs are prefetched three
// ahead in registers.
//
// Small problems (fewer tiles than CUs -- the 128-token fp32 layer has 24 to 96 of them, and a
// block walks K slab by slab with a barrier each) are split along K over grid.z: raw fp32
// partial sums go to the workspace and a second kernel adds them in split order (fixed order, no
// atomics: bitwise reproducible) and carries the epilogue.
#include "common.hpp"

namespace forge {
namespace {

constexpr int BM = 64, BN = 64, BK = 32, LDK = BK + 4;

__device__ inline void* split_dst(const QkvSplit& sp, int m, int n, size_t esz) {
  const int dh = sp.head_dim;
  const int b = m / sp.q_len, s = m % sp.q_len;
  const int nq = sp.q_heads * dh, nk = sp.kv_heads * dh;
  if (n < nq) {
    const int h = n / dh;
    return (char*)sp.q + ((((int64_t)b * sp.q_heads + h) * sp.q_len + s) * dh + n % dh) * esz;
  }
  const bool is_k = n < nq + nk;
  const int nn = is_k ? n - nq : n - nq - nk;
  const int h = nn / dh;
  char* basep = (char*)(is_k ? sp.k_cache : sp.v_cache);
  return basep + ((((int64_t)b * sp.kv_heads + h) * sp.kv_cap + seq_position(sp.pos, b, sp.pos0) + s) * dh + nn % dh) * esz;
}

template <int ACT, bool SPLIT>
__global__ __launch_bounds__(256) void gemm_f32_kernel(
    const float* __restrict__ x, const float* __restrict__ w, const float* __restrict__ bias,
    const float* residual, float* y, int M, int N, int K, int ldy, QkvSplit sp,
    int k_per_split, float* part) {
  constexpr bool SWIGLU = ACT == FORGE_ACT_SWIGLU;
  constexpr int NB = SWIGLU ? 2 : 1;
  __shared__ __attribute__((aligned(16))) float As[BM][LDK];
  __shared__ __attribute__((aligned(16))) float Bs[NB][BN][LDK];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;

  floatx16 acc[NB];
#pragma unroll
  for (int t = 0; t < NB; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;

  const int lrow = tid >> 3;        // 0..31
  const int lcol = (tid & 7) * 4;   // 0,4,..,28

  const int k_begin = blockIdx.z * k_per_split;           // multiple of BK
  const int k_end = min(K, k_begin + k_per_split);

  // Register prefetch, PF slabs ahead: a block of a small problem walks only a few slabs, and
  // with load -> LDS -> barrier -> multiply in sequence every slab would pay the full memory
  // latency.  Loads are unconditional from clamped (valid) addresses so that they stay
  // asynchronous; what lies outside the matrix is zeroed when the slab is written to LDS.
  constexpr int PF = 3;
  floatx4 va[PF][2], vb[PF][NB][2];
  const float* xrow[2];
  const float* wrow[NB][2];
  bool rowa_ok[2], rowb_ok[2];
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    const int row = lrow + 32 * r;
    rowa_ok[r] = m0 + row < M;
    rowb_ok[r] = n0 + row < N;
    xrow[r] = x + (int64_t)min(m0 + row, M - 1) * K;
#pragma unroll
    for (int t = 0; t < NB; ++t) wrow[t][r] = w + (int64_t)(min(n0 + row, N - 1) + t * N) * K;
  }
  auto gload = [&](int k0, int slot) {
    const int kk = min(k0 + lcol, K - 4);
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      va[slot][r] = *reinterpret_cast<const floatx4*>(xrow[r] + kk);
#pragma unroll
      for (int t = 0; t < NB; ++t) vb[slot][t][r] = *reinterpret_cast<const floatx4*>(wrow[t][r] + kk);
    }
  };
  auto lstore = [&](int k0, int slot) {
    const bool k_ok = k0 + lcol < K;
    const floatx4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const int row = lrow + 32 * r;
      *reinterpret_cast<floatx4*>(&As[row][lcol]) = rowa_ok[r] && k_ok ? va[slot][r] : zero;
#pragma unroll
      for (int t = 0; t < NB; ++t)
        *reinterpret_cast<floatx4*>(&Bs[t][row][lcol]) = rowb_ok[r] && k_ok ? vb[slot][t][r] : zero;
    }
  };
#pragma unroll
  for (int d = 0; d < PF; ++d) gload(k_begin + d * BK, d);
  for (int kb = k_begin; kb < k_end; kb += PF * BK) {
#pragma unroll
    for (int d = 0; d < PF; ++d) {
      const int k0 = kb + d * BK;
      if (k0 < k_end) {                       // block-uniform
        lstore(k0, d);
        __syncthreads();
        const int r = lane & 31, hk = (lane >> 5) * 16;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const floatx4 a = *reinterpret_cast<const floatx4*>(&As[wm * 32 + r][hk + 4 * j]);
          floatx4 b[NB];
#pragma unroll
          for (int t = 0; t < NB; ++t) b[t] = *reinterpret_cast<const floatx4*>(&Bs[t][wn * 32 + r][hk + 4 * j]);
#pragma unroll
          for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int t = 0; t < NB; ++t)
              acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[e], b[t][e], acc[t], 0, 0, 0);
        }
        __syncthreads();
      }
      gload(k0 + PF * BK, d);                 // slab k0 + PF slabs into the registers just consumed
    }
  }

  const int n = n0 + wn * 32 + (lane & 31);
  if (n >= N) return;
  if (part != nullptr) {       // split-K: raw partial sums [split, M, NB * N]; the reduce kernel does the rest
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int m = m0 + wm * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      if (m >= M) continue;
      float* dst = part + ((int64_t)blockIdx.z * M + m) * (NB * N) + n;
      dst[0] = acc[0][v];
      if (SWIGLU) dst[N] = acc[NB - 1][v];
    }
    return;
  }
  // epilogue on the accumulator: + bias, activation, + residual, store
  float bv = 0.f, bv2 = 0.f;
  if (bias != nullptr) {
    bv = bias[n];
    if (SWIGLU) bv2 = bias[n + N];
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int m = m0 + wm * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
    if (m >= M) continue;
    float val = acc[0][v] + bv;
    if (SWIGLU) val = silu_f(val) * (acc[NB - 1][v] + bv2);
    else val = apply_act<ACT>(val);
    if (SPLIT) {
      *reinterpret_cast<float*>(split_dst(sp, m, n, sizeof(float))) = val;
    } else {
      if (residual != nullptr) val += residual[(int64_t)m * ldy + n];
      y[(int64_t)m * ldy + n] = val;
    }
  }
}

// Second stage of the split: one thread per output element.
template <int ACT, bool SPLIT>
__global__ __launch_bounds__(256) void gemm_f32_reduce_kernel(
    const float* __restrict__ part, const float* __restrict__ bias, const float* residual, float* y,
    int M, int N, int ldy, int splits, QkvSplit sp) {
  constexpr bool SWIGLU = ACT == FORGE_ACT_SWIGLU;
  const int ncols = SWIGLU ? 2 * N : N;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (int64_t)M * N) return;
  const int m = (int)(gid / N), n = (int)(gid % N);
  const int64_t plane = (int64_t)M * ncols;
  const float* src = part + (int64_t)m * ncols + n;
  float a = 0.f, u = 0.f;
  for (int z = 0; z < splits; ++z) {
    a += src[z * plane];
    if (SWIGLU) u += src[z * plane + N];
  }
  if (bias != nullptr) {
    a += bias[n];
    if (SWIGLU) u += bias[n + N];
  }
  float val = SWIGLU ? silu_f(a) * u : apply_act<ACT>(a);
  if (SPLIT) {
    *reinterpret_cast<float*>(split_dst(sp, m, n, sizeof(float))) = val;
  } else {
    if (residual != nullptr) val += residual[(int64_t)m * ldy + n];
    y[(int64_t)m * ldy + n] = val;
  }
}

// k ranges for a problem: none while the tiles fill the chip; otherwise towards two blocks per
// CU, each with at least four slabs.
struct SplitPlan { int splits, k_per_split; };
SplitPlan plan_split(int M, int N, int K) {
  const int tiles = ceil_div(M, BM) * ceil_div(N, BN);
  const int slabs = ceil_div(K, BK);
  int want = tiles >= 256 ? 1 : min(ceil_div(256, tiles), slabs / 4);
  want = max(1, want);
  const int per = ceil_div(slabs, want);
  return SplitPlan{ceil_div(slabs, per), per * BK};
}

}  // namespace

size_t gemm_f32_workspace_bytes(int M, int N, int K, forge_act act) {
  const SplitPlan sp = plan_split(M, N, K);
  if (sp.splits == 1) return 0;
  return (size_t)sp.splits * M * (act == FORGE_ACT_SWIGLU ? 2 * N : N) * sizeof(float);
}

forge_status launch_gemm_f32(const GemmArgs& a, hipStream_t s) {
  SplitPlan pl = plan_split(a.M, a.N, a.K);
  const size_t need = gemm_f32_workspace_bytes(a.M, a.N, a.K, a.act);
  if (need > a.workspace_bytes || (need > 0 && a.workspace == nullptr)) pl = SplitPlan{1, a.K};   // unsplit
  float* part = pl.splits > 1 ? (float*)a.workspace : nullptr;
  dim3 grid(ceil_div(a.N, BN), ceil_div(a.M, BM), pl.splits), block(256);
  const unsigned rblocks = (unsigned)ceil_div64((int64_t)a.M * a.N, 256);
  const float* x = (const float*)a.x;
  const float* w = (const float*)a.w;
  const float* bias = (const float*)a.bias;
  const float* res = (const float*)a.residual;
  float* y = (float*)a.y;
  QkvSplit sp = {};
  const int ldy = a.ldy > 0 ? a.ldy : a.N;
  if (a.split != nullptr) {
    if (a.act != FORGE_ACT_NONE || a.residual != nullptr) return FORGE_ERR_UNSUPPORTED;
    sp = *a.split;
    gemm_f32_kernel<FORGE_ACT_NONE, true><<<grid, block, 0, s>>>(x, w, bias, res, y, a.M, a.N, a.K, ldy, sp,
                                                                 pl.k_per_split, part);
    if (part != nullptr)
      gemm_f32_reduce_kernel<FORGE_ACT_NONE, true><<<rblocks, 256, 0, s>>>(part, bias, res, y, a.M, a.N, ldy, pl.splits, sp);
    return launch_status();
  }
  switch (a.act) {
#define FORGE_CASE(ACT)                                                                                        \
  case ACT:                                                                                                    \
    gemm_f32_kernel<ACT, false><<<grid, block, 0, s>>>(x, w, bias, res, y, a.M, a.N, a.K, ldy, sp,             \
                                                       pl.k_per_split, part);                                  \
    if (part != nullptr)                                                                                       \
      gemm_f32_reduce_kernel<ACT, false><<<rblocks, 256, 0, s>>>(part, bias, res, y, a.M, a.N, ldy, pl.splits, sp); \
    break
    FORGE_CASE(FORGE_ACT_NONE);
    FORGE_CASE(FORGE_ACT_GELU_TANH);
    FORGE_CASE(FORGE_ACT_RELU);
    FORGE_CASE(FORGE_ACT_SILU);
    FORGE_CASE(FORGE_ACT_SWIGLU);
    FORGE_CASE(FORGE_ACT_GELU_ERF);
#undef FORGE_CASE
    default: return FORGE_ERR_INVALID_ARG;
  }
  return launch_status();
}

}  // namespace forge
