// bf16 fused linear on the gfx950 matrix cores:  y = act(x . w^T + bias) (+ residual).
//
// x [M,K] and w [N,K] are both K-contiguous, which is exactly what v_mfma_f32_32x32x16_bf16
// wants: each lane feeds 8 consecutive k of one row of either operand (one 128-bit read), so no
// operand is ever transposed.  Accumulation is fp32; bias, activation and the residual are
// applied to the accumulator and the result is rounded to bf16 once, at the store.
//
// Tiling (template parameters): a block of WM x WN waves owns a BM x BN tile of y; each wave
// owns (BM/WM) x (BN/WN) as TM x TN accumulators of 32 x 32.  K is walked in slabs of 64.  The
// x and w slabs go HBM -> registers -> LDS with 128-bit accesses, double buffered: the loads of
// slab k+1 are issued before the MFMAs of slab k and stored to the other LDS buffer after them
// (one barrier per slab).
//
// LDS layout: a slab row is 64 bf16 = 8 chunks of 16 B; chunk c of row r is stored at chunk
// position c ^ ((r >> 1) & 7).  A fragment read has lanes 0-31 on 32 consecutive rows at one
// logical chunk; with the swizzle any 16 consecutive rows hit 16 distinct 16-byte bank groups
// (two rows fill the 64 x 4 B banks), so 128-bit reads are conflict free.
//
// SwiGLU: the w slab of a block is half gate rows and half up rows of the SAME output columns,
// arranged so that accumulator (tm, t) is the gate and (tm, t + TN/2) the up projection of one
// column block; the epilogue writes silu(gate) * up and no extra accumulators are needed.
//
// Work-group order: blocks are dealt round-robin over the 8 XCDs (each with its own L2), so the
// block id is first remapped to give every XCD one contiguous run of tiles, and tiles are
// numbered in groups of GROUP_M tile rows, column-major inside a group, so that the tiles
// resident in one XCD at a time share x and w panels in that L2.
#include "common.hpp"

namespace forge {
namespace {

constexpr int BK = 64;            // k per slab
constexpr int CHUNKS = BK / 8;    // 16-byte chunks per slab row

__device__ inline int lds_chunk_off(int r, int c) { return (r * CHUNKS + (c ^ ((r >> 1) & 7))) * 16; }

__device__ inline bf16* split_dst_bf16(const QkvSplit& sp, int m, int n) {
  const int dh = sp.head_dim;
  const int b = m / sp.q_len, s = m % sp.q_len;
  const int nq = sp.q_heads * dh, nk = sp.kv_heads * dh;
  if (n < nq) {
    const int h = n / dh;
    return (bf16*)sp.q + (((int64_t)b * sp.q_heads + h) * sp.q_len + s) * dh + n % dh;
  }
  const bool is_k = n < nq + nk;
  const int nn = is_k ? n - nq : n - nq - nk;
  const int h = nn / dh;
  bf16* basep = (bf16*)(is_k ? sp.k_cache : sp.v_cache);
  return basep + (((int64_t)b * sp.kv_heads + h) * sp.kv_cap + sp.pos0 + s) * dh + nn % dh;
}

struct GemmParams {
  const bf16* x;
  const bf16* w;
  const bf16* bias;
  const bf16* residual;
  bf16* y;
  int M, N, K;        // N: output columns
  int tiles_m, tiles_n;
  int k_per_split;    // split-K: k range of one block (multiple of 64); otherwise >= K
  float* part;        // split-K: fp32 partial sums [splits, M, N]
  QkvSplit sp;
};

enum Mode { MODE_PLAIN = 0, MODE_QKV = 1, MODE_SPLITK = 2 };

template <int BM, int BN, int WM, int WN, int ACT, int MODE>
__global__ __launch_bounds__(WM* WN * 64) void gemm_bf16_kernel(GemmParams p) {
  constexpr int NT = WM * WN * 64;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr bool SWIGLU = ACT == FORGE_ACT_SWIGLU;
  constexpr int BN_OUT = SWIGLU ? BN / 2 : BN;      // output columns per block
  constexpr int LA = BM * CHUNKS / NT, LB = BN * CHUNKS / NT;
  static_assert(BM * CHUNKS % NT == 0 && BN * CHUNKS % NT == 0, "tile / thread mismatch");
  static_assert(!SWIGLU || TN % 2 == 0, "SwiGLU pairs accumulators");
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  // [A0 | B0 | A1 | B1]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

  // ---- tile of this block: XCD-contiguous runs, grouped tile order --------------------------
  int tile;
  {
    const int pid = blockIdx.x, nwg = gridDim.x;   // grid.y indexes the k split
    const int xcd = pid & 7, idx = pid >> 3;
    const int per = nwg >> 3, rem = nwg & 7;
    tile = xcd * per + min(xcd, rem) + idx;
  }
  constexpr int GROUP_M = 8;
  const int in_group = GROUP_M * p.tiles_n;
  const int group = tile / in_group;
  const int first_m = group * GROUP_M;
  const int gsz = min(p.tiles_m - first_m, GROUP_M);
  const int tile_m = first_m + (tile % in_group) % gsz;
  const int tile_n = (tile % in_group) / gsz;
  const int m0 = tile_m * BM, n0 = tile_n * BN_OUT;

  const int M = p.M, N = p.N, K = p.K;

  // ---- per-thread global source rows for the slab copies -----------------------------------
  const bf16* a_src[LA];
  const bf16* b_src[LB];
  int a_lds[LA], b_lds[LB];
  const int c_ld = tid % CHUNKS;
#pragma unroll
  for (int i = 0; i < LA; ++i) {
    const int r = (tid + i * NT) / CHUNKS;
    const int gm = min(m0 + r, M - 1);            // rows past the end re-read the last row
    a_src[i] = p.x + (int64_t)gm * K + c_ld * 8;
    a_lds[i] = lds_chunk_off(r, c_ld);
  }
#pragma unroll
  for (int i = 0; i < LB; ++i) {
    const int r = (tid + i * NT) / CHUNKS;
    int gn;
    if (SWIGLU) {
      // LDS row r = (wave column, accumulator t, row in tile): first TN/2 accumulators gate, rest up
      const int wcol = r / (32 * TN), t = (r / 32) % TN, rr = r % 32;
      const int col = n0 + (wcol * (TN / 2) + t % (TN / 2)) * 32 + rr;
      gn = min(col, N - 1) + (t >= TN / 2 ? N : 0);
    } else {
      gn = min(n0 + r, N - 1);
    }
    b_src[i] = p.w + (int64_t)gn * K + c_ld * 8;
    b_lds[i] = lds_chunk_off(r, c_ld);
  }

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  u32x4 ra[LA], rb[LB];
  auto load_slab = [&](int k0) {
    const bool ok = k0 + c_ld * 8 < K;            // K % 8 == 0: a chunk is all in or all out
#pragma unroll
    for (int i = 0; i < LA; ++i)
      ra[i] = ok ? *reinterpret_cast<const u32x4*>(a_src[i] + k0) : u32x4{0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < LB; ++i)
      rb[i] = ok ? *reinterpret_cast<const u32x4*>(b_src[i] + k0) : u32x4{0, 0, 0, 0};
  };
  auto store_slab = [&](int buf) {
    char* sa = smem + buf * (A_BYTES + B_BYTES);
    char* sb = sa + A_BYTES;
#pragma unroll
    for (int i = 0; i < LA; ++i) *reinterpret_cast<u32x4*>(sa + a_lds[i]) = ra[i];
#pragma unroll
    for (int i = 0; i < LB; ++i) *reinterpret_cast<u32x4*>(sb + b_lds[i]) = rb[i];
  };

  const int fr = lane & 31, fh = lane >> 5;
  auto compute_slab = [&](int buf) {
    const char* sa = smem + buf * (A_BYTES + B_BYTES);
    const char* sb = sa + A_BYTES;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        fa[i] = *reinterpret_cast<const bf16x8*>(sa + lds_chunk_off((wm * TM + i) * 32 + fr, 2 * ks + fh));
#pragma unroll
      for (int j = 0; j < TN; ++j)
        fb[j] = *reinterpret_cast<const bf16x8*>(sb + lds_chunk_off((wn * TN + j) * 32 + fr, 2 * ks + fh));
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  };

  const int k_begin = MODE == MODE_SPLITK ? blockIdx.y * p.k_per_split : 0;
  const int k_end = MODE == MODE_SPLITK ? min(K, k_begin + p.k_per_split) : K;
  const int nk = ceil_div(k_end - k_begin, BK);
  load_slab(k_begin);
  store_slab(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const bool more = kt + 1 < nk;
    if (more) load_slab(k_begin + (kt + 1) * BK);
    compute_slab(kt & 1);
    if (more) store_slab((kt + 1) & 1);
    __syncthreads();
  }

  // ---- epilogue -------------------------------------------------------------------------------
  // accumulator (i, j): lane holds column n = .. + (lane & 31) and rows 8*(v/4) + 4*(lane>>5) + v%4
  constexpr int TN_OUT = SWIGLU ? TN / 2 : TN;
#pragma unroll
  for (int j = 0; j < TN_OUT; ++j) {
    const int n = n0 + (wn * TN_OUT + j) * 32 + fr;
    if (n >= N) continue;
    float bv = 0.f, bv2 = 0.f;
    if (p.bias != nullptr) {
      bv = (float)p.bias[n];
      if (SWIGLU) bv2 = (float)p.bias[n + N];
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = m0 + (wm * TM + i) * 32 + 8 * (v >> 2) + 4 * fh + (v & 3);
        if (m >= M) continue;
        if (MODE == MODE_SPLITK) {   // raw partial sum; bias / activation happen in the reduce
          p.part[((int64_t)blockIdx.y * M + m) * N + n] = acc[i][j][v];
          continue;
        }
        float val = acc[i][j][v] + bv;
        if (SWIGLU) val = silu_f(val) * (acc[i][SWIGLU ? j + TN / 2 : j][v] + bv2);
        else val = apply_act<ACT>(val);
        if (MODE == MODE_QKV) {
          *split_dst_bf16(p.sp, m, n) = (bf16)val;
        } else {
          if (p.residual != nullptr) val += (float)p.residual[(int64_t)m * N + n];
          p.y[(int64_t)m * N + n] = (bf16)val;
        }
      }
    }
  }
}

// Split-K second stage: sums the fp32 partials of one output element in split order (fixed
// order, no atomics), then applies the same epilogue as the single-pass kernel.  One thread
// owns 4 consecutive columns.  For SwiGLU the partials hold 2N columns: gate n and up n + N.
template <int ACT, bool QKV>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(GemmParams p, int splits, int ncols) {
  constexpr bool SWIGLU = ACT == FORGE_ACT_SWIGLU;
  const int N = p.N;                        // output columns
  const int groups = ceil_div(N, 4);
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (int64_t)p.M * groups) return;
  const int m = (int)(gid / groups), n0 = (int)(gid % groups) * 4;
  const int64_t plane = (int64_t)p.M * ncols;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int n = n0 + e;
    if (n >= N) break;
    float a = 0.f, u = 0.f;
    for (int z = 0; z < splits; ++z) {
      a += p.part[z * plane + (int64_t)m * ncols + n];
      if (SWIGLU) u += p.part[z * plane + (int64_t)m * ncols + n + N];
    }
    if (p.bias != nullptr) {
      a += (float)p.bias[n];
      if (SWIGLU) u += (float)p.bias[n + N];
    }
    float val = SWIGLU ? silu_f(a) * u : apply_act<ACT>(a);
    if (QKV) {
      *split_dst_bf16(p.sp, m, n) = (bf16)val;
    } else {
      if (p.residual != nullptr) val += (float)p.residual[(int64_t)m * N + n];
      p.y[(int64_t)m * N + n] = (bf16)val;
    }
  }
}

template <int BM, int BN, int WM, int WN, int ACT, int MODE>
forge_status launch_cfg(const GemmParams& p0, int splits, hipStream_t s) {
  GemmParams p = p0;
  constexpr int BN_OUT = ACT == FORGE_ACT_SWIGLU ? BN / 2 : BN;
  p.tiles_m = ceil_div(p.M, BM);
  p.tiles_n = ceil_div(p.N, BN_OUT);
  constexpr int smem = 2 * (BM + BN) * BK * 2;
  auto kern = gemm_bf16_kernel<BM, BN, WM, WN, ACT, MODE>;
  static bool configured = false;   // idempotent attribute, set once per instantiation
  if (!configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
      return FORGE_ERR_HIP;
    configured = true;
  }
  dim3 grid(p.tiles_m * p.tiles_n, splits), block(WM * WN * 64);
  kern<<<grid, block, smem, s>>>(p);
  return launch_status();
}

// tile choice: big tiles when they still give every CU work, smaller ones otherwise; problems
// with at most 64 rows (decode) stream the weight once and are split over K to fill the chip
enum Variant { V_256x256 = 0, V_128x128 = 1, V_SKINNY = 2 };
inline Variant choose_variant(int M, int N, int K, forge_act act) {
  (void)K;
  if (M <= 64) return V_SKINNY;
  const int64_t big = (int64_t)ceil_div(M, 256) * ceil_div(N, act == FORGE_ACT_SWIGLU ? 128 : 256);
  return big >= 512 ? V_256x256 : V_128x128;
}

struct SkinnyPlan {
  int ncols;        // columns of the partial planes (2N for SwiGLU)
  int splits;
  int k_per_split;
};
inline SkinnyPlan plan_skinny(int N, int K, forge_act act) {
  SkinnyPlan sp;
  sp.ncols = act == FORGE_ACT_SWIGLU ? 2 * N : N;
  const int tiles = ceil_div(sp.ncols, 64);
  const int slabs = ceil_div(K, BK);
  int want = ceil_div(512, tiles);                 // aim at >= 512 blocks
  want = max(1, min(want, slabs / 4));             // but at least 4 slabs of work per block
  const int per = ceil_div(slabs, want);
  sp.splits = ceil_div(slabs, per);
  sp.k_per_split = per * BK;
  return sp;
}

template <int ACT, int MODE>
forge_status launch_act(const GemmParams& p, hipStream_t s) {
  switch (choose_variant(p.M, p.N, p.K, (forge_act)ACT)) {
    case V_256x256: return launch_cfg<256, 256, 2, 4, ACT, MODE>(p, 1, s);
    case V_128x128: return launch_cfg<128, 128, 2, 2, ACT, MODE>(p, 1, s);
    default: break;
  }
  // skinny: raw split-K GEMM over all weight rows into fp32 partials, then reduce + epilogue
  const SkinnyPlan sk = plan_skinny(p.N, p.K, (forge_act)ACT);
  GemmParams q = p;
  q.N = sk.ncols;
  q.k_per_split = sk.k_per_split;
  forge_status st = launch_cfg<64, 64, 2, 2, FORGE_ACT_NONE, MODE_SPLITK>(q, sk.splits, s);
  if (st != FORGE_OK) return st;
  GemmParams r = p;
  const int64_t threads = (int64_t)p.M * ceil_div(p.N, 4);
  splitk_reduce_kernel<ACT, MODE == MODE_QKV><<<(unsigned)ceil_div64(threads, 256), 256, 0, s>>>(r, sk.splits, sk.ncols);
  return launch_status();
}

}  // namespace

size_t gemm_bf16_workspace_bytes(int M, int N, int K, forge_act act) {
  if (choose_variant(M, N, K, act) != V_SKINNY) return 0;
  const SkinnyPlan sk = plan_skinny(N, K, act);
  return (size_t)sk.splits * M * sk.ncols * sizeof(float);
}

const char* gemm_bf16_variant(int M, int N, int K, forge_act act) {
  switch (choose_variant(M, N, K, act)) {
    case V_256x256: return "gemm_bf16<256,256,2,4>";
    case V_128x128: return "gemm_bf16<128,128,2,2>";
    default: return "gemm_bf16<64,64,2,2>+splitk";
  }
}

forge_status launch_gemm_bf16(const GemmArgs& a, hipStream_t s) {
  GemmParams p = {};
  p.x = (const bf16*)a.x;
  p.w = (const bf16*)a.w;
  p.bias = (const bf16*)a.bias;
  p.residual = (const bf16*)a.residual;
  p.y = (bf16*)a.y;
  p.M = a.M;
  p.N = a.N;
  p.K = a.K;
  p.k_per_split = a.K;
  p.part = (float*)a.workspace;
  if (gemm_bf16_workspace_bytes(a.M, a.N, a.K, a.act) > a.workspace_bytes ||
      (gemm_bf16_workspace_bytes(a.M, a.N, a.K, a.act) > 0 && a.workspace == nullptr))
    return FORGE_ERR_WORKSPACE;
  if (a.split != nullptr) {
    if (a.act != FORGE_ACT_NONE || a.residual != nullptr) return FORGE_ERR_UNSUPPORTED;
    p.sp = *a.split;
    return launch_act<FORGE_ACT_NONE, MODE_QKV>(p, s);
  }
  switch (a.act) {
    case FORGE_ACT_NONE: return launch_act<FORGE_ACT_NONE, MODE_PLAIN>(p, s);
    case FORGE_ACT_GELU_TANH: return launch_act<FORGE_ACT_GELU_TANH, MODE_PLAIN>(p, s);
    case FORGE_ACT_RELU: return launch_act<FORGE_ACT_RELU, MODE_PLAIN>(p, s);
    case FORGE_ACT_SILU: return launch_act<FORGE_ACT_SILU, MODE_PLAIN>(p, s);
    case FORGE_ACT_SWIGLU: return launch_act<FORGE_ACT_SWIGLU, MODE_PLAIN>(p, s);
    default: return FORGE_ERR_INVALID_ARG;
  }
}

}  // namespace forge
