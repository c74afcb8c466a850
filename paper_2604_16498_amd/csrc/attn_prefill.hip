// bf16 fused causal attention for prefill on the gfx950 matrix cores: scores, scale, mask,
// softmax and the product with V in one kernel; S and P live only in registers.
//
// Work split: a 512-thread block (8 waves, one block per CU) owns 256 consecutive queries of one
// (batch, head); each wave owns 32 of them and walks the keys in tiles of 64 up to its diagonal.
//
// Both contractions are computed TRANSPOSED so that the two MFMAs chain without any data
// movement:
//   S^T[key, query] = K . Q^T   : A operand = K rows (LDS, 128-bit reads along dh),
//                                 B operand = Q^T, i.e. each lane's own query row (registers).
//   O^T[d, query]   = V^T . P^T : B operand = P^T, which is exactly the accumulator layout of
//                                 S^T (lane = query, registers = keys) rounded to bf16;
//                                 A operand = V^T, read from the row-major V tile in LDS with
//                                 the transposing LDS read (ds_read_b64_tr_b16: within 16 lanes,
//                                 lane 4q+r receives element r of the 8-byte rows addressed by
//                                 lanes q, q+4, q+8, q+12).
// A lane therefore owns ONE query throughout: its 32 scores per tile sit in its own registers,
// the row maximum needs a single exchange with lane^32 (the other half of the keys), the row
// sum is kept as a per-lane partial and combined once at the end, and the rescale factor of
// the online softmax is a per-lane scalar (applied only when some lane's maximum moved).
//
// The contraction order over keys inside a 16-key MFMA step is permuted (the same permutation
// on both operands, so the sum is unchanged): element e of lane-half h is key
// 16 s + 8 (e / 4) + 4 h + e % 4, which is what the S^T accumulator registers 8 (s % 2) + e hold.
//
// Pipeline: per wave and tile of 64 keys the softmax is ~1000 cycles of vector ALU work and the two
// contractions ~1100 cycles of MFMA, and a wave issues in order.  The matrix pipe and the vector ALU
// of a SIMD do overlap when they are fed by two DIFFERENT waves (measured: the MFMA stream keeps its
// pace, the vector stream loses about a quarter), so the work of a tile is cut into a pure vector
// phase (mask, maximum, rescale, all exponentials, rounding of P) and a pure matrix phase
// (P.V of that tile, then S of the next one), and the two waves that share a SIMD (w and w+4) run
// the same sequence HALF A TILE APART: while one is in its vector phase the other is in its matrix
// phase.  A block barrier ends every half tile.  Only one set of score registers is alive per wave.
//
// LDS: K tile rows padded by 16 B and V tile rows by 64 B so that the row reads (K) and the
// 4-rows-by-64-B transposing reads (V) of a half wave fall on disjoint banks; two buffers each.
// Tiles go HBM -> registers -> LDS, moved by the early waves (0-3): the loads of K(t+1) are issued
// before the softmax of tile t and stored after it, those of V(t+1) before and after the matrix
// phase of tile t.  (The same loads issue two to four times slower from waves 4-7, and
// direct-to-LDS loads were measured slower still: +15 %.)
#include "common.hpp"

namespace forge {
namespace {

typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v4i16 lds_v4i16;

struct AttnParams {
  const bf16* q;
  const bf16* k;
  const bf16* v;
  bf16* out;
  int q_heads, kv_heads, q_len, kv_len;
  int64_t kv_bs, kv_hs;
  float scale_log2e;
  int causal;
  int n_qblocks;
  const float* mask;        // additive, fp32 [*, *, q_len, kv_len]; only read by the MASKED kernel
  int64_t mask_bs, mask_hs;
  int mask_vec;             // every group of 4 consecutive keys of a mask row is one aligned 16-byte load
};

__device__ inline float xchg32_max(float x) {
  // max over the lane pair (l, l^32)
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ inline float xchg32_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// MASKED: an additive mask (the optional mask node of the paper's attention chain) is added to
// the scaled scores before the softmax.  A lane's 32 mask values of a tile (its query row, the keys
// its score registers hold: 8 groups of 4 consecutive keys) are requested at the end of the
// preceding matrix phase, 16 bytes per load, and arrive behind the half-tile barrier.
template <int DH, bool MASKED>
__global__ __launch_bounds__(512) void attn_prefill_kernel(AttnParams p) {
  constexpr int BQ = 256, BKV = 64;
  constexpr int CPR = DH / 8;                 // 16-byte chunks per row
  constexpr int KS = DH * 2 + 16;             // K row stride in LDS (bytes)
  constexpr int VS = DH * 2 + 64;             // V row stride in LDS (bytes)
  constexpr int K_BYTES = BKV * KS, V_BYTES = BKV * VS;
  // chunks per thread, tensor and tile: the early waves move the tiles (measured: the same loads
  // issue two to four times slower from the second wave of a SIMD)
  constexpr int LPT = BKV * CPR / 256;        // per thread of the early waves; the late waves copy nothing
  constexpr int NKS = DH / 16;                // MFMA k-steps over dh
  constexpr int NDT = DH / 32;                // 32-row tiles of O^T
  extern __shared__ __attribute__((aligned(16))) char smem[];   // [K0 | K1 | V0 | V1]
  char* const kbuf = smem;
  char* const vbuf = smem + 2 * K_BYTES;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int fr = lane & 31, fh = lane >> 5;
  // late (long) query blocks first, over all heads: they carry the most key tiles under the
  // causal mask, and blocks are handed out in launch order
  const int qb = p.n_qblocks - 1 - blockIdx.y;
  const int h = blockIdx.x % p.q_heads, b = blockIdx.x / p.q_heads;
  const int g = h / (p.q_heads / p.kv_heads);
  const int q0 = qb * BQ, q0w = q0 + wave * 32;
  const int off = p.kv_len - p.q_len;
  const bool late = wave >= 4;                // the second wave of each SIMD runs half a tile behind (see above)

  const bf16* kbase = p.k + (int64_t)b * p.kv_bs + (int64_t)g * p.kv_hs;
  const bf16* vbase = p.v + (int64_t)b * p.kv_bs + (int64_t)g * p.kv_hs;

  // ---- this lane's query row as the B operand of S^T (registers for the whole kernel) ------
  const int my_q = q0w + fr;
  bf16x8 qf[NKS];
  {
    const int qr = min(my_q, p.q_len - 1);
    const bf16* qrow = p.q + (((int64_t)b * p.q_heads + h) * p.q_len + qr) * DH;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks)
      qf[ks] = *reinterpret_cast<const bf16x8*>(qrow + (2 * ks + fh) * 8);
    // pin the fragments in registers: otherwise the compiler re-loads them from global memory
    // inside the key loop and the score MFMAs wait on that latency every tile
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) asm volatile("" : "+v"(qf[ks]));
  }

  // keys a query may see: [0, limit]
  const int last_q_blk = min(q0 + BQ, p.q_len) - 1;
  const int n_tiles = ceil_div((p.causal ? last_q_blk + off : p.kv_len - 1) + 1, BKV);
  const int my_limit = p.causal ? my_q + off : p.kv_len - 1;
  const int wave_max_limit = p.causal ? min(q0w + 31, p.q_len - 1) + off : p.kv_len - 1;
  const int wave_min_limit = p.causal ? q0w + off : p.kv_len - 1;

  // ---- global -> registers -> LDS copy plan: each early wave moves a quarter of a tile -------------
  int ld_row[LPT], ld_c[LPT];
#pragma unroll
  for (int i = 0; i < LPT; ++i) {
    const int idx = (tid & 255) + i * 256;
    ld_row[i] = idx / CPR;
    ld_c[i] = idx % CPR;
  }
  u32x4 rk[LPT], rv[LPT];
  auto load_rows = [&](const bf16* base, int t, u32x4 (&r)[LPT]) {
    if (late) return;
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
      const int key = min(t * BKV + ld_row[i], p.kv_len - 1);   // rows past the end re-read the last key
      r[i] = *reinterpret_cast<const u32x4*>(base + (int64_t)key * DH + ld_c[i] * 8);
    }
  };
  auto store_k = [&](int buf) {
    if (late) return;
#pragma unroll
    for (int i = 0; i < LPT; ++i)
      *reinterpret_cast<u32x4*>(kbuf + buf * K_BYTES + ld_row[i] * KS + ld_c[i] * 16) = rk[i];
  };
  auto store_v = [&](int buf) {
    if (late) return;
#pragma unroll
    for (int i = 0; i < LPT; ++i)
      *reinterpret_cast<u32x4*>(vbuf + buf * V_BYTES + ld_row[i] * VS + ld_c[i] * 16) = rv[i];
  };

  floatx16 o_acc[NDT];
#pragma unroll
  for (int i = 0; i < NDT; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) o_acc[i][e] = 0.f;
  float m_run = -1e30f, l_run = 0.f;   // finite start: no inf - inf anywhere
  // MASKED works on pre-scaled scores (s * scale * log2e + mask * log2e), so the factor inside
  // the softmax is 1 there
  const float c = MASKED ? 1.0f : p.scale_log2e;
  const float* mask_row = nullptr;
  if (MASKED)
    mask_row = p.mask + b * p.mask_bs + h * p.mask_hs + (int64_t)min(my_q, p.q_len - 1) * p.kv_len;
  floatx4 mk[MASKED ? 8 : 1];      // mask values of the tile whose vector phase comes next
  auto mask_prefetch = [&](int t) {
    if (!MASKED) return;
#pragma unroll
    for (int g8 = 0; g8 < 8; ++g8) {
      const int key0 = t * BKV + (g8 >> 2) * 32 + 8 * (g8 & 3) + 4 * fh;     // registers 4 (g8 & 3) .. + 3 of block g8 >> 2
      floatx4 m = {0.f, 0.f, 0.f, 0.f};                                     // keys past the end are cut in the softmax
      if (p.mask_vec) {
        if (key0 < p.kv_len) m = *reinterpret_cast<const floatx4*>(mask_row + key0);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (key0 + e < p.kv_len) m[e] = mask_row[key0 + e];
      }
      mk[g8] = m;
    }
  };

  // per-lane byte offset of the transposing V read inside a tile (without key step / d tile)
  const int vt_lane = (((lane & 15) >> 2) + 4 * fh) * VS + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;

  // ---- matrix phase, part 2: S^T = K . Q^T of one tile ---------------------------------------------
  floatx16 sc[2];                  // the scores of the tile in flight, then its probabilities
  bf16x8 pf[4];                    // P^T of the tile whose vector phase has run: B operand of P.V
  auto scores = [&](int t) {
    const char* sk = kbuf + (t & 1) * K_BYTES;
    // (the first MFMA of each key block takes a zero accumulator as an inline constant)
    // K fragments run LA MFMAs ahead of their use so that no MFMA waits on an LDS read
    constexpr int NF = 2 * NKS, LA = 4;
    bf16x8 kf[LA];
    auto kread = [&](int i) {
      const int kb = i / NKS, ks = i % NKS;
      return *reinterpret_cast<const bf16x8*>(sk + (kb * 32 + fr) * KS + (2 * ks + fh) * 16);
    };
#pragma unroll
    for (int i = 0; i < LA; ++i) kf[i] = kread(i);
#pragma unroll
    for (int i = 0; i < NF; ++i) {
      __builtin_amdgcn_sched_barrier(0);
      const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      sc[i / NKS] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i % LA], qf[i % NKS], i % NKS == 0 ? zero : sc[i / NKS], 0, 0, 0);
      if (i + LA < NF) kf[i % LA] = kread(i + LA);
    }
    __builtin_amdgcn_sched_barrier(0);
  };

  // ---- vector phase: mask, online softmax, P rounded to bf16 (no matrix instruction) ----------------
  auto softmax = [&](int t) {
    const int kv0 = t * BKV;
    if (MASKED) {
      constexpr float LOG2E = 1.4426950408889634f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) sc[kb][v] = sc[kb][v] * p.scale_log2e + mk[kb * 4 + (v >> 2)][v & 3] * LOG2E;
    }
    if (kv0 + BKV - 1 > wave_min_limit) {       // diagonal / tail tiles only
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = kv0 + kb * 32 + 8 * (v >> 2) + 4 * fh + (v & 3);
          if (key > my_limit) sc[kb][v] = -INFINITY;
        }
    }
    float mx = sc[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sc[kb][v]);
    mx = xchg32_max(mx);
    const float m_new = fmaxf(m_run, mx);
    if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {   // wave-uniform: some maximum moved
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
      l_run *= alpha;
#pragma unroll
      for (int i = 0; i < NDT; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) o_acc[i][e] *= alpha;
      m_run = m_new;
    }
    const float mc = m_run * c;
    float psum = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float pv = __builtin_amdgcn_exp2f(sc[kb][v] * c - mc);
        sc[kb][v] = pv;
        psum += pv;
      }
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
        for (int e = 0; e < 8; ++e) pf[2 * kb + s2][e] = (bf16)sc[kb][8 * s2 + e];
    }
    l_run += psum;
  };

  // ---- matrix phase, part 1: O^T += V^T . P^T --------------------------------------------------------
  auto pv_mm = [&](int t) {
    const char* sv = vbuf + (t & 1) * V_BYTES;
    // V^T fragments (two transposing reads each) run LA MFMAs ahead of their use
    constexpr int NF = 4 * NDT, LA = 4;
    typedef short v8i16 __attribute__((ext_vector_type(8)));
    v4i16 lo[LA], hi[LA];
    auto vread = [&](int i, v4i16& l, v4i16& hh) {
      const int s = i / NDT, dt = i % NDT;
      const char* va = sv + vt_lane + (16 * s) * VS + dt * 64;
      l = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16*)(va));
      hh = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16*)(va + 8 * VS));
    };
#pragma unroll
    for (int i = 0; i < LA; ++i) vread(i, lo[i], hi[i]);
#pragma unroll
    for (int i = 0; i < NF; ++i) {
      __builtin_amdgcn_sched_barrier(0);
      const v4i16 l = lo[i % LA], hh = hi[i % LA];
      v8i16 both = {l[0], l[1], l[2], l[3], hh[0], hh[1], hh[2], hh[3]};
      o_acc[i % NDT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pf[i / NDT], o_acc[i % NDT], 0, 0, 0);
      if (i + LA < NF) vread(i + LA, lo[i % LA], hi[i % LA]);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  auto wave_needs = [&](int t) { return t < n_tiles && t * BKV <= wave_max_limit; };   // wave-uniform

  // ---- prologue: K(0), V(0), K(1) in LDS, S(0) in registers ---------------------------------------
  load_rows(kbase, 0, rk);
  load_rows(vbase, 0, rv);
  store_k(0);
  store_v(0);
  __syncthreads();
  if (wave_needs(0)) {
    scores(0);
    mask_prefetch(0);
  }
  __syncthreads();

  // Steps of half a tile, a block barrier after each; the late waves run one step behind:
  //   step 2t   : early waves  softmax(t), copy of K(t+1)           late waves  P.V(t-1), S(t)
  //   step 2t+1 : early waves  P.V(t), S(t+1), copy of V(t+1)      late waves  softmax(t)
  // K(t+1) goes into K buffer (t+1)&1, whose last reader was the late waves' S(t-1) in step 2t-2, and
  // is first read by the early waves' S(t+1) in step 2t+1.  V(t+1) goes into V buffer (t+1)&1, last
  // read by the late waves' P.V(t-1) in step 2t, first read by the early waves' P.V(t+1) in step 2t+3.
  auto matrix_phase = [&](int t) {
    if (wave_needs(t)) pv_mm(t);
    if (wave_needs(t + 1)) {
      scores(t + 1);
      mask_prefetch(t + 1);
    }
  };
  if (!late) {
    for (int t = 0; t < n_tiles; ++t) {
      // step 2t: K(t+1) travels behind the softmax; step 2t+1: V(t+1) behind the MFMAs
      if (t + 1 < n_tiles) load_rows(kbase, t + 1, rk);
      if (wave_needs(t)) softmax(t);
      if (t + 1 < n_tiles) store_k((t + 1) & 1);
      __syncthreads();
      if (t + 1 < n_tiles) load_rows(vbase, t + 1, rv);
      matrix_phase(t);
      if (t + 1 < n_tiles) store_v((t + 1) & 1);
      __syncthreads();
    }
    __syncthreads();                   // the late waves' last step
  } else {
    __syncthreads();                   // the early waves' first step
    for (int t = 0; t < n_tiles; ++t) {
      if (wave_needs(t)) softmax(t);
      __syncthreads();
      matrix_phase(t);
      __syncthreads();
    }
  }

  // ---- normalise and store: lane owns query my_q; registers 4g..4g+3 are 4 consecutive d -----
  const float l_tot = xchg32_sum(l_run);
  if (my_q < p.q_len) {
    const float inv = 1.0f / l_tot;
    bf16* orow = p.out + ((int64_t)b * p.q_len + my_q) * ((int64_t)p.q_heads * DH) + (int64_t)h * DH;
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
      for (int gg = 0; gg < 4; ++gg) {
        u32x2 pk;
        pk[0] = pack_bf2(o_acc[dt][4 * gg] * inv, o_acc[dt][4 * gg + 1] * inv);
        pk[1] = pack_bf2(o_acc[dt][4 * gg + 2] * inv, o_acc[dt][4 * gg + 3] * inv);
        *reinterpret_cast<u32x2*>(orow + dt * 32 + 8 * gg + 4 * fh) = pk;
      }
  }
}

template <int DH, bool MASKED>
forge_status launch_dh(const AttnArgs& a, hipStream_t s) {
  AttnParams p;
  p.q = (const bf16*)a.q;
  p.k = (const bf16*)a.k;
  p.v = (const bf16*)a.v;
  p.out = (bf16*)a.out;
  p.q_heads = a.q_heads;
  p.kv_heads = a.kv_heads;
  p.q_len = a.q_len;
  p.kv_len = a.kv_len;
  p.kv_bs = a.kv_batch_stride;
  p.kv_hs = a.kv_head_stride;
  p.scale_log2e = a.scale * 1.4426950408889634f;
  p.causal = a.causal;
  p.n_qblocks = ceil_div(a.q_len, 256);
  p.mask = a.mask;
  p.mask_bs = a.mask_batch_stride;
  p.mask_hs = a.mask_head_stride;
  p.mask_vec = a.mask != nullptr && a.kv_len % 4 == 0 && (reinterpret_cast<uintptr_t>(a.mask) & 15u) == 0 &&
               a.mask_batch_stride % 4 == 0 && a.mask_head_stride % 4 == 0;
  constexpr int smem = 2 * 64 * ((DH * 2 + 16) + (DH * 2 + 64));
  auto kern = attn_prefill_kernel<DH, MASKED>;
  static std::atomic<uint64_t> lds_raised{0};   // per kernel instantiation
  if (raise_lds_limit(reinterpret_cast<const void*>(kern), smem, lds_raised) != FORGE_OK) return FORGE_ERR_HIP;
  dim3 grid(a.q_heads * a.batch, p.n_qblocks), block(512);
  kern<<<grid, block, smem, s>>>(p);
  return launch_status();
}

}  // namespace

forge_status launch_attn_prefill_bf16(const AttnArgs& a, hipStream_t s) {
  if (a.head_dim == 64) return a.mask ? launch_dh<64, true>(a, s) : launch_dh<64, false>(a, s);
  if (a.head_dim == 128) return a.mask ? launch_dh<128, true>(a, s) : launch_dh<128, false>(a, s);
  return FORGE_ERR_UNSUPPORTED;
}

}  // namespace forge
