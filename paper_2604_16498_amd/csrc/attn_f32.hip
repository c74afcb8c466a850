// Fused attention in full fp32 on the fp32 matrix cores (v_mfma_f32_32x32x2_f32): the FORGE_F32
// path for a prompt (config 1).  Same chain as the bf16 prefill kernel (Sec. "Pass 4: Attention
// Fusion": scores, scale, causal mask, softmax, P.V in one kernel, S and P never leave the
// registers), nothing is rounded below fp32.
//
// A 256-thread block owns 32 consecutive queries of one (batch, head); its 4 waves share those
// queries and split the KEY tiles among themselves (wave w takes tiles w, w + 4, ...; a short
// prompt is a handful of tiles, and walking them one after the other would leave the kernel
// latency-bound), each with a running maximum / sum / output of its own; the four partial results
// are merged through LDS in wave order (fixed order: bitwise reproducible).  A wave stages its
// K and V tile (32 keys) in its own LDS region (rows padded by 4 floats: conflict-free 128-bit
// reads), so no block barrier is needed inside the loop.
//   scores  S^T[key, query] = K . Q^T: the MFMA contracts two dims per issue, lanes 0-31 supply
//           one and lanes 32-63 the other; lanes 0-31 walk the first half of head_dim and lanes
//           32-63 the second half, so a lane reads 4 consecutive floats of its key row per LDS
//           access and keeps its half of its query row in registers.  Lane = query column: a lane
//           holds 16 of its query's 32 scores, lane ^ 32 the other 16.
//   softmax online, per lane: running maximum / sum of its query (both half-lanes keep the same
//           values), one exchange with lane ^ 32 per tile; exp in fp32.
//   P . V   O^T[d, query] += V^T . P^T with the keys contracted in the order the score
//           accumulator already holds them: step s takes accumulator register s of either
//           half-lane as the P operand (no data movement) and reads the matching V row.
#include "common.hpp"

namespace forge {
namespace {

constexpr int F32_BQ = 32;       // queries per block
constexpr int F32_BK = 32;       // keys per tile
// waves per block = key-tile groups (each wave stages a K and a V tile of its own: 17 / 33 KB)
template <int DH> struct F32Cfg { static constexpr int NW = DH == 64 ? 4 : 2; };

// key held by accumulator register v of half-lane hb (the C layout of a 32 x 32 MFMA)
__device__ inline int acc_row(int v, int hb) { return 8 * (v >> 2) + 4 * hb + (v & 3); }

// lanes of one wave exchange data through LDS
__device__ inline void wave_sync_lds() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int DH>
__global__ __launch_bounds__((F32Cfg<DH>::NW * 64)) void attn_f32_kernel(
    const float* __restrict__ q, const float* __restrict__ k, const float* __restrict__ v,
    float* __restrict__ out, int q_heads, int kv_heads, int q_len, int kv_len, int64_t kv_bs,
    int64_t kv_hs, float scale, int causal) {
  constexpr int LD = DH + 4;                 // padded LDS row (floats)
  constexpr int HD = DH / 2;                 // dims per half-lane
  constexpr int NB = DH / 32;                // 32-row blocks of O^T
  constexpr int F32_NW = F32Cfg<DH>::NW;
  constexpr int TILE = F32_BK * LD;          // floats of one staged tile
  // per wave: K tile, V tile (the merge reuses the K region for O and the V region for m, l)
  extern __shared__ __attribute__((aligned(16))) float lds[];   // [NW][2][TILE]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, hb = lane >> 5;
  const int h = blockIdx.y, b = blockIdx.z;
  const int g = h / (q_heads / kv_heads);
  const int q0 = blockIdx.x * F32_BQ;
  const int qi = q0 + col;                                 // this lane's query
  const int off = kv_len - q_len;                          // query i sees keys j <= i + off
  const float* kb = k + (int64_t)b * kv_bs + (int64_t)g * kv_hs;
  const float* vb = v + (int64_t)b * kv_bs + (int64_t)g * kv_hs;
  float* ks = lds + (wave * 2 + 0) * TILE;
  float* vs = lds + (wave * 2 + 1) * TILE;

  // this lane's half of its query row, pre-scaled (rows past the end re-read the last query)
  float qr[HD];
  {
    const float* qrow = q + (((int64_t)b * q_heads + h) * q_len + min(qi, q_len - 1)) * DH + hb * HD;
#pragma unroll
    for (int e = 0; e < HD; e += 4) {
      const floatx4 t = *reinterpret_cast<const floatx4*>(qrow + e);
#pragma unroll
      for (int u = 0; u < 4; ++u) qr[e + u] = t[u] * scale;
    }
  }

  floatx16 oacc[NB];
#pragma unroll
  for (int t = 0; t < NB; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[t][e] = 0.f;
  float m_run = -1e30f, l_run = 0.f;         // finite start: a wave without tiles merges with weight 0

  // keys this block needs: up to the last query's limit
  const int q_last = min(q0 + F32_BQ, q_len) - 1;
  const int k_end = causal ? min(kv_len, q_last + off + 1) : kv_len;
  const int limit = causal ? min(kv_len, qi + off + 1) : kv_len;   // this lane's keys [0, limit)

  for (int j0 = wave * F32_BK; j0 < k_end; j0 += F32_NW * F32_BK) {   // wave-uniform
    wave_sync_lds();                         // this wave has consumed its previous tile
    // stage K and V rows j0 .. j0+31 (rows past the end re-read the last row; masked below)
    for (int idx = lane; idx < F32_BK * (DH / 4); idx += 64) {
      const int r = idx / (DH / 4), c4 = idx % (DH / 4);
      const int64_t src = (int64_t)min(j0 + r, kv_len - 1) * DH + c4 * 4;
      *reinterpret_cast<floatx4*>(&ks[r * LD + c4 * 4]) = *reinterpret_cast<const floatx4*>(kb + src);
      *reinterpret_cast<floatx4*>(&vs[r * LD + c4 * 4]) = *reinterpret_cast<const floatx4*>(vb + src);
    }
    wave_sync_lds();

    // ---- scores: S^T[key, query] -------------------------------------------------------------
    floatx16 sacc;
#pragma unroll
    for (int e = 0; e < 16; ++e) sacc[e] = 0.f;
#pragma unroll
    for (int e = 0; e < HD; e += 4) {
      const floatx4 kf = *reinterpret_cast<const floatx4*>(&ks[col * LD + hb * HD + e]);   // key row = col
#pragma unroll
      for (int u = 0; u < 4; ++u)
        sacc = __builtin_amdgcn_mfma_f32_32x32x2f32(kf[u], qr[e + u], sacc, 0, 0, 0);
    }
    // ---- mask, running maximum ---------------------------------------------------------------
    float mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      if (j0 + acc_row(e, hb) >= limit) sacc[e] = -INFINITY;
      mx = fmaxf(mx, sacc[e]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float alpha = __expf(m_run - m_new);
    float ps = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      sacc[e] = __expf(sacc[e] - m_new);     // exp(-inf) = 0 for masked keys
      ps += sacc[e];
    }
    ps += __shfl_xor(ps, 32, 64);
    l_run = l_run * alpha + ps;
    m_run = m_new;
#pragma unroll
    for (int t = 0; t < NB; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[t][e] *= alpha;
    // ---- P . V: O^T[d, query] += V[key, d] P[key, query], keys in accumulator order -------------
#pragma unroll
    for (int s = 0; s < 16; ++s) {
      const float* vrow = &vs[acc_row(s, hb) * LD];
#pragma unroll
      for (int t = 0; t < NB; ++t)
        oacc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(vrow[t * 32 + col], sacc[s], oacc[t], 0, 0, 0);
    }
  }

  // ---- merge the four waves, in wave order ---------------------------------------------------------
  // each wave publishes O[query][d] (unnormalised) in its K region and (m, l) in its V region
  wave_sync_lds();
#pragma unroll
  for (int t = 0; t < NB; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) ks[col * LD + t * 32 + acc_row(e, hb)] = oacc[t][e];
  if (hb == 0) { vs[2 * col] = m_run; vs[2 * col + 1] = l_run; }
  __syncthreads();
  // thread = (query, 4 consecutive dims); DH / 4 threads per query
  for (int idx = tid; idx < F32_BQ * (DH / 4); idx += F32_NW * 64) {
    const int qq = idx / (DH / 4), c4 = idx % (DH / 4);
    if (q0 + qq >= q_len) continue;
    float mw[F32_NW], mmax = -1e30f;
#pragma unroll
    for (int w = 0; w < F32_NW; ++w) { mw[w] = lds[(w * 2 + 1) * TILE + 2 * qq]; mmax = fmaxf(mmax, mw[w]); }
    floatx4 o = {0.f, 0.f, 0.f, 0.f};
    float lt = 0.f;
#pragma unroll
    for (int w = 0; w < F32_NW; ++w) {
      const float a = __expf(mw[w] - mmax);    // a wave that saw no key: exp(-1e30 - m) = 0
      lt += lds[(w * 2 + 1) * TILE + 2 * qq + 1] * a;
      o += *reinterpret_cast<const floatx4*>(&lds[(w * 2) * TILE + qq * LD + c4 * 4]) * a;
    }
    const float inv = 1.0f / lt;
    float* orow = out + ((int64_t)b * q_len + q0 + qq) * ((int64_t)q_heads * DH) + (int64_t)h * DH;
    *reinterpret_cast<floatx4*>(orow + c4 * 4) = o * inv;
  }
}

template <int DH>
forge_status launch_f32(const AttnArgs& a, hipStream_t s) {
  constexpr int NW = F32Cfg<DH>::NW;
  constexpr int smem = NW * 2 * F32_BK * (DH + 4) * (int)sizeof(float);
  auto kern = attn_f32_kernel<DH>;
  static std::atomic<uint64_t> lds_raised{0};   // per kernel instantiation
  if (raise_lds_limit(reinterpret_cast<const void*>(kern), smem, lds_raised) != FORGE_OK) return FORGE_ERR_HIP;
  dim3 grid(ceil_div(a.q_len, F32_BQ), a.q_heads, a.batch), block(NW * 64);
  kern<<<grid, block, smem, s>>>((const float*)a.q, (const float*)a.k, (const float*)a.v, (float*)a.out,
                                 a.q_heads, a.kv_heads, a.q_len, a.kv_len, a.kv_batch_stride,
                                 a.kv_head_stride, a.scale, a.causal);
  return launch_status();
}

}  // namespace

forge_status launch_attn_f32_mfma(const AttnArgs& a, hipStream_t s) {
  if (a.head_dim == 64) return launch_f32<64>(a, s);
  if (a.head_dim == 128) return launch_f32<128>(a, s);
  return FORGE_ERR_UNSUPPORTED;
}

}  // namespace forge
