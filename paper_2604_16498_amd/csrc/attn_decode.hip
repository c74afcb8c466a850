// bf16 fused attention for one new query per sequence over a KV cache (decode).  HBM-bound:
// every cached K and V row is read exactly once, with 128-bit loads, and nothing else of
// comparable size moves.
//
// Split-KV: block (split, kv head, batch) streams one contiguous range of cache rows of ONE kv
// head for all G = Hq/Hkv query heads that share it (grouped-query attention reads the cache
// once per group, not once per query head).  The 4 waves of a block take the 16-row tiles of the
// range in turn (wave w: tiles w, w + 4, ...) and each keeps two tiles of K and V loads in flight
// ahead of the one it is working on.  The number of splits is chosen on the host so that about
// two blocks per compute unit exist: a large batch needs no split at all (one block per
// (kv head, sequence) walks the whole cache and writes the final output itself: no partials, no
// second kernel), a small batch is cut into ranges that are multiples of 128 rows, 256 at least.
//
// Per tile of 16 rows:
//   scores   S[row, head] = K . q^T on the matrix cores (v_mfma_f32_16x16x32_bf16, heads padded
//            to 16).  K is loaded straight from HBM in the MFMA A layout: lane = (row l%16, 16-byte
//            chunk), the contraction order over dh is permuted so that one wave-wide load reads 64
//            contiguous bytes of each row.  No LDS, no transposition.
//   softmax  in the accumulator layout (lane = head, 4 rows per lane): running maximum per head
//            with LAZY rescaling (the accumulators are only rescaled when some row beats the
//            maximum, which becomes rare after the first tiles), exp2 domain.
//   P . V    each lane owns 8 output columns for every head.  P goes through a 16 x G float
//            patch of LDS (the only cross-lane traffic), is packed with its neighbour row to
//            bf16 pairs, V rows of two steps are interleaved with byte permutes, and the
//            accumulation runs on v_dot2_f32_bf16: two rows per instruction, fp32 accumulate.
// Wave and block partials are merged in a fixed order; with more than one split the block writes
// (m, l, o) per query head to the workspace and a second kernel merges the splits in split order
// -- no atomics, so the result is bitwise reproducible.
#include "common.hpp"

namespace forge {
namespace {

constexpr int NWAVES = 4;                 // waves per block
constexpr int TILE = 16;                  // cache rows per MFMA tile
constexpr int GRAIN = 2 * NWAVES * TILE;  // a split is a multiple of this many rows (two tiles per wave)
constexpr int MAX_SPLITS = 64;            // the combine holds one split per lane

struct DecParams {
  const bf16* q;
  const bf16* k;
  const bf16* v;
  float* part;     // [B, Hkv, splits, G, dh + 2]
  bf16* out;       // [B, Hq * dh]: written directly when splits == 1
  int q_heads, kv_heads, kv_len, splits;   // kv_heads counts blockIdx.y: cache heads x passes
  int passes;           // blocks (of G query heads each) that share one cache head
  int rows_per_split;   // multiple of GRAIN
  int64_t kv_bs, kv_hs;
  float scale_log2e;
  const int* kv_pos;   // per-sequence: rows [0, kv_pos[b]] (clamped to kv_len - 1); NULL: kv_len rows
};

// Lanes of one wave exchange data through LDS: the hardware runs a wave's LDS instructions in
// order, but the compiler must be told that other lanes wrote between this lane's accesses.
__device__ inline void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ inline float xor16_max(float x) { return fmaxf(x, __shfl_xor(x, 16, 64)); }
__device__ inline float xor32_max(float x) { return fmaxf(x, __shfl_xor(x, 32, 64)); }

// G: query heads per KV head, 1 ... 8 (the MFMA's 16 head columns hold them zero-padded; the
// P . V accumulators grow with G, so the larger groups run at two blocks per SIMD instead of three)
template <int DH, int G>
__global__ __launch_bounds__(NWAVES * 64, G > 4 ? 2 : 3) void attn_decode_kernel(DecParams p) {
  constexpr int NJ = DH / 32;          // MFMAs (and K loads) per tile
  constexpr int LPR = DH / 8;          // lanes per V row
  constexpr int KPS = 64 / LPR;        // rows per wave-wide V load
  constexpr int VSTEPS = TILE / KPS;   // V loads per tile
  constexpr int NPAIR = VSTEPS / 2;    // row pairs per lane per tile
  __shared__ __attribute__((aligned(16))) float pbuf[NWAVES][TILE][G];
  __shared__ __attribute__((aligned(16))) float abuf[NWAVES][G];
  __shared__ float sm[NWAVES][G][DH + 2];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int krow = lane & 15, kg = lane >> 4;          // MFMA layout: row in tile / lane group
  const int head = lane & 15;                          // ... and the accumulator's column
  const int slot = lane / LPR, c = lane % LPR;         // V layout: row in step / 16-byte chunk

  // query heads g G ... g G + G - 1 attend to cache head g / passes
  const int64_t cache_head = (int64_t)b * p.kv_bs + (int64_t)(g / p.passes) * p.kv_hs;
  const bf16* kb = p.k + cache_head;
  const bf16* vb = p.v + cache_head;
  const int split_begin = split * p.rows_per_split;
  // tiles of this wave that begin before the end of the range, rounded up to a pair (the loop
  // takes two per trip; the loads stay unconditional so that their count per trip is fixed)
  // a split that lies wholly past the end of a short sequence writes a neutral partial
  // (maximum -1e30, sum 0), which the combine weighs with exactly 0
  const int kv_len = p.kv_pos != nullptr ? min(max(p.kv_pos[b], 0), p.kv_len - 1) + 1 : p.kv_len;
  const int row_end = min(kv_len, split_begin + p.rows_per_split);
  const int rows_w = row_end - split_begin - wave * TILE;          // <= 0: no tile for this wave
  const int ntile = rows_w > 0 ? (ceil_div(rows_w, NWAVES * TILE) + 1) / 2 * 2 : 0;
  const int last = kv_len - 1;

  // q as the MFMA B operand: lane = (head, chunk 4j + kg); heads >= G are zero columns
  bf16x8 qf[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    u32x4 t = {0, 0, 0, 0};
    if (head < G) t = *reinterpret_cast<const u32x4*>(p.q + ((int64_t)b * p.q_heads + g * G + head) * DH + (4 * j + kg) * 8);
    qf[j] = __builtin_bit_cast(bf16x8, t);
  }

  u32x4 kr[2][NJ], vr[2][VSTEPS];
  // tile t of this wave: rows base .. base + 15 (the waves take the tiles of the range in turn)
  auto tile_base = [&](int t) { return split_begin + (t * NWAVES + wave) * TILE; };
  auto load_tile = [&](int t, u32x4 (&kk)[NJ], u32x4 (&vv)[VSTEPS]) {
    const int base = tile_base(t);
#pragma unroll
    for (int j = 0; j < NJ; ++j)   // rows past the end re-read the last row (masked below)
      kk[j] = *reinterpret_cast<const u32x4*>(kb + (int64_t)min(base + krow, last) * DH + (4 * j + kg) * 8);
#pragma unroll
    for (int s = 0; s < VSTEPS; ++s)
      vv[s] = *reinterpret_cast<const u32x4*>(vb + (int64_t)min(base + s * KPS + slot, last) * DH + c * 8);
  };
  load_tile(0, kr[0], vr[0]);
  load_tile(1, kr[1], vr[1]);

  float m_run = -1e30f, l_part = 0.f;      // accumulator layout: this lane's head
  float acc[G][8];                         // V layout: this lane's 8 columns, all heads
#pragma unroll
  for (int h = 0; h < G; ++h)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[h][e] = 0.f;
  const float cl = p.scale_log2e;

  for (int t0 = 0; t0 < ntile; t0 += 2) {
#pragma unroll
   for (int u = 0; u < 2; ++u) {
    const int t = t0 + u;
    u32x4 (&kk)[NJ] = kr[u];
    u32x4 (&vv)[VSTEPS] = vr[u];
    const int base = tile_base(t);
    if (base < row_end) {     // wave-uniform: tiles wholly past the end contribute nothing
      // ---- scores ------------------------------------------------------------------------------
      floatx4 sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < NJ; ++j)
        sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kk[j]), qf[j], sacc, 0, 0, 0);
      float sc[4];
      float mx = -INFINITY;
#pragma unroll
      for (int v = 0; v < 4; ++v) {     // accumulator register v is row 4 kg + v
        sc[v] = base + 4 * kg + v < row_end ? sacc[v] * cl : -INFINITY;
        mx = fmaxf(mx, sc[v]);
      }
      mx = xor32_max(xor16_max(mx));
      // ---- lazy rescale --------------------------------------------------------------------------
      if (__any(mx > m_run)) {
        const float m_new = fmaxf(m_run, mx);
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        l_part *= alpha;
        if (lane < G) abuf[wave][lane] = alpha;      // lane = head (kg == 0)
        wave_lds_sync();
        float al[G];
#pragma unroll
        for (int h = 0; h < G; ++h) al[h] = abuf[wave][h];
#pragma unroll
        for (int h = 0; h < G; ++h)
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[h][e] *= al[h];
      }
      // ---- probabilities, through LDS to the V layout ---------------------------------------------
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const float pr = __builtin_amdgcn_exp2f(sc[v] - m_run);   // exp2(-inf) = 0 past the end
        l_part += pr;
        if (head < G) pbuf[wave][4 * kg + v][head] = pr;
      }
      wave_lds_sync();
      // ---- P . V on dot2: rows (s, s+1) of this lane's slot packed as bf16 pairs ---------------------
#pragma unroll
      for (int pi = 0; pi < NPAIR; ++pi) {
        const int ra = (2 * pi) * KPS + slot, rb = (2 * pi + 1) * KPS + slot;
        bf16x2 pp[G];
#pragma unroll
        for (int h = 0; h < G; ++h) {
          pp[h][0] = (bf16)pbuf[wave][ra][h];
          pp[h][1] = (bf16)pbuf[wave][rb][h];
        }
        const u32x4 va = vv[2 * pi], vb2 = vv[2 * pi + 1];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          // (va.lo, vb.lo) and (va.hi, vb.hi): element 2d and 2d+1 of both rows
          const uint32_t lo = __builtin_amdgcn_perm(vb2[d], va[d], 0x05040100);
          const uint32_t hi = __builtin_amdgcn_perm(vb2[d], va[d], 0x07060302);
          const bf16x2 vlo = __builtin_bit_cast(bf16x2, lo), vhi = __builtin_bit_cast(bf16x2, hi);
#pragma unroll
          for (int h = 0; h < G; ++h) {
            acc[h][2 * d] = __builtin_amdgcn_fdot2_f32_bf16(vlo, pp[h], acc[h][2 * d], false);
            acc[h][2 * d + 1] = __builtin_amdgcn_fdot2_f32_bf16(vhi, pp[h], acc[h][2 * d + 1], false);
          }
        }
      }
    }
    wave_lds_sync();   // this tile's LDS reads are done before the next tile's writes
    // refill the registers just consumed (unconditional: past the end the last row is read
    // again, which keeps the number of loads per trip, and with it the wait counts, fixed)
    load_tile(t + 2, kr[u], vr[u]);
   }
  }

  // ---- merge inside the wave: plain sums (one running maximum per head for the whole wave) -------
#pragma unroll
  for (int o = LPR; o < 64; o <<= 1)
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[h][e] += __shfl_xor(acc[h][e], o, 64);
  l_part += __shfl_xor(l_part, 16, 64);
  l_part += __shfl_xor(l_part, 32, 64);
  if (slot == 0) {
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
      for (int e = 0; e < 8; ++e) sm[wave][h][c * 8 + e] = acc[h][e];
  }
  if (lane < G) { sm[wave][lane][DH] = m_run; sm[wave][lane][DH + 1] = l_part; }
  __syncthreads();
  // ---- merge the waves, fixed order -------------------------------------------------------------------
  float* dst = p.part + ((((int64_t)b * p.kv_heads + g) * p.splits + split) * G) * (DH + 2);
  for (int idx = tid; idx < G * DH; idx += NWAVES * 64) {
    const int h = idx / DH, d = idx % DH;
    float mn = sm[0][h][DH];
#pragma unroll
    for (int w = 1; w < NWAVES; ++w) mn = fmaxf(mn, sm[w][h][DH]);
    float o = 0.f, lt = 0.f;
#pragma unroll
    for (int w = 0; w < NWAVES; ++w) {
      const float a = __builtin_amdgcn_exp2f(sm[w][h][DH] - mn);
      o += sm[w][h][d] * a;
      lt += sm[w][h][DH + 1] * a;
    }
    if (p.splits == 1) {   // the whole cache in one block: this is the result
      p.out[((int64_t)b * p.q_heads + g * G + h) * DH + d] = (bf16)(o / lt);
    } else {
      dst[h * (DH + 2) + d] = o;
      if (d == 0) { dst[h * (DH + 2) + DH] = mn; dst[h * (DH + 2) + DH + 1] = lt; }
    }
  }
}

// one block per (batch, query head): merge the splits in split order and normalise.  Lane s of
// the first wave fetches (m, l) of split s, so the maximum and the weights cost one round trip;
// the weighted sums then run with independent loads, four splits per step.
template <int DH>
__global__ __launch_bounds__(DH) void attn_decode_combine(const float* __restrict__ part,
                                                          bf16* __restrict__ out, int q_heads,
                                                          int kv_heads, int splits) {
  __shared__ float wgt[64];
  __shared__ float ltot;
  const int h = blockIdx.x, b = blockIdx.y, d = threadIdx.x;
  const int G = q_heads / kv_heads;
  const int g = h / G, hh = h % G;
  const float* src = part + ((((int64_t)b * kv_heads + g) * splits) * G + hh) * (DH + 2);
  const int64_t stride = (int64_t)G * (DH + 2);
  if (d < 64) {
    float m = -1e30f, l = 0.f;
    if (d < splits) { m = src[d * stride + DH]; l = src[d * stride + DH + 1]; }
    const float mn = wave_max(m);
    const float a = __builtin_amdgcn_exp2f(m - mn);
    wgt[d] = a;
    // fixed-order sum of l over the splits: butterfly (the same tree every run)
    const float lt = wave_sum(l * a);
    if (d == 0) ltot = lt;
  }
  __syncthreads();
  float o = 0.f;
  int s = 0;
  for (; s + 4 <= splits; s += 4) {
    const float v0 = src[(s + 0) * stride + d], v1 = src[(s + 1) * stride + d];
    const float v2 = src[(s + 2) * stride + d], v3 = src[(s + 3) * stride + d];
    o += v0 * wgt[s];
    o += v1 * wgt[s + 1];
    o += v2 * wgt[s + 2];
    o += v3 * wgt[s + 3];
  }
  for (; s < splits; ++s) o += src[s * stride + d] * wgt[s];
  out[((int64_t)b * q_heads + h) * DH + d] = (bf16)(o / ltot);
}

// Number of row ranges: about two blocks per compute unit, but no range shorter than
// MIN_SPLIT_ROWS: a block streams that many rows in less time than the second launch (the merge of
// the ranges) costs, so a cache shorter than twice that is walked by one block per (head, sequence)
// however few of those there are.
constexpr int MIN_SPLIT_ROWS = 2 * GRAIN;
struct SplitPlan { int splits, rows_per_split; };
// the most ranges a batch is ever cut into, whatever the cache length
inline int max_splits(int batch, int kv_heads) {
  const int64_t pairs = (int64_t)batch * kv_heads;
  const int64_t for_two_per_cu = ceil_div64(2 * (int64_t)compute_units(), pairs);
  return for_two_per_cu < MAX_SPLITS ? (int)for_two_per_cu : MAX_SPLITS;
}
inline SplitPlan plan_splits(int batch, int kv_heads, int kv_len) {
  const int want = max(1, min(max_splits(batch, kv_heads), kv_len / MIN_SPLIT_ROWS));
  const int rows = ceil_div(ceil_div(kv_len, want), GRAIN) * GRAIN;
  return SplitPlan{ceil_div(kv_len, rows), rows};   // rows >= kv_len / want, so splits <= want
}
// Upper bound of plan_splits(.., len).splits over every len <= kv_len: the number of ranges is
// not monotone in the length (the range size is rounded up to GRAIN), the scratch size must be,
// because a generation loop sizes its scratch once, for the capacity of its cache.
inline int splits_bound(int batch, int kv_heads, int kv_len) {
  return max(1, min(max_splits(batch, kv_heads), kv_len / MIN_SPLIT_ROWS));
}

// Query heads per block for `group` heads sharing one cache head: the whole group up to 8, else
// its largest divisor up to 8 -- several blocks then each stream that cache head for their share of
// the query heads (16 heads: two passes of 8).  More than four passes (a prime group above 8) are
// left to the vector-ALU kernel.
constexpr int MAX_G = 8, MAX_PASSES = 4;
inline int heads_per_block(int group) {
  if (group <= MAX_G) return group;
  for (int d = MAX_G; d >= 1; --d)
    if (group % d == 0) return group / d <= MAX_PASSES ? d : 0;
  return 0;
}
// blocks along y: cache heads x passes (the split plan counts these)
inline int block_heads(int q_heads, int kv_heads) {
  const int gb = heads_per_block(q_heads / kv_heads);
  return gb > 0 ? q_heads / gb : kv_heads;
}

template <int DH, int G>
forge_status launch_dg(const AttnArgs& a, hipStream_t s) {
  const int yheads = a.q_heads / G;
  const SplitPlan pl = plan_splits(a.batch, yheads, a.kv_len);
  DecParams p;
  p.q = (const bf16*)a.q;
  p.k = (const bf16*)a.k;
  p.v = (const bf16*)a.v;
  p.part = (float*)a.workspace;
  p.out = (bf16*)a.out;
  p.q_heads = a.q_heads;
  p.kv_heads = yheads;
  p.passes = yheads / a.kv_heads;
  p.kv_len = a.kv_len;
  p.splits = pl.splits;
  p.rows_per_split = pl.rows_per_split;
  p.kv_bs = a.kv_batch_stride;
  p.kv_hs = a.kv_head_stride;
  p.scale_log2e = a.scale * 1.4426950408889634f;
  p.kv_pos = a.kv_pos;
  attn_decode_kernel<DH, G><<<dim3(p.splits, yheads, a.batch), NWAVES * 64, 0, s>>>(p);
  if (p.splits == 1) return launch_status();
  if (hipGetLastError() != hipSuccess) return FORGE_ERR_HIP;
  attn_decode_combine<DH><<<dim3(a.q_heads, a.batch), DH, 0, s>>>(p.part, (bf16*)a.out, a.q_heads,
                                                                  yheads, p.splits);
  return launch_status();
}

template <int DH>
forge_status launch_d(const AttnArgs& a, hipStream_t s) {
  switch (heads_per_block(a.q_heads / a.kv_heads)) {
    case 1: return launch_dg<DH, 1>(a, s);
    case 2: return launch_dg<DH, 2>(a, s);
    case 3: return launch_dg<DH, 3>(a, s);
    case 4: return launch_dg<DH, 4>(a, s);
    case 5: return launch_dg<DH, 5>(a, s);
    case 6: return launch_dg<DH, 6>(a, s);
    case 7: return launch_dg<DH, 7>(a, s);
    case 8: return launch_dg<DH, 8>(a, s);
    default: return launch_attn_simple_bf16(a, s);   // groups no pass count covers: vector-ALU path
  }
}

}  // namespace

size_t attn_decode_workspace_bytes(int batch, int q_heads, int kv_heads, int kv_len, int head_dim) {
  const int splits = splits_bound(batch, block_heads(q_heads, kv_heads), kv_len);
  if (splits == 1) return 0;       // one block per (kv head, sequence) writes the output itself
  return (size_t)batch * q_heads * splits * (head_dim + 2) * sizeof(float);
}

// ---- scratch that nobody allocates -----------------------------------------------------------
// For callers that can neither allocate nor bring a workspace: the split-KV partials go to a
// fixed array in the library's own device image.  Each GPU holds its own copy at its own address;
// the name below is only a host-side handle for it, so host code looks the address up once per
// device (with that device current) and passes the pointer on, as it would a caller's workspace.
constexpr size_t kStaticScratchBytes = (size_t)4 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;

size_t attn_decode_static_scratch_bytes() { return kStaticScratchBytes; }

forge_status attn_decode_static_scratch(void** ptr) {
  static std::atomic<void*> per_device[kMaxDevices];   // zero-initialised; filled on first use
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return FORGE_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return FORGE_ERR_UNSUPPORTED;
  void* p = per_device[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    // racing first calls look the same address up twice: harmless
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return FORGE_ERR_HIP;
    per_device[dev].store(p, std::memory_order_release);
  }
  *ptr = p;
  return FORGE_OK;
}

forge_status launch_attn_decode_bf16(const AttnArgs& a, hipStream_t s) {
  // what THIS launch writes (at most the bound the size query reports for any cache >= kv_len)
  const int splits = plan_splits(a.batch, block_heads(a.q_heads, a.kv_heads), a.kv_len).splits;
  const size_t need = splits == 1 ? 0 : (size_t)a.batch * a.q_heads * splits * (a.head_dim + 2) * sizeof(float);
  if (need > 0 && (a.workspace == nullptr || a.workspace_bytes < need)) return FORGE_ERR_WORKSPACE;
  if (a.head_dim == 64) return launch_d<64>(a, s);
  if (a.head_dim == 128) return launch_d<128>(a, s);
  return FORGE_ERR_UNSUPPORTED;
}

}  // namespace forge
