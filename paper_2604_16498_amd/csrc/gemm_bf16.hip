// bf16 fused linear on the gfx950 matrix cores:  y = act(x . w^T + bias) (+ residual).
//
// x [M,K] and w [N,K] are both K-contiguous, which is exactly what v_mfma_f32_32x32x16_bf16
// wants: each lane feeds 8 consecutive k of one row of either operand (one 128-bit read), so no
// operand is ever transposed.  Accumulation is fp32; bias, activation and the residual are
// applied to the accumulator and the result is rounded to bf16 once, at the store.
//
// Two kernels share the tiling (a block of WM x WN waves owns a BM x BN tile of y, each wave
// (BM/WM) x (BN/WN) as TM x TN accumulators of 32 x 32, K walked in slabs of 64):
//
//  * gemm_bf16_pers_kernel -- the fast path (K % 64 == 0, output rows 16-byte aligned, operands
//    below 4 GB).  Slabs go HBM -> LDS directly (global_load_lds_dwordx4: each wave-wide load drops
//    1 KB into LDS at lane*16, no staging registers, no LDS store instructions) into a 2-stage
//    ring: the loads of slab k+1 are in flight while slab k is multiplied; one barrier per slab.
//    w is the MFMA A operand and x the B operand, so an accumulator holds D[n, m]: a lane owns
//    ONE output row m and, after a permlane32 swap of register groups, two runs of 8 consecutive
//    columns.  The finished tile is transposed through LDS into whole output rows.  Blocks are
//    persistent: see the comment at the kernel.
//  * gemm_bf16_generic_kernel -- any K % 8 == 0 and any row stride: HBM -> registers -> LDS
//    double buffering with zero fill of the K tail, x as the A operand, element stores.
//
// LDS layout (both): a slab row is 64 bf16 = 8 chunks of 16 B; chunk c of row r sits at chunk
// position c ^ ((r >> 1) & 7).  A fragment read has lanes 0-31 on 32 consecutive rows at one
// logical chunk; with the swizzle any 16 consecutive rows hit 16 distinct 16-byte bank groups,
// so the 128-bit reads are conflict free.  The direct loads apply the inverse mapping on the
// global side: the lane that lands on (row, position p) fetches logical chunk p ^ f(row).
//
// SwiGLU: the w slab of a block is half gate rows and half up rows of the SAME output columns,
// arranged so that accumulator (., t) is the gate and (., t + TN/2) the up projection of one
// column block; the epilogue writes silu(gate) * up and no extra accumulators are needed.
//
// Work-group order: blocks are dealt round-robin over the 8 XCDs (each with its own L2), so every
// XCD gets one contiguous run of tiles, and tiles are numbered in groups of 8 tile rows,
// column-major inside a group, so that the tiles resident in one XCD at a time share x and w
// panels in that L2.
//
// M <= 64 (decode): the weight is streamed once by gemm_bf16_wstream_kernel (128 or 256 weight
// rows per block, K split over grid.y to about one block per CU), fp32 partials, and fixed-order
// reduce kernels that carry the epilogue (and, inside a decoder layer, RoPE or the following norm).
// Prompt-sized M with few tiles and a long K: the tile kernel itself walks (k range, tile) items.
#include <type_traits>
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
  return basep + (((int64_t)b * sp.kv_heads + h) * sp.kv_cap + seq_position(sp.pos, b, sp.pos0) + s) * dh + nn % dh;
}

struct GemmParams {
  const bf16* x;
  const bf16* w;
  const bf16* bias;
  const bf16* residual;
  bf16* y;
  int M, N, K;        // N: output columns
  int ldy;            // row stride of y and residual (elements)
  int tiles_m, tiles_n;
  int k_per_split;    // split-K: k range of one block (multiple of 64); otherwise >= K
  int splits;         // split-K in the persistent kernel: number of k ranges
  float* part;        // split-K: fp32 partial sums [splits, M, N]
  size_t part_bytes;  // bytes behind part
  QkvSplit sp;
  NormTail nt;        // nt.y_norm == nullptr: none
  const int8_t* w8;     // weight-only int8 (M <= 64 streaming path): [N, K] bytes; w is NULL then
  const float* wscale;  // one scale per weight row, applied to the reduced sum before the bias
  int row0;             // row of the whole problem that row 0 of this launch is (head split only)
  int col0;             // column of the whole problem that column 0 of this launch is (head split only)
};

// MODE_QKV_ROPE: the head split with the rotary embedding applied in the epilogue (prompt-sized
// problems; the decode-sized ones rotate in their reduce kernel)
enum Mode { MODE_PLAIN = 0, MODE_QKV = 1, MODE_SPLITK = 2, MODE_QKV_ROPE = 3 };

template <int BM, int BN, int WM, int WN, int ACT, int MODE>
__global__ __launch_bounds__(WM* WN * 64) void gemm_bf16_generic_kernel(GemmParams p) {
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
        const float ws1 = p.wscale != nullptr ? p.wscale[n] : 1.0f;
        const float ws2 = SWIGLU && p.wscale != nullptr ? p.wscale[n + N] : 1.0f;
        float val = acc[i][j][v] * ws1 + bv;
        if (SWIGLU) val = silu_f(val) * (acc[i][SWIGLU ? j + TN / 2 : j][v] * ws2 + bv2);
        else val = apply_act<ACT>(val);
        if (MODE == MODE_QKV) {
          *split_dst_bf16(p.sp, p.row0 + m, n) = (bf16)val;
        } else {
          if (p.residual != nullptr) val += (float)p.residual[(int64_t)m * p.ldy + n];
          p.y[(int64_t)m * p.ldy + n] = (bf16)val;
        }
      }
    }
  }
}

typedef __attribute__((address_space(3))) void lds_void;

// Block barrier for data exchanged through LDS only: this wave's LDS traffic has completed
// (lgkmcnt 0), vector-memory loads and stores stay in flight (__syncthreads would drain them too).
__device__ inline void lds_barrier() {
  __builtin_amdgcn_s_waitcnt(0xc07f);
  __builtin_amdgcn_s_barrier();
}

// Persistent fast path: one block per LDS/register slot of the chip walks over a strided list
// of tiles.
//
// Epilogue: a lane's own 16-byte runs sit on 32 different rows, and written that way the stores
// reach a fraction of the write bandwidth.  So the finished tile is rounded to bf16 and
// transposed through LDS (the operand ring is dead by then) into whole output rows: 16-byte chunk
// c of staged row r sits at position c ^ (r mod chunks-per-row), which makes both the
// accumulator-side accesses (32 rows, one chunk) and the row-side accesses (one row, all chunks)
// bank-conflict free.  A residual tile is fetched INTO the staging area first (direct-to-LDS,
// whole rows); each lane adds its runs in fp32 and overwrites them with the rounded result, so
// there is still one rounding, at the end.
//
// Overlap across tiles:
//  * the first slab of the next tile is requested BEFORE the epilogue of the current one (into
//    ring buffer 0; the tile is staged through buffer 1, in row halves if it is larger than a
//    buffer), so its latency hides behind the epilogue;
//  * a tile that is staged in one pass (128 x 128, and the SwiGLU 256 x 128) is then parked in
//    registers (16 or 32 per lane) and the next tile's k loop issues a few of these row stores per slab
//    instead of all blocks of the chip storing at once.  The vector-memory counter retires in
//    order, so the wait for slab k tolerates exactly the stores issued after its loads
//    (STORES_PER_IT).  Stores of tiles that touch the matrix edge are predicated, hence not
//    countable, and are issued at once.  The 256 x 256 tile has no registers to spare (its
//    accumulators are half the file) and stores at once, pass by pass.
//
// Tiles: XCD x (blocks with id = x mod 8) owns a contiguous run of the grouped tile order, its
// blocks stride through that run together, so at any time one L2 serves a compact patch of y.
template <int BM, int BN, int WM, int WN, int ACT, int MODE>
__global__ __launch_bounds__(WM* WN * 64) void gemm_bf16_pers_kernel(GemmParams p) {
  constexpr bool SPLITK = MODE == MODE_SPLITK;   // raw fp32 partial tiles over grid-wide k ranges
  constexpr bool QKV = MODE == MODE_QKV || MODE == MODE_QKV_ROPE;
  // ROPE: the w slab rows are arranged so that accumulator (., 0) holds a 32-column block of the
  // FIRST half of a head and accumulator (., 1) the block dh/2 columns further on: a lane then owns
  // both members of every rotation pair (i, i + dh/2) of its row and rotates them in fp32, with
  // cos / sin from a table indexed by (row of the sequence, i), before the single rounding.
  constexpr bool ROPE = MODE == MODE_QKV_ROPE;
  static_assert(!ROPE || (ACT == FORGE_ACT_NONE && BN / WN / 32 == 2), "rotation pairs two accumulators");
  static_assert(!SPLITK || ACT == FORGE_ACT_NONE, "the reduce kernel carries the epilogue");
  constexpr int NW = WM * WN;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr bool SWIGLU = ACT == FORGE_ACT_SWIGLU;
  constexpr int BN_OUT = SWIGLU ? BN / 2 : BN;
  constexpr int TN_OUT = SWIGLU ? TN / 2 : TN;
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;
  constexpr int IA = BM / 8 / NW, IB = BN / 8 / NW;   // wave-wide 1 KB loads per wave per slab
  static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "tile / wave mismatch");
  static_assert(!SWIGLU || TN % 2 == 0, "SwiGLU pairs accumulators");
  // output staging
  constexpr int NCH = BN_OUT / 8;                     // 16-byte chunks per output row
  constexpr int RPL = 64 / NCH;                       // rows per wave-wide 1 KB access
  constexpr int NPASS = (BM * BN_OUT * 2 + STAGE - 1) / STAGE;   // staging passes (row ranges)
  constexpr int BMP = BM / NPASS;                     // rows per pass
  constexpr int NITP = BMP / RPL / NW;                // wave-wide accesses per wave and pass
  constexpr int NIT = NITP * NPASS;                   // 16-byte row pieces per lane and tile
  // a tile staged in one pass is parked in registers; the large tile (two passes, accumulators
  // alone take half the register file) is stored at once, pass by pass
  constexpr bool PARK = NPASS == 1 && !SPLITK;
  constexpr int NPARK = PARK ? NIT : 1;
  constexpr int STORE_ITS = !PARK ? 1 : (NPARK < 8 ? NPARK : 8);   // k iterations that carry stores
  constexpr int STORES_PER_IT = PARK ? NPARK / STORE_ITS : 0;
  static_assert(BM % NPASS == 0 && BMP * BN_OUT * 2 <= STAGE, "a pass must fit one ring buffer");
  static_assert(64 % NCH == 0 && BMP % (RPL * NW) == 0 && BMP % 32 == 0 && NCH <= 32, "staging plan");
  static_assert(!PARK || (NPARK % STORE_ITS == 0 && STORES_PER_IT <= 3), "store plan");
  extern __shared__ __attribute__((aligned(16))) char smem[];   // [A0 | B0 | A1 | B1]
  char* const stg = smem + STAGE;                     // staging area = ring buffer 1

  // (the wave index is held in a scalar register: everything derived from it alone -- the LDS
  // destinations of the direct loads above all -- is then computed on the scalar unit)
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int fr = lane & 31, fh = lane >> 5;
  const int M = p.M, N = p.N, K = p.K;

  // ---- this block's work items: tiles, or (k range, tile) pairs when K is split -----------------
  // (k range major, so that the items resident at one time are neighbouring tiles of one range)
  const int ntiles = p.tiles_m * p.tiles_n;
  const int nitems = SPLITK ? ntiles * p.splits : ntiles;
  const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3, bpx = gridDim.x >> 3;
  const int lo = xcd * (nitems >> 3) + min(xcd, nitems & 7);
  const int cnt = (nitems >> 3) + (xcd < (nitems & 7) ? 1 : 0);
  if (idx >= cnt) return;                             // uniform over the block
  auto k_range = [&](int item, int& k_begin, int& n_slabs) {
    const int z = SPLITK ? item / ntiles : 0;
    k_begin = z * p.k_per_split;
    n_slabs = (min(K, k_begin + p.k_per_split) - k_begin) / BK;
  };
  constexpr int GROUP_M = 8;
  auto tile_origin = [&](int item, int& m0, int& n0) {
    const int tile = SPLITK ? item % ntiles : item;
    const int in_group = GROUP_M * p.tiles_n;
    const int group = tile / in_group;
    const int first_m = group * GROUP_M;
    const int gsz = min(p.tiles_m - first_m, GROUP_M);
    m0 = (first_m + (tile % in_group) % gsz) * BM;
    n0 = ((tile % in_group) / gsz) * BN_OUT;
  };

  // ROPE: 32-column block of the tile that accumulator t of wave column wcol holds.  A head is
  // 2 * hb blocks wide (hb = dh / 64: 1 or 2); wave columns go over (head, block of its first
  // half), and t = 1 is the partner block hb further on.  dh = 64 gives the natural order.
  const int rope_hb = ROPE ? p.sp.head_dim / 64 : 1;
  auto rope_block = [&](int wcol, int t) { return (wcol / rope_hb) * (2 * rope_hb) + wcol % rope_hb + t * rope_hb; };

  // ---- direct-to-LDS copy plan, sources as 32-bit byte offsets ------------------------------------
  // wave-wide load i of this wave fills LDS rows (i*NW + wave)*8 .. +8 of a slab (1 KB at
  // lane*16): lane -> (row = base + lane/8, position = lane%8) -> logical chunk = position ^ f(row)
  unsigned a_off[IA], b_off[IB];
  auto set_sources = [&](int m0, int n0) {
#pragma unroll
    for (int i = 0; i < IA; ++i) {
      const int r = (i * NW + wave) * 8 + (lane >> 3);
      const int c = (lane & 7) ^ ((r >> 1) & 7);
      a_off[i] = ((unsigned)min(m0 + r, M - 1) * (unsigned)K + c * 8) * 2u;
    }
#pragma unroll
    for (int i = 0; i < IB; ++i) {
      const int r = (i * NW + wave) * 8 + (lane >> 3);
      const int c = (lane & 7) ^ ((r >> 1) & 7);
      int gn;
      if (SWIGLU) {
        const int wcol = r / (32 * TN), t = (r / 32) % TN, rr = r % 32;
        const int col = n0 + (wcol * (TN / 2) + t % (TN / 2)) * 32 + rr;
        gn = min(col, N - 1) + (t >= TN / 2 ? N : 0);
      } else if (ROPE) {
        // wave column wcol, accumulator t -> 32-column block of the tile (see rope_block)
        const int wcol = r / 64, t = (r / 32) & 1, rr = r % 32;
        gn = min(n0 + rope_block(wcol, t) * 32 + rr, N - 1);
      } else {
        gn = min(n0 + r, N - 1);
      }
      b_off[i] = ((unsigned)gn * (unsigned)K + c * 8) * 2u;
    }
  };
  auto issue = [&](int k0, int buf) {
    char* sa = smem + buf * STAGE;
    char* sb = sa + A_BYTES;
    // uniform base + 32-bit lane offset: the offsets are pinned so that they are not turned into
    // eight running 64-bit pointers (two registers each, live across the whole loop)
    const char* xb = reinterpret_cast<const char*>(p.x);
    const char* wb = reinterpret_cast<const char*>(p.w);
    const unsigned kb = (unsigned)k0 * 2u;
#pragma unroll
    for (int i = 0; i < IA; ++i) {
      unsigned o = a_off[i] + kb;
      asm volatile("" : "+v"(o));
      __builtin_amdgcn_global_load_lds((const void*)(xb + o), (lds_void*)(sa + (i * NW + wave) * 1024), 16, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < IB; ++i) {
      unsigned o = b_off[i] + kb;
      asm volatile("" : "+v"(o));
      __builtin_amdgcn_global_load_lds((const void*)(wb + o), (lds_void*)(sb + (i * NW + wave) * 1024), 16, 0, 0);
    }
  };

  floatx16 acc[TM][TN];
  auto compute = [&](int buf, int ks0, int ks1) {
    const char* sa = smem + buf * STAGE;
    const char* sb = sa + A_BYTES;
#pragma unroll
    for (int ks = ks0; ks < ks1; ++ks) {
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
        for (int j = 0; j < TN; ++j)   // D[n, m]: w fragment is the A operand
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
  };

  // ---- output pieces ---------------------------------------------------------------------------
  // piece `it` of a tile: tile row and logical chunk of this lane (pass-major, the staging plan)
  auto piece_row = [&](int it) { return (it / NITP) * BMP + ((it % NITP) * NW + wave) * RPL + lane / NCH; };
  auto piece_chunk = [&](int row) { return (lane % NCH) ^ (row & (NCH - 1)); };
  // head split: n / head_dim by multiplication (exact for n * head_dim < 2^32), (batch, position)
  // of a row from those of the tile's first row
  const unsigned dh_magic = QKV ? 0xffffffffu / (unsigned)p.sp.head_dim + 1u : 0u;
  auto dst_of = [&](int t_b, int t_s, int m0_, int row, int n) -> bf16* {
    if (QKV) {
      // 8 consecutive columns never straddle a head (head_dim % 8 == 0, n % 8 == 0)
      n += p.col0;
      int sb_ = t_b, ss_ = t_s + row;
      while (ss_ >= p.sp.q_len) { ss_ -= p.sp.q_len; ++sb_; }
      const int dh = p.sp.head_dim, nq = p.sp.q_heads * dh, nkv = p.sp.kv_heads * dh;
      const bool is_q = n < nq, is_k = n < nq + nkv;
      const int nn = is_q ? n : (is_k ? n - nq : n - nq - nkv);
      const int h = (int)__umulhi((unsigned)nn, dh_magic);
      const int d = nn - h * dh;
      if (is_q) return (bf16*)p.sp.q + (((int64_t)sb_ * p.sp.q_heads + h) * p.sp.q_len + ss_) * dh + d;
      return (bf16*)(is_k ? p.sp.k_cache : p.sp.v_cache) +
             (((int64_t)sb_ * p.sp.kv_heads + h) * p.sp.kv_cap + seq_position(p.sp.pos, sb_, p.sp.pos0) + ss_) * dh + d;
    }
    return p.y + (int64_t)(m0_ + row) * p.ldy + n;
  };
  u32x4 parked[NPARK];
  bool pending = false;                  // uniform
  bool flushed = false;                  // uniform: the last NIT vector-memory operations of this wave
                                         // are the unpredicated stores of the previous tile
  int pm0 = 0, pn0 = 0, pb = 0, ps = 0;  // parked tile: origin, (batch, position) of its first row
  // interior tiles only: every piece is a full, valid 16-byte store
  auto store_parked = [&](int first, int count) {
#pragma unroll
    for (int it = 0; it < NPARK; ++it) {
      if (it < first || it >= first + count) continue;
      const int row = piece_row(it);
      *reinterpret_cast<u32x4*>(dst_of(pb, ps, pm0, row, pn0 + piece_chunk(row) * 8)) = parked[it];
    }
  };

  auto runs_of = [&](const floatx16& a, float (&run)[2][8]) {
#pragma unroll
    for (int gp = 0; gp < 2; ++gp)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(a[4 * gp + r]),
                                                   __float_as_uint(a[4 * (gp + 2) + r]), false, false);
        run[gp][r] = __uint_as_float(sw[0]);
        run[gp][4 + r] = __uint_as_float(sw[1]);
      }
  };
  const bool has_res = MODE == MODE_PLAIN && p.residual != nullptr;

  // The two waves that share a SIMD (w and w + 4) start their copies of the next slab half a slab
  // apart: a wave sits in the issue of its direct-to-LDS loads for several hundred cycles, and this
  // way the other wave of the SIMD is multiplying meanwhile instead of issuing its own.
  constexpr bool STAG = NW == 8;
  constexpr int STAG_AT = BK / 32;
  const bool late = STAG && __builtin_amdgcn_readfirstlane(wave) >= NW / 2;
  int tt = idx, m0, n0, kb0, nk;
  tile_origin(lo + tt, m0, n0);
  k_range(lo + tt, kb0, nk);
  set_sources(m0, n0);
  if (nk > 0) issue(kb0, 0);
  for (;;) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // ---- k loop: slab kt multiplied while slab kt+1 loads and parked rows drain -----------------
    auto k_loop = [&](auto late_c) {
      constexpr bool LATE = decltype(late_c)::value;
      for (int kt = 0; kt < nk; ++kt) {
        // younger than the loads of slab kt: only the stores issued right after them
        if (PARK && pending && kt >= 1 && kt <= STORE_ITS) __builtin_amdgcn_s_waitcnt(0x0f70 | STORES_PER_IT);
        else if (!PARK && kt == 0 && flushed) __builtin_amdgcn_s_waitcnt(0x0f70 | (NIT & 0xf) | ((NIT >> 4) << 14));
        else __builtin_amdgcn_s_waitcnt(0x0f70);
        __builtin_amdgcn_s_barrier();   // slab kt is in LDS for everyone; buffer (kt+1)&1 is free
        if (LATE) {
          compute(kt & 1, 0, STAG_AT);
          __builtin_amdgcn_sched_barrier(0);
        }
        if (kt + 1 < nk) issue(kb0 + (kt + 1) * BK, (kt + 1) & 1);
        __builtin_amdgcn_sched_barrier(0);   // the wait above counts on loads first, stores second
        if (PARK && pending && kt < STORE_ITS) {
#pragma unroll
          for (int c = 0; c < STORE_ITS; ++c)
            if (c == kt) store_parked(c * STORES_PER_IT, STORES_PER_IT);
        }
        __builtin_amdgcn_sched_barrier(0);
        compute(kt & 1, LATE ? STAG_AT : 0, BK / 16);
      }
    };
    if (STAG && late) k_loop(std::true_type{});
    else k_loop(std::false_type{});
    if (PARK && pending && nk < STORE_ITS) {
#pragma unroll
      for (int c = 0; c < STORE_ITS; ++c)
        if (c >= nk) store_parked(c * STORES_PER_IT, STORES_PER_IT);
    }
    pending = false;

    // ---- next tile's first slab, then the epilogue of this one ------------------------------------
    const int next = tt + bpx;
    const bool has_next = next < cnt;
    int nm0 = 0, nn0 = 0, nkb0 = 0, nnk = 0;
    lds_barrier();                    // every wave is done with the operand slabs
    if (has_next) {
      tile_origin(lo + next, nm0, nn0);
      k_range(lo + next, nkb0, nnk);
      set_sources(nm0, nn0);
      if (nnk > 0) issue(nkb0, 0);
    }
    if (SPLITK) {
      // raw partial sums of this k range: lane = row m, two runs of 8 columns per accumulator
      const int z = (lo + tt) / ntiles;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int m = m0 + (wm * TM + i) * 32 + fr;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          float run[2][8];
          runs_of(acc[i][j], run);
#pragma unroll
          for (int gp = 0; gp < 2; ++gp) {
            const int n = n0 + (wn * TN + j) * 32 + 16 * fh + 8 * gp;
            if (m >= M || n >= N) continue;       // N % 8 == 0 (host): a run is all in or all out
            Vec8<float>::store(p.part + ((int64_t)z * M + m) * N + n, run[gp]);
          }
        }
      }
      if (!has_next) break;
      tt = next; m0 = nm0; n0 = nn0; kb0 = nkb0; nk = nnk;
      continue;
    }
    const bool interior = m0 + BM <= M && n0 + BN_OUT <= N;
    int tb = 0, ts = 0;
    if (QKV) { tb = m0 / p.sp.q_len; ts = m0 - tb * p.sp.q_len; }
#pragma unroll
    for (int pass = 0; pass < NPASS; ++pass) {
      if (pass > 0) lds_barrier();    // the previous pass has been read out
      if (has_res) {
        // the residual rows of this pass land in the staging area first (whole rows, swizzled)
#pragma unroll
        for (int itp = 0; itp < NITP; ++itp) {
          const int row = piece_row(pass * NITP + itp);
          const int gm = min(m0 + row, M - 1);
          // a chunk that starts inside the row lies inside its padded stride (ldy % 8 == 0, host);
          // chunks wholly past the end fetch something valid, unused
          int gn = n0 + piece_chunk(row) * 8;
          if (gn >= N) gn = 0;
          __builtin_amdgcn_global_load_lds((const void*)(p.residual + (int64_t)gm * p.ldy + gn),
                                           (lds_void*)(stg + (itp * NW + wave) * 1024), 16, 0, 0);
        }
        __builtin_amdgcn_s_waitcnt(0x0f70);
        lds_barrier();
      }
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int rl = (wm * TM + i) * 32 + fr;       // row inside the tile
        if (rl / BMP != pass) continue;               // uniform over the wave
        const int rp = rl - pass * BMP;               // row inside the pass
        if constexpr (ROPE) {
          // this lane's row of the sequence: the table row of its angles
          int ss_ = ts + rl;
          while (ss_ >= p.sp.q_len) ss_ -= p.sp.q_len;
          const int dh = p.sp.head_dim, half = dh / 2;
          const float* tab = p.sp.rope_tab + (int64_t)ss_ * dh;      // [half] x (cos, sin)
          float lo[2][8], hi[2][8];
          runs_of(acc[i][0], lo);
          runs_of(acc[i][1], hi);
          const int blk = rope_block(wn, 0);
#pragma unroll
          for (int gp = 0; gp < 2; ++gp) {
            const int cl = blk * 4 + 2 * fh + gp, ch = cl + rope_hb * 4;   // chunks of the pair's two halves
            const int n_lo = n0 + cl * 8, n_hi = n0 + ch * 8;
            if (p.wscale != nullptr && n_hi + 8 <= N) {   // dequantised int8 weight: one scale per weight row
#pragma unroll
              for (int e = 0; e < 8; ++e) {
                lo[gp][e] *= p.wscale[n_lo + e];
                hi[gp][e] *= p.wscale[n_hi + e];
              }
            }
            if (p.bias != nullptr && n_hi + 8 <= N) {     // N % 8 == 0 (host): a chunk is all in or all out
              float bb[8];
              Vec8<bf16>::load(p.bias + n_lo, bb);
#pragma unroll
              for (int e = 0; e < 8; ++e) lo[gp][e] += bb[e];
              Vec8<bf16>::load(p.bias + n_hi, bb);
#pragma unroll
              for (int e = 0; e < 8; ++e) hi[gp][e] += bb[e];
            }
            if (p.col0 + n_lo < (p.sp.q_heads + p.sp.kv_heads) * dh) {    // q and k heads rotate, v heads do not
              const int d0 = (cl * 8) & (half - 1);              // pair index of the chunk's first column
              float cs[16];
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                const floatx4 t4 = *reinterpret_cast<const floatx4*>(tab + 2 * d0 + 4 * e);
                cs[4 * e] = t4[0]; cs[4 * e + 1] = t4[1]; cs[4 * e + 2] = t4[2]; cs[4 * e + 3] = t4[3];
              }
#pragma unroll
              for (int e = 0; e < 8; ++e) {
                const float c = cs[2 * e], sn = cs[2 * e + 1], a = lo[gp][e], d = hi[gp][e];
                lo[gp][e] = a * c - d * sn;
                hi[gp][e] = d * c + a * sn;
              }
            }
            Vec8<bf16>::store(reinterpret_cast<bf16*>(stg + (rp * NCH + (cl ^ (rp & (NCH - 1)))) * 16), lo[gp]);
            Vec8<bf16>::store(reinterpret_cast<bf16*>(stg + (rp * NCH + (ch ^ (rp & (NCH - 1)))) * 16), hi[gp]);
          }
          continue;
        }
#pragma unroll
        for (int j = 0; j < TN_OUT; ++j) {
          float run[2][8], run2[2][8];
          runs_of(acc[i][j], run);
          if (SWIGLU) runs_of(acc[i][SWIGLU ? j + TN / 2 : j], run2);
#pragma unroll
          for (int gp = 0; gp < 2; ++gp) {
            const int cl = (wn * TN_OUT + j) * 4 + 2 * fh + gp;   // chunk inside the tile row
            const int n = n0 + cl * 8;
            // the last chunk of a row may be ragged (N % 8 != 0, never with SwiGLU: host); its
            // columns past N are computed on whatever the padding holds and never stored
            const bool in = n + 8 <= N;
            float o[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = run[gp][e];
            if (p.wscale != nullptr) {      // dequantised int8 weight: one scale per weight row
#pragma unroll
              for (int e = 0; e < 8; ++e) {
                const int ne = min(n + e, N - 1);
                o[e] *= p.wscale[ne];
                if (SWIGLU) run2[gp][e] *= p.wscale[N + ne];
              }
            }
            if (p.bias != nullptr && in) {
              float bb[8];
              Vec8<bf16>::load(p.bias + n, bb);
#pragma unroll
              for (int e = 0; e < 8; ++e) o[e] += bb[e];
              if (SWIGLU) {
                Vec8<bf16>::load(p.bias + N + n, bb);
#pragma unroll
                for (int e = 0; e < 8; ++e) run2[gp][e] += bb[e];
              }
            } else if (!SWIGLU && p.bias != nullptr && n < N) {
#pragma unroll
              for (int e = 0; e < 8; ++e)
                if (n + e < N) o[e] += (float)p.bias[n + e];
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = SWIGLU ? silu_f(o[e]) * run2[gp][e] : apply_act<ACT>(o[e]);
            bf16* slot = reinterpret_cast<bf16*>(stg + (rp * NCH + (cl ^ (rp & (NCH - 1)))) * 16);
            if (has_res && n < N) {
              float rr[8];
              Vec8<bf16>::load(slot, rr);
#pragma unroll
              for (int e = 0; e < 8; ++e) o[e] += rr[e];
            }
            Vec8<bf16>::store(slot, o);
          }
        }
      }
      lds_barrier();
      if (interior && PARK) {
#pragma unroll
        for (int itp = 0; itp < NITP; ++itp)
          parked[itp] = *reinterpret_cast<const u32x4*>(stg + (itp * NW + wave) * 1024 + lane * 16);
      } else if (interior) {
#pragma unroll
        for (int itp = 0; itp < NITP; ++itp) {
          const int row = piece_row(pass * NITP + itp);
          *reinterpret_cast<u32x4*>(dst_of(tb, ts, m0, row, n0 + piece_chunk(row) * 8)) =
              *reinterpret_cast<const u32x4*>(stg + (itp * NW + wave) * 1024 + lane * 16);
        }
      } else {
        // edge tile: predicated stores straight from the staging area
#pragma unroll 1
        for (int itp = 0; itp < NITP; ++itp) {
          const int row = pass * BMP + (itp * NW + wave) * RPL + lane / NCH;
          const int m = m0 + row, n = n0 + piece_chunk(row) * 8;
          if (m >= M || n >= N) continue;
          const u32x4 v = *reinterpret_cast<const u32x4*>(stg + (itp * NW + wave) * 1024 + lane * 16);
          bf16* dst = dst_of(tb, ts, m0, row, n);
          if (n + 8 <= N) {
            *reinterpret_cast<u32x4*>(dst) = v;
          } else {
            const bf16* src = reinterpret_cast<const bf16*>(stg + (itp * NW + wave) * 1024 + lane * 16);
            for (int e = 0; n + e < N; ++e) dst[e] = src[e];
          }
        }
      }
    }
    flushed = !PARK && interior && !has_res;
    if (interior && PARK) {
      pending = true;
      pm0 = m0;
      pn0 = n0;
      pb = tb;
      ps = ts;
    }
    if (!has_next) break;
    // the staging area is ring buffer 1: the barrier of the next k loop's first iteration comes
    // before anything is loaded into it
    tt = next;
    m0 = nm0;
    n0 = nn0;
    kb0 = nkb0;
    nk = nnk;
  }
  if (PARK && pending) store_parked(0, NPARK);
}

// Weight-streaming kernel for M <= 64 (decode): HBM-bound, every weight byte is read once.
// A block owns BN weight rows (output columns) and one k range.  Weight slabs (BN x 64) and
// activation slabs (64 x 64, L2 resident) both arrive by direct-to-LDS loads, but in SEPARATE rings
// filled by different waves: the first half of the waves only issue weight loads, the second half
// only activation loads.  The vector-memory counter retires in order within a wave, so mixing the
// two streams in one wave would tie the HBM stream to the depth of the L2 stream.
//
// What bounds this kernel is the number of requests a CU's vector-memory pipeline keeps in
// flight, and an activation line (an L2 hit) occupies a slot just like a weight line (an HBM
// miss): with BN = 64 half of all requests are activation re-reads and the weight stream gets
// half of the pipeline.  Wider blocks re-read the activations less often per weight byte
// (1 : 2 at BN = 128, 1 : 4 at BN = 256); the launcher picks the widest block that still gives
// every CU work.  All waves multiply: a wave owns 32 weight rows and both halves of the
// activation rows.  Output: fp32 partial sums D[n, m] for the fixed-order split-K reduce.
template <int BN, bool W8>
struct WStream {
  static constexpr int NWV = BN >= 256 ? 8 : 4;            // waves per block
  static constexpr int NG = BN / 32;                       // 32-row groups of weight rows
  static constexpr int TMW = NG >= NWV ? 2 : 1;            // activation halves per wave
  static constexpr int NWL = NWV / 2, NXL = NWV - NWL;     // loader waves per stream
  // A weight row of a slab is 128 bytes either way: 64 bf16 or 128 int8 elements.  What an
  // iteration costs is mostly fixed (barrier, issue of the loads), so the int8 variant keeps the
  // weight bytes per iteration and doubles the k extent instead of halving the bytes.
  static constexpr int BKS = W8 ? 2 * BK : BK;             // k elements per slab
  static constexpr int LPW_W = BN / 8 / NWL;               // wave-wide 1 KB loads per loader and slab
  static constexpr int SLAB_W = BN * 128, SLAB_X = 64 * BKS * 2;
  static constexpr int LPW_X = SLAB_X / 1024 / NXL;
  static constexpr int WS_W = (BN == 128 || W8) ? 3 : 4;   // weight ring depth
  static constexpr int WS_X = W8 ? 2 : 3;                  // activation ring depth
  static constexpr int SMEM = WS_W * SLAB_W + WS_X * SLAB_X;
  static_assert(NG * (2 / TMW) == NWV, "waves cover the block tile");
  static_assert(SMEM <= 160 * 1024, "fits the LDS of a CU");
};

// 8 signed bytes -> 8 bf16 (exact: |q| <= 127 has 7 significant bits)
__device__ inline bf16x8 cvt_i8x8_bf16(u32x2 v) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int b = (int)(int8_t)((v[e >> 2] >> (8 * (e & 3))) & 0xff);
    r[e] = (bf16)(float)b;
  }
  return r;
}

// FACT < 0: fp32 partial sums for the split-K reduce (any number of k ranges).
// FACT >= 0 (an activation code): ONE k range, and the block finishes its outputs itself -- weight
// scale, bias, activation, residual, one rounding -- with the arithmetic of the reduce kernel, so
// the result is bit-identical to partials + reduce over one range; no partial planes, no second
// launch.  For the gated activation a block owns 64 gate rows and the 64 up rows that pair with
// them (waves 0-1 and 2-3; the up halves cross over through LDS once the ring is dead).
template <int BN, bool W8, int FACT>
__global__ __launch_bounds__((WStream<BN, W8>::NWV * 64)) void gemm_bf16_wstream_kernel(GemmParams p) {
  using C = WStream<BN, W8>;
  constexpr bool FUSE = FACT >= 0;
  constexpr bool GATED = FACT == FORGE_ACT_SWIGLU;
  static_assert(!FUSE || (BN == 128 && C::TMW == 2), "the fused finish is written for 4 waves of 32 x 64");
  extern __shared__ __attribute__((aligned(16))) char smem[];   // [W ring | x ring]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wn = wave % C::NG, wm0 = wave / C::NG;   // wm0: the activation half of a TMW == 1 wave
  const int fr = lane & 31, fh = lane >> 5;
  const int M = p.M, N = p.N, K = p.K;               // N: weight rows (twice the outputs when GATED)
  const int NO = GATED ? N / 2 : N;                  // output columns
  const int n0 = blockIdx.x * (GATED ? BN / 2 : BN); // first output column (FUSE) / weight row of the block
  // weight row behind row r of the block's slab
  auto w_row = [&](int r) {
    if (GATED) return r < BN / 2 ? min(n0 + r, NO - 1) : NO + min(n0 + r - BN / 2, NO - 1);
    return min(n0 + r, N - 1);
  };
  const bool w_loader = wave < C::NWL;        // wave-uniform role
  const int lw = w_loader ? wave : wave - C::NWL;   // index among the loaders of a stream

  // loader plan: wave-wide load i of loader lw fills slab rows (i * loaders + lw)*8 .. +8
  constexpr int LPW_MAX = C::LPW_W > C::LPW_X ? C::LPW_W : C::LPW_X;
  // (the activation slab of the int8 variant is two 64 x 64 sub-slabs, 8 loads each)
  constexpr int WESZ = W8 ? 1 : 2;     // bytes per weight element
  const char* src[LPW_MAX];
#pragma unroll
  for (int i = 0; i < LPW_MAX; ++i) {
    const int j = i * (w_loader ? C::NWL : C::NXL) + lw;     // which 1 KB piece of the slab
    const int r = (w_loader ? j : j % 8) * 8 + (lane >> 3);
    const int c = (lane & 7) ^ ((r >> 1) & 7);
    src[i] = w_loader ? (W8 ? (const char*)p.w8 : (const char*)p.w) + ((int64_t)w_row(r) * K * WESZ + c * 16)
                      : (const char*)(p.x + (int64_t)min(r, M - 1) * K + (j / 8) * BK + c * 8);
  }
  const int k_begin = blockIdx.y * p.k_per_split;
  const int k_end = min(K, k_begin + p.k_per_split);
  const int nk = (k_end - k_begin) / C::BKS;
  char* const xring = smem + C::WS_W * C::SLAB_W;

  // slab kt of this wave's stream; past the end the last slab is re-loaded into its own buffer
  // (same bytes, harmless), so every iteration issues the same number of loads per wave and the
  // in-order wait count is a constant per role
  auto issue = [&](int kt) {
    const int k = min(kt, nk - 1);
    if (w_loader) {
      char* dst = smem + (k % C::WS_W) * C::SLAB_W;
#pragma unroll
      for (int i = 0; i < C::LPW_W; ++i)
        __builtin_amdgcn_global_load_lds((const void*)(src[i] + (int64_t)(k_begin + k * C::BKS) * WESZ),
                                         (lds_void*)(dst + (i * C::NWL + lw) * 1024), 16, 0, 0);
    } else {
      char* dst = xring + (k % C::WS_X) * C::SLAB_X;
#pragma unroll
      for (int i = 0; i < C::LPW_X; ++i)
        __builtin_amdgcn_global_load_lds((const void*)(src[i] + (int64_t)(k_begin + k * C::BKS) * 2),
                                         (lds_void*)(dst + (i * C::NXL + lw) * 1024), 16, 0, 0);
    }
  };

  floatx16 acc[C::TMW];
#pragma unroll
  for (int t = 0; t < C::TMW; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;

  if (w_loader) {
    for (int st = 0; st < C::WS_W - 1; ++st) issue(st);
  } else {
    for (int st = 0; st < C::WS_X - 1; ++st) issue(st);
  }
  for (int kt = 0; kt < nk; ++kt) {
    // slab kt of my stream has landed when at most (depth - 2) younger slabs are outstanding
    constexpr int AW = (C::WS_W - 2) * C::LPW_W, AX = (C::WS_X - 2) * C::LPW_X;
    if (w_loader) __builtin_amdgcn_s_waitcnt(0x0f70 | (AW & 0xf) | ((AW >> 4) << 14));
    else __builtin_amdgcn_s_waitcnt(0x0f70 | (AX & 0xf) | ((AX >> 4) << 14));
    // a bare s_barrier: __syncthreads() carries a fence that drains ALL outstanding loads
    // (vmcnt(0)) and would collapse the ring to a single slab in flight
    __builtin_amdgcn_s_barrier();   // both streams' slab kt are in LDS; slab kt-1's buffers are free
    issue(kt + (w_loader ? C::WS_W : C::WS_X) - 1);
    const char* sw = smem + (kt % C::WS_W) * C::SLAB_W;
    const char* sx = xring + (kt % C::WS_X) * C::SLAB_X;
#pragma unroll
    for (int ks = 0; ks < C::BKS / 16; ++ks) {
      // 16 k of a weight row: one 32-byte run (bf16) or one 16-byte chunk (int8), halves by fh
      bf16x8 wf;
      if constexpr (W8)
        wf = cvt_i8x8_bf16(*reinterpret_cast<const u32x2*>(sw + lds_chunk_off(wn * 32 + fr, ks) + fh * 8));
      else
        wf = *reinterpret_cast<const bf16x8*>(sw + lds_chunk_off(wn * 32 + fr, 2 * ks + fh));
      const char* sxs = sx + (ks / 4) * (64 * BK * 2);      // 64-k sub-slab of the activations
#pragma unroll
      for (int t = 0; t < C::TMW; ++t) {
        const int mh = C::TMW == 2 ? t : wm0;
        const bf16x8 xf = *reinterpret_cast<const bf16x8*>(sxs + lds_chunk_off(mh * 32 + fr, 2 * (ks % 4) + fh));
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf, acc[t], 0, 0, 0);
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0f70);   // drain the re-loads of the tail before the block ends
  __syncthreads();

  // ---- lane = row m, registers = columns (see the fast kernel's epilogue) ---------------------------
  auto runs_of = [&](const floatx16& a, float (&run)[2][8]) {
#pragma unroll
    for (int gp = 0; gp < 2; ++gp)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        auto sw2 = __builtin_amdgcn_permlane32_swap(__float_as_uint(a[4 * gp + r]),
                                                    __float_as_uint(a[4 * (gp + 2) + r]), false, false);
        run[gp][r] = __uint_as_float(sw2[0]);
        run[gp][4 + r] = __uint_as_float(sw2[1]);
      }
  };
  if constexpr (FUSE) {
    // the same steps, in the same order, as splitk_reduce_kernel takes on the sum of one k range
    float* const xch = reinterpret_cast<float*>(smem);    // [2 wave pairs][2 halves][2 runs][64 lanes][8]
    const bool up_wave = GATED && wn >= 2;
    const int wcol = GATED ? (wn & 1) : wn;                // 32-column group of the block's outputs
    float run[2][2][8];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      runs_of(acc[t], run[t]);
#pragma unroll
      for (int gp = 0; gp < 2; ++gp) {
        const int n = n0 + wcol * 32 + 16 * fh + 8 * gp;   // output column of element 0
        const int wr = up_wave ? NO + n : n;               // weight row of element 0
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          if (n + e >= NO) continue;
          if (p.wscale != nullptr) run[t][gp][e] *= p.wscale[wr + e];
          if (p.bias != nullptr) run[t][gp][e] += (float)p.bias[wr + e];
        }
        if (up_wave) Vec8<float>::store(xch + ((((wn & 1) * 2 + t) * 2 + gp) * 64 + lane) * 8, run[t][gp]);
      }
    }
    if (GATED) __syncthreads();
    if (!up_wave) {
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const int m = t * 32 + fr;
        if (m >= M) continue;
#pragma unroll
        for (int gp = 0; gp < 2; ++gp) {
          const int n = n0 + wcol * 32 + 16 * fh + 8 * gp;
          if (n >= NO) continue;
          float uv[8], o[8];
          if (GATED) Vec8<float>::load(xch + (((wcol * 2 + t) * 2 + gp) * 64 + lane) * 8, uv);
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] = GATED ? silu_f(run[t][gp][e]) * uv[e] : apply_act<FACT>(run[t][gp][e]);
          bf16* dst = p.y + (int64_t)m * p.ldy + n;
          const bf16* res = p.residual != nullptr ? p.residual + (int64_t)m * p.ldy + n : nullptr;
          if (n + 8 <= NO && (p.ldy & 7) == 0) {
            if (res != nullptr) {
              float rr[8];
              Vec8<bf16>::load(res, rr);
#pragma unroll
              for (int e = 0; e < 8; ++e) o[e] += rr[e];
            }
            Vec8<bf16>::store(dst, o);
          } else {
            for (int e = 0; e < 8 && n + e < NO; ++e) dst[e] = (bf16)(o[e] + (res != nullptr ? (float)res[e] : 0.f));
          }
        }
      }
    }
    return;
  }
  const bool vec_part = (N & 3) == 0;
#pragma unroll
  for (int t = 0; t < C::TMW; ++t) {
    float run[2][8];
    runs_of(acc[t], run);
    const int m = (C::TMW == 2 ? t : wm0) * 32 + fr;
    if (m >= M) continue;
#pragma unroll
    for (int gp = 0; gp < 2; ++gp) {
      const int n = n0 + wn * 32 + 16 * fh + 8 * gp;
      if (n >= N) continue;
      float* dst = p.part + ((int64_t)blockIdx.y * M + m) * N + n;
      if (n + 8 <= N && vec_part) {
        Vec8<float>::store(dst, run[gp]);
      } else {
        for (int e = 0; e < 8 && n + e < N; ++e) dst[e] = run[gp][e];
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
  const float* src = p.part + (int64_t)m * ncols + n0;
  float a[4] = {0.f, 0.f, 0.f, 0.f}, u[4] = {0.f, 0.f, 0.f, 0.f};
  const bool vec = (ncols & 3) == 0 && n0 + 4 <= N && (!SWIGLU || (N & 3) == 0);
  if (vec) {
    // independent 128-bit loads, summed in split order
#pragma unroll 4
    for (int z = 0; z < splits; ++z) {
      const floatx4 v = *reinterpret_cast<const floatx4*>(src + z * plane);
#pragma unroll
      for (int e = 0; e < 4; ++e) a[e] += v[e];
      if (SWIGLU) {
        const floatx4 w = *reinterpret_cast<const floatx4*>(src + z * plane + N);
#pragma unroll
        for (int e = 0; e < 4; ++e) u[e] += w[e];
      }
    }
  } else {
    for (int z = 0; z < splits; ++z)
      for (int e = 0; e < 4 && n0 + e < N; ++e) {
        a[e] += src[z * plane + e];
        if (SWIGLU) u[e] += src[z * plane + e + N];
      }
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int n = n0 + e;
    if (n >= N) break;
    float av = a[e], uv = u[e];
    if (p.wscale != nullptr) {
      av *= p.wscale[n];
      if (SWIGLU) uv *= p.wscale[n + N];
    }
    if (p.bias != nullptr) {
      av += (float)p.bias[n];
      if (SWIGLU) uv += (float)p.bias[n + N];
    }
    float val = SWIGLU ? silu_f(av) * uv : apply_act<ACT>(av);
    if (QKV) {
      *split_dst_bf16(p.sp, p.row0 + m, n) = (bf16)val;
    } else {
      if (p.residual != nullptr) val += (float)p.residual[(int64_t)m * p.ldy + n];
      p.y[(int64_t)m * p.ldy + n] = (bf16)val;
    }
  }
}

// Split-K second stage of the QKV projection with the rotary embedding applied to the q and k
// heads before the single rounding to bf16.  One thread owns 4 consecutive pair indices of one
// head of one row: columns d..d+3 and d+dh/2..d+dh/2+3.  Angles as in rope_kernel: fp64
// position * theta, theta_i = base^(-2i/dh).
__global__ __launch_bounds__(256) void splitk_reduce_qkv_rope_kernel(GemmParams p, int splits) {
  const int dh = p.sp.head_dim, half = dh / 2, groups = half / 4;
  const int heads = p.sp.q_heads + 2 * p.sp.kv_heads;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (int64_t)p.M * heads * groups) return;
  const int j = (int)(gid % groups);
  const int hg = (int)((gid / groups) % heads);
  const int m = (int)(gid / ((int64_t)groups * heads));
  const int N = p.N;
  const int n_lo = hg * dh + 4 * j, n_hi = n_lo + half;
  const int64_t plane = (int64_t)p.M * N;
  const float* src = p.part + (int64_t)m * N;
  floatx4 lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
  for (int z = 0; z < splits; ++z) {       // split order, independent 128-bit loads
    lo += *reinterpret_cast<const floatx4*>(src + z * plane + n_lo);
    hi += *reinterpret_cast<const floatx4*>(src + z * plane + n_hi);
  }
  if (p.wscale != nullptr) {
    lo *= *reinterpret_cast<const floatx4*>(p.wscale + n_lo);
    hi *= *reinterpret_cast<const floatx4*>(p.wscale + n_hi);
  }
  if (p.bias != nullptr) {
#pragma unroll
    for (int e = 0; e < 4; ++e) { lo[e] += (float)p.bias[n_lo + e]; hi[e] += (float)p.bias[n_hi + e]; }
  }
  if (hg < p.sp.q_heads + p.sp.kv_heads) {   // q and k heads rotate, v heads do not
    const double pos = (double)(seq_position(p.sp.pos, (p.row0 + m) / p.sp.q_len, p.sp.pos0) + (p.row0 + m) % p.sp.q_len);
    const double l2b = log2((double)p.sp.rope_base);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const double theta = exp2(-2.0 * (double)(4 * j + e) / (double)dh * l2b);
      double sv, cv;
      sincos(pos * theta, &sv, &cv);
      const float c = (float)cv, sn = (float)sv, a = lo[e], d = hi[e];
      lo[e] = a * c - d * sn;
      hi[e] = d * c + a * sn;
    }
  }
  u32x2 plo, phi;
  plo[0] = pack_bf2(lo[0], lo[1]); plo[1] = pack_bf2(lo[2], lo[3]);
  phi[0] = pack_bf2(hi[0], hi[1]); phi[1] = pack_bf2(hi[2], hi[3]);
  *reinterpret_cast<u32x2*>(split_dst_bf16(p.sp, p.row0 + m, n_lo)) = plo;   // 4 columns stay inside a head half
  *reinterpret_cast<u32x2*>(split_dst_bf16(p.sp, p.row0 + m, n_hi)) = phi;
}

// Split-K second stage of a projection with residual, followed by the normalisation of the
// finished rows: one 1024-thread block per row (the partials of a row are 10^5 bytes that sit in
// L2; many loads in flight per CU are what makes a single CU per row fast enough); h = sum + bias
// + residual stays in fp32 registers, is stored rounded to y, and y_norm = Norm(h) is computed
// from the fp32 values (mean, then centred variance, as residual_norm_kernel does).
// N <= 1024 * 4 * NORM_TAIL_MAX_G columns.
constexpr int NORM_TAIL_MAX_G = 4;
constexpr int NORM_TAIL_THREADS = 1024;
__device__ inline float block_sum_1024(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();                      // red may still be read from the previous call
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < NORM_TAIL_THREADS / 64; ++i) t += red[i];
  return t;
}
__global__ __launch_bounds__(NORM_TAIL_THREADS) void splitk_reduce_norm_kernel(GemmParams p, int splits) {
  __shared__ float red[NORM_TAIL_THREADS / 64];
  const int N = p.N, m = blockIdx.x;
  const int64_t plane = (int64_t)p.M * N;
  const float* src = p.part + (int64_t)m * N;
  floatx4 h[NORM_TAIL_MAX_G];
  float sum = 0.f;
#pragma unroll
  for (int g = 0; g < NORM_TAIL_MAX_G; ++g) {
    const int n = (g * NORM_TAIL_THREADS + threadIdx.x) * 4;
    h[g] = floatx4{0.f, 0.f, 0.f, 0.f};
    if (n >= N) continue;                 // N % 4 == 0 (host)
    floatx4 a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
    for (int z = 0; z < splits; ++z) a += *reinterpret_cast<const floatx4*>(src + z * plane + n);
    if (p.wscale != nullptr) a *= *reinterpret_cast<const floatx4*>(p.wscale + n);
    const int64_t at = (int64_t)m * p.ldy + n;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (p.bias != nullptr) a[e] += (float)p.bias[n + e];
      if (p.residual != nullptr) a[e] += (float)p.residual[at + e];
      sum += a[e];
    }
    u32x2 pk;
    pk[0] = pack_bf2(a[0], a[1]); pk[1] = pack_bf2(a[2], a[3]);
    *reinterpret_cast<u32x2*>(p.y + at) = pk;
    h[g] = a;
  }
  const bool rms = p.nt.kind == FORGE_NORM_RMSNORM;
  const float mean = rms ? 0.f : block_sum_1024(sum, red) / (float)N;
  float sq = 0.f;
#pragma unroll
  for (int g = 0; g < NORM_TAIL_MAX_G; ++g) {
    const int n = (g * NORM_TAIL_THREADS + threadIdx.x) * 4;
    if (n >= N) continue;
#pragma unroll
    for (int e = 0; e < 4; ++e) { const float d = h[g][e] - mean; sq += d * d; }
  }
  const float rstd = rsqrtf(block_sum_1024(sq, red) / (float)N + p.nt.eps);
  const bf16* gamma = (const bf16*)p.nt.gamma;
  const bf16* beta = (const bf16*)p.nt.beta;
  bf16* yn = (bf16*)p.nt.y_norm + (int64_t)m * N;
#pragma unroll
  for (int g = 0; g < NORM_TAIL_MAX_G; ++g) {
    const int n = (g * NORM_TAIL_THREADS + threadIdx.x) * 4;
    if (n >= N) continue;
    float o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      o[e] = (h[g][e] - mean) * rstd * (float)gamma[n + e];
      if (beta != nullptr) o[e] += (float)beta[n + e];
    }
    u32x2 pk;
    pk[0] = pack_bf2(o[0], o[1]); pk[1] = pack_bf2(o[2], o[3]);
    *reinterpret_cast<u32x2*>(yn + n) = pk;
  }
}

template <int BM, int BN, int WM, int WN, int ACT, int MODE>
forge_status launch_generic(const GemmParams& p0, int splits, hipStream_t s) {
  GemmParams p = p0;
  constexpr int BN_OUT = ACT == FORGE_ACT_SWIGLU ? BN / 2 : BN;
  p.tiles_m = ceil_div(p.M, BM);
  p.tiles_n = ceil_div(p.N, BN_OUT);
  constexpr int smem = 2 * (BM + BN) * BK * 2;
  auto kern = gemm_bf16_generic_kernel<BM, BN, WM, WN, ACT, MODE>;
  static std::atomic<uint64_t> lds_raised{0};   // per kernel instantiation
  if (raise_lds_limit(reinterpret_cast<const void*>(kern), smem, lds_raised) != FORGE_OK) return FORGE_ERR_HIP;
  dim3 grid(p.tiles_m * p.tiles_n, splits), block(WM * WN * 64);
  kern<<<grid, block, smem, s>>>(p);
  return launch_status();
}

// Persistent launch: one block per resident slot (the 256 x 256 tile fills a CU, two 128 x 128
// blocks share one), in multiples of the 8 XCDs.
template <int BM, int BN, int WM, int WN, int ACT, int MODE>
forge_status launch_pers(const GemmParams& p0, hipStream_t s) {
  GemmParams p = p0;
  constexpr int BN_OUT = ACT == FORGE_ACT_SWIGLU ? BN / 2 : BN;
  p.tiles_m = ceil_div(p.M, BM);
  p.tiles_n = ceil_div(p.N, BN_OUT);
  constexpr int smem = 2 * (BM + BN) * BK * 2;
  constexpr int per_cu = smem <= 80 * 1024 ? 2 : 1;
  auto kern = gemm_bf16_pers_kernel<BM, BN, WM, WN, ACT, MODE>;
  static std::atomic<uint64_t> lds_raised{0};   // per kernel instantiation
  if (raise_lds_limit(reinterpret_cast<const void*>(kern), smem, lds_raised) != FORGE_OK) return FORGE_ERR_HIP;
  const int slots = compute_units() * per_cu / 8 * 8;
  const int nitems = p.tiles_m * p.tiles_n * (MODE == MODE_SPLITK ? p.splits : 1);
  const int blocks = min(slots, (nitems + 7) / 8 * 8);
  kern<<<dim3(blocks), dim3(WM * WN * 64), smem, s>>>(p);
  return launch_status();
}

// Which kernel and tile a problem gets.  Fast path: K a multiple of the slab and 16-byte aligned
// output rows (the head split and the fp32 partials have their own alignment rules).
enum Variant { V_FAST_256 = 0, V_FAST_128 = 1, V_GEN_256 = 2, V_GEN_128 = 3, V_SKINNY_FAST = 4, V_SKINNY_GEN = 5 };
inline Variant choose_variant(int M, int N, int K, int ldy, forge_act act, bool qkv) {
  const bool k_ok = K % BK == 0;
  // the fast kernels address x and w with 32-bit byte offsets
  const int64_t w_rows = act == FORGE_ACT_SWIGLU ? 2 * (int64_t)N : N;
  const bool small_ok = (int64_t)M * K * 2 < (1ll << 32) && w_rows * K * 2 < (1ll << 32);
  if (M <= 64) return k_ok ? V_SKINNY_FAST : V_SKINNY_GEN;
  const bool rows_ok = qkv ? N % 8 == 0 : (ldy % 8 == 0 && (N % 8 == 0 || act != FORGE_ACT_SWIGLU));
  const bool fast = k_ok && rows_ok && small_ok;
  // the 256-row tile multiplies faster (half the operand traffic per flop) but fills a CU on its
  // own: take it when its tiles come to whole rounds over the CUs, or to many rounds
  const int64_t big = (int64_t)ceil_div(M, 256) * ceil_div(N, act == FORGE_ACT_SWIGLU ? 128 : 256);
  const int64_t cus = compute_units();
  const int64_t rounds = (big + cus - 1) / cus;
  const bool use_256 = big >= 4 * cus || (big * 10 >= cus * 9 && big * 100 >= rounds * cus * 85);
  if (use_256) return fast ? V_FAST_256 : V_GEN_256;
  return fast ? V_FAST_128 : V_GEN_128;
}

// Few 128-tiles and a long reduction (a 128-token prompt against the 8B-shaped weights: 32 tiles
// of 224 slabs): the persistent kernel then walks (k range, tile) items instead of tiles and a
// reduce kernel adds the fp32 partial tiles in range order.  Only with workspace from the caller.
struct PersSplit {
  int splits, k_per_split;
};
inline PersSplit plan_pers_split(int M, int ncols, int K) {
  const int tiles = ceil_div(M, 128) * ceil_div(ncols, 128);
  const int slots = compute_units() * 2;
  const int slabs = K / BK;
  if (K % BK != 0 || ncols % 8 != 0 || tiles * 2 > slots || slabs < 16) return PersSplit{1, K};
  const int want = min(min(slots / tiles, slabs / 8), 16);
  if (want < 2) return PersSplit{1, K};
  const int per = ceil_div(slabs, want);
  return PersSplit{ceil_div(slabs, per), per * BK};
}

struct SkinnyPlan {
  int ncols;        // columns of the partial planes (2N for SwiGLU)
  int bn;           // weight rows per block of the streaming kernel
  int splits;
  int k_per_split;
  bool fused;       // one k range of 128-row blocks: a plain output can be finished inside the GEMM
};
inline SkinnyPlan plan_skinny(int N, int K, forge_act act, int bk = BK) {
  SkinnyPlan sp;
  sp.ncols = act == FORGE_ACT_SWIGLU ? 2 * N : N;
  sp.fused = false;
  const int slabs = ceil_div(K, bk);
  const int cus = compute_units();
  // Enough weight rows for 128-row blocks to cover three quarters of the chip with ONE k range
  // (8B gate + up: 224 blocks; an LM head): no partial planes and no second launch, and measured
  // faster than two k ranges of 256-row blocks even before the reduce is counted (51 vs 55 us for
  // the 8B gate + up at 64 rows).  bf16 weights only: with int8 weights the activation re-reads of
  // a 128-row block are as large as its weight stream.
  if (bk == BK && ceil_div(sp.ncols, 128) * 4 >= cus * 3) {
    sp.bn = 128;
    sp.splits = 1;
    sp.k_per_split = slabs * bk;
    sp.fused = true;
    return sp;
  }
  // About one block per CU measured best on the decode shapes: more blocks mean more k ranges,
  // i.e. more partial-sum traffic and a longer reduce.  256-row blocks (fewest activation re-reads
  // per weight byte) when two k ranges of them already cover the chip, 128-row blocks otherwise.
  sp.bn = ceil_div(sp.ncols, 256) * 8 >= cus * 3 ? 256 : 128;
  const int tiles = ceil_div(sp.ncols, sp.bn);
  int want = (cus + tiles / 2) / tiles;              // k ranges for ~ one block per CU
  want = max(1, min(want, min(8, slabs * bk / 512)));   // at least 512 k of work per block
  const int per = ceil_div(slabs, want);
  sp.splits = ceil_div(slabs, per);
  sp.k_per_split = per * bk;
  // a short reduction (K < 1024) comes to one k range as well: the second launch would cost more
  // than the few blocks lose by streaming alone
  sp.fused = bk == BK && sp.bn == 128 && sp.splits == 1;
  return sp;
}

template <int BN, bool W8, int FACT = -1>
forge_status launch_wstream(const GemmParams& q, int splits, hipStream_t s) {
  using C = WStream<BN, W8>;
  auto kern = gemm_bf16_wstream_kernel<BN, W8, FACT>;
  static std::atomic<uint64_t> lds_raised{0};   // per kernel instantiation
  if (raise_lds_limit(reinterpret_cast<const void*>(kern), C::SMEM, lds_raised) != FORGE_OK) return FORGE_ERR_HIP;
  // (a block of the gated fused finish covers BN / 2 outputs = BN weight rows: the same count)
  kern<<<dim3(ceil_div(q.N, BN), splits), C::NWV * 64, C::SMEM, s>>>(q);
  return launch_status();
}

template <int ACT, int MODE>
forge_status launch_act(const GemmParams& p, hipStream_t s) {
  const Variant v = choose_variant(p.M, p.N, p.K, p.ldy, (forge_act)ACT, MODE == MODE_QKV || MODE == MODE_QKV_ROPE);
  if constexpr (MODE == MODE_QKV || MODE == MODE_QKV_ROPE) {
    // A head split whose 256-tiles do not come to whole rounds over the CUs (4096 x 6144: 384 tiles
    // on 256 CUs) is cut by columns: as many columns as make whole rounds of 256-tiles, the rest on
    // 128-tiles (4096 + 2048 columns: one round each).  Worth it from K = 2048 on, where the large
    // tile multiplies faster.  Each part writes its own heads; two launches.
    if (v == V_FAST_128 && p.K >= 2048 && p.col0 == 0) {
      const int cus = compute_units(), tm = ceil_div(p.M, 256);
      int g = tm, r = cus;
      while (r != 0) { const int t = g % r; g = r; r = t; }          // gcd(tm, cus)
      const int64_t cols_per_round = (int64_t)(cus / g) * 256;
      const int c = (int)(p.N / cols_per_round * cols_per_round);
      if (c >= 256 && c < p.N && 2 * (int64_t)c >= p.N) {
        GemmParams a = p, b = p;
        a.N = c;
        b.N = p.N - c;
        b.col0 = c;
        b.part = nullptr;          // the parts run unsplit along K: the reduce kernels know no column offset
        b.part_bytes = 0;
        b.w = p.w + (int64_t)c * p.K;
        if (p.bias != nullptr) b.bias = p.bias + c;
        if (p.wscale != nullptr) b.wscale = p.wscale + c;
        const forge_status st = launch_act<ACT, MODE>(a, s);
        return st != FORGE_OK ? st : launch_act<ACT, MODE>(b, s);
      }
    }
  }
  if constexpr (MODE == MODE_QKV_ROPE) {
    // only the persistent kernels rotate in their epilogue; gemm_qkv_fuses_rope() has vouched for
    // the fast path, and the 128-tile takes the wave layout with two accumulators per wave
    if (v == V_FAST_256) return launch_pers<256, 256, 2, 4, ACT, MODE>(p, s);
    if (v == V_FAST_128) return launch_pers<128, 128, 2, 2, ACT, MODE>(p, s);
    return FORGE_ERR_UNSUPPORTED;
  } else {
  switch (v) {
    case V_FAST_256: return launch_pers<256, 256, 2, 4, ACT, MODE>(p, s);
    case V_FAST_128: {
      const int ncols = ACT == FORGE_ACT_SWIGLU ? 2 * p.N : p.N;
      const PersSplit ps = plan_pers_split(p.M, ncols, p.K);
      if (ps.splits > 1 && p.part != nullptr &&
          p.part_bytes >= (size_t)ps.splits * p.M * ncols * sizeof(float)) {
        GemmParams q = p;       // the gated weight is a plain [2N, K] matrix here: gate columns, then up
        q.N = ncols;
        q.splits = ps.splits;
        q.k_per_split = ps.k_per_split;
        const forge_status st = launch_pers<128, 128, 2, 4, FORGE_ACT_NONE, MODE_SPLITK>(q, s);
        if (st != FORGE_OK) return st;
        const int64_t threads = (int64_t)p.M * ceil_div(p.N, 4);
        splitk_reduce_kernel<ACT, MODE == MODE_QKV><<<(unsigned)ceil_div64(threads, 256), 256, 0, s>>>(p, ps.splits, ncols);
        return launch_status();
      }
      // 8 waves of 64 x 32 (16 waves per CU) hide the L2 latency of the small tile better than 4
      // waves of 64 x 64 (measured 7-13 % on the d_model = 768 shapes); the gated epilogue pairs
      // two accumulator columns per wave and keeps the 2 x 2 layout
      if constexpr (ACT == FORGE_ACT_SWIGLU) return launch_pers<128, 128, 2, 2, ACT, MODE>(p, s);
      else return launch_pers<128, 128, 2, 4, ACT, MODE>(p, s);
    }
    case V_GEN_256: return launch_generic<256, 256, 2, 4, ACT, MODE>(p, 1, s);
    case V_GEN_128: return launch_generic<128, 128, 2, 2, ACT, MODE>(p, 1, s);
    default: break;
  }
  // skinny: raw split-K GEMM over all weight rows into fp32 partials, then reduce + epilogue
  const SkinnyPlan sk = plan_skinny(p.N, p.K, (forge_act)ACT, p.w8 != nullptr ? 2 * BK : BK);
  GemmParams q = p;
  q.N = sk.ncols;
  q.k_per_split = sk.k_per_split;
  forge_status st;
  if (v == V_SKINNY_FAST && sk.fused && q.w8 == nullptr && MODE == MODE_PLAIN && p.nt.y_norm == nullptr)
    return launch_wstream<128, false, ACT>(q, 1, s);     // finishes its outputs itself
  if (v == V_SKINNY_FAST) {
    if (q.w8 != nullptr) st = sk.bn == 256 ? launch_wstream<256, true>(q, sk.splits, s) : launch_wstream<128, true>(q, sk.splits, s);
    else st = sk.bn == 256 ? launch_wstream<256, false>(q, sk.splits, s) : launch_wstream<128, false>(q, sk.splits, s);
  } else {
    st = launch_generic<64, 64, 2, 2, FORGE_ACT_NONE, MODE_SPLITK>(q, sk.splits, s);
  }
  if (st != FORGE_OK) return st;
  if (MODE == MODE_QKV && p.sp.rope) {
    const int64_t threads = (int64_t)p.M * (p.sp.q_heads + 2 * p.sp.kv_heads) * (p.sp.head_dim / 8);
    splitk_reduce_qkv_rope_kernel<<<(unsigned)ceil_div64(threads, 256), 256, 0, s>>>(p, sk.splits);
    return launch_status();
  }
  if (MODE == MODE_PLAIN && ACT == FORGE_ACT_NONE && p.nt.y_norm != nullptr) {
    splitk_reduce_norm_kernel<<<p.M, NORM_TAIL_THREADS, 0, s>>>(p, sk.splits);
    return launch_status();
  }
  const int64_t threads = (int64_t)p.M * ceil_div(p.N, 4);
  splitk_reduce_kernel<ACT, MODE == MODE_QKV><<<(unsigned)ceil_div64(threads, 256), 256, 0, s>>>(p, sk.splits, sk.ncols);
  return launch_status();
  }
}

// int8 -> bf16, exact (|q| <= 127 has 7 significant bits); one thread per 16 weights (K % 128 == 0)
__global__ __launch_bounds__(256) void dequant_int8_kernel(const int8_t* __restrict__ q, bf16* __restrict__ w,
                                                           int64_t n16) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n16) return;
  const u32x4 v = *reinterpret_cast<const u32x4*>(q + i * 16);
  const bf16x8 lo = cvt_i8x8_bf16(u32x2{v[0], v[1]}), hi = cvt_i8x8_bf16(u32x2{v[2], v[3]});
  *reinterpret_cast<bf16x8*>(w + i * 16) = lo;
  *reinterpret_cast<bf16x8*>(w + i * 16 + 8) = hi;
}

// cos / sin of the rotary embedding for rows 0 .. q_len-1 of a prompt at positions pos0 + s:
// tab[s][i] = (cos, sin)(p * theta_i), theta_i = base^(-2i/dh), evaluated in fp64 as rope_kernel
// does (p * theta reaches thousands of radians) and stored as fp32.
__global__ __launch_bounds__(256) void rope_table_kernel(float* __restrict__ tab, int q_len, int head_dim,
                                                         int pos0, float base) {
  const int half = head_dim / 2;
  const int gid = blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= q_len * half) return;
  const int i = gid % half, s = gid / half;
  const double theta = exp2(-2.0 * (double)i / (double)head_dim * log2((double)base));
  double sv, cv;
  sincos((double)(pos0 + s) * theta, &sv, &cv);
  floatx2 o = {(float)cv, (float)sv};
  *reinterpret_cast<floatx2*>(tab + 2 * (int64_t)gid) = o;
}

}  // namespace

// bytes of the bf16 copy of an int8 weight (prompt-sized problems), 256-byte aligned
inline size_t w8_dequant_bytes(int N, int K, forge_act act) {
  const size_t b = (size_t)(act == FORGE_ACT_SWIGLU ? 2 : 1) * N * K * sizeof(bf16);
  return (b + 255) / 256 * 256;
}

bool gemm_qkv_fuses_rope(int M, int N, int K, int head_dim, int q_len, forge_dtype dt, bool w8) {
  if (dt != FORGE_BF16) return false;
  if (M <= 64) return gemm_fuses_tail(M, N, dt);     // the reduce step of the weight-streaming path rotates
  if (w8 && K % (2 * BK) != 0) return false;         // (an int8 prompt runs the bf16 kernels on a bf16 copy of the weight)
  if (q_len == 1) return false;                      // a wide decode step may carry per-sequence positions
  if (head_dim != 64 && head_dim != 128) return false;
  const Variant v = choose_variant(M, N, K, N, FORGE_ACT_NONE, true);
  if (v != V_FAST_256 && v != V_FAST_128) return false;
  // a 128-tile problem that would rather split its reduction keeps the separate rotation
  return v == V_FAST_256 || plan_pers_split(M, N, K).splits == 1;
}

size_t gemm_qkv_workspace_bytes(int M, int N, int K, forge_dtype dt, bool w8, bool rope, int q_len, int head_dim) {
  if (rope && M > 64 && gemm_qkv_fuses_rope(M, N, K, head_dim, q_len, dt, w8))   // [bf16 copy of an int8 weight |] cos / sin table
    return (w8 ? w8_dequant_bytes(N, K, FORGE_ACT_NONE) : 0) + (size_t)q_len * head_dim * sizeof(float);
  if (w8) return gemm_w8_workspace_bytes(M, N, K, FORGE_ACT_NONE);
  return dt == FORGE_BF16 ? gemm_bf16_workspace_bytes(M, N, K, FORGE_ACT_NONE, false) : gemm_f32_workspace_bytes(M, N, K, FORGE_ACT_NONE);
}

size_t gemm_bf16_workspace_bytes(int M, int N, int K, forge_act act, bool plain) {
  // plain: a dense output with bias / activation / residual only (no head split, no norm tail)
  if (M <= 64 && plain && K % BK == 0 && plan_skinny(N, K, act).fused) return 0;   // finished inside the GEMM
  if (M > 64) {     // optional: without it the problem runs unsplit
    const int ncols = act == FORGE_ACT_SWIGLU ? 2 * N : N;
    const PersSplit ps = plan_pers_split(M, ncols, K);
    return ps.splits > 1 ? (size_t)ps.splits * M * ncols * sizeof(float) : 0;
  }
  const SkinnyPlan sk = plan_skinny(N, K, act);
  return (size_t)sk.splits * M * sk.ncols * sizeof(float);
}

size_t gemm_w8_workspace_bytes(int M, int N, int K, forge_act act) {
  if (M > 64) return w8_dequant_bytes(N, K, act) + gemm_bf16_workspace_bytes(M, N, K, act, false);
  const SkinnyPlan sk = plan_skinny(N, K, act, 2 * BK);
  return (size_t)sk.splits * M * sk.ncols * sizeof(float);
}

bool gemm_fuses_tail(int M, int N, forge_dtype dt) {
  return dt == FORGE_BF16 && M <= 64 && N % 4 == 0 && N <= NORM_TAIL_THREADS * 4 * NORM_TAIL_MAX_G;
}

const char* gemm_bf16_variant(int M, int N, int K, int ldy, forge_act act) {
  switch (choose_variant(M, N, K, ldy, act, false)) {   // the call launch_act makes for a plain output
    case V_FAST_256: return "gemm_bf16_pers<256,256,2,4>";
    case V_FAST_128: return act == FORGE_ACT_SWIGLU ? "gemm_bf16_pers<128,128,2,2>" : "gemm_bf16_pers<128,128,2,4>";
    case V_GEN_256: return "gemm_bf16_generic<256,256,2,4>";
    case V_GEN_128: return "gemm_bf16_generic<128,128,2,2>";
    case V_SKINNY_FAST: return plan_skinny(N, K, act).fused ? "gemm_bf16_wstream_fused<128>" : "gemm_bf16_wstream+splitk";
    default: return "gemm_bf16_generic<64,64,2,2>+splitk";
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
  p.ldy = a.ldy > 0 ? a.ldy : a.N;
  p.k_per_split = a.K;
  p.part = (float*)a.workspace;
  p.part_bytes = a.workspace != nullptr ? a.workspace_bytes : 0;
  p.splits = 1;
  const bool w8 = a.w_scale != nullptr;
  // the decode path needs its partial-sum planes; the k split of larger problems is optional
  const bool tails = gemm_fuses_tail(a.M, a.N, FORGE_BF16);
  const bool plain = a.split == nullptr && !(a.norm != nullptr && tails && a.act == FORGE_ACT_NONE);
  const size_t need = w8 ? (a.M > 64 ? w8_dequant_bytes(a.N, a.K, a.act) : gemm_w8_workspace_bytes(a.M, a.N, a.K, a.act))
                         : (a.M <= 64 ? gemm_bf16_workspace_bytes(a.M, a.N, a.K, a.act, plain) : 0);
  if (need > a.workspace_bytes || (need > 0 && a.workspace == nullptr)) return FORGE_ERR_WORKSPACE;
  if (a.norm != nullptr && tails && a.split == nullptr && a.act == FORGE_ACT_NONE) {
    if (p.ldy != a.N) return FORGE_ERR_UNSUPPORTED;   // the norm tail writes dense rows
    p.nt = *a.norm;
  }
  bool rope_epilogue = false;
  if (a.split != nullptr) {
    if (a.act != FORGE_ACT_NONE || a.residual != nullptr) return FORGE_ERR_UNSUPPORTED;
    p.sp = *a.split;
    if (p.sp.rope && a.M > 64) {
      // prompt-sized: the epilogue rotates, with cos / sin from a table written into the workspace
      if (!gemm_qkv_fuses_rope(a.M, a.N, a.K, p.sp.head_dim, p.sp.q_len, FORGE_BF16, w8) || p.sp.pos != nullptr)
        return FORGE_ERR_UNSUPPORTED;
      const size_t tab_bytes = (size_t)p.sp.q_len * p.sp.head_dim * sizeof(float);
      const size_t tab_at = w8 ? w8_dequant_bytes(a.N, a.K, FORGE_ACT_NONE) : 0;   // behind the bf16 copy of an int8 weight
      if (a.workspace == nullptr || a.workspace_bytes < tab_at + tab_bytes) return FORGE_ERR_WORKSPACE;
      float* tab = (float*)((char*)a.workspace + tab_at);
      const int n_tab = p.sp.q_len * (p.sp.head_dim / 2);
      rope_table_kernel<<<ceil_div(n_tab, 256), 256, 0, s>>>(tab, p.sp.q_len, p.sp.head_dim, p.sp.pos0, p.sp.rope_base);
      if (hipGetLastError() != hipSuccess) return FORGE_ERR_HIP;
      p.sp.rope_tab = tab;
      p.part = nullptr;
      p.part_bytes = 0;
      rope_epilogue = true;
    } else if (!tails) {
      p.sp.rope = 0;
    }
  }
  auto dispatch = [&](const GemmParams& q) -> forge_status {
    if (rope_epilogue) return launch_act<FORGE_ACT_NONE, MODE_QKV_ROPE>(q, s);
    if (a.split != nullptr) return launch_act<FORGE_ACT_NONE, MODE_QKV>(q, s);
    switch (a.act) {
      case FORGE_ACT_NONE: return launch_act<FORGE_ACT_NONE, MODE_PLAIN>(q, s);
      case FORGE_ACT_GELU_TANH: return launch_act<FORGE_ACT_GELU_TANH, MODE_PLAIN>(q, s);
      case FORGE_ACT_RELU: return launch_act<FORGE_ACT_RELU, MODE_PLAIN>(q, s);
      case FORGE_ACT_SILU: return launch_act<FORGE_ACT_SILU, MODE_PLAIN>(q, s);
      case FORGE_ACT_SWIGLU: return launch_act<FORGE_ACT_SWIGLU, MODE_PLAIN>(q, s);
      case FORGE_ACT_GELU_ERF: return launch_act<FORGE_ACT_GELU_ERF, MODE_PLAIN>(q, s);
      default: return FORGE_ERR_INVALID_ARG;
    }
  };
  if (!w8) return dispatch(p);

  // Weight-only int8.  At most 64 rows: the streaming kernel reads the int8 rows as they are.  More
  // rows (a prompt): the integers are written out once as bf16 (exact) into the workspace and the
  // bf16 kernels run on them, with the row scale applied to the finished sums in their epilogues,
  // so both sizes compute scale * sum(x q) and the weight is read once either way.
  if (a.K % (2 * BK) != 0) return FORGE_ERR_UNSUPPORTED;
  p.wscale = a.w_scale;
  if (a.M <= 64) {
    p.w = nullptr;
    p.w8 = (const int8_t*)a.w;
    return dispatch(p);
  }
  const int64_t w_elems = (a.act == FORGE_ACT_SWIGLU ? 2 : 1) * (int64_t)a.N * a.K;
  const size_t w_bytes = w8_dequant_bytes(a.N, a.K, a.act);
  bf16* wd = (bf16*)a.workspace;
  dequant_int8_kernel<<<(unsigned)ceil_div64(w_elems / 16, 256), 256, 0, s>>>((const int8_t*)a.w, wd, w_elems / 16);
  if (hipGetLastError() != hipSuccess) return FORGE_ERR_HIP;
  p.w = wd;
  p.w8 = nullptr;
  if (!rope_epilogue) {            // (with the rotation in the epilogue the table sits there, and K is not split)
    p.part = (float*)((char*)a.workspace + w_bytes);
    p.part_bytes = a.workspace_bytes - w_bytes;
  }
  return dispatch(p);
}

}  // namespace forge
