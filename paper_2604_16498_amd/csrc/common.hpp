// Shared device/host helpers of the forge HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include <atomic>

#include "../../include/forge.h"

namespace forge {

constexpr int kWave = 64;

typedef __bf16 bf16;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__host__ __device__ inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
__host__ __device__ inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- bf16 <-> fp32 ---------------------------------------------------------------------
__device__ inline float bf2f(bf16 v) { return (float)v; }
__device__ inline bf16 f2bf(float v) { return (bf16)v; }   // round-to-nearest-even

// low / high half of a packed pair of bf16 -> fp32 (exact: bf16 is the top half of an fp32)
__device__ inline float bf_lo(uint32_t p) { return __uint_as_float(p << 16); }
__device__ inline float bf_hi(uint32_t p) { return __uint_as_float(p & 0xffff0000u); }
__device__ inline uint32_t pack_bf2(float lo, float hi) {
  bf16x2 t;
  t[0] = (bf16)lo;
  t[1] = (bf16)hi;
  return __builtin_bit_cast(uint32_t, t);
}

// ---- element access templated on the storage type --------------------------------------
// Vec8<T>: eight consecutive elements held as fp32, loaded / stored with 128-bit accesses.
template <typename T> struct Vec8;

template <> struct Vec8<float> {
  static __device__ inline void load(const float* p, float (&v)[8]) {
    floatx4 a = *reinterpret_cast<const floatx4*>(p);
    floatx4 b = *reinterpret_cast<const floatx4*>(p + 4);
#pragma unroll
    for (int i = 0; i < 4; ++i) { v[i] = a[i]; v[4 + i] = b[i]; }
  }
  static __device__ inline void store(float* p, const float (&v)[8]) {
    floatx4 a, b;
#pragma unroll
    for (int i = 0; i < 4; ++i) { a[i] = v[i]; b[i] = v[4 + i]; }
    *reinterpret_cast<floatx4*>(p) = a;
    *reinterpret_cast<floatx4*>(p + 4) = b;
  }
};

template <> struct Vec8<bf16> {
  static __device__ inline void load(const bf16* p, float (&v)[8]) {
    u32x4 r = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
    for (int i = 0; i < 4; ++i) { v[2 * i] = bf_lo(r[i]); v[2 * i + 1] = bf_hi(r[i]); }
  }
  static __device__ inline void store(bf16* p, const float (&v)[8]) {
    u32x4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = pack_bf2(v[2 * i], v[2 * i + 1]);
    *reinterpret_cast<u32x4*>(p) = r;
  }
};

template <typename T> __device__ inline float to_f32(T v);
template <> __device__ inline float to_f32<float>(float v) { return v; }
template <> __device__ inline float to_f32<bf16>(bf16 v) { return (float)v; }
template <typename T> __device__ inline T from_f32(float v);
template <> __device__ inline float from_f32<float>(float v) { return v; }
template <> __device__ inline bf16 from_f32<bf16>(float v) { return (bf16)v; }

// ---- wave reductions (all 64 lanes take part, every lane gets the result) ---------------
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// ---- activations on the fp32 accumulator ------------------------------------------------
// tanh-GELU written through the logistic form: 0.5 x (1 + tanh u) = x / (1 + exp(-2u)),
// u = sqrt(2/pi) (x + 0.044715 x^3).
__device__ inline float gelu_tanh_f(float x) {
  // exp(-2u) = exp2(x (a + b x^2)) with a = -2 sqrt(2/pi) log2(e), b = 0.044715 a: three
  // multiply-adds in front of the two transcendentals (v_exp_f32, v_rcp_f32)
  const float a = -2.302208198f, b = -0.1029432397f;
  const float e = __builtin_amdgcn_exp2f(x * __builtin_fmaf(x * x, b, a));
  // x * sigmoid(2u); hardware reciprocal (1 ulp) instead of an IEEE division
  return x * __builtin_amdgcn_rcpf(1.0f + e);
}
__device__ inline float silu_f(float x) { return x * __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }
__device__ inline float gelu_erf_f(float x) { return 0.5f * x * (1.0f + erff(x * 0.7071067811865476f)); }

template <int ACT> __device__ inline float apply_act(float x) {
  if (ACT == FORGE_ACT_GELU_TANH) return gelu_tanh_f(x);
  if (ACT == FORGE_ACT_RELU) return fmaxf(x, 0.0f);
  if (ACT == FORGE_ACT_SILU) return silu_f(x);
  if (ACT == FORGE_ACT_GELU_ERF) return gelu_erf_f(x);
  return x;
}

// ---- host-side checks --------------------------------------------------------------------
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline forge_status launch_status() {
  return hipGetLastError() == hipSuccess ? FORGE_OK : FORGE_ERR_HIP;
}

// Compute units of the current device (256 when no device answers, e.g. a size query on a
// host without a GPU).  Read once: the launch heuristics assume a homogeneous node.
inline int compute_units() {
  static const int cus = [] {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0)
      v = 256;
    return v;
  }();
  return cus;
}

// Raise a kernel's dynamic-LDS limit to `bytes`, once per device: the attribute belongs to the
// (kernel, device) pair.  `done` is a bit mask over device ordinals owned by the caller (one per
// kernel instantiation); callers may race, setting the attribute twice is harmless.
inline forge_status raise_lds_limit(const void* kernel, int bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return FORGE_ERR_HIP;
  const uint64_t bit = 1ull << (dev & 63);
  if (done.load(std::memory_order_acquire) & bit) return FORGE_OK;
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess)
    return FORGE_ERR_HIP;
  done.fetch_or(bit, std::memory_order_release);
  return FORGE_OK;
}

// ---- internal launchers (one per kernel family; defined in the .hip files) ---------------

// Where a GEMM writes its result.  Plain: y[m*N + n].  QKV split: column n of row
// t = b*q_len + s goes to q[b, n/dh, s, n%dh] (n < Hq*dh), else to the K or V cache row
// pos0 + s of head (n - Hq*dh)/dh resp. (n - (Hq+Hkv)*dh)/dh.
struct QkvSplit {
  void* q;        // [B,Hq,q_len,dh]
  void* k_cache;  // [B,Hkv,kv_cap,dh]
  void* v_cache;
  int q_heads, kv_heads, head_dim, q_len, kv_cap, pos0;
  int rope;         // the GEMM rotates the new q and k rows itself (only where gemm_qkv_fuses_rope() says so)
  float rope_base;
  // Per-sequence positions (decode step of a generation loop, q_len == 1): device array [B];
  // sequence b writes cache row pos[b] and rotates by pos[b].  pos0 is then the largest position
  // the caller vouches for: values are clamped to [0, pos0] so a bad entry cannot leave the cache.
  const int* pos;
  const float* rope_tab;   // set by the launcher: cos / sin table of a prompt-sized rotating projection
};

__device__ inline int seq_position(const int* pos, int b, int pos0) {
  return pos != nullptr ? min(max(pos[b], 0), pos0) : pos0;
}

// Optional tail of a GEMM with a residual: y_norm = Norm(y) of the rows just produced, from the
// fp32 values before y is rounded (the contract of the residual + norm operator).
struct NormTail {
  const void* gamma;
  const void* beta;   // NULL: no shift
  void* y_norm;       // [M, N]
  float eps;
  forge_norm kind;
};

struct GemmArgs {
  const void* x;
  const void* w;
  const void* bias;
  const void* residual;
  void* y;
  int M, N, K;            // N = number of OUTPUT columns (SWIGLU: w has 2N rows)
  int ldy;                // row stride of y and residual in elements (0: N)
  forge_act act;
  const QkvSplit* split;  // NULL: plain row-major output
  const NormTail* norm;   // NULL: none; honoured only where gemm_fuses_tail() says so
  void* workspace;
  size_t workspace_bytes;
  const float* w_scale;   // non-NULL: w is int8 [N, K] (bf16 activations only), one scale per weight row
};

forge_status launch_gemm_f32(const GemmArgs& a, hipStream_t s);
forge_status launch_gemm_bf16(const GemmArgs& a, hipStream_t s);
// True when this problem takes the split-K path (M <= 64), whose reduce kernel can also rotate
// the q / k heads of a head split (QkvSplit::rope) and normalise the rows of a residual GEMM
// (GemmArgs::norm).  Otherwise both fields are ignored and the caller launches those operators.
bool gemm_fuses_tail(int M, int N, forge_dtype dt);
// True when the QKV projection of this size rotates q and k itself (QkvSplit::rope): the reduce
// kernel of the split-K path (M <= 64), or the epilogue of the persistent kernels (prompts), which
// then needs gemm_qkv_workspace_bytes() of workspace for its cos / sin table.
bool gemm_qkv_fuses_rope(int M, int N, int K, int head_dim, int q_len, forge_dtype dt, bool w8);
size_t gemm_qkv_workspace_bytes(int M, int N, int K, forge_dtype dt, bool w8, bool rope, int q_len, int head_dim);
// plain: the output is a dense matrix with bias / activation / residual only (no head split, no norm
// tail); a decode-sized problem that is finished inside the streaming kernel then needs nothing
size_t gemm_bf16_workspace_bytes(int M, int N, int K, forge_act act, bool plain);
size_t gemm_w8_workspace_bytes(int M, int N, int K, forge_act act);   // required, any M
// Symmetric int8 quantisation of a weight, one scale per row.
forge_status launch_quantize_int8(const void* w, int8_t* q, float* scale, int N, int K, forge_dtype dt,
                                  hipStream_t s);
const char* gemm_bf16_variant(int M, int N, int K, int ldy, forge_act act);
size_t gemm_f32_workspace_bytes(int M, int N, int K, forge_act act);

struct AttnArgs {
  const void* q;
  const void* k;
  const void* v;
  void* out;
  int batch, q_heads, kv_heads, q_len, kv_len, head_dim;
  int64_t kv_batch_stride, kv_head_stride;
  float scale;
  int causal;
  void* workspace;
  size_t workspace_bytes;
  const float* mask;                 // additive fp32 [*, *, q_len, kv_len], NULL: none
  int64_t mask_batch_stride, mask_head_stride;   // elements; 0 broadcasts
  // Per-sequence lengths (q_len == 1, no mask): device array [B]; sequence b attends to rows
  // [0, kv_pos[b]] (clamped to kv_len - 1); kv_len is then the upper bound that sizes the launch.
  const int* kv_pos;
};

forge_status launch_attn_f32(const AttnArgs& a, hipStream_t s);
forge_status launch_attn_f32_mfma(const AttnArgs& a, hipStream_t s);   // prompts: no mask, one length
forge_status launch_attn_simple_bf16(const AttnArgs& a, hipStream_t s);
forge_status launch_attn_prefill_bf16(const AttnArgs& a, hipStream_t s);
forge_status launch_attn_decode_bf16(const AttnArgs& a, hipStream_t s);
size_t attn_decode_workspace_bytes(int batch, int q_heads, int kv_heads, int kv_len, int head_dim);
// The library's own fixed scratch array for the decode attention (one per GPU): its size, and its
// address on the current device.  Every call on a GPU shares it.
size_t attn_decode_static_scratch_bytes();
forge_status attn_decode_static_scratch(void** ptr);

forge_status launch_residual_norm(const void* x, const void* delta, const void* gamma,
                                  const void* beta, void* h_out, void* y, int rows, int d,
                                  float eps, forge_norm kind, forge_dtype dt, hipStream_t s);
// pos (device, [batch], or NULL): per-sequence position instead of pos0 (then pos0 is the clamp);
// rows_at_pos: the rows to rotate start at row pos[b] of each head (a KV cache) instead of row0.
forge_status launch_rope(void* x, int batch, int heads, int n_rows, int head_dim,
                         int64_t batch_stride, int64_t head_stride, int row0, int pos0, float base,
                         forge_dtype dt, hipStream_t s, const int* pos = nullptr, bool rows_at_pos = false);
forge_status launch_embed(const int32_t* ids, const void* wte, const void* wpe, void* h, int batch,
                          int seq, int d, int vocab, int n_pos, int pos0, forge_dtype dt,
                          hipStream_t s, const int* pos = nullptr);

}  // namespace forge
