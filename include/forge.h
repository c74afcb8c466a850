/*
 * forge.h -- C ABI of the fused transformer decoder-block forward for MI355X (gfx950).
 *
 * The library implements the *products* of the paper's two fusion passes as GPU kernels:
 *   - the fused scaled-dot-product attention op that replaces the chain
 *     Q.K^T -> scale -> [mask] -> softmax -> .V   (Sec. "Pass 4: Attention Fusion",
 *     the attention-chain equation and the SDPA equation), taking the UN-transposed K;
 *   - the fused linear op  matmul -> bias add -> activation  with the weight stored
 *     [out_features, in_features], and the "matmul + residual add" pattern
 *     (Sec. "Pass 5: Operator Fusion", the fused-op listing and its four patterns);
 *   - a launcher that runs one decoder layer as a fixed list of launches with no
 *     allocation and no host synchronisation, the three properties the paper states for
 *     its compiled executor (Sec. "Code Generation: CompiledNPUExecutor").
 *
 * Conventions for EVERY entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller; the library never
 *     allocates, frees or synchronises.  Descriptor structs are HOST memory.
 *   - Tensors are dense, row-major (innermost index last), base pointers 16-byte aligned.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *     enqueued asynchronously on it; results are valid after the stream is synchronised.
 *   - `dt` selects the storage type of all activations, weights, biases and gains of the
 *     call: FORGE_F32 (fp32 storage, fp32 arithmetic) or FORGE_BF16 (bf16 storage, fp32
 *     accumulation, one rounding to bf16 at each kernel's store).
 *   - Return value: FORGE_OK, or an error.  Argument errors are detected on the host
 *     BEFORE anything is enqueued.  FORGE_ERR_HIP reports a launch failure.
 *   - `workspace` is caller-provided device scratch of `workspace_bytes` bytes (16-byte
 *     aligned); the matching *_workspace_bytes() function gives the size needed (may be 0,
 *     then NULL is accepted).  Too small -> FORGE_ERR_WORKSPACE.
 *   - No global mutable state beyond per-device caches of launch attributes (safe to fill
 *     from several host threads); calls on different streams with disjoint buffers are
 *     independent.  Results are bitwise reproducible run to run (no atomics in reductions).
 *   - Size limits of one call, beyond which FORGE_ERR_UNSUPPORTED is returned (and the
 *     *_workspace_bytes() query returns 0): batch * q_len <= 2^24 rows; batch and head
 *     counts <= 65535; GEMM M, N <= 2^24 with M * N <= 2^36.  Element offsets inside the
 *     kernels are 64-bit.  Position arithmetic (pos0 + q_len against kv_cap or n_pos) is
 *     checked without overflow.
 */
#ifndef FORGE_H_
#define FORGE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FORGE_OK = 0,
  FORGE_ERR_INVALID_ARG = 1,   /* NULL / misaligned required pointer, non-positive size   */
  FORGE_ERR_UNSUPPORTED = 2,   /* a shape or mode the kernels do not cover                */
  FORGE_ERR_WORKSPACE = 3,     /* workspace missing or too small                          */
  FORGE_ERR_HIP = 4            /* hipGetLastError() after a launch was not hipSuccess     */
} forge_status;

typedef enum { FORGE_F32 = 0, FORGE_BF16 = 1 } forge_dtype;

typedef enum {
  FORGE_ACT_NONE = 0,
  FORGE_ACT_GELU_TANH = 1,     /* 0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3)))         */
  FORGE_ACT_RELU = 2,
  FORGE_ACT_SILU = 3,          /* x / (1 + exp(-x))                                       */
  FORGE_ACT_SWIGLU = 4,        /* silu(gate) * up, gate and up from one [2N,K] weight     */
  FORGE_ACT_GELU_ERF = 5       /* 0.5 x (1 + erf(x / sqrt 2)): the exact form; the paper says
                                  "GELU" only, the tanh form is the reading taken for it    */
} forge_act;

typedef enum { FORGE_NORM_LAYERNORM = 0, FORGE_NORM_RMSNORM = 1 } forge_norm;

/* Human-readable name of a status code (static storage, never NULL). */
const char* forge_status_string(forge_status s);

/* Library version as major*10000 + minor*100 + patch. */
int forge_version(void);

/* ---------------------------------------------------------------------------------------
 * Fused causal scaled-dot-product attention (Sec. "Pass 4: Attention Fusion", SDPA eq.).
 *
 *   out[b, i, h*dh : (h+1)*dh] = sum_j P[b,h,i,j] * v[b, g(h), j, :]
 *   P[b,h,i,:] = softmax_j( mask( scale * q[b,h,i,:] . k[b,g(h),j,:] ) ),  g(h) = h / (Hq/Hkv)
 *   mask (causal != 0): keys j > i + (kv_len - q_len) are excluded.
 *
 * S and P never reach memory (online softmax, fp32).  q: [B,Hq,q_len,dh] dense.
 * k, v: [B,Hkv,*,dh] with row stride dh and explicit batch / head strides IN ELEMENTS, so the
 * same call reads a packed prefill tensor or a KV cache with capacity > kv_len.
 * out: [B,q_len,Hq*dh] dense (heads concatenated per token).  out must not alias q, k, v.
 * Requirements: Hq % Hkv == 0; dh in {64,128}; q_len >= 1; kv_len >= q_len when causal;
 * strides multiples of 8 elements; scale positive and finite (else FORGE_ERR_INVALID_ARG: the
 * paper's scale is 1/sqrt(d_k)).  q_len == 1 takes the split-KV (decode) path, which needs
 * workspace; the size reported for (.., q_len 1, kv_len L, ..) also serves every shorter
 * length, so a generation loop asks once, for the capacity of its cache.
 * ------------------------------------------------------------------------------------ */
size_t forge_attn_fused_workspace_bytes(int batch, int q_heads, int kv_heads, int q_len,
                                        int kv_len, int head_dim, forge_dtype dt);

forge_status forge_attn_fused(const void* q, const void* k, const void* v, void* out,
                              int batch, int q_heads, int kv_heads, int q_len, int kv_len,
                              int head_dim, int64_t kv_batch_stride, int64_t kv_head_stride,
                              float scale, int causal, forge_dtype dt,
                              void* workspace, size_t workspace_bytes, void* stream);

/* The same operator with the optional mask node of the paper's attention chain
 * (Sec. "Pass 4: Attention Fusion": Q.K^T -> scale -> [mask] -> softmax -> [dropout] -> .V):
 *   P[b,h,i,:] = softmax_j( scale * q.k + mask[b,h,i,j] ),  causal != 0 cuts keys as above too.
 * mask: fp32 device pointer, 4-byte aligned, rows of kv_len values ([q_len, kv_len] per plane);
 * mask_batch_stride / mask_head_stride in elements, 0 broadcasts over that axis; values are
 * finite or -inf (a padded key).  Every query row must keep at least one key with a finite
 * mask; rows that do not have no defined result.  No workspace; q_len == 1 is allowed.
 * Same requirements and errors as forge_attn_fused otherwise. */
forge_status forge_attn_fused_masked(const void* q, const void* k, const void* v, const float* mask,
                                     void* out, int batch, int q_heads, int kv_heads, int q_len,
                                     int kv_len, int head_dim, int64_t kv_batch_stride,
                                     int64_t kv_head_stride, int64_t mask_batch_stride,
                                     int64_t mask_head_stride, float scale, int causal,
                                     forge_dtype dt, void* stream);

/* ---------------------------------------------------------------------------------------
 * Fused linear: y = act(x . w^T + bias) (+ residual)   (Sec. "Pass 5: Operator Fusion").
 *
 * x: [M,K]; w: [N,K] ([out_features, in_features]); bias: [N] or NULL; residual: [M,N] or
 * NULL (may alias y); y: [M,N].  Order on the fp32 accumulator: + bias, activation,
 * + residual, one rounding to the storage type.
 * act == FORGE_ACT_SWIGLU: w is [2N,K] (rows 0..N-1 gate, rows N..2N-1 up), bias [2N] or
 * NULL, y[m,n] = silu(gate[m,n]) * up[m,n].
 * The name is the paper's "linear+gelu" pattern; act = NONE with a residual is its
 * "mm+add" pattern, act = RELU / SILU its other two.
 * ldy: row stride of y and residual in elements (0 = dense, N).  A stride that is a multiple of
 * 8 elements keeps every output row 16-byte aligned, which the fast store path needs; a
 * vocabulary-sized N such as 50257 is best given a padded stride (50264).
 * Requirements: M,N,K >= 1; K % 8 == 0 for bf16, K % 4 == 0 for fp32; ldy == 0 or ldy >= N.
 * Workspace: problems with fewer output tiles than the chip has room for are split along K and
 * keep fp32 partial sums in forge_gemm_workspace_bytes() bytes of device memory (0 when the
 * problem is not split); the partial sums are added in a fixed order, so results stay bitwise
 * reproducible.  bf16 problems with M <= 64 (a decode step) cannot run without it
 * (FORGE_ERR_WORKSPACE) unless the size function returns 0 for them (enough weight rows for one
 * k range to fill the chip: such a problem is finished inside the streaming kernel); all others
 * run unsplit, slower, when less is given.
 * ------------------------------------------------------------------------------------ */
size_t forge_gemm_workspace_bytes(int M, int N, int K, forge_act act, forge_dtype dt);

/* Diagnostic: the name of the kernel variant (tile shape and wave layout) that
 * forge_gemm_bias_gelu launches for this problem, e.g. "gemm_bf16_pers<256,256,2,4>"; static
 * storage, never NULL.  Lets a profiler trace be matched to the calls that produced it. */
const char* forge_gemm_variant(int M, int N, int K, int ldy, forge_act act, forge_dtype dt);

forge_status forge_gemm_bias_gelu(const void* x, const void* w, const void* bias,
                                  const void* residual, void* y, int M, int N, int K, int ldy,
                                  forge_act act, forge_dtype dt,
                                  void* workspace, size_t workspace_bytes, void* stream);

/* A gated weight whose rows alternate (gate 0, up 0, gate 1, up 1, ...) re-laid once, out of
 * place, into the layout FORGE_ACT_SWIGLU takes (all gate rows, then all up rows): row r of
 * dst = row 2r of src, row n_pairs + r of dst = row 2r + 1 of src, rows of row_bytes bytes
 * (K * element size for a weight, the element size for a bias; any element type, int8 rows and
 * their fp32 scales included).  src, dst: device pointers to 2 * n_pairs rows each, not
 * overlapping (FORGE_ERR_INVALID_ARG); no alignment required. */
forge_status forge_deinterleave_gated_rows(const void* src, void* dst, int n_pairs, size_t row_bytes,
                                          void* stream);

/* ---------------------------------------------------------------------------------------
 * Weight-only int8 (Sec. "Precision Strategy for Llama-3.1-8B": symmetric int8 weights with
 * 16-bit activations).  The paper gives no granularity or rounding; taken here: one fp32 scale
 * per weight row (output channel), no zero point, q in [-127, 127].
 *
 * forge_quantize_int8: scale[n] = max_k |w[n,k]| / 127, q[n,k] = rint(w[n,k] / scale[n]) (ties
 *   to even), both correctly rounded fp32 divisions; a row of zeros gets scale 1.  w [N,K] in
 *   `dt`, q [N,K] int8, scale [N] fp32, all device pointers (w 16-byte aligned).
 * forge_gemm_w8: y[M,N] = act(x[M,K] . (wq[N,K] * wscale[N])^T + bias) (+ residual), x, bias,
 *   residual, y in bf16, fp32 accumulation; the scale multiplies the finished sum (the same
 *   value as multiplying every weight, one rounding fewer).  Arguments as forge_gemm_bias_gelu
 *   (SWIGLU: wq [2N,K], wscale [2N]).  K % 128 != 0 -> FORGE_ERR_UNSUPPORTED.  The workspace of
 *   forge_gemm_w8_workspace_bytes is REQUIRED for every M.  M <= 64 (a decode step): the int8
 *   weight is streamed once at half the bytes of bf16.  Larger M (a prompt): the integers are
 *   written out once as bf16 (exact) into the workspace, which therefore holds a bf16 copy of
 *   the weight, and the bf16 kernels run on that copy with the row scale applied to the finished
 *   sums: the same arithmetic at both sizes, about the speed of the bf16 call plus one pass
 *   over the weight.
 * ------------------------------------------------------------------------------------ */
forge_status forge_quantize_int8(const void* w, int8_t* q, float* scale, int N, int K,
                                 forge_dtype dt, void* stream);
size_t forge_gemm_w8_workspace_bytes(int M, int N, int K, forge_act act);
forge_status forge_gemm_w8(const void* x, const int8_t* wq, const float* wscale, const void* bias,
                           const void* residual, void* y, int M, int N, int K, int ldy,
                           forge_act act, void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * Fused residual add + normalisation:  h = x (+ delta);  y = Norm(h).
 *
 * x, delta (may be NULL), h_out (may be NULL, may alias x), y: [rows,d].  gamma: [d];
 * beta: [d] or NULL (ignored for RMSNorm).  LayerNorm: biased variance, eps inside the
 * square root, y = (h-mean)/sqrt(var+eps)*gamma+beta.  RMSNorm: y = h/sqrt(mean(h^2)+eps)*gamma.
 * The sum is normalised in fp32 BEFORE h_out is rounded to the storage type.
 * Requirements: d % 8 == 0, 8 <= d <= 16384.
 * ------------------------------------------------------------------------------------ */
forge_status forge_residual_norm(const void* x, const void* delta, const void* gamma,
                                 const void* beta, void* h_out, void* y, int rows, int d,
                                 float eps, forge_norm kind, forge_dtype dt, void* stream);

/* ---------------------------------------------------------------------------------------
 * Rotary position embedding, in place, rotate-half pairing (i, i + dh/2):
 *   theta_i = base^(-2i/dh);  position of row s is pos0 + s.
 * x: [B,H,*,dh] with batch / head strides in elements and row stride dh; rows
 * row0 .. row0+n_rows-1 of every (b,h) are rotated (a KV cache passes row0 = pos0).
 * ------------------------------------------------------------------------------------ */
forge_status forge_rope(void* x, int batch, int heads, int n_rows, int head_dim,
                        int64_t batch_stride, int64_t head_stride, int row0, int pos0,
                        float base, forge_dtype dt, void* stream);

/* ---------------------------------------------------------------------------------------
 * Token + learned-position embedding:  h[b,s,:] = wte[ids[b,s],:] + wpe[pos0+s,:].
 * ids: int32 [B,S] (device).  Ids outside [0,vocab) are clamped into range.
 * ------------------------------------------------------------------------------------ */
forge_status forge_embed(const int32_t* ids, const void* wte, const void* wpe, void* h,
                         int batch, int seq, int d, int vocab, int n_pos, int pos0,
                         forge_dtype dt, void* stream);

/* ---------------------------------------------------------------------------------------
 * One pre-norm decoder layer as a fixed launch list:
 *   y = Norm1(x);  q,k,v = split_heads(y.Wqkv^T + b);  RoPE(q,k) if use_rope;
 *   k,v -> cache rows pos0..pos0+q_len-1;  o = attention(q, cache[0..pos0+q_len));
 *   h = x + o.Wo^T + b_o;  m = Norm2(h);  u = act(m.Wup^T + b_up);  x_out = h + u.Wdown^T + b_down
 * w_qkv rows: Hq*dh query rows, then Hkv*dh key rows, then Hkv*dh value rows.
 * mlp_act: FORGE_ACT_GELU_TANH / GELU_ERF / RELU / SILU (w_up [d_ff,d]) or FORGE_ACT_SWIGLU
 * (w_up [2*d_ff,d]).
 * Biases and norm shifts may be NULL.  All pointers in the descriptor are device pointers.
 * With at most 64 rows (a decode step) the projections take a split-K path whose reduce step
 * also carries RoPE (QKV projection) and Norm2 (output projection): same results up to rounding
 * order, fewer launches.
 * ------------------------------------------------------------------------------------ */
typedef struct {
  int d_model, q_heads, kv_heads, head_dim, d_ff;
  forge_norm norm;
  float eps;
  forge_act mlp_act;
  int use_rope;
  float rope_base;
  forge_dtype dt;
  const void *norm1_g, *norm1_b, *w_qkv, *b_qkv, *w_o, *b_o;
  const void *norm2_g, *norm2_b, *w_up, *b_up, *w_down, *b_down;
  /* Weight-only int8 (Sec. "Precision Strategy for Llama-3.1-8B"): all four NULL = weights in
   * `dt`; all four set = w_qkv, w_o, w_up, w_down are int8 [out, in] with these fp32 per-row
   * scales (as forge_quantize_int8 writes them); dt must be FORGE_BF16 and d_model, d_ff and
   * q_heads*head_dim multiples of 128, else FORGE_ERR_UNSUPPORTED. */
  const float *s_qkv, *s_o, *s_up, *s_down;
} forge_block_desc;

size_t forge_decoder_block_workspace_bytes(const forge_block_desc* desc, int batch, int q_len,
                                           int kv_cap);

/* x_in, x_out: [B,q_len,d] residual stream (may alias).  k_cache, v_cache: [B,Hkv,kv_cap,dh];
 * rows pos0..pos0+q_len-1 are written, rows < pos0 are read.  Prefill: pos0 = 0.
 * Decode: q_len = 1, pos0 = number of cached positions.  pos0 + q_len <= kv_cap. */
forge_status forge_decoder_block(const forge_block_desc* desc, const void* x_in, void* x_out,
                                 void* k_cache, void* v_cache, int batch, int q_len, int pos0,
                                 int kv_cap, void* workspace, size_t workspace_bytes,
                                 void* stream);

/* ---------------------------------------------------------------------------------------
 * Whole model: [embedding ->] L decoder layers -> final norm [-> tied LM head].
 * The LM head multiplies by the token table itself: one physical tensor serves both uses
 * (Sec. "Tied Weight Resolution").
 * layers: HOST array of n_layers descriptors.  wte/wpe NULL: `input` is a hidden state
 * [B,q_len,d] and `output` receives the final normed hidden state [B,q_len,d]; otherwise
 * `input` is int32 ids [B,q_len] and `output` receives logits [B,q_len,vocab] with row stride
 * logits_ld (padding columns, if any, are left untouched).
 * k_cache, v_cache: [n_layers,B,Hkv,kv_cap,dh].
 * In a bf16 step of at most 64 rows (a decode step) the reduce step of a layer's MLP down
 * projection also produces the next layer's Norm1 (after the last layer: the final norm), so
 * only the first layer launches a norm of its own: same results up to rounding order (the norm
 * takes the fp32 sum before it is rounded to bf16).
 * ------------------------------------------------------------------------------------ */
typedef struct {
  int n_layers, vocab, n_pos;
  int logits_ld;   /* row stride of the logits in elements; 0 = vocab (dense) */
  const forge_block_desc* layers;
  const void *wte, *wpe, *normf_g, *normf_b;
} forge_model_desc;

size_t forge_model_workspace_bytes(const forge_model_desc* model, int batch, int q_len, int kv_cap);

forge_status forge_model_forward(const forge_model_desc* model, const void* input, void* output,
                                 void* k_cache, void* v_cache, int batch, int q_len, int pos0,
                                 int kv_cap, void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * Decode step with per-sequence lengths (the generation loop of the paper's language-modelling
 * workload, Sec. "Datasets": a prompt, then one token at a time; here for a batch whose sequences
 * have different lengths).  q_len is 1.  seq_pos: DEVICE int32 [batch]; sequence b has seq_pos[b]
 * cached positions and its new token sits at position seq_pos[b]: its k and v go to cache row
 * seq_pos[b], RoPE / the learned position embedding use seq_pos[b], and its query attends to
 * rows [0, seq_pos[b]].  max_pos: HOST upper bound of seq_pos (max_pos < kv_cap; it sizes
 * launches and workspace, as pos0 does in the calls above).  The kernels clamp every entry to
 * [0, max_pos], so a bad entry gives a wrong result for that sequence, never an access outside
 * the cache.  Because the positions live in device memory the same launch list serves every
 * step: advance seq_pos on the device and launch again (forge_compiled_bind_decode records it
 * once for a whole generation, for positions up to the max_pos the handle was compiled with as
 * pos0).  Workspace: forge_attn_fused_workspace_bytes(.., q_len 1, kv_len max_pos + 1, ..),
 * forge_decoder_block_workspace_bytes / forge_model_workspace_bytes(.., q_len 1, kv_cap).
 * Other arguments, layouts and errors as forge_attn_fused (causal), forge_decoder_block and
 * forge_model_forward.
 * ------------------------------------------------------------------------------------ */
forge_status forge_attn_decode_varlen(const void* q, const void* k, const void* v, void* out,
                                      const int32_t* seq_pos, int batch, int q_heads, int kv_heads,
                                      int max_pos, int head_dim, int64_t kv_batch_stride,
                                      int64_t kv_head_stride, float scale, forge_dtype dt,
                                      void* workspace, size_t workspace_bytes, void* stream);
/* For callers that cannot allocate device memory and have no workspace to hand over (code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation): forge_attn_fused for
 * one new query per sequence (q_len 1, causal, bf16), with the split-KV partial results kept in a
 * fixed array inside the library's device image instead of a caller workspace.  Same kernels,
 * same order, bit-identical output.  The call allocates nothing and frees nothing; its first use
 * on a device looks the array's address up once.
 * Limit: forge_attn_fused_workspace_bytes(batch, q_heads, kv_heads, 1, kv_len, head_dim,
 * FORGE_BF16) must not exceed forge_attn_decode_static_max_bytes() (4 MiB; each GPU the library
 * runs on holds that much until the process ends), else FORGE_ERR_WORKSPACE and nothing is
 * enqueued.  Every call on one GPU shares the array: calls that may overlap on one GPU (different
 * streams, different threads) race and must be ordered by the caller.  Nothing in it needs
 * clearing between calls: every partial a call reads it has written first.
 * Other arguments, layouts and errors as forge_attn_fused. */
size_t forge_attn_decode_static_max_bytes(void);
forge_status forge_attn_decode_static(const void* q, const void* k, const void* v, void* out,
                                      int batch, int q_heads, int kv_heads, int kv_len, int head_dim,
                                      int64_t kv_batch_stride, int64_t kv_head_stride, float scale,
                                      void* stream);
forge_status forge_decoder_block_decode(const forge_block_desc* desc, const void* x_in, void* x_out,
                                        void* k_cache, void* v_cache, const int32_t* seq_pos,
                                        int batch, int max_pos, int kv_cap, void* workspace,
                                        size_t workspace_bytes, void* stream);
forge_status forge_model_decode(const forge_model_desc* model, const void* input, void* output,
                                void* k_cache, void* v_cache, const int32_t* seq_pos, int batch,
                                int max_pos, int kv_cap, void* workspace, size_t workspace_bytes,
                                void* stream);

/* ---------------------------------------------------------------------------------------
 * Static buffer plan of a flat instruction list (Sec. "Phase 4: IR Analysis & Optimization").
 * HOST functions on HOST arrays; they never touch the GPU.
 * A program has n_instr instructions over registers 0..n_regs-1: instruction j writes
 * out_reg[j] (-1: none) and reads in_regs[in_begin[j] .. in_begin[j+1]) (in_begin has
 * n_instr+1 entries, in_begin[0] = 0).  Malformed input -> FORGE_ERR_INVALID_ARG, outputs
 * untouched.
 *
 * forge_plan_liveness (Eq. "liveness"): start[r] = index of the instruction that writes r,
 *   end[r] = index of the last one that reads it.  A register that is only read (a scratch
 *   area) starts at its first mention, one that is never read ends where it starts, one that
 *   is never mentioned gets start = end = -1.
 * forge_plan_dead_after: the dead-after map in CSR form: dead_regs[dead_begin[j] ..
 *   dead_begin[j+1]) = registers (ascending) whose last use is instruction j.  dead_begin has
 *   n_instr+1 entries, dead_regs one per register with end >= 0.
 * forge_plan_linear_scan (Alg. "Linear-Scan Buffer Allocation"): intervals in order of start
 *   (ties: register number); before each, active intervals that ended strictly before its
 *   start release their buffers; the interval takes the lowest-numbered free buffer (the
 *   algorithm leaves the choice open), else a new one, numbered in order of creation;
 *   *n_bufs = M.  reg_to_buf[r] = -1 where start[r] < 0.  The buffer reduction ratio of
 *   Eq. "buf_reduction" is 1 - M/N.
 * forge_plan_workspace: byte offsets in one workspace.  Registers of equal nbytes share
 *   buffers through a linear scan of their own; registers that live within one instruction
 *   (start == end, e.g. scratch areas) form one further group sized to its largest member; the
 *   groups follow each other in the order of their first register; each buffer spans its
 *   group's size rounded up to 256.  offset[r] = (size_t)-1 where start[r] < 0.
 * ------------------------------------------------------------------------------------ */
forge_status forge_plan_liveness(int n_instr, const int* out_reg, const int* in_begin,
                                 const int* in_regs, int n_regs, int* start, int* end);
forge_status forge_plan_dead_after(int n_regs, const int* end, int n_instr, int* dead_begin,
                                   int* dead_regs);
forge_status forge_plan_linear_scan(int n_regs, const int* start, const int* end, int* reg_to_buf,
                                    int* n_bufs);
forge_status forge_plan_workspace(int n_regs, const int* start, const int* end,
                                  const size_t* nbytes, size_t* offset, size_t* total_bytes,
                                  int* n_bufs);

/* ---------------------------------------------------------------------------------------
 * Compiled executor (Sec. "Code Generation: CompiledNPUExecutor"): the launch list of
 * forge_model_forward for ONE fixed (batch, q_len, pos0, kv_cap), lowered to a flat
 * instruction list over virtual registers (Alg. "FX -> NPUIR Lowering"), placed in one
 * workspace by forge_plan_liveness + forge_plan_workspace, and recorded into a HIP graph.
 * Same kernels, same order, same results as forge_model_forward, bit for bit.
 *
 * Registers are the intermediate tensors and per-launch scratch areas; tensors the caller owns
 * (input, output, KV cache, weights) are constants.  Register numbering: in program order, per
 * instruction its output, then its second result, then its scratch area (size 0 where the
 * launch needs none).
 *
 * forge_compile_model   builds the handle (host memory only; copies the descriptors, keeps the
 *                       weight POINTERS: the weights must outlive the handle).
 * forge_compiled_counts / forge_compiled_program   report the program and its plan: op[j]
 *                       (forge_op), out_reg / in_begin / in_regs as for forge_plan_liveness,
 *                       reg_bytes and reg_offset per register.  HOST arrays sized from the
 *                       counts: op and out_reg n_instr entries, in_begin n_instr + 1, in_regs
 *                       n_reads, reg_bytes and reg_offset n_regs.  Any output pointer may be
 *                       NULL.
 * forge_compiled_bind   fixes input / output / caches / workspace (device pointers as for
 *                       forge_model_forward, workspace >= forge_compiled_workspace_bytes) and
 *                       records the graph on `stream`, which must not be the NULL stream.  It
 *                       runs the launch list once on `stream` before recording (so output and
 *                       cache rows are already written when it returns) and creates the graph
 *                       objects: the only call besides compile/destroy that allocates.  May be
 *                       called again with other pointers.
 * forge_compiled_run    replays the graph on `stream`: one launch call, no allocation, no
 *                       synchronisation.  FORGE_ERR_INVALID_ARG before a successful bind.
 * A handle is not thread-safe; replays of one handle must not overlap (they share the workspace).
 * ------------------------------------------------------------------------------------ */
typedef enum {
  FORGE_OP_EMBED = 0, FORGE_OP_NORM = 1, FORGE_OP_GEMM_QKV = 2, FORGE_OP_ROPE_Q = 3,
  FORGE_OP_ROPE_K = 4, FORGE_OP_ATTN = 5, FORGE_OP_GEMM_RES = 6, FORGE_OP_GEMM_ACT = 7,
  FORGE_OP_GEMM = 8
} forge_op;

typedef struct forge_compiled forge_compiled;

forge_status forge_compile_model(const forge_model_desc* model, int batch, int q_len, int pos0,
                                 int kv_cap, forge_compiled** out);
void forge_compiled_destroy(forge_compiled* c);
size_t forge_compiled_workspace_bytes(const forge_compiled* c);
forge_status forge_compiled_counts(const forge_compiled* c, int* n_instr, int* n_regs, int* n_reads,
                                   int* n_bufs);
forge_status forge_compiled_program(const forge_compiled* c, int* op, int* out_reg, int* in_begin,
                                    int* in_regs, size_t* reg_bytes, size_t* reg_offset);
forge_status forge_compiled_bind(forge_compiled* c, const void* input, void* output, void* k_cache,
                                 void* v_cache, void* workspace, size_t workspace_bytes,
                                 void* stream);
/* as forge_compiled_bind for a handle compiled with q_len 1, with per-sequence positions: the
 * handle's pos0 is the max_pos of forge_model_decode */
forge_status forge_compiled_bind_decode(forge_compiled* c, const void* input, void* output,
                                        void* k_cache, void* v_cache, const int32_t* seq_pos,
                                        void* workspace, size_t workspace_bytes, void* stream);
forge_status forge_compiled_run(forge_compiled* c, void* stream);

/* ---------------------------------------------------------------------------------------
 * Where a step's time goes (Sec. "Evaluation Protocol" measures whole-model latency; this is the
 * per-operator breakdown of the same launch list).  Between forge_trace_start and
 * forge_trace_stop, forge_decoder_block, forge_model_forward and their *_decode forms record one
 * HIP event on their stream after every operator of the list (forge_op: a launch, or the two
 * launches of a split-K projection); operator i took the time between events i and i + 1, launch
 * gaps included.  forge_trace_start creates capacity + 1 events and records the first on `stream`
 * (operators past `capacity` are not recorded); forge_trace_stop waits for the last recorded
 * event, writes min(*n_ops, capacity) operator codes and durations in milliseconds, and destroys
 * the events.  One trace at a time (a second start -> FORGE_ERR_INVALID_ARG); a profiling aid,
 * not for use under stream capture.  The compiled executor's replays are not traced.
 * ------------------------------------------------------------------------------------ */
forge_status forge_trace_start(int capacity, void* stream);
forge_status forge_trace_stop(int* n_ops, int* ops, float* ms, int capacity);

#ifdef __cplusplus
}
#endif
#endif /* FORGE_H_ */
