// Compiled executor of the decoder stack: the model's launch list is lowered once into a flat
// instruction list over virtual registers (Alg. "FX -> NPUIR Lowering": one output register per
// instruction, caller-owned tensors are constants), the registers get static places in one
// workspace from their live intervals and a linear scan (Sec. "Phase 4: IR Analysis &
// Optimization"), and the list is recorded into a HIP graph that later runs replay.  This gives
// the three properties the paper asks of its executor (Sec. "Code Generation:
// CompiledNPUExecutor"): callables resolved ahead of time, no allocation while running, and an
// order fixed at compile time.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <new>
#include <vector>

#include "api_internal.hpp"
#include "plan.hpp"

using namespace forge;

namespace {

constexpr int REG_NONE = -2;   // operand absent
constexpr int REG_EXT = -1;    // the caller's input (as operand) or output (as result)

struct Instr {
  int op;      // forge_op
  int layer;   // which layer's weights; -1: model level
  int which;   // norm: 0 first, 1 second, 2 final; gemm_res: 0 output projection, 1 MLP down
  int out;     // result register, REG_EXT = caller's output, REG_NONE = works in place / on the cache
  int x;       // main operand
  int res;     // residual operand
  int aux;     // second result: the rows the next consumer normalises (output projection: the
               // layer's second norm; MLP down: the next layer's first norm or the final norm,
               // REG_EXT when that is the caller's output)
  int ws;      // scratch register
};

}  // namespace

struct forge_compiled {
  std::vector<forge_block_desc> layers;
  forge_model_desc model;
  int batch, q_len, pos0, kv_cap;
  std::vector<Instr> prog;
  std::vector<int> out_reg, in_begin, in_regs, start, end;
  std::vector<size_t> reg_bytes, reg_offset;
  int n_bufs = 0;
  size_t ws_bytes = 0;
  // binding
  const void* input = nullptr;
  void* output = nullptr;
  void* k_cache = nullptr;
  void* v_cache = nullptr;
  char* workspace = nullptr;
  const int* seq_pos = nullptr;   // per-sequence positions of a decode step (device), or NULL
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
};

namespace {

struct Lowering {
  forge_compiled* c;
  int new_reg(size_t bytes) {
    c->reg_bytes.push_back(bytes);
    return (int)c->reg_bytes.size() - 1;
  }
  // registers are numbered in creation order: per instruction its output, then its second
  // result, then its scratch area; `ins` lists what the planner counts as reads
  void emit(const Instr& in, std::initializer_list<int> ins) {
    c->prog.push_back(in);
    c->out_reg.push_back(in.out >= 0 ? in.out : -1);
    for (int r : ins)
      if (r >= 0) c->in_regs.push_back(r);
    c->in_begin.push_back((int)c->in_regs.size());
  }
};

void lower(forge_compiled* c) {
  const forge_model_desc& m = c->model;
  const forge_block_desc& d0 = c->layers[0];
  const forge_dtype dt = d0.dt;
  const size_t es = esize(dt);
  const size_t T = (size_t)c->batch * c->q_len;
  const int Ti = (int)T, dm = d0.d_model;
  const bool tokens = m.wte != nullptr;
  const size_t h_bytes = T * dm * es;
  Lowering lo{c};
  c->in_begin.push_back(0);

  int h = REG_EXT;
  if (tokens) {
    h = lo.new_reg(h_bytes);
    lo.emit({FORGE_OP_EMBED, -1, 0, h, REG_EXT, REG_NONE, REG_NONE, REG_NONE}, {});
  }
  // decode-sized steps chain the norms: the reduce step of a layer's MLP down projection also
  // produces what the next consumer normalises (the plain launcher does the same)
  const bool chain = gemm_fuses_tail(Ti, dm, dt);
  int y_chained = REG_NONE;
  for (int l = 0; l < m.n_layers; ++l) {
    const forge_block_desc& d = c->layers[l];
    const int hd = d.q_heads * d.head_dim, nqkv = (d.q_heads + 2 * d.kv_heads) * d.head_dim;
    const bool rope_in_gemm = d.use_rope && gemm_qkv_fuses_rope(Ti, nqkv, dm, d.head_dim, c->q_len, dt, block_w8(&d));
    const bool norm_in_gemm = gemm_fuses_tail(Ti, dm, dt);
    const bool w8 = block_w8(&d);

    int y = y_chained;
    if (!chain || l == 0) {
      y = lo.new_reg(h_bytes);
      lo.emit({FORGE_OP_NORM, l, 0, y, h, REG_NONE, REG_NONE, REG_NONE}, {h});
    }
    const int q = lo.new_reg(T * hd * es);
    int ws = lo.new_reg(gemm_qkv_workspace_bytes(Ti, nqkv, dm, dt, w8, d.use_rope != 0, c->q_len, d.head_dim));
    lo.emit({FORGE_OP_GEMM_QKV, l, rope_in_gemm ? 1 : 0, q, y, REG_NONE, REG_NONE, ws}, {y, ws});
    if (d.use_rope && !rope_in_gemm) {
      lo.emit({FORGE_OP_ROPE_Q, l, 0, REG_NONE, q, REG_NONE, REG_NONE, REG_NONE}, {q});
      lo.emit({FORGE_OP_ROPE_K, l, 0, REG_NONE, REG_NONE, REG_NONE, REG_NONE, REG_NONE}, {});
    }
    const int o = lo.new_reg(T * hd * es);
    ws = lo.new_reg(attn_ws(c->batch, d.q_heads, d.kv_heads, c->q_len, c->pos0 + c->q_len, d.head_dim, dt));
    lo.emit({FORGE_OP_ATTN, l, 0, o, q, REG_NONE, REG_NONE, ws}, {q, ws});
    const int h_mid = lo.new_reg(h_bytes);
    int y2;
    if (norm_in_gemm) {
      y2 = lo.new_reg(h_bytes);
      ws = lo.new_reg(gemm_ws(Ti, dm, hd, FORGE_ACT_NONE, dt, w8));
      lo.emit({FORGE_OP_GEMM_RES, l, 0, h_mid, o, h, y2, ws}, {o, h, y2, ws});
    } else {
      ws = lo.new_reg(gemm_ws(Ti, dm, hd, FORGE_ACT_NONE, dt, w8));
      lo.emit({FORGE_OP_GEMM_RES, l, 0, h_mid, o, h, REG_NONE, ws}, {o, h, ws});
      y2 = lo.new_reg(h_bytes);
      lo.emit({FORGE_OP_NORM, l, 1, y2, h_mid, REG_NONE, REG_NONE, REG_NONE}, {h_mid});
    }
    const int u = lo.new_reg(T * d.d_ff * es);
    ws = lo.new_reg(gemm_ws(Ti, d.d_ff, dm, d.mlp_act, dt, w8, true));
    lo.emit({FORGE_OP_GEMM_ACT, l, 0, u, y2, REG_NONE, REG_NONE, ws}, {y2, ws});
    if (chain && l + 1 == m.n_layers && !tokens) {
      // the final norm is the caller's output; nobody reads the last residual stream, which is
      // added in place (no register of its own)
      y_chained = REG_EXT;
      ws = lo.new_reg(gemm_ws(Ti, dm, d.d_ff, FORGE_ACT_NONE, dt, w8));
      lo.emit({FORGE_OP_GEMM_RES, l, 1, REG_NONE, u, h_mid, y_chained, ws}, {u, h_mid, ws});
      h = h_mid;
    } else {
      const int h_out = lo.new_reg(h_bytes);
      if (chain) y_chained = lo.new_reg(h_bytes);
      ws = lo.new_reg(gemm_ws(Ti, dm, d.d_ff, FORGE_ACT_NONE, dt, w8));
      lo.emit({FORGE_OP_GEMM_RES, l, 1, h_out, u, h_mid, chain ? y_chained : REG_NONE, ws},
              {u, h_mid, chain ? y_chained : REG_NONE, ws});
      h = h_out;
    }
  }
  if (tokens) {
    int yf = y_chained;
    if (!chain) {
      yf = lo.new_reg(h_bytes);
      lo.emit({FORGE_OP_NORM, -1, 2, yf, h, REG_NONE, REG_NONE, REG_NONE}, {h});
    }
    const int ws = lo.new_reg(gemm_ws(Ti, m.vocab, dm, FORGE_ACT_NONE, dt, false, true));
    lo.emit({FORGE_OP_GEMM, -1, 0, REG_EXT, yf, REG_NONE, REG_NONE, ws}, {yf, ws});
  } else if (!chain) {
    lo.emit({FORGE_OP_NORM, -1, 2, REG_EXT, h, REG_NONE, REG_NONE, REG_NONE}, {h});
  }

  const int n_regs = (int)c->reg_bytes.size();
  c->start.resize(n_regs);
  c->end.resize(n_regs);
  c->reg_offset.resize(n_regs);
  plan_liveness((int)c->prog.size(), c->out_reg.data(), c->in_begin.data(), c->in_regs.data(), n_regs,
                c->start.data(), c->end.data());
  c->ws_bytes = plan_workspace(n_regs, c->start.data(), c->end.data(), c->reg_bytes.data(),
                               c->reg_offset.data(), &c->n_bufs);
}

// the launches of the instruction list, in order, on stream s
forge_status run_program(const forge_compiled* c, hipStream_t s) {
  const forge_model_desc& m = c->model;
  const forge_block_desc& d0 = c->layers[0];
  const forge_dtype dt = d0.dt;
  const int T = c->batch * c->q_len, dm = d0.d_model;
  const size_t layer_kv_bytes = (size_t)c->batch * d0.kv_heads * c->kv_cap * d0.head_dim * esize(dt);
  auto in = [&](int r) -> const void* {
    return r >= 0 ? c->workspace + c->reg_offset[r] : (r == REG_EXT ? c->input : nullptr);
  };
  auto out = [&](int r) -> void* {
    return r >= 0 ? c->workspace + c->reg_offset[r] : (r == REG_EXT ? c->output : nullptr);
  };
  auto bytes = [&](int r) -> size_t { return r >= 0 ? c->reg_bytes[r] : 0; };

  for (const Instr& I : c->prog) {
    const forge_block_desc* d = I.layer >= 0 ? &c->layers[I.layer] : &d0;
    const int dh = d->head_dim, hd = d->q_heads * dh, nqkv = (d->q_heads + 2 * d->kv_heads) * dh;
    const int64_t kv_hs = (int64_t)c->kv_cap * dh, kv_bs = kv_hs * d->kv_heads;
    char* kc = static_cast<char*>(c->k_cache) + (I.layer >= 0 ? I.layer : 0) * layer_kv_bytes;
    char* vc = static_cast<char*>(c->v_cache) + (I.layer >= 0 ? I.layer : 0) * layer_kv_bytes;
    forge_status st = FORGE_OK;
    switch (I.op) {
      case FORGE_OP_EMBED:
        st = launch_embed(static_cast<const int32_t*>(c->input), m.wte, m.wpe, out(I.out), c->batch,
                          c->q_len, dm, m.vocab, m.n_pos, c->pos0, dt, s, c->seq_pos);
        break;
      case FORGE_OP_NORM: {
        const void* g = I.which == 0 ? d->norm1_g : (I.which == 1 ? d->norm2_g : m.normf_g);
        const void* b = I.which == 0 ? d->norm1_b : (I.which == 1 ? d->norm2_b : m.normf_b);
        st = launch_residual_norm(in(I.x), nullptr, g, b, nullptr, out(I.out), T, dm, d->eps, d->norm, dt, s);
        break;
      }
      case FORGE_OP_GEMM_QKV: {
        QkvSplit sp = {out(I.out), kc, vc, d->q_heads, d->kv_heads, dh, c->q_len, c->kv_cap, c->pos0,
                       I.which, d->rope_base, c->seq_pos, nullptr};
        GemmArgs g = {in(I.x), d->w_qkv, d->b_qkv, nullptr, nullptr, T, nqkv, dm, 0, FORGE_ACT_NONE,
                      &sp, nullptr, out(I.ws), bytes(I.ws), d->s_qkv};
        st = gemm_dispatch(g, dt, s);
        break;
      }
      case FORGE_OP_ROPE_Q:
        st = launch_rope(out(I.x), c->batch, d->q_heads, c->q_len, dh, (int64_t)d->q_heads * c->q_len * dh,
                         (int64_t)c->q_len * dh, 0, c->pos0, d->rope_base, dt, s, c->seq_pos, false);
        break;
      case FORGE_OP_ROPE_K:
        st = launch_rope(kc, c->batch, d->kv_heads, c->q_len, dh, kv_bs, kv_hs, c->pos0, c->pos0,
                         d->rope_base, dt, s, c->seq_pos, true);
        break;
      case FORGE_OP_ATTN: {
        AttnArgs at = {in(I.x), kc, vc, out(I.out), c->batch, d->q_heads, d->kv_heads, c->q_len,
                       c->pos0 + c->q_len, dh, kv_bs, kv_hs, 1.0f / sqrtf((float)dh), 1,
                       out(I.ws), bytes(I.ws), nullptr, 0, 0, c->seq_pos};
        st = attn_dispatch(at, dt, s);
        break;
      }
      case FORGE_OP_GEMM_RES: {
        const bool o_proj = I.which == 0;
        // whose norm rides on this projection: the layer's second, the next layer's first, the final one
        const forge_block_desc* nx = I.layer + 1 < m.n_layers ? &c->layers[I.layer + 1] : nullptr;
        NormTail nt = o_proj ? NormTail{d->norm2_g, d->norm2_b, out(I.aux), d->eps, d->norm}
                             : (nx != nullptr ? NormTail{nx->norm1_g, nx->norm1_b, out(I.aux), nx->eps, nx->norm}
                                              : NormTail{m.normf_g, m.normf_b, out(I.aux), d0.eps, d0.norm});
        // out == REG_NONE: the sum replaces the residual operand
        void* y = I.out == REG_NONE ? const_cast<void*>(in(I.res)) : out(I.out);
        GemmArgs g = {in(I.x), o_proj ? d->w_o : d->w_down, o_proj ? d->b_o : d->b_down, in(I.res),
                      y, T, dm, o_proj ? hd : d->d_ff, 0, FORGE_ACT_NONE, nullptr,
                      I.aux != REG_NONE ? &nt : nullptr, out(I.ws), bytes(I.ws), o_proj ? d->s_o : d->s_down};
        st = gemm_dispatch(g, dt, s);
        break;
      }
      case FORGE_OP_GEMM_ACT: {
        GemmArgs g = {in(I.x), d->w_up, d->b_up, nullptr, out(I.out), T, d->d_ff, dm, 0, d->mlp_act,
                      nullptr, nullptr, out(I.ws), bytes(I.ws), d->s_up};
        st = gemm_dispatch(g, dt, s);
        break;
      }
      case FORGE_OP_GEMM: {
        // tied LM head: the token table is the weight of the last projection
        GemmArgs g = {in(I.x), m.wte, nullptr, nullptr, out(I.out), T, m.vocab, dm, m.logits_ld,
                      FORGE_ACT_NONE, nullptr, nullptr, out(I.ws), bytes(I.ws)};
        st = gemm_dispatch(g, dt, s);
        break;
      }
      default: st = FORGE_ERR_INVALID_ARG;
    }
    if (st != FORGE_OK) return st;
  }
  return FORGE_OK;
}

void drop_graph(forge_compiled* c) {
  if (c->exec != nullptr) (void)hipGraphExecDestroy(c->exec);
  if (c->graph != nullptr) (void)hipGraphDestroy(c->graph);
  c->exec = nullptr;
  c->graph = nullptr;
}

}  // namespace

extern "C" {

forge_status forge_compile_model(const forge_model_desc* model, int batch, int q_len, int pos0,
                                 int kv_cap, forge_compiled** out) {
  if (out == nullptr) return FORGE_ERR_INVALID_ARG;
  *out = nullptr;
  forge_status st = check_model(model);
  if (st != FORGE_OK) return st;
  if (batch < 1 || !span_ok(pos0, q_len, kv_cap)) return FORGE_ERR_INVALID_ARG;
  if (model->wte != nullptr && !span_ok(pos0, q_len, model->n_pos)) return FORGE_ERR_INVALID_ARG;
  if (!grid_ok(batch, 1) || !rows_ok(batch, q_len)) return FORGE_ERR_UNSUPPORTED;
  forge_compiled* c = nullptr;
  try {
    c = new forge_compiled();
    c->layers.assign(model->layers, model->layers + model->n_layers);
    c->model = *model;
    c->model.layers = c->layers.data();
    c->batch = batch;
    c->q_len = q_len;
    c->pos0 = pos0;
    c->kv_cap = kv_cap;
    lower(c);
  } catch (...) {   // host memory exhausted
    delete c;
    return FORGE_ERR_UNSUPPORTED;
  }
  *out = c;
  return FORGE_OK;
}

void forge_compiled_destroy(forge_compiled* c) {
  if (c == nullptr) return;
  drop_graph(c);
  delete c;
}

size_t forge_compiled_workspace_bytes(const forge_compiled* c) { return c != nullptr ? c->ws_bytes : 0; }

forge_status forge_compiled_counts(const forge_compiled* c, int* n_instr, int* n_regs, int* n_reads,
                                   int* n_bufs) {
  if (c == nullptr) return FORGE_ERR_INVALID_ARG;
  if (n_instr != nullptr) *n_instr = (int)c->prog.size();
  if (n_regs != nullptr) *n_regs = (int)c->reg_bytes.size();
  if (n_reads != nullptr) *n_reads = (int)c->in_regs.size();
  if (n_bufs != nullptr) *n_bufs = c->n_bufs;
  return FORGE_OK;
}

forge_status forge_compiled_program(const forge_compiled* c, int* op, int* out_reg, int* in_begin,
                                    int* in_regs, size_t* reg_bytes, size_t* reg_offset) {
  if (c == nullptr) return FORGE_ERR_INVALID_ARG;
  const size_t ni = c->prog.size(), nr = c->reg_bytes.size();
  for (size_t j = 0; j < ni; ++j) {
    if (op != nullptr) op[j] = c->prog[j].op;
    if (out_reg != nullptr) out_reg[j] = c->out_reg[j];
  }
  if (in_begin != nullptr) std::copy(c->in_begin.begin(), c->in_begin.end(), in_begin);
  if (in_regs != nullptr) std::copy(c->in_regs.begin(), c->in_regs.end(), in_regs);
  for (size_t r = 0; r < nr; ++r) {
    if (reg_bytes != nullptr) reg_bytes[r] = c->reg_bytes[r];
    if (reg_offset != nullptr) reg_offset[r] = c->reg_offset[r];
  }
  return FORGE_OK;
}

static forge_status bind(forge_compiled* c, const void* input, void* output, void* k_cache,
                         void* v_cache, void* workspace, size_t workspace_bytes, void* stream,
                         const int* seq_pos) {
  if (c == nullptr) return FORGE_ERR_INVALID_ARG;
  if (input == nullptr || !req(output) || !req(k_cache) || !req(v_cache) || !req(workspace))
    return FORGE_ERR_INVALID_ARG;
  if (c->model.wte == nullptr && !aligned16(input)) return FORGE_ERR_INVALID_ARG;
  if (stream == nullptr) return FORGE_ERR_INVALID_ARG;   // the legacy default stream cannot record
  if (workspace_bytes < c->ws_bytes) return FORGE_ERR_WORKSPACE;
  drop_graph(c);
  c->input = input;
  c->output = output;
  c->k_cache = k_cache;
  c->v_cache = v_cache;
  c->workspace = static_cast<char*>(workspace);
  c->seq_pos = seq_pos;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // one plain pass first: it settles the one-time kernel attributes outside the recording and
  // reports a launch that cannot run as an ordinary status
  forge_status st = run_program(c, s);
  if (st != FORGE_OK) return st;
  if (hipStreamBeginCapture(s, hipStreamCaptureModeRelaxed) != hipSuccess) return FORGE_ERR_HIP;
  st = run_program(c, s);
  hipGraph_t g = nullptr;
  const hipError_t e = hipStreamEndCapture(s, &g);
  if (st != FORGE_OK || e != hipSuccess || g == nullptr) {
    if (g != nullptr) (void)hipGraphDestroy(g);
    (void)hipGetLastError();
    return st != FORGE_OK ? st : FORGE_ERR_HIP;
  }
  c->graph = g;
  if (hipGraphInstantiate(&c->exec, g, nullptr, nullptr, 0) != hipSuccess) {
    drop_graph(c);
    (void)hipGetLastError();
    return FORGE_ERR_HIP;
  }
  return FORGE_OK;
}

forge_status forge_compiled_bind(forge_compiled* c, const void* input, void* output, void* k_cache,
                                 void* v_cache, void* workspace, size_t workspace_bytes,
                                 void* stream) {
  return bind(c, input, output, k_cache, v_cache, workspace, workspace_bytes, stream, nullptr);
}

forge_status forge_compiled_bind_decode(forge_compiled* c, const void* input, void* output,
                                        void* k_cache, void* v_cache, const int32_t* seq_pos,
                                        void* workspace, size_t workspace_bytes, void* stream) {
  if (c == nullptr || c->q_len != 1) return FORGE_ERR_INVALID_ARG;
  if (seq_pos == nullptr || (reinterpret_cast<uintptr_t>(seq_pos) & 3u) != 0) return FORGE_ERR_INVALID_ARG;
  return bind(c, input, output, k_cache, v_cache, workspace, workspace_bytes, stream, seq_pos);
}

forge_status forge_compiled_run(forge_compiled* c, void* stream) {
  if (c == nullptr || c->exec == nullptr) return FORGE_ERR_INVALID_ARG;
  return hipGraphLaunch(c->exec, static_cast<hipStream_t>(stream)) == hipSuccess ? FORGE_OK : FORGE_ERR_HIP;
}

}  // extern "C"
