// The LM train step: forward, backward and optimiser update as an ordered list of kernel launches on one
// stream.  The workload is the decoder-only Transformer of the paper's large-scale evaluation (Section
// 5.3: embedding lookup in front, Transformer layers of model dimension d and hidden dimension F, a
// softmax layer at the end); it is a "compiled function" in the sense of Section 3: every shape is
// known up front, so every buffer is allocated once, at model creation.
//
// bf16 mode keeps fp32 where rounding would accumulate: the residual stream x, LayerNorm statistics,
// softmax statistics, the loss, every GEMM accumulator, weight gradients, master weights and optimiser
// state.  GEMM and attention operands (LayerNorm outputs, qkv, attention output, FFN activations and
// their gradients, logits) are bf16.
#include "lm.hpp"

#include <cmath>
#include <cstdio>

#include "kernels.hpp"

namespace pw {

namespace {

OptimizerConfig opt_of(const pw_lm_config& c) { return OptimizerConfig{c.optimizer, c.lr, c.beta1, c.beta2, c.eps}; }

// The weight-gradient GEMM of a [in, out] weight over N tokens, as far as the launcher's choice of kernel goes.
GemmArgs wgrad_shape(int64_t N, int64_t in, int64_t out) {
  GemmArgs a{};
  a.dtype = kBF16; a.a_kmajor = 1; a.b_kmajor = 1;
  a.M = in; a.N = out; a.K = N; a.lda = in; a.ldb = out; a.ldc = out;
  a.epilogue = kEpiStore; a.out_dtype = kF32;
  return a;
}

// Which weights of a layer (and the head) get their Adam update inside the weight-gradient GEMM: those whose GEMM
// runs on the ring kernel's full tiles, alone or - QKV and out-projection - in their shared launch.
struct FusedPlan { bool qkv = false, wo = false, w1 = false, w2 = false, wh = false; };
FusedPlan fused_plan(const pw_lm_config& c) {
  FusedPlan f;
  if (!c.fused_update || !c.bf16 || c.optimizer != 2 || !c.has_head) return f;
  const int64_t N = (int64_t)c.batch * c.seq, d = c.d_model, F = c.d_ff, V = c.vocab;
  const GemmArgs pair[2] = {wgrad_shape(N, d, 3 * d), wgrad_shape(N, d, d)};
  const bool shared = gemm_group_shares_launch(pair, 2);
  f.qkv = gemm_adam_fusable(pair[0], shared);
  f.wo = gemm_adam_fusable(pair[1], shared);
  if (shared && f.qkv != f.wo) f.qkv = f.wo = false;   // one launch, one kind of epilogue
  f.w1 = gemm_adam_fusable(wgrad_shape(N, d, F), false);
  f.w2 = gemm_adam_fusable(wgrad_shape(N, F, d), false);
  f.wh = gemm_adam_fusable(wgrad_shape(N, d, V), false);
  return f;
}

void build_param_table(const pw_lm_config& c, std::vector<ParamInfo>& t, int64_t& total, int64_t& fused_from) {
  ParamTableBuilder tb{t};
  const FusedPlan fp = fused_plan(c);
  auto add = [&](const std::string& n, int64_t numel, bool fused = false) { tb.add(n, numel, fused); };
  const int64_t d = c.d_model, F = c.d_ff, V = c.vocab, T = c.seq;
  if (c.has_embed) {
    add("wte", V * d);
    add("wpe", T * d);
  }
  for (int l = 0; l < c.n_layer; ++l) {
    const std::string p = "l" + std::to_string(l) + ".";
    add(p + "ln1_g", d); add(p + "ln1_b", d);
    add(p + "wqkv", d * 3 * d, fp.qkv); add(p + "bqkv", 3 * d);
    add(p + "wo", d * d, fp.wo); add(p + "bo", d);
    add(p + "ln2_g", d); add(p + "ln2_b", d);
    add(p + "w1", d * F, fp.w1); add(p + "b1", F);
    add(p + "w2", F * d, fp.w2); add(p + "b2", d);
  }
  if (c.has_head) {
    add("lnf_g", d); add("lnf_b", d);
    add("wh", d * V, fp.wh);
  }
  tb.finish(total, fused_from);
}

// Assigns every activation / scratch pointer; with base == nullptr only measures.
size_t plan(Model* m, unsigned char* base) {
  const pw_lm_config& c = m->cfg;
  const size_t N = (size_t)m->N(), d = c.d_model, F = c.d_ff, V = c.vocab, L = c.n_layer;
  const size_t es = c.bf16 ? 2 : 4;
  const size_t BHT = (size_t)c.batch * c.n_head * c.seq;
  Carver cv;
  cv.base = base;
  const size_t n_mb = (size_t)c.n_microbatch;
  m->defer_wgrad = !c.has_embed && !c.has_head && c.bf16 && n_mb > 1;
  m->slots.resize(n_mb);
  m->pending.assign(n_mb, 0);
  for (auto& s : m->slots) {
    s.layer.resize(L);
    for (size_t l = 0; l < L; ++l) {
      auto& a = s.layer[l];
      a.x_in = cv.take<float>(N * d * 4);
      a.x_mid = cv.take<float>(N * d * 4);
      a.lse = cv.take<float>(BHT * 4);
      a.mean1 = cv.take<float>(N * 4);
      a.rstd1 = cv.take<float>(N * 4);
      a.mean2 = cv.take<float>(N * 4);
      a.rstd2 = cv.take<float>(N * 4);
      a.qkv = cv.take<void>(N * 3 * d * es);
      a.u = cv.take<void>(N * F * es);
      if (!m->defer_wgrad) {
        a.a = cv.take<void>(N * d * es);
        a.o = cv.take<void>(N * d * es);
        a.mm = cv.take<void>(N * d * es);
        a.h = cv.take<void>(N * F * es);
      }
    }
    s.x_out = cv.take<float>(N * d * 4);
  }
  if (m->defer_wgrad) {
    // operands of the weight-gradient GEMMs: per layer and tensor one block [micro-batch][token][feature], so that
    // any run of consecutive micro-batches is one k-major operand
    auto block = [&](size_t l, void* Model::LayerActs::*field, size_t width) {
      unsigned char* b0 = cv.take<unsigned char>(n_mb * N * width * es);
      for (size_t mb = 0; mb < n_mb; ++mb) m->slots[mb].layer[l].*field = b0 ? b0 + mb * N * width * es : nullptr;
    };
    for (size_t l = 0; l < L; ++l) {
      block(l, &Model::LayerActs::a, d);
      block(l, &Model::LayerActs::o, d);
      block(l, &Model::LayerActs::mm, d);
      block(l, &Model::LayerActs::h, F);
      block(l, &Model::LayerActs::g_y2, d);
      block(l, &Model::LayerActs::g_u, F);
      block(l, &Model::LayerActs::g_yo, d);
      block(l, &Model::LayerActs::g_qkv, 3 * d);
    }
  }
  if (c.has_head) {
    m->y = cv.take<void>(N * d * es);
    m->logits = cv.take<void>(N * V * es);
    m->meanf = cv.take<float>(N * 4);
    m->rstdf = cv.take<float>(N * 4);
    m->row_loss = cv.take<float>(N * 4);
    if (m->fused_head) {   // statistics instead of a second use of the logits buffer
      m->xe_part = cv.take<float>(N * (V / 64) * 2 * 4);
      m->xe_zt = cv.take<float>(N * 4);
      m->xe_lse = cv.take<float>(N * 4);
    }
  }
  m->dx_a = cv.take<float>(N * d * 4);
  m->dx_b = cv.take<float>(N * d * 4);
  m->delta = cv.take<float>(BHT * 4);
  m->dx_lp = cv.take<void>(N * d * es);
  m->dx_lp2 = cv.take<void>(N * d * es);
  m->dx_lp3 = cv.take<void>(N * d * es);
  m->d_big = cv.take<void>(N * F * es);
  m->d_qkv = cv.take<void>(N * 3 * d * es);
  m->d_small = cv.take<void>(N * d * es);
  int64_t wsf = layernorm_bwd_ws_floats((int)N, (int)d);
  const int64_t widest = (int64_t)std::max(std::max(3 * d, F), d);
  wsf = std::max(wsf, colsum_ws_floats((int64_t)(m->defer_wgrad ? n_mb * N : N), widest));
  m->ws = cv.take<float>((size_t)wsf * 4);
  return cv.off;
}

const ParamInfo& P(const Model* m, size_t idx) { return m->params[idx]; }

size_t layer_base(const Model* m, int l) { return (m->cfg.has_embed ? 2 : 0) + (size_t)l * 12; }

hipError_t layers_forward(Model* m, Model::Slot& s) {
  const pw_lm_config& c = m->cfg;
  const int N = m->N(), d = c.d_model, F = c.d_ff;
  const int dt = m->act_dtype();
  for (int l = 0; l < c.n_layer; ++l) {
    auto& A = s.layer[l];
    const size_t e = layer_base(m, l);
    float* x_next = l + 1 < c.n_layer ? s.layer[l + 1].x_in : s.x_out;
    PW_TRY(launch_layernorm_fwd(m->stream, dt, A.x_in, m->w + P(m, e).offset, m->w + P(m, e + 1).offset, A.a, A.mean1, A.rstd1, N, d), "ln1 fwd");
    PW_TRY(gemm_fwd(m, A.a, e + 2, m->w + P(m, e + 3).offset, N, d, 3 * d, kEpiBias, dt, nullptr, A.qkv, nullptr), "qkv gemm");
    PW_TRY(launch_attention_fwd(m->stream, dt, A.qkv, A.o, A.lse, c.batch, c.seq, c.n_head, m->hd()), "attention fwd");
    PW_TRY(gemm_fwd(m, A.o, e + 4, m->w + P(m, e + 5).offset, N, d, d, kEpiBiasResidual, kF32, A.x_in, A.x_mid, nullptr), "out-proj gemm");
    PW_TRY(launch_layernorm_fwd(m->stream, dt, A.x_mid, m->w + P(m, e + 6).offset, m->w + P(m, e + 7).offset, A.mm, A.mean2, A.rstd2, N, d), "ln2 fwd");
    PW_TRY(gemm_fwd(m, A.mm, e + 8, m->w + P(m, e + 9).offset, N, d, F, kEpiBiasGelu, dt, nullptr, A.u, A.h), "ffn1 gemm");
    PW_TRY(gemm_fwd(m, A.h, e + 10, m->w + P(m, e + 11).offset, N, F, d, kEpiBiasResidual, kF32, A.x_mid, x_next, nullptr), "ffn2 gemm");
  }
  return hipSuccess;
}

// On entry m->dx_a holds the gradient w.r.t. the stack output (fp32) and, in bf16 mode, m->dx_lp its bf16
// copy.  On exit m->dx_a holds the gradient w.r.t. the stack input.
// The bias gradients of the two projections that write the residual stream (b2, bo) are column sums of the
// stream's gradient; the LayerNorm backward that produces that gradient delivers them.  top_b2_done says
// whether the caller's producer of dx_a already did so for the last layer's b2.
// defer: with deferred weight gradients (see lm.hpp) the four gradients that feed them go to this micro-batch's own
// storage instead of the shared scratch, and the weight-gradient GEMMs are left to flush_wgrads.
hipError_t layers_backward(Model* m, Model::Slot& s, int accumulate, bool top_b2_done, bool defer) {
  const pw_lm_config& c = m->cfg;
  const int N = m->N(), d = c.d_model, F = c.d_ff;
  const int dt = m->act_dtype();
  float* g = m->g;
  const FusedPlan fz = (m->fused_from >= 0 && !accumulate && !defer) ? fused_plan(c) : FusedPlan{};
  const OptimizerConfig opt = opt_of(c);
  for (int l = c.n_layer - 1; l >= 0; --l) {
    auto& A = s.layer[l];
    const size_t e = layer_base(m, l);
    void* const d_big = defer ? A.g_u : m->d_big;
    void* const d_qkv = defer ? A.g_qkv : m->d_qkv;
    void* const lp_mid = defer ? A.g_yo : m->dx_lp2;                                   // bf16 copy of dx_b
    // All weight gradients of the layer at its end (bf16, not deferred): the bf16 copy of the layer's incoming gradient,
    // which the FFN2 weight gradient reads, must then survive LN1's backward - the copies of consecutive layers
    // alternate between two buffers.
    const bool late = c.bf16 && !defer;
    const bool odd = ((c.n_layer - 1 - l) & 1) != 0;
    void* const lp_in = late && odd ? m->dx_lp3 : m->dx_lp;
    void* const lp_below = defer && l > 0 ? s.layer[l - 1].g_y2 : (late && !odd ? m->dx_lp3 : m->dx_lp);   // bf16 copy of the new dx_a
    const void* dx_op = c.bf16 ? (defer ? (const void*)A.g_y2 : (const void*)lp_in) : (const void*)m->dx_a;
    const void* const dx_in = dx_op;
    // Every data gradient comes BEFORE the weight gradient of the same layer: a weight gradient whose epilogue
    // applies the optimizer (fused update) rewrites the weight its data gradient still has to read.
    // FFN2: x_out = x_mid + h W2 + b2
    if (l == c.n_layer - 1 && !top_b2_done)
      PW_TRY(launch_colsum(m->stream, kF32, m->dx_a, g + P(m, e + 11).offset, m->ws, N, d, accumulate), "b2 grad");
    PW_TRY(gemm_dgrad(m, dx_op, e + 10, N, F, d, kEpiGeluBwd, A.u, d_big, dt, 0), "ffn2 dgrad + gelu'");
    // FFN1: u = m W1 + b1
    // (b1 gradient = column sums of d_big: delivered by the weight-gradient GEMM where that is free)
    PW_TRY(gemm_dgrad(m, d_big, e + 8, N, d, F, kEpiStore, nullptr, m->d_small, dt, 0), "ffn1 dgrad");
    // LN2 and the residual branch: dx_b = dx_a + LN2'(d_small).  The chain FFN2 data gradient -> FFN1 data gradient ->
    // LN2 backward runs without the two weight-gradient GEMMs in between, which need nothing of it: those GEMMs (and,
    // fused, the optimizer traffic of their epilogues) would otherwise push d_big, d_small and the residual gradient
    // out of the caches before their one reader gets to them.
    PW_TRY(launch_layernorm_bwd(m->stream, dt, m->d_small, A.x_mid, m->w + P(m, e + 6).offset, A.mean2, A.rstd2, m->dx_a,
                                m->dx_b, c.bf16 ? lp_mid : nullptr, g + P(m, e + 6).offset, g + P(m, e + 7).offset,
                                g + P(m, e + 5).offset /* bo */, m->ws, N, d, accumulate), "ln2 bwd");
    auto ffn_wgrads = [&]() -> hipError_t {
      PW_TRY(launch_gemm(m->stream, fz.w2 ? wgrad_adam_args(m, opt, A.h, dx_in, e + 10, N, F, d)
                                          : wgrad_args(m, A.h, dx_in, e + 10, N, F, d, accumulate)), "ffn2 wgrad");
      PW_TRY(gemm_wgrad_bias(m, A.mm, d_big, e + 8, e + 9, N, d, F, accumulate, m->ws, fz.w1 ? &opt : nullptr), "ffn1 wgrad + b1 grad");
      return hipSuccess;
    };
    if (!defer && !late) {
      const hipError_t er = ffn_wgrads();
      if (er != hipSuccess) return er;
    }
    dx_op = c.bf16 ? (const void*)lp_mid : (const void*)m->dx_b;
    // out-proj: x_mid = x_in + o Wo + bo
    // (its weight gradient is computed together with the QKV one below: neither fills the chip alone)
    const void* dy_out = dx_op;
    PW_TRY(gemm_dgrad(m, dx_op, e + 4, N, d, d, kEpiStore, nullptr, m->d_small, dt, 0), "out-proj dgrad");
    PW_TRY(launch_attention_bwd(m->stream, dt, A.qkv, A.o, m->d_small, A.lse, m->delta, d_qkv, c.batch, c.seq,
                                c.n_head, m->hd()), "attention bwd");
    // QKV: qkv = a Wqkv + bqkv
    PW_TRY(gemm_dgrad(m, d_qkv, e + 2, N, d, 3 * d, kEpiStore, nullptr, m->d_small, dt, 0), "qkv dgrad");
    // LN1 and the residual branch: dx_a = dx_b + LN1'(d_small); again right behind the producer of d_small.  Its bf16
    // output goes to the other of the two low-precision buffers, so dy_out stays intact for the weight gradients below.
    PW_TRY(launch_layernorm_bwd(m->stream, dt, m->d_small, A.x_in, m->w + P(m, e).offset, A.mean1, A.rstd1, m->dx_b,
                                m->dx_a, c.bf16 ? lp_below : nullptr, g + P(m, e).offset, g + P(m, e + 1).offset,
                                l > 0 ? g + P(m, layer_base(m, l - 1) + 11).offset /* b2 of the layer below */ : nullptr,
                                m->ws, N, d, accumulate), "ln1 bwd");
    if (late) {
      const hipError_t er = ffn_wgrads();
      if (er != hipSuccess) return er;
    }
    if (!defer) {
      const WgradJob jobs[2] = {{fz.qkv ? wgrad_adam_args(m, opt, A.a, d_qkv, e + 2, N, d, 3 * d)
                                        : wgrad_args(m, A.a, d_qkv, e + 2, N, d, 3 * d, accumulate), (int64_t)e + 3},
                                {fz.wo ? wgrad_adam_args(m, opt, A.o, dy_out, e + 4, N, d, d)
                                       : wgrad_args(m, A.o, dy_out, e + 4, N, d, d, accumulate), -1}};
      PW_TRY(gemm_wgrad_group(m, jobs, 2, m->ws), "qkv + out-proj wgrad + bqkv grad");
    }
  }
  return hipSuccess;
}

// The weight gradients that the backward passes of the pending micro-batches left undone: per layer four GEMMs
// (three launches) over each run of consecutive pending micro-batches - one run, all of them, after a full
// schedule - accumulated into g.
hipError_t flush_wgrads(Model* m) {
  if (!m->defer_wgrad) return hipSuccess;
  const pw_lm_config& c = m->cfg;
  const int N = m->N(), d = c.d_model, F = c.d_ff, n_mb = c.n_microbatch;
  for (int first = 0; first < n_mb;) {
    if (!m->pending[first]) {
      ++first;
      continue;
    }
    int last = first;
    while (last + 1 < n_mb && m->pending[last + 1]) ++last;
    const int64_t K = (int64_t)(last - first + 1) * N;
    const int acc = m->wgrads_zero ? 0 : 1;   // into freshly zeroed gradients: no need to read the zeros back
    for (int l = c.n_layer - 1; l >= 0; --l) {
      const auto& A = m->slots[first].layer[l];
      const size_t e = layer_base(m, l);
      PW_TRY(launch_gemm(m->stream, wgrad_args(m, A.h, A.g_y2, e + 10, K, F, d, acc)), "ffn2 wgrad");
      PW_TRY(gemm_wgrad_bias(m, A.mm, A.g_u, e + 8, e + 9, K, d, F, acc, m->ws), "ffn1 wgrad + b1 grad");
      const WgradJob jobs[2] = {{wgrad_args(m, A.a, A.g_qkv, e + 2, K, d, 3 * d, acc), (int64_t)e + 3},
                                {wgrad_args(m, A.o, A.g_yo, e + 4, K, d, d, acc), -1}};
      PW_TRY(gemm_wgrad_group(m, jobs, 2, m->ws), "qkv + out-proj wgrad + bqkv grad");
    }
    m->wgrads_zero = false;
    for (int mb = first; mb <= last; ++mb) m->pending[mb] = 0;
    first = last + 1;
  }
  return hipSuccess;
}

}  // namespace

bool model_config_ok(const pw_lm_config& c, std::string* why) {
  auto bad = [&](const char* s) {
    if (why) *why = s;
    return false;
  };
  if (c.n_layer < 1 || c.d_model < 1 || c.n_head < 1 || c.d_ff < 1 || c.seq < 1 || c.batch < 1) return bad("non-positive dimension");
  if (c.d_model % c.n_head) return bad("d_model must be a multiple of n_head");
  const int hd = c.d_model / c.n_head;
  if (hd != 64 && hd != 128) return bad("head_dim must be 64 or 128");
  if (c.d_model % 64 || c.d_ff % 64) return bad("d_model and d_ff must be multiples of 64");
  if (c.d_model > 8192) return bad("d_model above 8192 is not supported by the row kernels");
  if (c.has_head && (c.vocab < 8 || c.vocab % 8)) return bad("vocab must be a positive multiple of 8");
  if (c.has_embed != c.has_head) return bad("has_embed and has_head must be set together (full LM) or both clear (stage)");
  if (c.has_embed && c.vocab < 1) return bad("vocab missing");
  if (c.n_microbatch < 1 || c.n_microbatch > 64) return bad("n_microbatch out of range");
  if (c.has_head && c.n_microbatch != 1) return bad("a full LM step uses one micro-batch");
  if (c.optimizer != 1 && c.optimizer != 2) return bad("optimizer must be 1 (SGD) or 2 (Adam)");
  if ((int64_t)c.batch * c.n_head > 65535) return bad("batch * n_head too large");
  if ((int64_t)c.batch * c.seq > (1 << 24)) return bad("too many tokens");
  // the token count is the contraction length of every weight-gradient GEMM, and bf16 operands move in 16-byte pieces
  if (c.bf16 && ((int64_t)c.batch * c.seq) % 8) return bad("bf16 needs batch * seq to be a multiple of 8");
  return true;
}

// The LM-head GEMM [N, d] . [d, V], as far as the launcher's choice of kernel goes.
static GemmArgs head_fwd_shape(const pw_lm_config& c) {
  GemmArgs a{};
  a.dtype = kBF16; a.a_kmajor = 0; a.b_kmajor = 1;
  a.M = (int64_t)c.batch * c.seq; a.N = c.vocab; a.K = c.d_model; a.lda = a.K; a.ldb = a.N; a.ldc = a.N;
  a.epilogue = kEpiStore; a.out_dtype = kBF16;
  return a;
}

hipError_t model_create(const pw_lm_config& cfg, hipStream_t stream, Model** out, std::string* err) {
  std::string why;
  if (!model_config_ok(cfg, &why)) {
    if (err) *err = why;
    return hipErrorInvalidValue;
  }
  Model* m = new Model();
  m->cfg = cfg;
  m->stream = stream;
  m->bf16 = cfg.bf16 ? 1 : 0;
  build_param_table(cfg, m->params, m->total, m->fused_from);
  m->fused_head = cfg.fused_head_loss && cfg.bf16 && cfg.has_head && gemm_xent_fusable(head_fwd_shape(cfg));
  hipError_t e = model_state_alloc(m, opt_of(cfg), err);
  if (e != hipSuccess) {
    delete m;
    return e;
  }
  m->act_bytes = plan(m, nullptr);
  if ((e = hipMalloc(&m->act, m->act_bytes)) != hipSuccess) {
    if (err) *err = std::string("alloc activations: ") + hipGetErrorString(e);
    model_destroy(m);
    return e;
  }
  plan(m, m->act);
  m->flush_pending = [](ModelBase* base) {   // someone outside is about to read or write the gradients
    Model* self = static_cast<Model*>(base);
    const hipError_t e = flush_wgrads(self);
    self->wgrads_zero = false;
    return e;
  };
  *out = m;
  return hipSuccess;
}

void model_destroy(Model* m) {
  if (!m) return;
  model_state_free(m);
  (void)hipFree(m->act);
  delete m;
}

hipError_t model_refresh_lowp(Model* m, int64_t offset, int64_t numel) { return model_state_refresh_lowp(m, offset, numel); }

hipError_t model_zero_grads(Model* m) {
  std::fill(m->pending.begin(), m->pending.end(), 0);   // contributions held back go the way of the ones in g
  PW_TRY(launch_fill_f32(m->stream, m->g, m->total, 0.f), "zero grads");
  m->wgrads_zero = true;
  return hipSuccess;
}

hipError_t model_before_graph(Model* m, bool backward) {
  const hipError_t e = flush_wgrads(m);   // with acc = 0 only into gradients that nothing has touched since zeroing
  if (e != hipSuccess) return e;
  if (backward) m->wgrads_zero = false;
  return hipSuccess;
}

hipError_t model_apply_optimizer(Model* m) {
  const pw_lm_config& c = m->cfg;
  hipError_t e = flush_wgrads(m);
  if (e != hipSuccess) return e;
  return model_state_apply_optimizer(m, opt_of(c));
}

hipError_t model_train_step(Model* m, const int32_t* tokens, float* loss) {
  const pw_lm_config& c = m->cfg;
  if (!c.has_embed || !c.has_head) {
    m->error = "train step needs a full LM (has_embed and has_head)";
    return hipErrorInvalidValue;
  }
  const int N = m->N(), d = c.d_model, V = c.vocab;
  const int dt = m->act_dtype();
  Model::Slot& s = m->slots[0];
  const size_t tail = layer_base(m, c.n_layer);
  PW_TRY(launch_embedding_fwd(m->stream, tokens, m->w + P(m, 0).offset, m->w + P(m, 1).offset, s.layer[0].x_in, c.batch, c.seq, d, V), "embedding fwd");
  hipError_t e = layers_forward(m, s);
  if (e != hipSuccess) return e;
  PW_TRY(launch_layernorm_fwd(m->stream, dt, s.x_out, m->w + P(m, tail).offset, m->w + P(m, tail + 1).offset, m->y, m->meanf, m->rstdf, N, d), "lnf fwd");
  if (m->fused_head) {
    // The head GEMM fused with the loss: the logits never reach memory.  A first pass over the product leaves only
    // softmax statistics per 64-column group (and the target's logit); a second pass over the same product writes
    // the gradient of the logits straight from the accumulators.
    GemmArgs hz = head_fwd_shape(c);
    hz.A = m->y;
    hz.B = (const uint16_t*)m->wlp + P(m, tail + 2).offset;
    hz.epilogue = kEpiXentStats;
    hz.C = nullptr;
    hz.xent = XentEpi{tokens, c.seq, m->xe_part, m->xe_zt, m->xe_lse, 1.f / (float)N};
    PW_TRY(launch_gemm(m->stream, hz), "head gemm + softmax statistics");
    PW_TRY(launch_xent_from_stats(m->stream, m->xe_part, m->xe_zt, m->xe_lse, m->row_loss, loss, N, V / 64), "loss from statistics");
    hz.epilogue = kEpiXentGrad;
    hz.C = m->logits;
    PW_TRY(launch_gemm(m->stream, hz), "head gemm + gradient of the logits");
  } else {
    PW_TRY(gemm_fwd(m, m->y, tail + 2, nullptr, N, d, V, kEpiStore, dt, nullptr, m->logits, nullptr), "head gemm");
    PW_TRY(launch_softmax_xent(m->stream, dt, m->logits, tokens, loss, m->row_loss, c.batch, c.seq, V), "softmax-xent");
  }
  // head backward: logits now hold dlogits (the data gradient first: see layers_backward)
  PW_TRY(gemm_dgrad(m, m->logits, tail + 2, N, d, V, kEpiStore, nullptr, m->d_small, dt, 0), "head dgrad");
  PW_TRY(launch_gemm(m->stream, fused_plan(c).wh && m->fused_from >= 0 ? wgrad_adam_args(m, opt_of(c), m->y, m->logits, tail + 2, N, d, V)
                                                                         : wgrad_args(m, m->y, m->logits, tail + 2, N, d, V, 0)), "head wgrad");
  PW_TRY(launch_layernorm_bwd(m->stream, dt, m->d_small, s.x_out, m->w + P(m, tail).offset, m->meanf, m->rstdf, nullptr, m->dx_a,
                              c.bf16 ? m->dx_lp : nullptr, m->g + P(m, tail).offset, m->g + P(m, tail + 1).offset,
                              c.n_layer > 0 ? m->g + P(m, layer_base(m, c.n_layer - 1) + 11).offset : nullptr, m->ws, N, d, 0), "lnf bwd");
  e = layers_backward(m, s, 0, true, false);
  if (e != hipSuccess) return e;
  PW_TRY(launch_embedding_bwd(m->stream, tokens, m->dx_a, m->g + P(m, 0).offset, m->g + P(m, 1).offset, c.batch, c.seq, d, V), "embedding bwd");
  return model_apply_optimizer(m);
}

hipError_t model_stage_fwd(Model* m, int mb, const float* x, float* y) {
  const pw_lm_config& c = m->cfg;
  if (c.has_embed || c.has_head || mb < 0 || mb >= c.n_microbatch) {
    m->error = "stage_fwd: not a pipeline-stage model or bad micro-batch index";
    return hipErrorInvalidValue;
  }
  Model::Slot& s = m->slots[mb];
  if (m->pending[mb]) {   // the activations about to be overwritten are operands of weight gradients held back
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    PW_TRY(hipStreamIsCapturing(m->stream, &cap), "capture status");
    if (cap != hipStreamCaptureStatusNone) {
      m->error = "stage_fwd under graph capture while weight gradients of this micro-batch are held back: apply the optimizer or zero the gradients first";
      return hipErrorInvalidValue;
    }
    hipError_t e = flush_wgrads(m);
    if (e != hipSuccess) return e;
  }
  const int64_t bytes = (int64_t)m->N() * c.d_model * 4;
  PW_TRY(launch_copy_bytes(m->stream, x, s.layer[0].x_in, bytes), "stage input copy");
  hipError_t e = layers_forward(m, s);
  if (e != hipSuccess) return e;
  PW_TRY(launch_copy_bytes(m->stream, s.x_out, y, bytes), "stage output copy");
  return hipSuccess;
}

hipError_t model_stage_bwd(Model* m, int mb, const float* dy, float* dx) {
  const pw_lm_config& c = m->cfg;
  if (c.has_embed || c.has_head || mb < 0 || mb >= c.n_microbatch) {
    m->error = "stage_bwd: not a pipeline-stage model or bad micro-batch index";
    return hipErrorInvalidValue;
  }
  Model::Slot& s = m->slots[mb];
  // Work held back lives in host-side bookkeeping, which the replay of a captured graph would not repeat: a call
  // that is being captured does all of its work at once.
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  PW_TRY(hipStreamIsCapturing(m->stream, &cap), "capture status");
  const bool capturing = cap != hipStreamCaptureStatusNone;
  if (m->pending[mb]) {   // a second backward pass of this micro-batch: the first one's contribution goes in first
    if (capturing) {
      m->error = "stage_bwd under graph capture while weight gradients of this micro-batch are held back: apply the optimizer or zero the gradients first";
      return hipErrorInvalidValue;
    }
    hipError_t e = flush_wgrads(m);
    if (e != hipSuccess) return e;
  }
  const bool defer = m->defer_wgrad && !capturing;
  const int64_t n = (int64_t)m->N() * c.d_model;
  PW_TRY(launch_copy_bytes(m->stream, dy, m->dx_a, n * 4), "stage grad-output copy");
  if (c.bf16)
    PW_TRY(launch_f32_to_bf16(m->stream, dy, defer ? s.layer[c.n_layer - 1].g_y2 : m->dx_lp, n), "stage grad-output to bf16");
  hipError_t e = layers_backward(m, s, 1, false, defer);
  if (e != hipSuccess) return e;
  if (defer) m->pending[mb] = 1;
  else m->wgrads_zero = false;
  PW_TRY(launch_copy_bytes(m->stream, m->dx_a, dx, n * 4), "stage grad-input copy");
  return hipSuccess;
}

double model_step_flops(const pw_lm_config& c) {
  const double N = (double)c.batch * c.seq, d = c.d_model, F = c.d_ff, V = c.has_head ? c.vocab : 0, L = c.n_layer;
  const double per_layer = d * 3 * d + d * d + 2 * d * F;          // multiply-adds per token, forward
  const double gemm = 6.0 * N * (L * per_layer + d * V);           // x2 flops, x3 fwd + dgrad + wgrad
  const double attn = 6.0 * c.batch * (double)c.seq * c.seq * d * L;   // causal half of QK^T, PV and their 4 backward products
  return (gemm + attn) * c.n_microbatch;
}

}  // namespace pw
