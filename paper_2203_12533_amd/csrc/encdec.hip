// The encoder-decoder train step: forward, backward and optimiser update as an ordered list of kernel launches
// on one stream.  The workload stands for the text-to-text Transformers of the paper's Table 1, whose recipe
// the paper does not give; it is assembled from the residual sub-blocks of the decoder-only model (lm.hip):
//   encoder layer: x += SelfAttn_unmasked(LN x);  x += FFN(LN x)
//   decoder layer: y += SelfAttn_causal(LN y);  y += Attn(q from LN y; keys, values from mem);  y += FFN(LN y)
//   mem = LN(encoder stack output);  logits = LN(decoder stack output) Wh;  next-token loss on the target side.
// Every sub-block has the form x_out = x_in + f(LN(x_in)) and ends in a projection with a bias; the gradient of
// that bias is the column sum of the gradient w.r.t. x_out, which the LayerNorm backward that produces that
// gradient delivers for free (its `dsum` output) - so each sub-block's backward takes the address of the bias
// gradient of the sub-block below it.
// Precision as in lm.hip: bf16 operands, fp32 residual stream, statistics, accumulators, gradients and state.
// One thing more: every attention keeps, next to its bf16 output, what the rounding left over (o_lo), so that the
// backward pass's delta = rowsum(dO * O) is exact to fp32.  Here the query projection of the cross-attention has a
// weight tensor of its own, and at initialisation (near-uniform attention over keys that share a common
// component) that one rounding alone put 3 to 4 per cent of error into its gradient.
#include "encdec.hpp"

#include <algorithm>
#include <cmath>

#include "kernels.hpp"

namespace pw {

namespace {

constexpr int kSelfParams = 6, kCrossParams = 8, kFfnParams = 6;
constexpr int kEncLayerParams = kSelfParams + kFfnParams, kDecLayerParams = kSelfParams + kCrossParams + kFfnParams;

OptimizerConfig opt_of(const pw_encdec_config& c) { return OptimizerConfig{c.optimizer, c.lr, c.beta1, c.beta2, c.eps}; }

// Whether every GEMM weight of the step gets its Adam update inside its weight-gradient GEMM: all of them or none, and
// all only if each of those GEMMs - alone or as a member of the launch it shares - runs on the ring kernel's full tiles.
bool fused_update_possible(const pw_encdec_config& c) {
  if (!c.fused_update || !c.bf16 || c.optimizer != 2) return false;
  const int64_t Ns = (int64_t)c.batch * c.src_len, Nt = (int64_t)c.batch * c.tgt_len, d = c.d_model, F = c.d_ff, V = c.vocab;
  auto shape = [](int64_t N, int64_t in, int64_t out) {
    GemmArgs a{};
    a.dtype = kBF16; a.a_kmajor = 1; a.b_kmajor = 1;
    a.M = in; a.N = out; a.K = N; a.lda = in; a.ldb = out; a.ldc = out;
    a.epilogue = kEpiStore; a.out_dtype = kF32;
    return a;
  };
  auto group_ok = [](const GemmArgs* g, int n) {
    const bool shared = gemm_group_shares_launch(g, n);
    for (int i = 0; i < n; ++i)
      if (!gemm_adam_fusable(g[i], shared)) return false;
    return true;
  };
  bool ok = true;
  for (int64_t N : {Ns, Nt}) {
    const GemmArgs pair[2] = {shape(N, d, 3 * d), shape(N, d, d)};
    ok = ok && group_ok(pair, 2) && gemm_adam_fusable(shape(N, d, F), false) && gemm_adam_fusable(shape(N, F, d), false);
  }
  const GemmArgs cross[3] = {shape(Ns, d, 2 * d), shape(Nt, d, d), shape(Nt, d, d)};
  return ok && group_ok(cross, 3) && gemm_adam_fusable(shape(Nt, d, V), false);
}

void build_param_table(const pw_encdec_config& c, std::vector<ParamInfo>& t, int64_t& total, int64_t& fused_from) {
  ParamTableBuilder tb{t};
  const bool fz = fused_update_possible(c);
  auto add = [&](const std::string& n, int64_t numel, bool gemm_weight = false) { tb.add(n, numel, gemm_weight && fz); };
  const int64_t d = c.d_model, F = c.d_ff, V = c.vocab;
  auto self = [&](const std::string& p) {
    add(p + "ln1_g", d); add(p + "ln1_b", d);
    add(p + "wqkv", d * 3 * d, true); add(p + "bqkv", 3 * d);
    add(p + "wo", d * d, true); add(p + "bo", d);
  };
  auto ffn = [&](const std::string& p) {
    add(p + "ln2_g", d); add(p + "ln2_b", d);
    add(p + "w1", d * F, true); add(p + "b1", F);
    add(p + "w2", F * d, true); add(p + "b2", d);
  };
  add("enc.wte", V * d);
  add("enc.wpe", (int64_t)c.src_len * d);
  for (int l = 0; l < c.n_enc_layer; ++l) {
    const std::string p = "e" + std::to_string(l) + ".";
    self(p);
    ffn(p);
  }
  add("enc.lnf_g", d); add("enc.lnf_b", d);
  add("dec.wte", V * d);
  add("dec.wpe", (int64_t)c.tgt_len * d);
  for (int l = 0; l < c.n_dec_layer; ++l) {
    const std::string p = "d" + std::to_string(l) + ".";
    self(p);
    add(p + "lnx_g", d); add(p + "lnx_b", d);
    add(p + "wq", d * d, true); add(p + "bq", d);
    add(p + "wkv", d * 2 * d, true); add(p + "bkv", 2 * d);
    add(p + "wox", d * d, true); add(p + "box", d);
    ffn(p);
  }
  add("dec.lnf_g", d); add("dec.lnf_b", d);
  add("wh", d * V, true);
  tb.finish(total, fused_from);
}

// parameter indices
size_t enc_layer_base(int l) { return 2 + (size_t)l * kEncLayerParams; }
size_t enc_tail(const pw_encdec_config& c) { return enc_layer_base(c.n_enc_layer); }          // lnf_g, lnf_b
size_t dec_embed(const pw_encdec_config& c) { return enc_tail(c) + 2; }                        // wte, wpe
size_t dec_layer_base(const pw_encdec_config& c, int l) { return dec_embed(c) + 2 + (size_t)l * kDecLayerParams; }
size_t dec_tail(const pw_encdec_config& c) { return dec_layer_base(c, c.n_dec_layer); }       // lnf_g, lnf_b, wh

// Assigns every activation / scratch pointer; with base == nullptr only measures.
size_t plan(EncDec* m, unsigned char* base) {
  const pw_encdec_config& c = m->cfg;
  const size_t Ns = (size_t)m->Ns(), Nt = (size_t)m->Nt(), Nmax = std::max(Ns, Nt);
  const size_t d = c.d_model, F = c.d_ff, V = c.vocab;
  const size_t es = c.bf16 ? 2 : 4;
  const size_t BH = (size_t)c.batch * c.n_head;
  Carver cv;
  cv.base = base;
  auto self = [&](EncDec::SelfActs& a, size_t N, size_t T) {
    a.x_in = cv.take<float>(N * d * 4);
    a.lse = cv.take<float>(BH * T * 4);
    a.mean = cv.take<float>(N * 4);
    a.rstd = cv.take<float>(N * 4);
    a.a = cv.take<void>(N * d * es);
    a.qkv = cv.take<void>(N * 3 * d * es);
    a.o = cv.take<void>(N * d * es);
    a.o_lo = c.bf16 ? cv.take<void>(N * d * es) : nullptr;
  };
  auto ffn = [&](EncDec::FfnActs& a, size_t N) {
    a.x_in = cv.take<float>(N * d * 4);
    a.mean = cv.take<float>(N * 4);
    a.rstd = cv.take<float>(N * 4);
    a.mm = cv.take<void>(N * d * es);
    a.u = cv.take<void>(N * F * es);
    a.h = cv.take<void>(N * F * es);
  };
  m->enc.resize(c.n_enc_layer);
  for (auto& L : m->enc) {
    self(L.sa, Ns, c.src_len);
    ffn(L.ff, Ns);
  }
  m->enc_x_out = cv.take<float>(Ns * d * 4);
  m->enc_meanf = cv.take<float>(Ns * 4);
  m->enc_rstdf = cv.take<float>(Ns * 4);
  m->mem = cv.take<void>(Ns * d * es);
  m->dec.resize(c.n_dec_layer);
  for (auto& L : m->dec) {
    self(L.sa, Nt, c.tgt_len);
    L.ca.x_in = cv.take<float>(Nt * d * 4);
    L.ca.lse = cv.take<float>(BH * c.tgt_len * 4);
    L.ca.mean = cv.take<float>(Nt * 4);
    L.ca.rstd = cv.take<float>(Nt * 4);
    L.ca.a = cv.take<void>(Nt * d * es);
    L.ca.q = cv.take<void>(Nt * d * es);
    L.ca.kv = cv.take<void>(Ns * 2 * d * es);
    L.ca.o = cv.take<void>(Nt * d * es);
    L.ca.o_lo = c.bf16 ? cv.take<void>(Nt * d * es) : nullptr;
    ffn(L.ff, Nt);
  }
  m->dec_x_out = cv.take<float>(Nt * d * 4);
  m->meanf = cv.take<float>(Nt * 4);
  m->rstdf = cv.take<float>(Nt * 4);
  m->row_loss = cv.take<float>(Nt * 4);
  m->y = cv.take<void>(Nt * d * es);
  m->logits = cv.take<void>(Nt * V * es);
  m->dx_a = cv.take<float>(Nmax * d * 4);
  m->dx_b = cv.take<float>(Nmax * d * 4);
  m->dmem = cv.take<float>(Ns * d * 4);
  m->delta = cv.take<float>(BH * std::max(c.src_len, c.tgt_len) * 4);
  m->dx_lp = cv.take<void>(Nmax * d * es);
  m->dx_lp2 = c.bf16 ? cv.take<void>(Nmax * d * es) : nullptr;
  m->d_big = cv.take<void>(Nmax * F * es);
  m->d_qkv = cv.take<void>(Nmax * 3 * d * es);
  m->d_small = cv.take<void>(Nmax * d * es);
  m->d_q = cv.take<void>(Nt * d * es);
  int64_t wsf = layernorm_bwd_ws_floats((int)Nmax, (int)d);
  wsf = std::max(wsf, colsum_ws_floats((int64_t)Nmax, (int64_t)std::max(3 * d, F)));
  m->ws = cv.take<float>((size_t)wsf * 4);
  return cv.off;
}

// The gradient w.r.t. the residual stream travels in two fp32 buffers that alternate (a LayerNorm backward reads
// one as the residual branch and writes the sum to the other) plus, in bf16 mode, a bf16 copy of the current
// one, the GEMM operand, which alternates between two buffers likewise: a sub-block's LayerNorm backward runs right
// behind the data-gradient GEMM that produced its input (while that is still in the caches) and writes the copy for
// the sub-block below, and the weight-gradient GEMMs that follow still read the copy of this sub-block.
struct GradStream {
  float* cur;
  float* other;
  void* lp_cur;     // bf16 copy of cur (bf16 mode)
  void* lp_other;
  void swap() { std::swap(cur, other); std::swap(lp_cur, lp_other); }
};

const void* grad_operand(const EncDec* m, const GradStream& gs) { return m->bf16 ? (const void*)gs.lp_cur : (const void*)gs.cur; }

// The weight-gradient GEMM of weight wi = x^T dy over N rows - with the weight's Adam update in its epilogue when the
// model updates its GEMM weights that way.  Such a GEMM rewrites the weight's bf16 copy, so every backward routine
// below runs a weight's data-gradient GEMM (which reads that copy) before its weight-gradient GEMM.
GemmArgs wgrad_of(EncDec* m, const void* x, const void* dy, int64_t wi, int64_t N, int64_t in, int64_t out) {
  return m->fused_from >= 0 ? wgrad_adam_args(m, opt_of(m->cfg), x, dy, wi, N, in, out) : wgrad_args(m, x, dy, wi, N, in, out, 0);
}

// x_out = x_in + Attn(LN(x_in) Wqkv + bqkv) Wo + bo over T positions per batch; parameters e .. e+5.
hipError_t self_fwd(EncDec* m, size_t e, const EncDec::SelfActs& A, float* x_out, int N, int T, int causal) {
  const pw_encdec_config& c = m->cfg;
  const int d = c.d_model, dt = m->act_dtype();
  PW_TRY(launch_layernorm_fwd(m->stream, dt, A.x_in, m->wp(e), m->wp(e + 1), A.a, A.mean, A.rstd, N, d), "self-attention LN fwd");
  PW_TRY(gemm_fwd(m, A.a, e + 2, m->wp(e + 3), N, d, 3 * d, kEpiBias, dt, nullptr, A.qkv, nullptr), "qkv gemm");
  const size_t es = m->bf16 ? 2 : 4;
  const char* qkv = (const char*)A.qkv;
  const MhaArgs a{dt, qkv, qkv + d * es, qkv + 2 * d * es, 3 * (int64_t)d, 3 * (int64_t)d, c.batch, T, T, c.n_head, m->hd(), causal};
  PW_TRY(launch_mha_fwd(m->stream, a, A.o, A.o_lo, A.lse), "self-attention fwd");
  PW_TRY(gemm_fwd(m, A.o, e + 4, m->wp(e + 5), N, d, d, kEpiBiasResidual, kF32, A.x_in, x_out, nullptr), "out-proj gemm");
  return hipSuccess;
}

// Backward of the above.  gs.cur: gradient w.r.t. x_out on entry, w.r.t. x_in on return (buffers swapped).
// below_bias: gradient slot of the bias of the projection that wrote x_in, or null.
hipError_t self_bwd(EncDec* m, size_t e, const EncDec::SelfActs& A, GradStream& gs, float* below_bias, int N, int T, int causal) {
  const pw_encdec_config& c = m->cfg;
  const int d = c.d_model, dt = m->act_dtype();
  const void* dy = grad_operand(m, gs);
  PW_TRY(gemm_dgrad(m, dy, e + 4, N, d, d, kEpiStore, nullptr, m->d_small, dt, 0), "out-proj dgrad");
  const size_t es = m->bf16 ? 2 : 4;
  const char* qkv = (const char*)A.qkv;
  char* dqkv = (char*)m->d_qkv;
  const MhaArgs a{dt, qkv, qkv + d * es, qkv + 2 * d * es, 3 * (int64_t)d, 3 * (int64_t)d, c.batch, T, T, c.n_head, m->hd(), causal};
  PW_TRY(launch_mha_bwd(m->stream, a, A.o, A.o_lo, m->d_small, A.lse, m->delta, dqkv, 3 * (int64_t)d, dqkv + d * es, dqkv + 2 * d * es,
                        3 * (int64_t)d), "self-attention bwd");
  // (d_small, the attention backward's input, is free again and takes the QKV data gradient)
  PW_TRY(gemm_dgrad(m, m->d_qkv, e + 2, N, d, 3 * d, kEpiStore, nullptr, m->d_small, dt, 0), "qkv dgrad");
  PW_TRY(launch_layernorm_bwd(m->stream, dt, m->d_small, A.x_in, m->wp(e), A.mean, A.rstd, gs.cur, gs.other,
                              m->bf16 ? gs.lp_other : nullptr, m->gp(e), m->gp(e + 1), below_bias, m->ws, N, d, 0), "self-attention LN bwd");
  {
    const WgradJob jobs[2] = {{wgrad_of(m, A.a, m->d_qkv, e + 2, N, d, 3 * d), (int64_t)e + 3},
                              {wgrad_of(m, A.o, dy, e + 4, N, d, d), -1}};
    PW_TRY(gemm_wgrad_group(m, jobs, 2, m->ws), "qkv + out-proj wgrad + bqkv grad");
  }
  gs.swap();
  return hipSuccess;
}

// y_out = y_in + Attn(q = LN(y_in) Wq + bq; [K|V] = mem Wkv + bkv) Wox + box; parameters e .. e+7
// (lnx_g, lnx_b, wq, bq, wkv, bkv, wox, box).
hipError_t cross_fwd(EncDec* m, size_t e, const EncDec::CrossActs& A, float* y_out) {
  const pw_encdec_config& c = m->cfg;
  const int d = c.d_model, dt = m->act_dtype(), Nt = m->Nt(), Ns = m->Ns();
  PW_TRY(launch_layernorm_fwd(m->stream, dt, A.x_in, m->wp(e), m->wp(e + 1), A.a, A.mean, A.rstd, Nt, d), "cross-attention LN fwd");
  PW_TRY(gemm_fwd(m, A.a, e + 2, m->wp(e + 3), Nt, d, d, kEpiBias, dt, nullptr, A.q, nullptr), "cross q gemm");
  PW_TRY(gemm_fwd(m, m->mem, e + 4, m->wp(e + 5), Ns, d, 2 * d, kEpiBias, dt, nullptr, A.kv, nullptr), "cross kv gemm");
  const size_t es = m->bf16 ? 2 : 4;
  const char* kv = (const char*)A.kv;
  const MhaArgs a{dt, A.q, kv, kv + d * es, (int64_t)d, 2 * (int64_t)d, c.batch, c.tgt_len, c.src_len, c.n_head, m->hd(), 0};
  PW_TRY(launch_mha_fwd(m->stream, a, A.o, A.o_lo, A.lse), "cross-attention fwd");
  PW_TRY(gemm_fwd(m, A.o, e + 6, m->wp(e + 7), Nt, d, d, kEpiBiasResidual, kF32, A.x_in, y_out, nullptr), "cross out-proj gemm");
  return hipSuccess;
}

// dmem_accumulate: 0 for the first sub-block visited (it overwrites dmem), 1 afterwards.
hipError_t cross_bwd(EncDec* m, size_t e, const EncDec::CrossActs& A, GradStream& gs, float* below_bias, int dmem_accumulate) {
  const pw_encdec_config& c = m->cfg;
  const int d = c.d_model, dt = m->act_dtype(), Nt = m->Nt(), Ns = m->Ns();
  const void* dy = grad_operand(m, gs);
  PW_TRY(gemm_dgrad(m, dy, e + 6, Nt, d, d, kEpiStore, nullptr, m->d_small, dt, 0), "cross out-proj dgrad");
  const size_t es = m->bf16 ? 2 : 4;
  const char* kv = (const char*)A.kv;
  char* dkv = (char*)m->d_qkv;
  const MhaArgs a{dt, A.q, kv, kv + d * es, (int64_t)d, 2 * (int64_t)d, c.batch, c.tgt_len, c.src_len, c.n_head, m->hd(), 0};
  PW_TRY(launch_mha_bwd(m->stream, a, A.o, A.o_lo, m->d_small, A.lse, m->delta, m->d_q, (int64_t)d, dkv, dkv + d * es, 2 * (int64_t)d),
         "cross-attention bwd");
  PW_TRY(gemm_dgrad(m, dkv, e + 4, Ns, d, 2 * d, kEpiStore, nullptr, m->dmem, kF32, dmem_accumulate), "cross kv dgrad");
  PW_TRY(gemm_dgrad(m, m->d_q, e + 2, Nt, d, d, kEpiStore, nullptr, m->d_small, dt, 0), "cross q dgrad");
  PW_TRY(launch_layernorm_bwd(m->stream, dt, m->d_small, A.x_in, m->wp(e), A.mean, A.rstd, gs.cur, gs.other,
                              m->bf16 ? gs.lp_other : nullptr, m->gp(e), m->gp(e + 1), below_bias, m->ws, Nt, d, 0), "cross-attention LN bwd");
  {
    // three weight gradients that each cover a quarter to a half of the chip: one launch
    const WgradJob jobs[3] = {{wgrad_of(m, m->mem, dkv, e + 4, Ns, d, 2 * d), (int64_t)e + 5},
                              {wgrad_of(m, A.a, m->d_q, e + 2, Nt, d, d), (int64_t)e + 3},
                              {wgrad_of(m, A.o, dy, e + 6, Nt, d, d), -1}};
    PW_TRY(gemm_wgrad_group(m, jobs, 3, m->ws), "cross kv + q + out-proj wgrad + bias grads");
  }
  gs.swap();
  return hipSuccess;
}

// x_out = x_in + gelu(LN(x_in) W1 + b1) W2 + b2; parameters e .. e+5.
hipError_t ffn_fwd(EncDec* m, size_t e, const EncDec::FfnActs& A, float* x_out, int N) {
  const int d = m->cfg.d_model, F = m->cfg.d_ff, dt = m->act_dtype();
  PW_TRY(launch_layernorm_fwd(m->stream, dt, A.x_in, m->wp(e), m->wp(e + 1), A.mm, A.mean, A.rstd, N, d), "ffn LN fwd");
  PW_TRY(gemm_fwd(m, A.mm, e + 2, m->wp(e + 3), N, d, F, kEpiBiasGelu, dt, nullptr, A.u, A.h), "ffn1 gemm");
  PW_TRY(gemm_fwd(m, A.h, e + 4, m->wp(e + 5), N, F, d, kEpiBiasResidual, kF32, A.x_in, x_out, nullptr), "ffn2 gemm");
  return hipSuccess;
}

hipError_t ffn_bwd(EncDec* m, size_t e, const EncDec::FfnActs& A, GradStream& gs, float* below_bias, int N) {
  const int d = m->cfg.d_model, F = m->cfg.d_ff, dt = m->act_dtype();
  const void* dy = grad_operand(m, gs);
  const OptimizerConfig opt = opt_of(m->cfg);
  PW_TRY(gemm_dgrad(m, dy, e + 4, N, F, d, kEpiGeluBwd, A.u, m->d_big, dt, 0), "ffn2 dgrad + gelu'");
  PW_TRY(gemm_dgrad(m, m->d_big, e + 2, N, d, F, kEpiStore, nullptr, m->d_small, dt, 0), "ffn1 dgrad");
  PW_TRY(launch_layernorm_bwd(m->stream, dt, m->d_small, A.x_in, m->wp(e), A.mean, A.rstd, gs.cur, gs.other,
                              m->bf16 ? gs.lp_other : nullptr, m->gp(e), m->gp(e + 1), below_bias, m->ws, N, d, 0), "ffn LN bwd");
  PW_TRY(launch_gemm(m->stream, wgrad_of(m, A.h, dy, e + 4, N, F, d)), "ffn2 wgrad");
  PW_TRY(gemm_wgrad_bias(m, A.mm, m->d_big, e + 2, e + 3, N, d, F, 0, m->ws, m->fused_from >= 0 ? &opt : nullptr), "ffn1 wgrad + b1 grad");
  gs.swap();
  return hipSuccess;
}

}  // namespace

bool encdec_config_ok(const pw_encdec_config& c, std::string* why) {
  auto bad = [&](const char* s) {
    if (why) *why = s;
    return false;
  };
  if (c.n_enc_layer < 1 || c.n_dec_layer < 1 || c.d_model < 1 || c.n_head < 1 || c.d_ff < 1 || c.src_len < 1 || c.tgt_len < 1 ||
      c.batch < 1)
    return bad("non-positive dimension");
  if (c.d_model % c.n_head) return bad("d_model must be a multiple of n_head");
  const int hd = c.d_model / c.n_head;
  if (hd != 64 && hd != 128) return bad("head_dim must be 64 or 128");
  if (c.d_model % 64 || c.d_ff % 64) return bad("d_model and d_ff must be multiples of 64");
  if (c.d_model > 8192) return bad("d_model above 8192 is not supported by the row kernels");
  if (c.vocab < 8 || c.vocab % 8) return bad("vocab must be a positive multiple of 8");
  if (c.optimizer != 1 && c.optimizer != 2) return bad("optimizer must be 1 (SGD) or 2 (Adam)");
  if ((int64_t)c.batch * c.n_head > 65535) return bad("batch * n_head too large");
  if ((int64_t)c.batch * std::max(c.src_len, c.tgt_len) > (1 << 24)) return bad("too many tokens");
  // the token count is the contraction length of every weight-gradient GEMM, and bf16 operands move in 16-byte pieces
  if (c.bf16 && (((int64_t)c.batch * c.src_len) % 8 || ((int64_t)c.batch * c.tgt_len) % 8))
    return bad("bf16 needs batch * src_len and batch * tgt_len to be multiples of 8");
  return true;
}

hipError_t encdec_create(const pw_encdec_config& cfg, hipStream_t stream, EncDec** out, std::string* err) {
  std::string why;
  if (!encdec_config_ok(cfg, &why)) {
    if (err) *err = why;
    return hipErrorInvalidValue;
  }
  EncDec* m = new EncDec();
  m->cfg = cfg;
  m->stream = stream;
  m->bf16 = cfg.bf16 ? 1 : 0;
  build_param_table(cfg, m->params, m->total, m->fused_from);
  hipError_t e = model_state_alloc(m, OptimizerConfig{cfg.optimizer, cfg.lr, cfg.beta1, cfg.beta2, cfg.eps}, err);
  if (e != hipSuccess) {
    delete m;
    return e;
  }
  m->act_bytes = plan(m, nullptr);
  if ((e = hipMalloc(&m->act, m->act_bytes)) != hipSuccess) {
    if (err) *err = std::string("alloc activations: ") + hipGetErrorString(e);
    encdec_destroy(m);
    return e;
  }
  plan(m, m->act);
  *out = m;
  return hipSuccess;
}

void encdec_destroy(EncDec* m) {
  if (!m) return;
  model_state_free(m);
  (void)hipFree(m->act);
  delete m;
}

hipError_t encdec_train_step(EncDec* m, const int32_t* src, const int32_t* tgt, float* loss) {
  const pw_encdec_config& c = m->cfg;
  const int Ns = m->Ns(), Nt = m->Nt(), d = c.d_model, V = c.vocab, dt = m->act_dtype();
  const int Le = c.n_enc_layer, Ld = c.n_dec_layer;
  const size_t et = enc_tail(c), de = dec_embed(c), dtl = dec_tail(c);

  // ---- forward: encoder
  PW_TRY(launch_embedding_fwd(m->stream, src, m->wp(0), m->wp(1), m->enc[0].sa.x_in, c.batch, c.src_len, d, V, c.src_len), "encoder embedding fwd");
  for (int l = 0; l < Le; ++l) {
    const size_t e = enc_layer_base(l);
    EncDec::EncLayer& L = m->enc[l];
    hipError_t er = self_fwd(m, e, L.sa, L.ff.x_in, Ns, c.src_len, 0);
    if (er != hipSuccess) return er;
    er = ffn_fwd(m, e + kSelfParams, L.ff, l + 1 < Le ? m->enc[l + 1].sa.x_in : m->enc_x_out, Ns);
    if (er != hipSuccess) return er;
  }
  PW_TRY(launch_layernorm_fwd(m->stream, dt, m->enc_x_out, m->wp(et), m->wp(et + 1), m->mem, m->enc_meanf, m->enc_rstdf, Ns, d), "encoder final LN fwd");

  // ---- forward: decoder
  PW_TRY(launch_embedding_fwd(m->stream, tgt, m->wp(de), m->wp(de + 1), m->dec[0].sa.x_in, c.batch, c.tgt_len, d, V, c.tgt_len + 1), "decoder embedding fwd");
  for (int l = 0; l < Ld; ++l) {
    const size_t e = dec_layer_base(c, l);
    EncDec::DecLayer& L = m->dec[l];
    hipError_t er = self_fwd(m, e, L.sa, L.ca.x_in, Nt, c.tgt_len, 1);
    if (er != hipSuccess) return er;
    er = cross_fwd(m, e + kSelfParams, L.ca, L.ff.x_in);
    if (er != hipSuccess) return er;
    er = ffn_fwd(m, e + kSelfParams + kCrossParams, L.ff, l + 1 < Ld ? m->dec[l + 1].sa.x_in : m->dec_x_out, Nt);
    if (er != hipSuccess) return er;
  }
  PW_TRY(launch_layernorm_fwd(m->stream, dt, m->dec_x_out, m->wp(dtl), m->wp(dtl + 1), m->y, m->meanf, m->rstdf, Nt, d), "decoder final LN fwd");
  PW_TRY(gemm_fwd(m, m->y, dtl + 2, nullptr, Nt, d, V, kEpiStore, dt, nullptr, m->logits, nullptr), "head gemm");
  PW_TRY(launch_softmax_xent(m->stream, dt, m->logits, tgt, loss, m->row_loss, c.batch, c.tgt_len, V), "softmax-xent");

  // ---- backward: head (logits now hold dlogits) and decoder
  PW_TRY(gemm_dgrad(m, m->logits, dtl + 2, Nt, d, V, kEpiStore, nullptr, m->d_small, dt, 0), "head dgrad");
  PW_TRY(launch_gemm(m->stream, wgrad_of(m, m->y, m->logits, dtl + 2, Nt, d, V)), "head wgrad");
  GradStream gs{m->dx_a, m->dx_b, m->dx_lp, m->dx_lp2};
  const size_t top_dec = dec_layer_base(c, Ld - 1);
  PW_TRY(launch_layernorm_bwd(m->stream, dt, m->d_small, m->dec_x_out, m->wp(dtl), m->meanf, m->rstdf, nullptr, gs.cur,
                              m->bf16 ? gs.lp_cur : nullptr, m->gp(dtl), m->gp(dtl + 1), m->gp(top_dec + kDecLayerParams - 1), m->ws,
                              Nt, d, 0), "decoder final LN bwd");
  for (int l = Ld - 1; l >= 0; --l) {
    const size_t e = dec_layer_base(c, l);
    EncDec::DecLayer& L = m->dec[l];
    // bias below each sub-block: box, bo, and the b2 of the layer underneath
    hipError_t er = ffn_bwd(m, e + kSelfParams + kCrossParams, L.ff, gs, m->gp(e + kSelfParams + kCrossParams - 1), Nt);
    if (er != hipSuccess) return er;
    er = cross_bwd(m, e + kSelfParams, L.ca, gs, m->gp(e + kSelfParams - 1), l == Ld - 1 ? 0 : 1);
    if (er != hipSuccess) return er;
    er = self_bwd(m, e, L.sa, gs, l > 0 ? m->gp(dec_layer_base(c, l - 1) + kDecLayerParams - 1) : nullptr, Nt, c.tgt_len, 1);
    if (er != hipSuccess) return er;
  }
  PW_TRY(launch_embedding_bwd(m->stream, tgt, gs.cur, m->gp(de), m->gp(de + 1), c.batch, c.tgt_len, d, V, c.tgt_len + 1), "decoder embedding bwd");

  // ---- backward: encoder, from the gradient the cross-attention sub-blocks left in dmem
  const void* dmem_op = m->dmem;
  if (m->bf16) {
    PW_TRY(launch_f32_to_bf16(m->stream, m->dmem, m->d_small, (int64_t)Ns * d), "dmem to bf16");
    dmem_op = m->d_small;
  }
  gs = GradStream{m->dx_a, m->dx_b, m->dx_lp, m->dx_lp2};
  const size_t top_enc = enc_layer_base(Le - 1);
  PW_TRY(launch_layernorm_bwd(m->stream, dt, dmem_op, m->enc_x_out, m->wp(et), m->enc_meanf, m->enc_rstdf, nullptr, gs.cur,
                              m->bf16 ? gs.lp_cur : nullptr, m->gp(et), m->gp(et + 1), m->gp(top_enc + kEncLayerParams - 1), m->ws, Ns,
                              d, 0), "encoder final LN bwd");
  for (int l = Le - 1; l >= 0; --l) {
    const size_t e = enc_layer_base(l);
    EncDec::EncLayer& L = m->enc[l];
    hipError_t er = ffn_bwd(m, e + kSelfParams, L.ff, gs, m->gp(e + kSelfParams - 1), Ns);
    if (er != hipSuccess) return er;
    er = self_bwd(m, e, L.sa, gs, l > 0 ? m->gp(enc_layer_base(l - 1) + kEncLayerParams - 1) : nullptr, Ns, c.src_len, 0);
    if (er != hipSuccess) return er;
  }
  PW_TRY(launch_embedding_bwd(m->stream, src, gs.cur, m->gp(0), m->gp(1), c.batch, c.src_len, d, V, c.src_len), "encoder embedding bwd");

  return model_state_apply_optimizer(m, opt_of(c));
}

double encdec_step_flops(const pw_encdec_config& c) {
  const double Ns = (double)c.batch * c.src_len, Nt = (double)c.batch * c.tgt_len, d = c.d_model, F = c.d_ff, V = c.vocab;
  const double self_ffn = d * 3 * d + d * d + 2 * d * F;             // multiply-adds per token, forward
  const double enc = Ns * c.n_enc_layer * self_ffn;
  const double dec = Nt * c.n_dec_layer * (self_ffn + 2 * d * d) + Ns * c.n_dec_layer * (d * 2 * d) + Nt * d * V;
  const double gemm = 6.0 * (enc + dec);                             // x2 flops, x3 fwd + dgrad + wgrad
  // attention: QK^T and PV forward plus their 4 backward products = 12 flops per (query, key, feature), halved
  // where the mask is causal
  const double B = c.batch, Ts = c.src_len, Tt = c.tgt_len;
  const double attn = 12.0 * B * d * (c.n_enc_layer * Ts * Ts + c.n_dec_layer * (0.5 * Tt * Tt + Tt * Ts));
  return gemm + attn;
}

}  // namespace pw
