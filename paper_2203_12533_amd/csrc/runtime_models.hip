// Model-level and single-kernel entry points of the C boundary (include/pw.h): the decoder-only LM and the
// encoder-decoder as objects with parameters, gradients and optimizer state, and every kernel of the step
// as a call of its own for the kernel-level parity tests.
#include "runtime_internal.hpp"

extern "C" {

// ---- model -------------------------------------------------------------------------------------------

pw_status pw_model_create(pw_ctx* c, const pw_lm_config* cfg, pw_model** out) {
  if (!c || !cfg || !out) return PW_ERR_INVALID;
  PW_API_LOCK(c);
  std::string why;
  if (!model_config_ok(*cfg, &why)) return fail(c, PW_ERR_UNSUPPORTED, "%s", why.c_str());
  Model* m = nullptr;
  hipError_t e = model_create(*cfg, c->exec, &m, &why);
  if (e != hipSuccess) return fail(c, e == hipErrorOutOfMemory ? PW_ERR_OOM : PW_ERR_DEVICE, "%s", why.c_str());
  c->models.push_back(m);
  *out = new pw_model{c, m};
  return PW_OK;
}

pw_status pw_model_destroy(pw_model* pm) {
  if (!pm) return PW_ERR_INVALID;
  pw_ctx* c = pm->ctx;
  PW_API_LOCK(c);   // the tables edited below are read by the dispatch calls, the scheduler and the executors
  (void)hipStreamSynchronize(c->exec);
  for (size_t i = 0; i < c->models.size(); ++i)
    if (c->models[i] == pm->impl) {
      c->models.erase(c->models.begin() + i);
      model_destroy(pm->impl);
      break;
    }
  for (auto& f : c->fns)
    if (f.live && f.model == pm->impl) f.live = false;   // functions of a dead model die with it
  delete pm;
  return PW_OK;
}

// Parameter-table access shared by the two kinds of model (both keep their state in a ModelBase).
static float* part_base(ModelBase* m, int part) {
  switch (part) {
    case PW_PARAMS: return m->w;
    case PW_GRADS: return m->g;
    case PW_ADAM_M: return m->m;
    case PW_ADAM_V: return m->v;
  }
  return nullptr;
}
static pw_status state_param_info(ModelBase* m, int64_t idx, char* name, int cap, int64_t* numel) {
  if (idx < 0 || idx >= (int64_t)m->params.size()) return PW_ERR_INVALID;
  const ParamInfo& p = m->params[idx];
  if (name && cap > 0) snprintf(name, cap, "%s", p.name.c_str());
  if (numel) *numel = p.numel;
  return PW_OK;
}
static pw_status state_import(pw_ctx* c, ModelBase* m, int part, int64_t idx, const float* src, int src_on_device) {
  if (!src || idx < 0 || idx >= (int64_t)m->params.size()) return PW_ERR_INVALID;
  float* base = part_base(m, part);
  if (!base) return fail(c, PW_ERR_INVALID, "this model has no such part");
  const ParamInfo& p = m->params[idx];
  if (m->flush_pending && m->flush_pending(m) != hipSuccess) return fail(c, PW_ERR_DEVICE, "%s", m->error.c_str());
  PW_HIP(c, hipMemcpyAsync(base + p.offset, src, (size_t)p.numel * 4, src_on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, c->exec));
  if (part == PW_PARAMS) {
    hipError_t e = model_state_refresh_lowp(m, p.offset, p.numel);
    if (e != hipSuccess) return fail(c, PW_ERR_DEVICE, "bf16 refresh: %s", hipGetErrorString(e));
  }
  PW_HIP(c, hipStreamSynchronize(c->exec));
  return PW_OK;
}
static pw_status state_export(pw_ctx* c, ModelBase* m, int part, int64_t idx, float* dst) {
  if (!dst || idx < 0 || idx >= (int64_t)m->params.size()) return PW_ERR_INVALID;
  float* base = part_base(m, part);
  if (!base) return fail(c, PW_ERR_INVALID, "this model has no such part");
  const ParamInfo& p = m->params[idx];
  if (part == PW_GRADS && m->fused_from >= 0 && p.offset >= m->fused_from)
    return fail(c, PW_ERR_UNSUPPORTED, "%s is updated inside its weight-gradient GEMM (fused_update): its gradient is never stored", p.name.c_str());
  if (m->flush_pending && m->flush_pending(m) != hipSuccess) return fail(c, PW_ERR_DEVICE, "%s", m->error.c_str());
  PW_HIP(c, hipStreamSynchronize(c->exec));
  PW_HIP(c, hipMemcpy(dst, base + p.offset, (size_t)p.numel * 4, hipMemcpyDeviceToHost));
  return PW_OK;
}
// Copies n elements of a device array in the activation type out as fp32, after draining the executor stream.
static pw_status export_activation(pw_ctx* c, const void* src, int64_t n, bool is_bf16, float* dst) {
  PW_HIP(c, hipStreamSynchronize(c->exec));
  if (!is_bf16) {
    PW_HIP(c, hipMemcpy(dst, src, (size_t)n * 4, hipMemcpyDeviceToHost));
    return PW_OK;
  }
  float* tmp = nullptr;
  PW_HIP(c, hipMalloc(&tmp, (size_t)n * 4));
  hipError_t e = launch_bf16_to_f32(c->exec, src, tmp, n);
  if (e == hipSuccess) e = hipStreamSynchronize(c->exec);
  if (e == hipSuccess) e = hipMemcpy(dst, tmp, (size_t)n * 4, hipMemcpyDeviceToHost);
  (void)hipFree(tmp);
  if (e != hipSuccess) return fail(c, PW_ERR_DEVICE, "activation export: %s", hipGetErrorString(e));
  return PW_OK;
}

int64_t pw_model_param_count(pw_model* pm) { return pm ? (int64_t)pm->impl->params.size() : -1; }
pw_status pw_model_param_info(pw_model* pm, int64_t idx, char* name, int cap, int64_t* numel) {
  return pm ? state_param_info(pm->impl, idx, name, cap, numel) : PW_ERR_INVALID;
}
// The calls below enqueue on the executor stream and touch the model's host-side bookkeeping, as the dispatch calls
// do that run one of its functions: they take the same lock.
pw_status pw_model_import(pw_model* pm, int part, int64_t idx, const float* src, int src_on_device) {
  if (!pm) return PW_ERR_INVALID;
  PW_API_LOCK(pm->ctx);
  return state_import(pm->ctx, pm->impl, part, idx, src, src_on_device);
}
pw_status pw_model_export(pw_model* pm, int part, int64_t idx, float* dst) {
  if (!pm) return PW_ERR_INVALID;
  PW_API_LOCK(pm->ctx);
  return state_export(pm->ctx, pm->impl, part, idx, dst);
}

pw_status pw_model_zero_grads(pw_model* pm) {
  if (!pm) return PW_ERR_INVALID;
  PW_API_LOCK(pm->ctx);
  if (model_zero_grads(pm->impl) != hipSuccess) return fail(pm->ctx, PW_ERR_DEVICE, "%s", pm->impl->error.c_str());
  return PW_OK;
}

pw_status pw_model_apply_optimizer(pw_model* pm) {
  if (!pm) return PW_ERR_INVALID;
  PW_API_LOCK(pm->ctx);
  if (model_apply_optimizer(pm->impl) != hipSuccess) return fail(pm->ctx, PW_ERR_DEVICE, "%s", pm->impl->error.c_str());
  return PW_OK;
}

pw_status pw_model_export_activation(pw_model* pm, const char* name, int mb, float* dst, int64_t numel) {
  if (!pm || !name || !dst) return PW_ERR_INVALID;
  pw_ctx* c = pm->ctx;
  Model* m = pm->impl;
  if (mb < 0 || mb >= m->cfg.n_microbatch) return fail(c, PW_ERR_INVALID, "micro-batch index out of range");
  const int64_t N = m->N(), d = m->cfg.d_model;
  const void* src = nullptr;
  int64_t n = 0;
  int dt = PW_F32;
  const std::string s(name);
  if (s == "x_out") { src = m->slots[mb].x_out; n = N * d; }
  else if (s == "dlogits" && m->logits) { src = m->logits; n = N * m->cfg.vocab; dt = m->act_dtype(); }
  else if (s == "dx_in") { src = m->dx_a; n = N * d; }
  else return fail(c, PW_ERR_INVALID, "unknown activation name");
  if (numel != n) return fail(c, PW_ERR_SHAPE, "activation has %lld elements", (long long)n);
  return export_activation(c, src, n, dt != PW_F32, dst);
}

double pw_model_step_flops(const pw_lm_config* cfg) { return cfg ? model_step_flops(*cfg) : 0.0; }

// ---- encoder-decoder model -------------------------------------------------------------------------------

pw_status pw_encdec_create(pw_ctx* c, const pw_encdec_config* cfg, pw_encdec** out) {
  if (!c || !cfg || !out) return PW_ERR_INVALID;
  PW_API_LOCK(c);
  std::string why;
  if (!encdec_config_ok(*cfg, &why)) return fail(c, PW_ERR_UNSUPPORTED, "%s", why.c_str());
  EncDec* m = nullptr;
  hipError_t e = encdec_create(*cfg, c->exec, &m, &why);
  if (e != hipSuccess) return fail(c, e == hipErrorOutOfMemory ? PW_ERR_OOM : PW_ERR_DEVICE, "%s", why.c_str());
  c->encdecs.push_back(m);
  *out = new pw_encdec{c, m};
  return PW_OK;
}

pw_status pw_encdec_destroy(pw_encdec* pm) {
  if (!pm) return PW_ERR_INVALID;
  pw_ctx* c = pm->ctx;
  PW_API_LOCK(c);
  (void)hipStreamSynchronize(c->exec);
  for (size_t i = 0; i < c->encdecs.size(); ++i)
    if (c->encdecs[i] == pm->impl) {
      c->encdecs.erase(c->encdecs.begin() + i);
      encdec_destroy(pm->impl);
      break;
    }
  for (auto& f : c->fns)
    if (f.live && f.encdec == pm->impl) f.live = false;   // functions of a dead model die with it
  delete pm;
  return PW_OK;
}

int64_t pw_encdec_param_count(pw_encdec* pm) { return pm ? (int64_t)pm->impl->params.size() : -1; }
pw_status pw_encdec_param_info(pw_encdec* pm, int64_t idx, char* name, int cap, int64_t* numel) {
  return pm ? state_param_info(pm->impl, idx, name, cap, numel) : PW_ERR_INVALID;
}
pw_status pw_encdec_import(pw_encdec* pm, int part, int64_t idx, const float* src, int src_on_device) {
  if (!pm) return PW_ERR_INVALID;
  PW_API_LOCK(pm->ctx);
  return state_import(pm->ctx, pm->impl, part, idx, src, src_on_device);
}
pw_status pw_encdec_export(pw_encdec* pm, int part, int64_t idx, float* dst) {
  if (!pm) return PW_ERR_INVALID;
  PW_API_LOCK(pm->ctx);
  return state_export(pm->ctx, pm->impl, part, idx, dst);
}

pw_status pw_encdec_export_activation(pw_encdec* pm, const char* name, float* dst, int64_t numel) {
  if (!pm || !name || !dst) return PW_ERR_INVALID;
  pw_ctx* c = pm->ctx;
  EncDec* m = pm->impl;
  if (std::string(name) != "dlogits") return fail(c, PW_ERR_INVALID, "unknown activation name");
  const int64_t n = (int64_t)m->Nt() * m->cfg.vocab;
  if (numel != n) return fail(c, PW_ERR_SHAPE, "activation has %lld elements", (long long)n);
  return export_activation(c, m->logits, n, m->bf16 != 0, dst);
}

double pw_encdec_step_flops(const pw_encdec_config* cfg) { return cfg ? encdec_step_flops(*cfg) : 0.0; }

// ---- single kernels ------------------------------------------------------------------------------------

#define PW_OP(c, expr)                                                                               \
  do {                                                                                               \
    if (!(c)) return PW_ERR_INVALID;                                                                 \
    hipError_t e_ = (expr);                                                                          \
    if (e_ == hipErrorInvalidValue) return fail(c, PW_ERR_INVALID, "arguments rejected by the launcher"); \
    if (e_ == hipErrorNotSupported) return fail(c, PW_ERR_UNSUPPORTED, "not supported");            \
    if (e_ != hipSuccess) return fail(c, PW_ERR_DEVICE, "%s", hipGetErrorString(e_));               \
    return PW_OK;                                                                                    \
  } while (0)

static GemmArgs gemm_args_of(const pw_gemm_args* a) {
  GemmArgs g{};
  g.dtype = a->dtype; g.a_kmajor = a->a_kmajor; g.b_kmajor = a->b_kmajor;
  g.M = a->M; g.N = a->N; g.K = a->K; g.lda = a->lda; g.ldb = a->ldb; g.ldc = a->ldc;
  g.epilogue = a->epilogue; g.out_dtype = a->out_dtype; g.accumulate = a->accumulate;
  g.A = a->A; g.B = a->B; g.bias = a->bias; g.aux = a->aux; g.C = a->C; g.C2 = a->C2;
  g.b_colsum = a->b_colsum;
  if (a->adam) g.adam = AdamEpi{a->adam->w, a->adam->m, a->adam->v, a->adam->w_bf16, a->adam->lr, a->adam->beta1,
                                a->adam->beta2, a->adam->eps, a->adam->t, nullptr};
  if (a->xent) g.xent = XentEpi{a->xent->tokens, a->xent->T, a->xent->part, a->xent->zt, a->xent->lse, a->xent->inv_n};
  return g;
}
pw_status pw_op_gemm(pw_ctx* c, const pw_gemm_args* a) {
  if (!c || !a) return PW_ERR_INVALID;
  PW_OP(c, launch_gemm(c->exec, gemm_args_of(a)));
}
pw_status pw_op_gemm_pair(pw_ctx* c, const pw_gemm_args* a0, const pw_gemm_args* a1) {
  if (!c || !a0 || !a1) return PW_ERR_INVALID;
  PW_OP(c, launch_gemm_pair(c->exec, gemm_args_of(a0), gemm_args_of(a1)));
}
pw_status pw_op_gemm_group(pw_ctx* c, const pw_gemm_args* a, int n) {
  if (!c || !a || n < 1 || n > 3) return PW_ERR_INVALID;
  GemmArgs g[3];
  for (int i = 0; i < n; ++i) g[i] = gemm_args_of(&a[i]);
  PW_OP(c, launch_gemm_group(c->exec, g, n));
}
pw_status pw_op_embedding_fwd(pw_ctx* c, const int32_t* tokens, const float* wte, const float* wpe, float* x, int B, int T, int d, int V) {
  PW_OP(c, launch_embedding_fwd(c->exec, tokens, wte, wpe, x, B, T, d, V));
}
pw_status pw_op_embedding_bwd(pw_ctx* c, const int32_t* tokens, const float* dx, float* dwte, float* dwpe, int B, int T, int d, int V) {
  PW_OP(c, launch_embedding_bwd(c->exec, tokens, dx, dwte, dwpe, B, T, d, V));
}
pw_status pw_op_layernorm_fwd(pw_ctx* c, int dtype, const float* x, const float* g, const float* b, void* y, float* mean, float* rstd, int N, int d) {
  PW_OP(c, launch_layernorm_fwd(c->exec, dtype, x, g, b, y, mean, rstd, N, d));
}
pw_status pw_op_layernorm_bwd(pw_ctx* c, int dtype, const void* dy, const float* x, const float* g, const float* mean, const float* rstd,
                              const float* dres, float* dx, void* dx_lp, float* dg, float* db, float* dxsum, float* ws, int N, int d, int accumulate) {
  PW_OP(c, launch_layernorm_bwd(c->exec, dtype, dy, x, g, mean, rstd, dres, dx, dx_lp, dg, db, dxsum, ws, N, d, accumulate));
}
int64_t pw_layernorm_bwd_ws_floats(int N, int d) { return layernorm_bwd_ws_floats(N, d); }
pw_status pw_op_layernorm_bwd_noalloc(pw_ctx* c, int dtype, const void* dy, const float* x, const float* g, const float* mean,
                                      const float* rstd, const float* dres, float* dx, void* dx_lp, float* dg, float* db,
                                      float* dxsum, int N, int d, int accumulate) {
  if (!c) return PW_ERR_INVALID;
  if (N >= 0 && d > 0 && layernorm_bwd_ws_floats(N, d) > layernorm_bwd_static_max_ws_floats())
    return fail(c, PW_ERR_UNSUPPORTED, "N = %d rows of d = %d columns need %lld floats of block sums, the library's fixed array holds %lld",
                N, d, (long long)layernorm_bwd_ws_floats(N, d), (long long)layernorm_bwd_static_max_ws_floats());
  PW_OP(c, launch_layernorm_bwd_static(c->exec, c->device, dtype, dy, x, g, mean, rstd, dres, dx, dx_lp, dg, db, dxsum, N, d, accumulate));
}
pw_status pw_op_attention_fwd(pw_ctx* c, int dtype, const void* qkv, void* o, float* lse, int B, int T, int H, int hd) {
  PW_OP(c, launch_attention_fwd(c->exec, dtype, qkv, o, lse, B, T, H, hd));
}
pw_status pw_op_attention_bwd(pw_ctx* c, int dtype, const void* qkv, const void* o, const void* dout, const float* lse, float* delta,
                              void* dqkv, int B, int T, int H, int hd) {
  PW_OP(c, launch_attention_bwd(c->exec, dtype, qkv, o, dout, lse, delta, dqkv, B, T, H, hd));
}
static MhaArgs mha_args_of(const pw_mha_args* a) {
  return MhaArgs{a->dtype, a->q, a->k, a->v, a->ldq, a->ldkv, a->B, a->Tq, a->Tk, a->H, a->hd, a->causal};
}
pw_status pw_op_mha_fwd(pw_ctx* c, const pw_mha_args* a, void* o, void* o_lo, float* lse) {
  if (!a) return PW_ERR_INVALID;
  PW_OP(c, launch_mha_fwd(c->exec, mha_args_of(a), o, o_lo, lse));
}
pw_status pw_op_mha_bwd(pw_ctx* c, const pw_mha_args* a, const void* o, const void* o_lo, const void* dout, const float* lse,
                        float* delta, void* dq, int64_t lddq, void* dk, void* dv, int64_t lddkv) {
  if (!a) return PW_ERR_INVALID;
  PW_OP(c, launch_mha_bwd(c->exec, mha_args_of(a), o, o_lo, dout, lse, delta, dq, lddq, dk, dv, lddkv));
}
pw_status pw_op_softmax_xent(pw_ctx* c, int dtype, void* z, const int32_t* tokens, float* loss, float* row_loss, int B, int T, int V) {
  PW_OP(c, launch_softmax_xent(c->exec, dtype, z, tokens, loss, row_loss, B, T, V));
}
pw_status pw_op_xent_from_stats(pw_ctx* c, const float* part, const float* zt, float* lse, float* row_loss, float* loss, int N, int groups) {
  PW_OP(c, launch_xent_from_stats(c->exec, part, zt, lse, row_loss, loss, N, groups));
}
pw_status pw_op_colsum(pw_ctx* c, int dtype, const void* in, float* out, float* ws, int64_t rows, int64_t cols, int accumulate) {
  PW_OP(c, launch_colsum(c->exec, dtype, in, out, ws, rows, cols, accumulate));
}
int64_t pw_colsum_ws_floats(int64_t rows, int64_t cols) { return colsum_ws_floats(rows, cols); }
pw_status pw_op_sgd(pw_ctx* c, float* w, const float* g, int64_t n, float lr) { PW_OP(c, launch_sgd(c->exec, w, g, n, lr)); }
pw_status pw_op_adam(pw_ctx* c, float* w, float* m, float* v, const float* g, void* w_bf16, int64_t n, float lr, float beta1, float beta2,
                     float eps, int t) {
  PW_OP(c, launch_adam(c->exec, w, m, v, g, w_bf16, n, lr, beta1, beta2, eps, t, nullptr));
}

pw_status pw_profile_begin(pw_ctx* c) {
  if (!c) return PW_ERR_INVALID;
  gemm_profile_begin();
  return PW_OK;
}
pw_status pw_profile_pause(pw_ctx* c) {
  if (!c) return PW_ERR_INVALID;
  gemm_profile_pause();
  return PW_OK;
}
pw_status pw_profile_end(pw_ctx* c, int64_t* launches, double* total_ms, double* total_flops) {
  if (!c) return PW_ERR_INVALID;
  hipError_t e = gemm_profile_end(launches, total_ms, total_flops);
  if (e != hipSuccess) return fail(c, PW_ERR_DEVICE, "profile read: %s", hipGetErrorString(e));
  return PW_OK;
}

pw_status pw_profile_fused_update(pw_ctx* c, int64_t* launches, double* total_ms, double* total_flops) {
  if (!c) return PW_ERR_INVALID;
  gemm_profile_fused(launches, total_ms, total_flops);
  return PW_OK;
}

pw_status pw_profile_gemm_shapes(pw_ctx* c, pw_gemm_shape_row* rows, int32_t cap, int32_t* n_rows) {
  if (!c || !n_rows || cap < 0 || (cap > 0 && !rows)) return PW_ERR_INVALID;
  std::vector<GemmShapeRow> r((size_t)cap);
  const int n = gemm_profile_shapes(r.data(), cap);
  for (int i = 0; i < n && i < cap; ++i) {
    const GemmShapeKey& k = r[i].key;
    rows[i] = pw_gemm_shape_row{k.M, k.N, k.K, k.a_kmajor, k.b_kmajor, k.epilogue, k.members, r[i].launches, r[i].total_ms, r[i].total_flops};
  }
  *n_rows = n;
  return PW_OK;
}

}  // extern "C"
