// Shared pieces of the train-step models: state arenas and the GEMM layouts of a linear layer.
#include "model_common.hpp"

namespace pw {

hipError_t model_state_alloc(ModelBase* m, const OptimizerConfig& o, std::string* err) {
  const int optimizer = o.kind;
  auto fail = [&](hipError_t e, const char* what) {
    if (err) *err = std::string(what) + ": " + hipGetErrorString(e);
    model_state_free(m);
    return e;
  };
  hipError_t e;
  const size_t bytes = (size_t)m->total * 4;
  if ((e = hipMalloc(&m->w, bytes)) != hipSuccess) return fail(e, "alloc params");
  if ((e = hipMalloc(&m->g, bytes)) != hipSuccess) return fail(e, "alloc grads");
  if (optimizer == 2) {
    if ((e = hipMalloc(&m->m, bytes)) != hipSuccess) return fail(e, "alloc adam m");
    if ((e = hipMalloc(&m->v, bytes)) != hipSuccess) return fail(e, "alloc adam v");
  }
  if (m->bf16 && (e = hipMalloc(&m->wlp, (size_t)m->total * 2)) != hipSuccess) return fail(e, "alloc bf16 weights");
  if ((e = hipMalloc(&m->step_dev, 256)) != hipSuccess) return fail(e, "alloc step counter");
  // zero everything that is read before it is written
  if ((e = launch_fill_f32(m->stream, m->w, m->total, 0.f)) != hipSuccess) return fail(e, "zero params");
  if ((e = launch_fill_f32(m->stream, m->g, m->total, 0.f)) != hipSuccess) return fail(e, "zero grads");
  if (m->m && (e = launch_fill_f32(m->stream, m->m, m->total, 0.f)) != hipSuccess) return fail(e, "zero m");
  if (m->v && (e = launch_fill_f32(m->stream, m->v, m->total, 0.f)) != hipSuccess) return fail(e, "zero v");
  if (m->wlp && (e = launch_f32_to_bf16(m->stream, m->w, m->wlp, m->total)) != hipSuccess) return fail(e, "zero bf16 weights");
  if ((e = launch_adam_step(m->stream, m->step_dev, 1, o.beta1, o.beta2)) != hipSuccess) return fail(e, "init step");
  if ((e = hipStreamSynchronize(m->stream)) != hipSuccess) return fail(e, "sync");
  return hipSuccess;
}

void model_state_free(ModelBase* m) {
  (void)hipFree(m->w); (void)hipFree(m->g); (void)hipFree(m->m); (void)hipFree(m->v);
  (void)hipFree(m->wlp); (void)hipFree(m->step_dev);
  m->w = m->g = m->m = m->v = nullptr;
  m->wlp = nullptr;
  m->step_dev = nullptr;
}

hipError_t model_state_refresh_lowp(ModelBase* m, int64_t offset, int64_t numel) {
  if (!m->wlp) return hipSuccess;
  return launch_f32_to_bf16(m->stream, m->w + offset, (uint16_t*)m->wlp + offset, numel);
}

hipError_t model_state_apply_optimizer(ModelBase* m, const OptimizerConfig& o) {
  if (o.kind == 1) {
    PW_TRY(launch_sgd(m->stream, m->w, m->g, m->total, o.lr), "sgd");
    if (m->wlp) PW_TRY(launch_f32_to_bf16(m->stream, m->w, m->wlp, m->total), "refresh bf16 weights");
  } else {
    const int64_t n = m->fused_from >= 0 ? m->fused_from : m->total;   // the rest was updated by its weight-gradient GEMMs
    PW_TRY(launch_adam(m->stream, m->w, m->m, m->v, m->g, m->wlp, n, o.lr, o.beta1, o.beta2, o.eps, 0, m->step_dev), "adam");
    PW_TRY(launch_adam_step(m->stream, m->step_dev, 0, o.beta1, o.beta2), "step counter");
  }
  return hipSuccess;
}

static const void* weight_operand(const ModelBase* m, int64_t wi) {
  return m->bf16 ? (const void*)((const uint16_t*)m->wlp + m->P(wi).offset) : (const void*)(m->w + m->P(wi).offset);
}

hipError_t gemm_fwd(ModelBase* m, const void* x, int64_t wi, const float* bias, int64_t N, int64_t in, int64_t out,
                    int epi, int out_dtype, const void* aux, void* C, void* C2) {
  GemmArgs a{};
  a.dtype = m->act_dtype();
  a.a_kmajor = 0;                      // x [N, in]
  a.b_kmajor = 1;                      // W [in, out]: stored [k][n]
  a.M = N; a.N = out; a.K = in; a.lda = in; a.ldb = out; a.ldc = out;
  a.epilogue = epi; a.out_dtype = out_dtype; a.accumulate = 0;
  a.A = x;
  a.B = weight_operand(m, wi);
  a.bias = bias; a.aux = aux; a.C = C; a.C2 = C2;
  return launch_gemm(m->stream, a);
}

hipError_t gemm_dgrad(ModelBase* m, const void* dy, int64_t wi, int64_t N, int64_t in, int64_t out, int epi,
                      const void* aux, void* C, int out_dtype, int accumulate) {
  GemmArgs a{};
  a.dtype = m->act_dtype();
  a.a_kmajor = 0;                      // dy [N, out]
  a.b_kmajor = 0;                      // W [in, out]: stored [n = in][k = out]
  a.M = N; a.N = in; a.K = out; a.lda = out; a.ldb = out; a.ldc = in;
  a.epilogue = epi; a.out_dtype = out_dtype; a.accumulate = accumulate;
  a.A = dy;
  a.B = weight_operand(m, wi);
  a.aux = aux; a.C = C;
  return launch_gemm(m->stream, a);
}

GemmArgs wgrad_args(ModelBase* m, const void* x, const void* dy, int64_t wi, int64_t N, int64_t in, int64_t out,
                    int accumulate) {
  GemmArgs a{};
  a.dtype = m->act_dtype();
  a.a_kmajor = 1;                      // x [N, in]: stored [k = N][m = in]
  a.b_kmajor = 1;                      // dy [N, out]: stored [k = N][n = out]
  a.M = in; a.N = out; a.K = N; a.lda = in; a.ldb = out; a.ldc = out;
  a.epilogue = kEpiStore; a.out_dtype = kF32; a.accumulate = accumulate;
  a.A = x; a.B = dy; a.C = m->g + m->P(wi).offset;
  return a;
}

GemmArgs wgrad_adam_args(ModelBase* m, const OptimizerConfig& o, const void* x, const void* dy, int64_t wi, int64_t N,
                         int64_t in, int64_t out) {
  GemmArgs a = wgrad_args(m, x, dy, wi, N, in, out, 0);
  const int64_t off = m->P(wi).offset;
  a.epilogue = kEpiAdam;
  a.C = nullptr;
  a.adam = AdamEpi{m->w + off, m->m + off, m->v + off, m->wlp ? (void*)((uint16_t*)m->wlp + off) : nullptr,
                   o.lr, o.beta1, o.beta2, o.eps, 0, m->adam_c()};
  return a;
}

hipError_t gemm_wgrad_bias(ModelBase* m, const void* x, const void* dy, int64_t wi, int64_t bi, int64_t N, int64_t in,
                           int64_t out, int accumulate, float* ws, const OptimizerConfig* fused) {
  GemmArgs wa = fused ? wgrad_adam_args(m, *fused, x, dy, wi, N, in, out) : wgrad_args(m, x, dy, wi, N, in, out, accumulate);
  wa.b_colsum = m->gp(bi);
  if (gemm_colsum_fusable(wa, false)) return launch_gemm(m->stream, wa);
  wa.b_colsum = nullptr;
  hipError_t e = launch_gemm(m->stream, wa);
  if (e != hipSuccess) return e;
  return launch_colsum(m->stream, m->act_dtype(), dy, m->gp(bi), ws, N, out, accumulate);
}

hipError_t gemm_wgrad_group(ModelBase* m, const WgradJob* jobs, int n, float* ws) {
  if (n < 1 || n > 3) return hipErrorInvalidValue;
  GemmArgs a[3];
  for (int i = 0; i < n; ++i) a[i] = jobs[i].args;
  const bool shared = gemm_group_shares_launch(a, n);
  bool fused[3] = {false, false, false};
  for (int i = 0; i < n; ++i) {
    if (jobs[i].bias < 0) continue;
    a[i].b_colsum = m->gp(jobs[i].bias);
    fused[i] = gemm_colsum_fusable(a[i], shared);
    if (!fused[i]) a[i].b_colsum = nullptr;
  }
  hipError_t e = launch_gemm_group(m->stream, a, n);
  for (int i = 0; i < n && e == hipSuccess; ++i)
    if (jobs[i].bias >= 0 && !fused[i])   // dy of a weight gradient is its B operand: [K = N rows][N = out columns]
      e = launch_colsum(m->stream, m->act_dtype(), a[i].B, m->gp(jobs[i].bias), ws, a[i].K, a[i].N, a[i].accumulate);
  return e;
}

}  // namespace pw
