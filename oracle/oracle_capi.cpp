// C entry points of the CPU oracle (test infrastructure only; see lm_oracle.hpp).
// Every array is a host pointer owned by the caller; functions return 0 on success.
#include "encdec_oracle.hpp"
#include "lm_oracle.hpp"

#include <chrono>
#include <cstdio>
#ifdef _OPENMP
#include <omp.h>
#endif

using namespace oracle;

extern "C" {

struct orc_lm_shape {
  int L, d, H, F, V, T, B, has_embed, has_head;
};
struct orc_opt {
  int kind;
  double lr, beta1, beta2, eps;
  int t;
};

static LMShape to_shape(const orc_lm_shape* c) {
  return LMShape{c->L, c->d, c->H, c->F, c->V, c->T, c->B, c->has_embed, c->has_head};
}

int orc_threads() {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

int orc_embedding_fwd(const int32_t* inp, const double* wte, const double* wpe, double* x, int B, int T, int d) {
  embedding_fwd<double>(inp, wte, wpe, x, B, T, d);
  return 0;
}
int orc_embedding_bwd(const int32_t* inp, const double* dx, double* dwte, double* dwpe, int B, int T, int d, int V) {
  embedding_bwd<double>(inp, dx, dwte, dwpe, B, T, d, V);
  return 0;
}
int orc_layernorm_fwd(const double* x, const double* g, const double* b, double* y, double* mean, double* rstd,
                      int N, int d) {
  layernorm_fwd<double>(x, g, b, y, mean, rstd, N, d);
  return 0;
}
int orc_layernorm_bwd(const double* dy, const double* x, const double* g, double* dx, double* dg, double* db,
                      int N, int d) {
  layernorm_bwd<double>(dy, x, g, dx, dg, db, N, d);
  return 0;
}
int orc_linear_fwd(const double* x, const double* W, const double* b, double* y, int N, int in, int out) {
  linear_fwd<double>(x, W, b, y, N, in, out);
  return 0;
}
int orc_linear_bwd(const double* x, const double* W, const double* dy, double* dx, double* dW, double* db,
                   int N, int in, int out) {
  linear_bwd<double>(x, W, dy, dx, dW, db, N, in, out);
  return 0;
}
int orc_gelu_fwd(const double* u, double* h, int64_t n) {
  for (int64_t i = 0; i < n; ++i) h[i] = gelu<double>(u[i]);
  return 0;
}
int orc_gelu_bwd(const double* u, const double* dh, double* du, int64_t n) {
  for (int64_t i = 0; i < n; ++i) du[i] = dh[i] * gelu_grad<double>(u[i]);
  return 0;
}
int orc_attention_fwd(const double* qkv, double* o, double* probs, int B, int T, int H, int hd) {
  attention_fwd<double>(qkv, o, probs, B, T, H, hd);
  return 0;
}
int orc_attention_bwd(const double* qkv, const double* dout, double* dqkv, int B, int T, int H, int hd) {
  attention_bwd<double>(qkv, dout, dqkv, B, T, H, hd);
  return 0;
}
int orc_softmax_xent(const double* z, const int32_t* tgt, int N, int V, double* loss, double* dz) {
  softmax_xent<double>(z, tgt, N, V, loss, dz);
  return 0;
}
int orc_sgd(double* w, const double* g, int64_t n, double lr) {
  sgd<double>(w, g, (size_t)n, lr);
  return 0;
}
int orc_adam(double* w, double* m, double* v, const double* g, int64_t n, double lr, double b1, double b2,
             double eps, int t) {
  adam<double>(w, m, v, g, (size_t)n, lr, b1, b2, eps, t);
  return 0;
}

int64_t orc_lm_param_count(const orc_lm_shape* c) { return (int64_t)param_table(to_shape(c)).size(); }
int64_t orc_lm_param_total(const orc_lm_shape* c) { return (int64_t)param_total(to_shape(c)); }
int orc_lm_param_info(const orc_lm_shape* c, int64_t idx, char* name, int name_cap, int64_t* offset, int64_t* numel) {
  const auto t = param_table(to_shape(c));
  if (idx < 0 || idx >= (int64_t)t.size()) return 1;
  std::snprintf(name, name_cap, "%s", t[idx].name.c_str());
  *offset = (int64_t)t[idx].offset;
  *numel = (int64_t)t[idx].numel;
  return 0;
}

int orc_lm_train_step(const orc_lm_shape* c, double* P, double* M, double* V, const int32_t* tokens,
                      const orc_opt* o, double* loss, double* G, double* logits, int do_bwd) {
  if (!c->has_embed || !c->has_head) return 1;
  OptConfig oc{o->kind, o->lr, o->beta1, o->beta2, o->eps, o->t};
  lm_train_step<double>(to_shape(c), P, M, V, tokens, oc, loss, G, logits, do_bwd);
  return 0;
}
int orc_lm_train_step_f32(const orc_lm_shape* c, float* P, float* M, float* V, const int32_t* tokens,
                          const orc_opt* o, float* loss, float* G, float* logits, int do_bwd) {
  if (!c->has_embed || !c->has_head) return 1;
  OptConfig oc{o->kind, o->lr, o->beta1, o->beta2, o->eps, o->t};
  lm_train_step<float>(to_shape(c), P, M, V, tokens, oc, loss, G, logits, do_bwd);
  return 0;
}
int orc_stage_fwd_bwd(const orc_lm_shape* c, const double* P, int n_mb, const double* X, const double* dY,
                      double* Y, double* dX, double* G) {
  if (c->has_embed || c->has_head) return 1;
  stage_fwd_bwd<double>(to_shape(c), P, n_mb, X, dY, Y, dX, G);
  return 0;
}

// ---- encoder-decoder workload (encdec_oracle.hpp) ------------------------------------------------

struct orc_encdec_shape {
  int Le, Ld, d, H, F, V, Ts, Tt, B;
};
static EncDecShape to_ed_shape(const orc_encdec_shape* c) {
  return EncDecShape{c->Le, c->Ld, c->d, c->H, c->F, c->V, c->Ts, c->Tt, c->B};
}

int orc_mha_fwd(const double* q, int64_t ldq, const double* k, const double* v, int64_t ldkv, double* o, int B, int Tq,
                int Tk, int H, int hd, int causal) {
  if (causal && Tq != Tk) return 1;
  mha_fwd<double>(q, (size_t)ldq, k, v, (size_t)ldkv, o, B, Tq, Tk, H, hd, causal);
  return 0;
}
int orc_mha_bwd(const double* q, int64_t ldq, const double* k, const double* v, int64_t ldkv, const double* dout,
                double* dq, int64_t lddq, double* dk, double* dv, int64_t lddkv, int B, int Tq, int Tk, int H, int hd,
                int causal) {
  if (causal && Tq != Tk) return 1;
  mha_bwd<double>(q, (size_t)ldq, k, v, (size_t)ldkv, dout, dq, (size_t)lddq, dk, dv, (size_t)lddkv, B, Tq, Tk, H, hd, causal);
  return 0;
}

int64_t orc_encdec_param_count(const orc_encdec_shape* c) { return (int64_t)encdec_param_table(to_ed_shape(c)).size(); }
int64_t orc_encdec_param_total(const orc_encdec_shape* c) { return (int64_t)encdec_param_total(to_ed_shape(c)); }
int orc_encdec_param_info(const orc_encdec_shape* c, int64_t idx, char* name, int name_cap, int64_t* offset, int64_t* numel) {
  const auto t = encdec_param_table(to_ed_shape(c));
  if (idx < 0 || idx >= (int64_t)t.size()) return 1;
  std::snprintf(name, name_cap, "%s", t[idx].name.c_str());
  *offset = (int64_t)t[idx].offset;
  *numel = (int64_t)t[idx].numel;
  return 0;
}
int orc_encdec_train_step(const orc_encdec_shape* c, double* P, double* M, double* V, const int32_t* src,
                          const int32_t* tgt, const orc_opt* o, double* loss, double* G, double* logits, int do_bwd) {
  if (c->Le < 1 || c->Ld < 1 || c->d % c->H) return 1;
  OptConfig oc{o->kind, o->lr, o->beta1, o->beta2, o->eps, o->t};
  encdec_train_step<double>(to_ed_shape(c), P, M, V, src, tgt, oc, loss, G, logits, do_bwd);
  return 0;
}

int orc_chain_add_f32(const float* x, float* y, int n, int L, float cst) {
  chain_add_f32(x, y, n, L, cst);
  return 0;
}
int orc_scalar_fn_f32(int kind, const float* x, float* y, int n, float cst) {
  if (kind < 0 || kind > 2) return 1;
  scalar_fn_f32(kind, x, y, n, cst);
  return 0;
}

}  // extern "C"
