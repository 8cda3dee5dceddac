// Host-side launchers of the gfx950 kernels.  Every launcher validates what its kernel assumes
// about shapes and alignment BEFORE launching, enqueues on `s`, and returns a hipError_t
// (hipErrorInvalidValue for a rejected argument).  Nothing here allocates or synchronises.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pw {

enum DType { kF32 = 0, kBF16 = 1, kI32 = 2 };
enum Epilogue {
  kEpiStore = 0, kEpiBias = 1, kEpiBiasResidual = 2, kEpiBiasGelu = 3, kEpiGeluBwd = 4,
  kEpiAdam = 5,        // the product is the gradient of a weight: the Adam update of that weight runs in the epilogue
  kEpiXentStats = 6,   // the product is a tile of logits: only softmax statistics leave the kernel
  kEpiXentGrad = 7     // the product is a tile of logits: what is stored is (softmax - onehot) / N in bf16
};

// kEpiAdam: w, m, v (fp32) and w_bf16 (optional) are laid out like the product [M, N] with leading dimension
// ldc; the gradient itself is stored to C only if C is non-null.  Bias corrections 1 / (1 - beta^t): read from
// c_dev[0..1] (device) when non-null - a captured graph then stays valid across steps - else computed from t.
struct AdamEpi {
  float *w, *m, *v;
  void* w_bf16;
  float lr, b1, b2, eps;
  int t;
  const float* c_dev;
};
// kEpiXentStats / kEpiXentGrad: rows of the product are token positions (row r = b*T + t, target
// tokens[b*(T+1) + t + 1]), columns the vocabulary.  Stats: part[r][N/64] receives (max, sum exp(z - max)) of each
// 64-column group, zt[r] the target's logit; C is not written.  Grad: lse[r] is the row's log-sum-exp;
// C (bf16) receives (exp(z - lse) - [column == target]) * inv_n.
struct XentEpi {
  const int32_t* tokens;
  int T;
  float* part;
  float* zt;
  const float* lse;
  float inv_n;
};

struct GemmArgs {
  int dtype;
  int a_kmajor, b_kmajor;
  int64_t M, N, K, lda, ldb, ldc;
  int epilogue, out_dtype, accumulate;
  const void* A;
  const void* B;
  const float* bias;
  const void* aux;
  void* C;
  void* C2;
  float* b_colsum;   // optional: column sums of op(B) over k (= or +=, following `accumulate`); see gemm_colsum_fusable
  AdamEpi adam;      // kEpiAdam
  XentEpi xent;      // kEpiXentStats, kEpiXentGrad
};

// elementwise.hip
// done / token (optional): the launch writes token to *done (pinned host memory) when its output is complete; only
// launches of one block can (scalar_fn_one_block).
hipError_t launch_scalar_fn(hipStream_t s, int kind, const float* x, float* y, int64_t n, float c, float busy_us, int reps,
                            uint32_t* done = nullptr, uint32_t token = 0);
bool scalar_fn_one_block(int64_t n);
hipError_t launch_add2(hipStream_t s, const float* a, const float* b, float* y, int64_t n);
hipError_t launch_fill_f32(hipStream_t s, float* p, int64_t n, float v);
hipError_t launch_f32_to_bf16(hipStream_t s, const float* src, void* dst, int64_t n);
hipError_t launch_bf16_to_f32(hipStream_t s, const void* src, float* dst, int64_t n);
hipError_t launch_copy_bytes(hipStream_t s, const void* src, void* dst, int64_t bytes);
// Spins (bounded by timeout_ticks of the 100 MHz wall clock) until *flag != 0.  *flag == 1 means
// "resolved"; any other value, or a timeout, writes 1 to *poison.  Both words live in pinned host memory.
hipError_t launch_gate(hipStream_t s, const uint32_t* flag, uint32_t* poison, uint64_t timeout_ticks);
hipError_t launch_sgd(hipStream_t s, float* w, const float* g, int64_t n, float lr);
hipError_t launch_adam(hipStream_t s, float* w, float* m, float* v, const float* g, void* w_bf16, int64_t n,
                       float lr, float b1, float b2, float eps, int t, const int* t_dev);
hipError_t launch_increment(hipStream_t s, int* counter);
// Adam's step state on the device (at least 32 bytes): state[0] (int) the step number t, state[4], state[5] (float,
// 16-byte aligned) the bias corrections 1 / (1 - beta1^t), 1 / (1 - beta2^t).  set_to > 0: t = set_to; set_to = 0: t += 1.
hipError_t launch_adam_step(hipStream_t s, int* state, int set_to, float b1, float b2);
// Mean cross-entropy from the statistics a kEpiXentStats GEMM left: lse[r] = log sum exp over the row's `groups`
// 64-column groups, row_loss[r] = lse[r] - zt[r], loss = mean.
hipError_t launch_xent_from_stats(hipStream_t s, const float* part, const float* zt, float* lse, float* row_loss,
                                  float* loss, int N, int groups);
// Whether launch_gemm can run this problem with epilogue kEpiAdam (alone, or as a member of a shared launch) /
// with kEpiXentStats and kEpiXentGrad.
bool gemm_adam_fusable(const GemmArgs& a, bool grouped);
bool gemm_xent_fusable(const GemmArgs& a);

// norm.hip
hipError_t launch_layernorm_fwd(hipStream_t s, int dtype, const float* x, const float* g, const float* b, void* y,
                                float* mean, float* rstd, int N, int d);
int64_t layernorm_bwd_ws_floats(int N, int d);
// The same with the workspace in a fixed device array of the library (no allocation anywhere on the path):
// _init looks the array's address up for `device`, which must be current; the launcher needs that to have happened
// (hipErrorNotInitialized) and takes problems whose workspace fits the array (hipErrorNotSupported otherwise).
hipError_t layernorm_bwd_static_init(int device);
int64_t layernorm_bwd_static_max_ws_floats();
hipError_t launch_layernorm_bwd_static(hipStream_t s, int device, int dtype, const void* dy, const float* x, const float* g,
                                       const float* mean, const float* rstd, const float* dres, float* dx, void* dx_lp,
                                       float* dg, float* db, float* dsum, int N, int d, int accumulate);
hipError_t launch_layernorm_bwd(hipStream_t s, int dtype, const void* dy, const float* x, const float* g,
                                const float* mean, const float* rstd, const float* dres, float* dx, void* dx_lp,
                                float* dg, float* db, float* dsum, float* ws, int N, int d, int accumulate);
int64_t colsum_ws_floats(int64_t rows, int64_t cols);
hipError_t launch_colsum(hipStream_t s, int dtype, const void* in, float* out, float* ws, int64_t rows, int64_t cols,
                         int accumulate);

// embed_xent.hip
// tokens: rows tok_stride ids apart, the first T of each row are looked up; tok_stride = 0 means T + 1 (the
// [B, T+1] arrays that carry inputs and next-token targets together).
hipError_t launch_embedding_fwd(hipStream_t s, const int32_t* tokens, const float* wte, const float* wpe, float* x,
                                int B, int T, int d, int V, int tok_stride = 0);
hipError_t launch_embedding_bwd(hipStream_t s, const int32_t* tokens, const float* dx, float* dwte, float* dwpe,
                                int B, int T, int d, int V, int tok_stride = 0);
hipError_t launch_softmax_xent(hipStream_t s, int dtype, void* z, const int32_t* tokens, float* loss, float* row_loss,
                               int B, int T, int V);

// attention.hip
// Multi-head attention of Tq queries over Tk keys per (batch, head), scale 1/sqrt(hd).  q, k, v point at element
// (batch 0, row 0, feature 0) of arrays in `dtype`; rows are ldq (q) and ldkv (k and v) elements apart, batch b
// starts at row b*Tq (q) or b*Tk (k, v), head h owns features h*hd .. of a row.  causal: query i sees keys j <= i
// (needs Tq == Tk).  Packed self-attention is q = qkv, k = qkv + d, v = qkv + 2d, ldq = ldkv = 3d.
struct MhaArgs {
  int dtype;
  const void *q, *k, *v;
  int64_t ldq, ldkv;
  int B, Tq, Tk, H, hd;
  int causal;
};
// o: dense [B*Tq, H*hd] in `dtype`; lse: [B, H, Tq] row log-sum-exp (kept for the backward pass).
// o_lo (optional, same shape and type as o): receives what the rounding of O to `dtype` left over; handed to
// launch_mha_bwd it makes the backward pass's delta = rowsum(dO * O) as exact as fp32 allows.  Without it the
// bf16 rounding of O becomes a common offset on every dS of a row, which keys that share a large common
// component turn into an error of several per cent in dq and dk.
hipError_t launch_mha_fwd(hipStream_t s, const MhaArgs& a, void* o, void* o_lo, float* lse);
// dq rows lddq elements apart, dk and dv rows lddkv; delta: [B, H, Tq] scratch.  Every feature of every row of
// dq, dk, dv is overwritten.
hipError_t launch_mha_bwd(hipStream_t s, const MhaArgs& a, const void* o, const void* o_lo, const void* dout,
                          const float* lse, float* delta, void* dq, int64_t lddq, void* dk, void* dv, int64_t lddkv);
// Causal self-attention over packed qkv [B*T, 3d] (the two calls above with the packed layout).
hipError_t launch_attention_fwd(hipStream_t s, int dtype, const void* qkv, void* o, float* lse, int B, int T, int H,
                                int hd);
hipError_t launch_attention_bwd(hipStream_t s, int dtype, const void* qkv, const void* o, const void* dout,
                                const float* lse, float* delta, void* dqkv, int B, int T, int H, int hd);

// One-time set-up of the head_dim-128 attention kernels' dynamic-LDS limits; call once before any capture.
hipError_t attention_dma_init();

// gemm.hip
hipError_t launch_gemm(hipStream_t s, const GemmArgs& a);
// Whether launch_gemm / launch_gemm_pair can deliver a.b_colsum for this problem (k-major bf16 operands on full
// 256 x 256 tiles: the weight-gradient GEMMs); callers fall back to launch_colsum otherwise.
bool gemm_colsum_fusable(const GemmArgs& a, bool paired);
bool gemm_pair_shares_launch(const GemmArgs& a0, const GemmArgs& a1);
bool gemm_group_shares_launch(const GemmArgs* a, int n);
// Two (or up to three) independent GEMMs; one launch is shared between them when that fills the chip better
// (same results either way).  Their outputs must not overlap each other or any operand.
hipError_t launch_gemm_pair(hipStream_t s, const GemmArgs& a0, const GemmArgs& a1);
hipError_t launch_gemm_group(hipStream_t s, const GemmArgs* a, int n);
// Timing of MFMA GEMM launches with HIP events on the launch stream (measurement aid).
void gemm_profile_begin();
void gemm_profile_pause();   // stop bracketing launches; what was recorded so far stays for gemm_profile_end
hipError_t gemm_profile_end(int64_t* launches, double* total_ms, double* total_flops);
// Launches that carried the Adam epilogue are kept out of those figures (they do the optimizer's memory traffic as
// well); this returns theirs, as of the last gemm_profile_end.
void gemm_profile_fused(int64_t* launches, double* total_ms, double* total_flops);
// The same launches (all of them) by shape, as of the last gemm_profile_end, largest total time first.  A launch
// shared by several GEMMs counts under its largest member's shape with members > 1 and the FLOPs of all of them.
struct GemmShapeKey { int64_t M, N, K; int a_kmajor, b_kmajor, epilogue, members; };
struct GemmShapeRow { GemmShapeKey key; int64_t launches; double total_ms, total_flops; };
int gemm_profile_shapes(GemmShapeRow* rows, int cap);   // returns how many rows there are
// One-time per-process set-up of kernel attributes (large dynamic LDS); call once before any capture.
hipError_t gemm_init();

}  // namespace pw
