// Decoder-only LM train step as a static list of kernel launches over a static buffer plan
// (the body of the PW_FN_LM_TRAIN_STEP / PW_FN_STAGE_* compiled functions).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "../../include/pw.h"
#include "model_common.hpp"

namespace pw {

struct Model : ModelBase {
  pw_lm_config cfg;

  // activations: one allocation, carved by plan()
  unsigned char* act = nullptr;
  size_t act_bytes = 0;
  struct LayerActs {
    float *x_in, *x_mid, *lse, *mean1, *rstd1, *mean2, *rstd2;
    void *a, *qkv, *o, *mm, *u, *h;
    // deferred weight gradients only: the four gradients that are the second operands of this layer's weight
    // gradients (w.r.t. the layer output, the FFN pre-activation, the attention sub-block output, qkv)
    void *g_y2 = nullptr, *g_u = nullptr, *g_yo = nullptr, *g_qkv = nullptr;
  };
  struct Slot {
    std::vector<LayerActs> layer;
    float* x_out;
  };
  std::vector<Slot> slots;    // one per micro-batch
  // A pipeline stage in bf16 with several micro-batches holds its weight gradients back: the backward pass of a
  // micro-batch leaves the operands of its four weight-gradient GEMMs per layer in per-micro-batch storage, which
  // is laid out micro-batch after micro-batch, and one GEMM per weight over ALL pending micro-batches (contraction
  // length n_microbatch x tokens) follows when the gradients are needed.  With HBM to spare this replaces
  // n_microbatch read-modify-write passes over every gradient tensor by one, and 32 k-tiles per output tile by
  // 32 x n_microbatch.  pending[mb]: the backward pass of micro-batch mb has run and its contribution is not in g yet.
  bool defer_wgrad = false;
  std::vector<char> pending;
  bool wgrads_zero = false;   // nothing has gone into the weight (and fused bias) gradients since they were zeroed:
                              // the next GEMMs over pending micro-batches may overwrite instead of accumulate
  // head
  void* y = nullptr;
  void* logits = nullptr;
  float *meanf = nullptr, *rstdf = nullptr, *row_loss = nullptr;
  // head fused with the loss (cfg.fused_head_loss on a shape the ring kernel takes): softmax statistics per
  // 64-column group, the targets' logits, the rows' log-sum-exp
  bool fused_head = false;
  float *xe_part = nullptr, *xe_zt = nullptr, *xe_lse = nullptr;
  // backward scratch
  float *dx_a = nullptr, *dx_b = nullptr, *delta = nullptr, *ws = nullptr;
  void *dx_lp = nullptr, *d_big = nullptr, *d_qkv = nullptr, *d_small = nullptr;
  void* dx_lp3 = nullptr;   // second home of the copy at a layer's input / output (the two alternate from layer to layer)
  void* dx_lp2 = nullptr;   // bf16 copy of the residual gradient at a layer's mid-point (dx_lp: at its input / output)

  int N() const { return cfg.batch * cfg.seq; }
  int hd() const { return cfg.d_model / cfg.n_head; }
};

// Each returns a hipError_t; on failure `model->error` says which launch was rejected.
hipError_t model_create(const pw_lm_config& cfg, hipStream_t stream, Model** out, std::string* err);
void model_destroy(Model* m);
hipError_t model_refresh_lowp(Model* m, int64_t offset, int64_t numel);
hipError_t model_train_step(Model* m, const int32_t* tokens_dev, float* loss_dev);
hipError_t model_stage_fwd(Model* m, int mb, const float* x_dev, float* y_dev);
hipError_t model_stage_bwd(Model* m, int mb, const float* dy_dev, float* dx_dev);
hipError_t model_zero_grads(Model* m);
// What the host must do for a stage function that is about to run as part of a HIP graph, captured now or replayed
// from the cache (a replay repeats the launches, not the host-side bookkeeping of held-back weight gradients):
// contributions still held back are enqueued first - the graph's forward pass overwrites their operands, its
// backward pass adds to the gradients at once - and a backward pass marks the gradients as written.
hipError_t model_before_graph(Model* m, bool backward);
hipError_t model_apply_optimizer(Model* m);
double model_step_flops(const pw_lm_config& cfg);
bool model_config_ok(const pw_lm_config& cfg, std::string* why);

}  // namespace pw
