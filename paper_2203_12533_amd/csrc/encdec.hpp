// Encoder-decoder Transformer train step (the text-to-text family of the paper's Table 1) as a static list of
// kernel launches over a static buffer plan: the body of the PW_FN_ENCDEC_TRAIN_STEP compiled function.
#pragma once
#include "../../include/pw.h"
#include "model_common.hpp"

namespace pw {

struct EncDec : ModelBase {
  pw_encdec_config cfg;

  // activations kept for the backward pass, one set per residual sub-block
  struct SelfActs { float *x_in, *lse, *mean, *rstd; void *a, *qkv, *o, *o_lo; };
  struct CrossActs { float *x_in, *lse, *mean, *rstd; void *a, *q, *kv, *o, *o_lo; };
  struct FfnActs { float *x_in, *mean, *rstd; void *mm, *u, *h; };
  struct EncLayer { SelfActs sa; FfnActs ff; };
  struct DecLayer { SelfActs sa; CrossActs ca; FfnActs ff; };
  unsigned char* act = nullptr;
  size_t act_bytes = 0;
  std::vector<EncLayer> enc;
  std::vector<DecLayer> dec;
  float *enc_x_out = nullptr, *enc_meanf = nullptr, *enc_rstdf = nullptr;
  void* mem = nullptr;         // encoder output after its final LayerNorm, [B*Ts, d]
  float *dec_x_out = nullptr, *meanf = nullptr, *rstdf = nullptr, *row_loss = nullptr;
  void *y = nullptr, *logits = nullptr;
  // backward scratch, sized for the longer of the two sides
  float *dx_a = nullptr, *dx_b = nullptr, *delta = nullptr, *ws = nullptr, *dmem = nullptr;
  void *dx_lp = nullptr, *dx_lp2 = nullptr, *d_big = nullptr, *d_qkv = nullptr, *d_small = nullptr, *d_q = nullptr;

  int Ns() const { return cfg.batch * cfg.src_len; }
  int Nt() const { return cfg.batch * cfg.tgt_len; }
  int hd() const { return cfg.d_model / cfg.n_head; }
};

bool encdec_config_ok(const pw_encdec_config& cfg, std::string* why);
hipError_t encdec_create(const pw_encdec_config& cfg, hipStream_t stream, EncDec** out, std::string* err);
void encdec_destroy(EncDec* m);
// src [B, Ts], tgt [B, Tt+1] token ids on the device; loss: one fp32 on the device.
hipError_t encdec_train_step(EncDec* m, const int32_t* src, const int32_t* tgt, float* loss);
double encdec_step_flops(const pw_encdec_config& cfg);

}  // namespace pw
