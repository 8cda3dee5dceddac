// What the train-step models (lm.hip, encdec.hip) share: the flat parameter / gradient / optimiser-state arenas
// with their offset table, the carving of one activation allocation, and the three GEMM layouts of a linear
// layer (forward, input gradient, weight gradient).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "kernels.hpp"

namespace pw {

struct ParamInfo {
  std::string name;
  int64_t offset, numel;
};

struct OptimizerConfig {
  int kind;   // 1 SGD, 2 Adam
  float lr, beta1, beta2, eps;
};

struct ModelBase {
  hipStream_t stream = nullptr;
  std::string error;
  int bf16 = 0;               // 1: bf16 GEMM/attention operands, fp32 accumulation and master weights

  // parameters and optimiser state: flat fp32 arenas with one shared offset table
  std::vector<ParamInfo> params;
  int64_t total = 0;
  float* w = nullptr;
  float* g = nullptr;
  float* m = nullptr;
  float* v = nullptr;
  void* wlp = nullptr;        // bf16 compute copy of w (bf16 mode only)
  int* step_dev = nullptr;    // Adam step state on the device (launch_adam_step), so that captured graphs stay valid
  // Parameters at offsets >= fused_from (-1: none) are updated inside the epilogue of their weight-gradient GEMM:
  // their gradients are never stored, and the optimizer launch covers [0, fused_from) only.
  int64_t fused_from = -1;
  const float* adam_c() const { return reinterpret_cast<const float*>(step_dev) + 4; }   // the two bias corrections
  // Set by a model that holds back gradient work (see lm.hpp): enqueues it.  Whoever is about to read or
  // overwrite `g` from outside the model calls it first.
  hipError_t (*flush_pending)(ModelBase*) = nullptr;

  int act_dtype() const { return bf16 ? kBF16 : kF32; }
  const ParamInfo& P(size_t idx) const { return params[idx]; }
  float* wp(size_t idx) const { return w + params[idx].offset; }
  float* gp(size_t idx) const { return g + params[idx].offset; }
};

constexpr int64_t kParamAlign = 64;   // elements; keeps every tensor 256-byte aligned in fp32 and 128 in bf16

// Appends to the offset table.
struct ParamTableBuilder {
  std::vector<ParamInfo>& t;
  int64_t off = 0;
  std::vector<char> late;   // per parameter: updated inside its weight-gradient GEMM
  void add(const std::string& n, int64_t numel, bool updated_in_gemm = false) {
    t.push_back({n, off, numel});
    late.push_back(updated_in_gemm ? 1 : 0);
    off += (numel + kParamAlign - 1) / kParamAlign * kParamAlign;
  }
  // Offsets again, in two runs: everything the optimizer launch updates first, then the weights updated by their
  // GEMMs, so that the launch covers one contiguous range [0, fused_from) (-1: no such weights).  Index order, which
  // is what the API shows, is unchanged.
  void finish(int64_t& total, int64_t& fused_from) {
    total = off;
    fused_from = -1;
    int64_t o = 0;
    for (int pass = 0; pass < 2; ++pass)
      for (size_t i = 0; i < t.size(); ++i) {
        if (late[i] != pass) continue;
        if (pass == 1 && fused_from < 0) fused_from = o;
        t[i].offset = o;
        o += (t[i].numel + kParamAlign - 1) / kParamAlign * kParamAlign;
      }
  }
};

// Hands out 256-byte aligned pieces of one allocation; with base == nullptr it only measures.
struct Carver {
  size_t off = 0;
  unsigned char* base = nullptr;
  template <class T> T* take(size_t bytes) {
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += (bytes + 255) / 256 * 256;
    return p;
  }
};

#define PW_TRY(expr, what)                                                        \
  do {                                                                            \
    hipError_t e_ = (expr);                                                       \
    if (e_ != hipSuccess) {                                                       \
      m->error = std::string(what) + ": " + hipGetErrorString(e_);                \
      return e_;                                                                  \
    }                                                                             \
  } while (0)

// Allocates and zeroes w, g, (m, v), (wlp) and the step counter for m->total elements; on failure frees what
// it allocated and says what failed in *err.
hipError_t model_state_alloc(ModelBase* m, const OptimizerConfig& o, std::string* err);
void model_state_free(ModelBase* m);
hipError_t model_state_refresh_lowp(ModelBase* m, int64_t offset, int64_t numel);
hipError_t model_state_apply_optimizer(ModelBase* m, const OptimizerConfig& o);

// GEMMs of a linear layer y = x W + b with W [in, out] row-major (parameter index wi).
// y[N, out] = x[N, in] . W with a fused epilogue.
hipError_t gemm_fwd(ModelBase* m, const void* x, int64_t wi, const float* bias, int64_t N, int64_t in, int64_t out,
                    int epi, int out_dtype, const void* aux, void* C, void* C2);
// dx[N, in] (=|+=) dy[N, out] . W^T; out_dtype kF32 is needed for accumulate = 1.
hipError_t gemm_dgrad(ModelBase* m, const void* dy, int64_t wi, int64_t N, int64_t in, int64_t out, int epi,
                      const void* aux, void* C, int out_dtype, int accumulate);
// dW[in, out] (=|+=) x^T[in, N] . dy[N, out], into the gradient arena.
GemmArgs wgrad_args(ModelBase* m, const void* x, const void* dy, int64_t wi, int64_t N, int64_t in, int64_t out,
                    int accumulate);
// The same GEMM with the Adam update of parameter wi in its epilogue (gradient not stored).
GemmArgs wgrad_adam_args(ModelBase* m, const OptimizerConfig& o, const void* x, const void* dy, int64_t wi, int64_t N,
                         int64_t in, int64_t out);
// Weight gradient plus the bias gradient db (= column sums of dy): fused into the GEMM where that is free,
// a separate column-sum launch otherwise.  ws: workspace of colsum_ws_floats(N, out) floats.
// fused (optional): the weight (not the bias) is updated by Adam in the GEMM's epilogue instead of its gradient being stored.
hipError_t gemm_wgrad_bias(ModelBase* m, const void* x, const void* dy, int64_t wi, int64_t bi, int64_t N, int64_t in,
                           int64_t out, int accumulate, float* ws, const OptimizerConfig* fused = nullptr);
// Several (up to three) weight gradients of one step, in one launch where that fills the chip better.  A job with
// bias >= 0 also delivers the bias gradient db = column sums of its dy [N, out] into that parameter's slot: fused
// where that is free, a separate column-sum launch otherwise.
struct WgradJob {
  GemmArgs args;       // from wgrad_args
  int64_t bias;        // parameter index of the bias, or -1
};
hipError_t gemm_wgrad_group(ModelBase* m, const WgradJob* jobs, int n, float* ws);

}  // namespace pw
