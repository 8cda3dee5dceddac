// Multi-head attention, forward and backward: causal or unmasked, queries and keys/values from separate
// arrays with their own row strides and lengths (MhaArgs).  One definition serves a decoder's causal
// self-attention over packed [Q|K|V] rows, an encoder's unmasked self-attention and a decoder's attention over
// the encoder output.
//
// Three families:
//  * "row" kernels (here): one thread per query (or key) row, fp32 ALU arithmetic, K/V (or Q/dO) tiles staged
//    through LDS and read as wave-wide broadcasts.  They serve the fp32 configuration (small, latency
//    bound) and whatever the MFMA kernels do not cover.
//  * bf16 MFMA kernels with direct global->LDS loads for head_dim 128 (attention_dma.hip): every layout and
//    mask - the ones that matter for throughput.
//  * bf16 MFMA kernels for packed causal self-attention at head_dim 64 (attention_mfma.hip).
// Scores and probabilities never touch HBM in any family: the forward keeps a running (max, sum)
// per row and writes only O and the row log-sum-exp; the backward recomputes P from Q, K and that
// log-sum-exp.  All reductions run in a fixed order: results are the same bits on every run.
#include <cstdlib>

#include "common.hpp"
#include "kernels.hpp"

namespace pw {

hipError_t launch_attention_fwd_mfma(hipStream_t s, const void* qkv, void* o, float* lse, int B, int T, int H, int hd);
hipError_t launch_attention_bwd_mfma(hipStream_t s, const void* qkv, const void* o, const void* dout, const float* lse,
                                     float* delta, void* dqkv, int B, int T, int H, int hd);
bool attention_mfma_supported(int T, int hd);
bool mha_dma_supported(const MhaArgs& a);
hipError_t launch_mha_fwd_dma(hipStream_t s, const MhaArgs& a, void* o, void* o_lo, float* lse);
hipError_t launch_mha_dq_dkv_dma(hipStream_t s, const MhaArgs& a, const void* o, const void* o_lo, const void* dout,
                                 const float* lse, float* delta, void* dq, int64_t lddq, void* dk, void* dv, int64_t lddkv);

// What the row kernels need of an MhaArgs, typed.
template <class T> struct RowArgs {
  const T *q, *k, *v;
  int64_t ldq, ldkv;
  int Tq, Tk, H, causal;
};

constexpr int kTileRows = 32;   // rows of the streamed operand staged in LDS per step

// Cooperative load of `rows` x HD elements (row stride ld) into LDS as fp32; rows past `limit` become 0.
template <class T, int HD, int NT>
__device__ __forceinline__ void stage_rows(const T* __restrict__ src, int64_t ld, int row0, int limit, float* dst) {
  constexpr int kChunks = kTileRows * HD / 4;
  for (int idx = threadIdx.x; idx < kChunks; idx += NT) {
    const int r = idx / (HD / 4), c = (idx % (HD / 4)) * 4;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (row0 + r < limit) {
      const T* p = src + (int64_t)(row0 + r) * ld + c;
      v = make_float4(to_f32(p[0]), to_f32(p[1]), to_f32(p[2]), to_f32(p[3]));
    }
    *reinterpret_cast<float4*>(dst + r * HD + c) = v;
  }
}

// ---- forward: thread = query row ---------------------------------------------------------------------
template <class T, int HD>
__global__ __launch_bounds__(128) void attention_fwd_row_kernel(RowArgs<T> a, T* __restrict__ o, T* __restrict__ o_lo,
                                                                float* __restrict__ lse) {
  __shared__ float Ks[kTileRows * HD];
  __shared__ float Vs[kTileRows * HD];
  const int Tn = a.Tq, Tk = a.Tk, H = a.H;
  const int d = H * HD;
  const int bh = blockIdx.y, b = bh / H, h = bh - b * H;
  const int i = blockIdx.x * 128 + threadIdx.x;
  const int64_t ld = a.ldkv;
  const T* qrow = a.q + ((int64_t)b * Tn + i) * a.ldq + h * HD;
  const T* kbase = a.k + (int64_t)b * Tk * ld + h * HD;
  const T* vbase = a.v + (int64_t)b * Tk * ld + h * HD;
  const float scale = 1.f / sqrtf((float)HD);
  float q[HD], acc[HD];
  const bool live = i < Tn;
#pragma unroll
  for (int c = 0; c < HD; ++c) {
    q[c] = live ? to_f32(qrow[c]) * scale : 0.f;
    acc[c] = 0.f;
  }
  float m = -INFINITY, l = 0.f;
  const int last_row = a.causal ? min(Tn, (int)(blockIdx.x + 1) * 128) - 1 : Tk - 1;
  for (int j0 = 0; j0 <= last_row; j0 += kTileRows) {
    __syncthreads();
    stage_rows<T, HD, 128>(kbase, ld, j0, Tk, Ks);
    stage_rows<T, HD, 128>(vbase, ld, j0, Tk, Vs);
    __syncthreads();
    if (!live) continue;
    const int jn = a.causal ? min(kTileRows, i - j0 + 1) : min(kTileRows, Tk - j0);
    for (int j = 0; j < jn; ++j) {
      float s = 0.f;
#pragma unroll
      for (int c = 0; c < HD; ++c) s += q[c] * Ks[j * HD + c];
      if (s > m) {
        const float a = __expf(m - s);
        l *= a;
#pragma unroll
        for (int c = 0; c < HD; ++c) acc[c] *= a;
        m = s;
      }
      const float p = __expf(s - m);
      l += p;
#pragma unroll
      for (int c = 0; c < HD; ++c) acc[c] += p * Vs[j * HD + c];
    }
  }
  if (live) {
    const float inv = 1.f / l;
    T* orow = o + ((int64_t)b * Tn + i) * d + h * HD;
#pragma unroll
    for (int c = 0; c < HD; ++c) orow[c] = from_f32<T>(acc[c] * inv);
    if (o_lo) {   // what the rounding of O left over (zero in fp32)
      T* lrow = o_lo + ((int64_t)b * Tn + i) * d + h * HD;
#pragma unroll
      for (int c = 0; c < HD; ++c) lrow[c] = from_f32<T>(acc[c] * inv - to_f32(from_f32<T>(acc[c] * inv)));
    }
    lse[(int64_t)bh * Tn + i] = m + logf(l);
  }
}

// ---- backward ------------------------------------------------------------------------------------------
// delta[b,h,i] = sum_c dO[i,c] O[i,c]
template <class T>
__global__ void attention_delta_kernel(const T* __restrict__ o, const T* __restrict__ o_lo, const T* __restrict__ dout,
                                       float* __restrict__ delta, int Tn, int H, int hd, int64_t total) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // over (b, t, h)
  if (idx >= total) return;
  const int h = idx % H;
  const int64_t n = idx / H;
  const int64_t b = n / Tn, t = n - b * Tn;
  const T* po = o + n * (int64_t)H * hd + (int64_t)h * hd;
  const T* pd = dout + n * (int64_t)H * hd + (int64_t)h * hd;
  float s = 0.f;
  const T* pl = o_lo ? o_lo + n * (int64_t)H * hd + (int64_t)h * hd : nullptr;
  for (int c = 0; c < hd; ++c) s += (to_f32(po[c]) + (pl ? to_f32(pl[c]) : 0.f)) * to_f32(pd[c]);
  delta[(b * H + h) * Tn + t] = s;
}

// dq_i = scale * sum_{j<=i} p_ij (dO_i.v_j - delta_i) k_j,  p_ij = exp(scale q_i.k_j - lse_i); thread = query row.
template <class T, int HD>
__global__ __launch_bounds__(64) void attention_dq_row_kernel(RowArgs<T> a, const T* __restrict__ dout,
                                                              const float* __restrict__ lse,
                                                              const float* __restrict__ delta, T* __restrict__ dq_out,
                                                              int64_t lddq) {
  __shared__ float Ks[kTileRows * HD];
  __shared__ float Vs[kTileRows * HD];
  const int Tn = a.Tq, Tk = a.Tk, H = a.H;
  const int d = H * HD;
  const int bh = blockIdx.y, b = bh / H, h = bh - b * H;
  const int i = blockIdx.x * 64 + threadIdx.x;
  const int64_t ld = a.ldkv;
  const T* qrow = a.q + ((int64_t)b * Tn + i) * a.ldq + h * HD;
  const T* kbase = a.k + (int64_t)b * Tk * ld + h * HD;
  const T* vbase = a.v + (int64_t)b * Tk * ld + h * HD;
  const float scale = 1.f / sqrtf((float)HD);
  const bool live = i < Tn;
  float q[HD], go[HD], dq[HD];
#pragma unroll
  for (int c = 0; c < HD; ++c) {
    q[c] = live ? to_f32(qrow[c]) * scale : 0.f;
    go[c] = live ? to_f32(dout[((int64_t)b * Tn + i) * d + h * HD + c]) : 0.f;
    dq[c] = 0.f;
  }
  const float li = live ? lse[(int64_t)bh * Tn + i] : 0.f;
  const float di = live ? delta[(int64_t)bh * Tn + i] : 0.f;
  const int last_row = a.causal ? min(Tn, (int)(blockIdx.x + 1) * 64) - 1 : Tk - 1;
  for (int j0 = 0; j0 <= last_row; j0 += kTileRows) {
    __syncthreads();
    stage_rows<T, HD, 64>(kbase, ld, j0, Tk, Ks);
    stage_rows<T, HD, 64>(vbase, ld, j0, Tk, Vs);
    __syncthreads();
    if (!live) continue;
    const int jn = a.causal ? min(kTileRows, i - j0 + 1) : min(kTileRows, Tk - j0);
    for (int j = 0; j < jn; ++j) {
      float s = 0.f, dp = 0.f;
#pragma unroll
      for (int c = 0; c < HD; ++c) {
        s += q[c] * Ks[j * HD + c];
        dp += go[c] * Vs[j * HD + c];
      }
      const float ds = __expf(s - li) * (dp - di);
#pragma unroll
      for (int c = 0; c < HD; ++c) dq[c] += ds * Ks[j * HD + c];
    }
  }
  if (live) {
    T* out = dq_out + ((int64_t)b * Tn + i) * lddq + h * HD;
#pragma unroll
    for (int c = 0; c < HD; ++c) out[c] = from_f32<T>(dq[c] * scale);
  }
}

// MODE 0: dv_j = sum_{i>=j} p_ij dO_i.   MODE 1: dk_j = scale * sum_{i>=j} p_ij (dO_i.v_j - delta_i) q_i.
// Thread = key row; Q and dO tiles stream through LDS.
template <class T, int HD, int MODE>
__global__ __launch_bounds__(64) void attention_dkv_row_kernel(RowArgs<T> a, const T* __restrict__ dout,
                                                               const float* __restrict__ lse,
                                                               const float* __restrict__ delta, T* __restrict__ out_base,
                                                               int64_t lddkv) {
  __shared__ float Qs[kTileRows * HD];
  __shared__ float Gs[kTileRows * HD];
  __shared__ float Ls[kTileRows], Ds[kTileRows];
  const int Tn = a.Tq, Tk = a.Tk, H = a.H;             // Tn queries stream past Tk keys
  const int d = H * HD;
  const int bh = blockIdx.y, b = bh / H, h = bh - b * H;
  const int j = blockIdx.x * 64 + threadIdx.x;
  const int64_t ld = a.ldq;
  const T* base = a.q + (int64_t)b * Tn * ld + h * HD;
  const T* gbase = dout + (int64_t)b * Tn * d + h * HD;
  const T* krow = a.k + ((int64_t)b * Tk + j) * a.ldkv + h * HD;
  const T* vrow = a.v + ((int64_t)b * Tk + j) * a.ldkv + h * HD;
  const float scale = 1.f / sqrtf((float)HD);
  const bool live = j < Tk;
  float k[HD], v[MODE == 1 ? HD : 1], acc[HD];
#pragma unroll
  for (int c = 0; c < HD; ++c) {
    k[c] = live ? to_f32(krow[c]) * scale : 0.f;
    if (MODE == 1) v[c] = live ? to_f32(vrow[c]) : 0.f;
    acc[c] = 0.f;
  }
  const int first = a.causal ? (blockIdx.x * 64 / kTileRows) * kTileRows : 0;
  for (int i0 = first; i0 < Tn; i0 += kTileRows) {
    __syncthreads();
    stage_rows<T, HD, 64>(base, ld, i0, Tn, Qs);
    stage_rows<T, HD, 64>(gbase, d, i0, Tn, Gs);
    if (threadIdx.x < kTileRows) {
      const int i = i0 + threadIdx.x;
      Ls[threadIdx.x] = i < Tn ? lse[(int64_t)bh * Tn + i] : 0.f;
      Ds[threadIdx.x] = i < Tn ? delta[(int64_t)bh * Tn + i] : 0.f;
    }
    __syncthreads();
    if (!live) continue;
    const int in = min(kTileRows, Tn - i0);
    for (int ii = a.causal ? max(0, j - i0) : 0; ii < in; ++ii) {
      float s = 0.f;
#pragma unroll
      for (int c = 0; c < HD; ++c) s += k[c] * Qs[ii * HD + c];
      const float p = __expf(s - Ls[ii]);
      if (MODE == 0) {
#pragma unroll
        for (int c = 0; c < HD; ++c) acc[c] += p * Gs[ii * HD + c];
      } else {
        float dp = 0.f;
#pragma unroll
        for (int c = 0; c < HD; ++c) dp += v[c] * Gs[ii * HD + c];
        const float ds = p * (dp - Ds[ii]);
#pragma unroll
        for (int c = 0; c < HD; ++c) acc[c] += ds * Qs[ii * HD + c];
      }
    }
  }
  if (live) {
    T* out = out_base + ((int64_t)b * Tk + j) * lddkv + h * HD;   // MODE 0: dv, MODE 1: dk
#pragma unroll
    for (int c = 0; c < HD; ++c) out[c] = from_f32<T>(MODE == 0 ? acc[c] : acc[c] * scale);
  }
}

template <class T> static RowArgs<T> row_args(const MhaArgs& a) {
  return RowArgs<T>{(const T*)a.q, (const T*)a.k, (const T*)a.v, a.ldq, a.ldkv, a.Tq, a.Tk, a.H, a.causal};
}

template <class T, int HD>
static hipError_t fwd_row(hipStream_t s, const MhaArgs& a, void* o, void* o_lo, float* lse) {
  dim3 grid((a.Tq + 127) / 128, a.B * a.H);
  attention_fwd_row_kernel<T, HD><<<grid, 128, 0, s>>>(row_args<T>(a), (T*)o, (T*)o_lo, lse);
  return hipGetLastError();
}
template <class T, int HD>
static hipError_t bwd_row(hipStream_t s, const MhaArgs& a, const void* o, const void* o_lo, const void* dout, const float* lse,
                          float* delta, void* dq, int64_t lddq, void* dk, void* dv, int64_t lddkv) {
  const int64_t total = (int64_t)a.B * a.Tq * a.H;
  attention_delta_kernel<T><<<(unsigned)((total + 255) / 256), 256, 0, s>>>((const T*)o, (const T*)o_lo, (const T*)dout, delta, a.Tq, a.H, HD, total);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const RowArgs<T> r = row_args<T>(a);
  dim3 grid_q((a.Tq + 63) / 64, a.B * a.H), grid_k((a.Tk + 63) / 64, a.B * a.H);
  attention_dq_row_kernel<T, HD><<<grid_q, 64, 0, s>>>(r, (const T*)dout, lse, delta, (T*)dq, lddq);
  attention_dkv_row_kernel<T, HD, 0><<<grid_k, 64, 0, s>>>(r, (const T*)dout, lse, delta, (T*)dv, lddkv);
  attention_dkv_row_kernel<T, HD, 1><<<grid_k, 64, 0, s>>>(r, (const T*)dout, lse, delta, (T*)dk, lddkv);
  return hipGetLastError();
}

static bool mha_args_ok(const MhaArgs& a) {
  if (!a.q || !a.k || !a.v || a.B <= 0 || a.Tq <= 0 || a.Tk <= 0 || a.H <= 0) return false;
  if (a.hd != 64 && a.hd != 128) return false;
  if (a.dtype != kF32 && a.dtype != kBF16) return false;
  if ((int64_t)a.B * a.H > 65535) return false;
  if (a.ldq < (int64_t)a.H * a.hd || a.ldkv < (int64_t)a.H * a.hd) return false;
  if (a.causal && a.Tq != a.Tk) return false;
  return true;
}

// head_dim 128 in bf16 runs the kernels of attention_dma.hip unless PW_ATTN_DMA=0 (A/B switch for measurements).
static bool use_dma_kernels() {
  static int v = -1;
  if (v < 0) {
    const char* e = getenv("PW_ATTN_DMA");
    v = !(e && e[0] == '0');
  }
  return v != 0;
}

// Packed causal self-attention: what the kernels of attention_mfma.hip are written for.
static bool is_packed_causal(const MhaArgs& a) {
  const int64_t d = (int64_t)a.H * a.hd;
  const size_t es = a.dtype == kBF16 ? 2 : 4;
  return a.causal && a.ldq == 3 * d && a.ldkv == 3 * d && (const char*)a.k == (const char*)a.q + d * es &&
         (const char*)a.v == (const char*)a.q + 2 * d * es;
}

hipError_t launch_mha_fwd(hipStream_t s, const MhaArgs& a, void* o, void* o_lo, float* lse) {
  if (!mha_args_ok(a) || !o || !lse) return hipErrorInvalidValue;
  if (use_dma_kernels() && mha_dma_supported(a) && !(((uintptr_t)o | (uintptr_t)o_lo) & 15)) return launch_mha_fwd_dma(s, a, o, o_lo, lse);
  if (a.dtype == kBF16 && is_packed_causal(a) && attention_mfma_supported(a.Tq, a.hd)) {
    if (o_lo) {   // these kernels keep no remainder: an all-zero one says so to the backward pass
      const int64_t n = (int64_t)a.B * a.Tq * a.H * a.hd;   // bf16 elements, an even number
      const hipError_t e = launch_fill_f32(s, (float*)o_lo, n / 2, 0.f);
      if (e != hipSuccess) return e;
    }
    return launch_attention_fwd_mfma(s, a.q, o, lse, a.B, a.Tq, a.H, a.hd);
  }
  if (a.dtype == kF32) return a.hd == 64 ? fwd_row<float, 64>(s, a, o, o_lo, lse) : fwd_row<float, 128>(s, a, o, o_lo, lse);
  return a.hd == 64 ? fwd_row<bf16, 64>(s, a, o, o_lo, lse) : fwd_row<bf16, 128>(s, a, o, o_lo, lse);
}

hipError_t launch_mha_bwd(hipStream_t s, const MhaArgs& a, const void* o, const void* o_lo, const void* dout,
                          const float* lse, float* delta, void* dq, int64_t lddq, void* dk, void* dv, int64_t lddkv) {
  if (!mha_args_ok(a) || !o || !dout || !lse || !delta || !dq || !dk || !dv) return hipErrorInvalidValue;
  const int64_t d = (int64_t)a.H * a.hd;
  if (lddq < d || lddkv < d) return hipErrorInvalidValue;
  if (use_dma_kernels() && mha_dma_supported(a) && !(((uintptr_t)o | (uintptr_t)o_lo | (uintptr_t)dout) & 15)) {
    return launch_mha_dq_dkv_dma(s, a, o, o_lo, dout, lse, delta, dq, lddq, dk, dv, lddkv);   // (delta comes from the dQ kernel)
  }
  const size_t es = a.dtype == kBF16 ? 2 : 4;
  const bool packed_out = lddq == 3 * d && lddkv == 3 * d && (char*)dk == (char*)dq + d * es && (char*)dv == (char*)dq + 2 * d * es;
  if (a.dtype == kBF16 && is_packed_causal(a) && packed_out && attention_mfma_supported(a.Tq, a.hd))
    return launch_attention_bwd_mfma(s, a.q, o, dout, lse, delta, dq, a.B, a.Tq, a.H, a.hd);   // (its forward left o_lo zero)
  if (a.dtype == kF32)
    return a.hd == 64 ? bwd_row<float, 64>(s, a, o, o_lo, dout, lse, delta, dq, lddq, dk, dv, lddkv)
                      : bwd_row<float, 128>(s, a, o, o_lo, dout, lse, delta, dq, lddq, dk, dv, lddkv);
  return a.hd == 64 ? bwd_row<bf16, 64>(s, a, o, o_lo, dout, lse, delta, dq, lddq, dk, dv, lddkv)
                    : bwd_row<bf16, 128>(s, a, o, o_lo, dout, lse, delta, dq, lddq, dk, dv, lddkv);
}

static MhaArgs packed_args(int dtype, const void* qkv, int B, int T, int H, int hd) {
  const int64_t d = (int64_t)H * hd;
  const size_t es = dtype == kBF16 ? 2 : 4;
  const char* base = (const char*)qkv;
  return MhaArgs{dtype, base, base + d * es, base + 2 * d * es, 3 * d, 3 * d, B, T, T, H, hd, 1};
}

hipError_t launch_attention_fwd(hipStream_t s, int dtype, const void* qkv, void* o, float* lse, int B, int T, int H,
                                int hd) {
  if (!qkv || (dtype != kF32 && dtype != kBF16)) return hipErrorInvalidValue;
  return launch_mha_fwd(s, packed_args(dtype, qkv, B, T, H, hd), o, nullptr, lse);
}

hipError_t launch_attention_bwd(hipStream_t s, int dtype, const void* qkv, const void* o, const void* dout,
                                const float* lse, float* delta, void* dqkv, int B, int T, int H, int hd) {
  if (!qkv || !dqkv || (dtype != kF32 && dtype != kBF16)) return hipErrorInvalidValue;
  const int64_t d = (int64_t)H * hd;
  const size_t es = dtype == kBF16 ? 2 : 4;
  char* g = (char*)dqkv;
  return launch_mha_bwd(s, packed_args(dtype, qkv, B, T, H, hd), o, nullptr, dout, lse, delta, g, 3 * d, g + d * es, g + 2 * d * es, 3 * d);
}

}  // namespace pw
