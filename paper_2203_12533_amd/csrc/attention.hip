// Causal multi-head attention, forward and backward.
//
// Two families live here:
//  * "row" kernels: one thread per query (or key) row, fp32 ALU arithmetic, K/V (or Q/dO) tiles staged
//    through LDS and read as wave-wide broadcasts.  They serve the fp32 configuration (small, latency
//    bound) and any head_dim/dtype the MFMA kernels do not cover.
//  * MFMA kernels for bf16 (see attention_mfma.hip) - the ones that matter for throughput.
// Scores and probabilities never touch HBM in either family: the forward keeps a running (max, sum)
// per row and writes only O and the row log-sum-exp; the backward recomputes P from Q, K and that
// log-sum-exp.  All reductions run in a fixed order: results are the same bits on every run.
#include "common.hpp"
#include "kernels.hpp"

namespace pw {

hipError_t launch_attention_fwd_mfma(hipStream_t s, const void* qkv, void* o, float* lse, int B, int T, int H, int hd);
hipError_t launch_attention_bwd_mfma(hipStream_t s, const void* qkv, const void* o, const void* dout, const float* lse,
                                     float* delta, void* dqkv, int B, int T, int H, int hd);
bool attention_mfma_supported(int T, int hd);

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
__global__ __launch_bounds__(128) void attention_fwd_row_kernel(const T* __restrict__ qkv, T* __restrict__ o,
                                                                float* __restrict__ lse, int Tn, int H) {
  __shared__ float Ks[kTileRows * HD];
  __shared__ float Vs[kTileRows * HD];
  const int d = H * HD;
  const int bh = blockIdx.y, b = bh / H, h = bh - b * H;
  const int i = blockIdx.x * 128 + threadIdx.x;
  const int64_t ld = 3 * (int64_t)d;
  const T* base = qkv + (int64_t)b * Tn * ld + h * HD;
  const float scale = 1.f / sqrtf((float)HD);
  float q[HD], acc[HD];
  const bool live = i < Tn;
#pragma unroll
  for (int c = 0; c < HD; ++c) {
    q[c] = live ? to_f32(base[(int64_t)i * ld + c]) * scale : 0.f;
    acc[c] = 0.f;
  }
  float m = -INFINITY, l = 0.f;
  const int last_row = min(Tn, (int)(blockIdx.x + 1) * 128) - 1;
  for (int j0 = 0; j0 <= last_row; j0 += kTileRows) {
    __syncthreads();
    stage_rows<T, HD, 128>(base + d, ld, j0, Tn, Ks);
    stage_rows<T, HD, 128>(base + 2 * d, ld, j0, Tn, Vs);
    __syncthreads();
    if (!live) continue;
    const int jn = min(kTileRows, i - j0 + 1);
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
    lse[(int64_t)bh * Tn + i] = m + logf(l);
  }
}

// ---- backward ------------------------------------------------------------------------------------------
// delta[b,h,i] = sum_c dO[i,c] O[i,c]
template <class T>
__global__ void attention_delta_kernel(const T* __restrict__ o, const T* __restrict__ dout, float* __restrict__ delta,
                                       int Tn, int H, int hd, int64_t total) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // over (b, t, h)
  if (idx >= total) return;
  const int h = idx % H;
  const int64_t n = idx / H;
  const int64_t b = n / Tn, t = n - b * Tn;
  const T* po = o + n * (int64_t)H * hd + (int64_t)h * hd;
  const T* pd = dout + n * (int64_t)H * hd + (int64_t)h * hd;
  float s = 0.f;
  for (int c = 0; c < hd; ++c) s += to_f32(po[c]) * to_f32(pd[c]);
  delta[(b * H + h) * Tn + t] = s;
}

// dq_i = scale * sum_{j<=i} p_ij (dO_i.v_j - delta_i) k_j,  p_ij = exp(scale q_i.k_j - lse_i); thread = query row.
template <class T, int HD>
__global__ __launch_bounds__(64) void attention_dq_row_kernel(const T* __restrict__ qkv, const T* __restrict__ dout,
                                                              const float* __restrict__ lse,
                                                              const float* __restrict__ delta, T* __restrict__ dqkv,
                                                              int Tn, int H) {
  __shared__ float Ks[kTileRows * HD];
  __shared__ float Vs[kTileRows * HD];
  const int d = H * HD;
  const int bh = blockIdx.y, b = bh / H, h = bh - b * H;
  const int i = blockIdx.x * 64 + threadIdx.x;
  const int64_t ld = 3 * (int64_t)d;
  const T* base = qkv + (int64_t)b * Tn * ld + h * HD;
  const float scale = 1.f / sqrtf((float)HD);
  const bool live = i < Tn;
  float q[HD], go[HD], dq[HD];
#pragma unroll
  for (int c = 0; c < HD; ++c) {
    q[c] = live ? to_f32(base[(int64_t)i * ld + c]) * scale : 0.f;
    go[c] = live ? to_f32(dout[((int64_t)b * Tn + i) * d + h * HD + c]) : 0.f;
    dq[c] = 0.f;
  }
  const float li = live ? lse[(int64_t)bh * Tn + i] : 0.f;
  const float di = live ? delta[(int64_t)bh * Tn + i] : 0.f;
  const int last_row = min(Tn, (int)(blockIdx.x + 1) * 64) - 1;
  for (int j0 = 0; j0 <= last_row; j0 += kTileRows) {
    __syncthreads();
    stage_rows<T, HD, 64>(base + d, ld, j0, Tn, Ks);
    stage_rows<T, HD, 64>(base + 2 * d, ld, j0, Tn, Vs);
    __syncthreads();
    if (!live) continue;
    const int jn = min(kTileRows, i - j0 + 1);
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
    T* out = dqkv + ((int64_t)b * Tn + i) * ld + h * HD;
#pragma unroll
    for (int c = 0; c < HD; ++c) out[c] = from_f32<T>(dq[c] * scale);
  }
}

// MODE 0: dv_j = sum_{i>=j} p_ij dO_i.   MODE 1: dk_j = scale * sum_{i>=j} p_ij (dO_i.v_j - delta_i) q_i.
// Thread = key row; Q and dO tiles stream through LDS.
template <class T, int HD, int MODE>
__global__ __launch_bounds__(64) void attention_dkv_row_kernel(const T* __restrict__ qkv, const T* __restrict__ dout,
                                                               const float* __restrict__ lse,
                                                               const float* __restrict__ delta, T* __restrict__ dqkv,
                                                               int Tn, int H) {
  __shared__ float Qs[kTileRows * HD];
  __shared__ float Gs[kTileRows * HD];
  __shared__ float Ls[kTileRows], Ds[kTileRows];
  const int d = H * HD;
  const int bh = blockIdx.y, b = bh / H, h = bh - b * H;
  const int j = blockIdx.x * 64 + threadIdx.x;
  const int64_t ld = 3 * (int64_t)d;
  const T* base = qkv + (int64_t)b * Tn * ld + h * HD;
  const T* gbase = dout + (int64_t)b * Tn * d + h * HD;
  const float scale = 1.f / sqrtf((float)HD);
  const bool live = j < Tn;
  float k[HD], v[MODE == 1 ? HD : 1], acc[HD];
#pragma unroll
  for (int c = 0; c < HD; ++c) {
    k[c] = live ? to_f32(base[(int64_t)j * ld + d + c]) * scale : 0.f;
    if (MODE == 1) v[c] = live ? to_f32(base[(int64_t)j * ld + 2 * d + c]) : 0.f;
    acc[c] = 0.f;
  }
  const int first = (blockIdx.x * 64 / kTileRows) * kTileRows;
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
    for (int ii = max(0, j - i0); ii < in; ++ii) {
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
    T* out = dqkv + ((int64_t)b * Tn + j) * ld + (MODE == 0 ? 2 * d : d) + h * HD;
#pragma unroll
    for (int c = 0; c < HD; ++c) out[c] = from_f32<T>(MODE == 0 ? acc[c] : acc[c] * scale);
  }
}

template <class T, int HD>
static hipError_t fwd_row(hipStream_t s, const void* qkv, void* o, float* lse, int B, int Tn, int H) {
  dim3 grid((Tn + 127) / 128, B * H);
  attention_fwd_row_kernel<T, HD><<<grid, 128, 0, s>>>((const T*)qkv, (T*)o, lse, Tn, H);
  return hipGetLastError();
}
template <class T, int HD>
static hipError_t bwd_row(hipStream_t s, const void* qkv, const void* o, const void* dout, const float* lse,
                          float* delta, void* dqkv, int B, int Tn, int H) {
  const int64_t total = (int64_t)B * Tn * H;
  attention_delta_kernel<T><<<(unsigned)((total + 255) / 256), 256, 0, s>>>((const T*)o, (const T*)dout, delta, Tn, H, HD, total);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  dim3 grid((Tn + 63) / 64, B * H);
  attention_dq_row_kernel<T, HD><<<grid, 64, 0, s>>>((const T*)qkv, (const T*)dout, lse, delta, (T*)dqkv, Tn, H);
  attention_dkv_row_kernel<T, HD, 0><<<grid, 64, 0, s>>>((const T*)qkv, (const T*)dout, lse, delta, (T*)dqkv, Tn, H);
  attention_dkv_row_kernel<T, HD, 1><<<grid, 64, 0, s>>>((const T*)qkv, (const T*)dout, lse, delta, (T*)dqkv, Tn, H);
  return hipGetLastError();
}

static bool attn_args_ok(const void* qkv, const void* o, int B, int T, int H, int hd) {
  if (!qkv || !o || B <= 0 || T <= 0 || H <= 0) return false;
  if (hd != 64 && hd != 128) return false;
  if ((int64_t)B * H > 65535) return false;
  return true;
}

hipError_t launch_attention_fwd(hipStream_t s, int dtype, const void* qkv, void* o, float* lse, int B, int T, int H,
                                int hd) {
  if (!attn_args_ok(qkv, o, B, T, H, hd) || !lse) return hipErrorInvalidValue;
  if (dtype == kBF16 && attention_mfma_supported(T, hd)) return launch_attention_fwd_mfma(s, qkv, o, lse, B, T, H, hd);
  if (dtype == kF32) return hd == 64 ? fwd_row<float, 64>(s, qkv, o, lse, B, T, H) : fwd_row<float, 128>(s, qkv, o, lse, B, T, H);
  if (dtype == kBF16) return hd == 64 ? fwd_row<bf16, 64>(s, qkv, o, lse, B, T, H) : fwd_row<bf16, 128>(s, qkv, o, lse, B, T, H);
  return hipErrorInvalidValue;
}

hipError_t launch_attention_bwd(hipStream_t s, int dtype, const void* qkv, const void* o, const void* dout,
                                const float* lse, float* delta, void* dqkv, int B, int T, int H, int hd) {
  if (!attn_args_ok(qkv, o, B, T, H, hd) || !dout || !lse || !delta || !dqkv) return hipErrorInvalidValue;
  if (dtype == kBF16 && attention_mfma_supported(T, hd))
    return launch_attention_bwd_mfma(s, qkv, o, dout, lse, delta, dqkv, B, T, H, hd);
  if (dtype == kF32)
    return hd == 64 ? bwd_row<float, 64>(s, qkv, o, dout, lse, delta, dqkv, B, T, H)
                    : bwd_row<float, 128>(s, qkv, o, dout, lse, delta, dqkv, B, T, H);
  if (dtype == kBF16)
    return hd == 64 ? bwd_row<bf16, 64>(s, qkv, o, dout, lse, delta, dqkv, B, T, H)
                    : bwd_row<bf16, 128>(s, qkv, o, dout, lse, delta, dqkv, B, T, H);
  return hipErrorInvalidValue;
}

}  // namespace pw
