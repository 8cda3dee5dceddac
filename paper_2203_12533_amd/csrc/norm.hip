// LayerNorm forward / backward and column sums (bias gradients).  HBM-bound: every row is read once
// from memory with 16-byte accesses, held in registers, and reduced with wave64 shuffles.  Rows of up to
// 2048 columns are handled by ONE wave each (no block-wide synchronisation at all, several rows in flight per
// compute unit); wider rows by one 256-thread block each.
#include "common.hpp"
#include "kernels.hpp"

namespace pw {

constexpr int kLnThreads = 256;
constexpr int kLnMaxVec = 8;   // float4 per thread: rows up to 256*4*8 = 8192 columns stay in registers

template <class T> __device__ __forceinline__ void store4(T* p, float a, float b, float c, float d);
template <> __device__ __forceinline__ void store4<float>(float* p, float a, float b, float c, float d) {
  *reinterpret_cast<float4*>(p) = make_float4(a, b, c, d);
}
template <> __device__ __forceinline__ void store4<bf16>(bf16* p, float a, float b, float c, float d) {
  bf16x4 o = {(bf16)a, (bf16)b, (bf16)c, (bf16)d};
  *reinterpret_cast<bf16x4*>(p) = o;
}
template <class T> __device__ __forceinline__ float4 load4(const T* p);
template <> __device__ __forceinline__ float4 load4<float>(const float* p) { return *reinterpret_cast<const float4*>(p); }
template <> __device__ __forceinline__ float4 load4<bf16>(const bf16* p) {
  const bf16x4 v = *reinterpret_cast<const bf16x4*>(p);
  return make_float4((float)v[0], (float)v[1], (float)v[2], (float)v[3]);
}

// One block per row (grid-stride over rows).  d % 4 == 0, d <= 8192.
template <class T>
__global__ __launch_bounds__(kLnThreads) void layernorm_fwd_kernel(const float* __restrict__ x, const float* __restrict__ g,
                                                                   const float* __restrict__ b, T* __restrict__ y,
                                                                   float* __restrict__ mean, float* __restrict__ rstd,
                                                                   int N, int d) {
  __shared__ float red[kLnThreads / 64];
  const int d4 = d >> 2;
  for (int n = blockIdx.x; n < N; n += gridDim.x) {
    const float* xr = x + (size_t)n * d;
    float4 v[kLnMaxVec];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < kLnMaxVec; ++i) {
      const int c4 = threadIdx.x + i * kLnThreads;
      if (c4 < d4) {
        v[i] = reinterpret_cast<const float4*>(xr)[c4];
        s += (v[i].x + v[i].y) + (v[i].z + v[i].w);
      }
    }
    const float mu = block_sum(s, red) / (float)d;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < kLnMaxVec; ++i) {
      const int c4 = threadIdx.x + i * kLnThreads;
      if (c4 < d4) {
        const float a = v[i].x - mu, bb = v[i].y - mu, c = v[i].z - mu, e = v[i].w - mu;
        q += (a * a + bb * bb) + (c * c + e * e);
      }
    }
    const float var = block_sum(q, red) / (float)d;
    const float rs = 1.f / sqrtf(var + 1e-5f);
#pragma unroll
    for (int i = 0; i < kLnMaxVec; ++i) {
      const int c4 = threadIdx.x + i * kLnThreads;
      if (c4 < d4) {
        const float4 gv = reinterpret_cast<const float4*>(g)[c4];
        const float4 bv = reinterpret_cast<const float4*>(b)[c4];
        store4<T>(y + (size_t)n * d + 4 * c4, (v[i].x - mu) * rs * gv.x + bv.x, (v[i].y - mu) * rs * gv.y + bv.y,
                  (v[i].z - mu) * rs * gv.z + bv.z, (v[i].w - mu) * rs * gv.w + bv.w);
      }
    }
    if (threadIdx.x == 0) {
      mean[n] = mu;
      rstd[n] = rs;
    }
  }
}

// One wave per row: lane l owns float4 columns l, l + 64, ...; VEC of them (d <= 256 * VEC).
constexpr int kLnWaveMaxD = 2048;
template <class T, int VEC>
__global__ __launch_bounds__(kLnThreads) void layernorm_fwd_wave_kernel(const float* __restrict__ x, const float* __restrict__ g,
                                                                        const float* __restrict__ b, T* __restrict__ y,
                                                                        float* __restrict__ mean, float* __restrict__ rstd,
                                                                        int N, int d) {
  const int d4 = d >> 2, lane = threadIdx.x & 63;
  const int wave = blockIdx.x * (kLnThreads / 64) + (threadIdx.x >> 6), nwaves = gridDim.x * (kLnThreads / 64);
  // The next row of this wave is requested before the current one is reduced and stored, so a wave always has
  // loads in flight.
  auto fetch = [&](int n, float4* r) {
    const float4* xr = reinterpret_cast<const float4*>(x + (size_t)n * d);
#pragma unroll
    for (int i = 0; i < VEC; ++i)
      if (lane + i * 64 < d4) r[i] = xr[lane + i * 64];
  };
  float4 v[VEC], nx[VEC];
  if (wave < N) fetch(wave, v);
  for (int n = wave; n < N; n += nwaves) {
    if (n + nwaves < N) fetch(n + nwaves, nx);
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < VEC; ++i)
      if (lane + i * 64 < d4) s += (v[i].x + v[i].y) + (v[i].z + v[i].w);
    const float mu = wave_sum(s) / (float)d;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
      if (lane + i * 64 < d4) {
        const float a = v[i].x - mu, bb = v[i].y - mu, c = v[i].z - mu, e = v[i].w - mu;
        q += (a * a + bb * bb) + (c * c + e * e);
      }
    }
    const float var = wave_sum(q) / (float)d;
    const float rs = 1.f / sqrtf(var + 1e-5f);
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
      const int c4 = lane + i * 64;
      if (c4 < d4) {
        const float4 gv = reinterpret_cast<const float4*>(g)[c4];
        const float4 bv = reinterpret_cast<const float4*>(b)[c4];
        store4<T>(y + (size_t)n * d + 4 * c4, (v[i].x - mu) * rs * gv.x + bv.x, (v[i].y - mu) * rs * gv.y + bv.y,
                  (v[i].z - mu) * rs * gv.z + bv.z, (v[i].w - mu) * rs * gv.w + bv.w);
      }
    }
    if (lane == 0) {
      mean[n] = mu;
      rstd[n] = rs;
    }
#pragma unroll
    for (int i = 0; i < VEC; ++i) v[i] = nx[i];
  }
}

template <class T>
static void launch_ln_fwd_wave(hipStream_t s, const float* x, const float* g, const float* b, T* y, float* mean,
                               float* rstd, int N, int d) {
  const int rows_per_block = kLnThreads / 64;
  int grid = (N + rows_per_block - 1) / rows_per_block;
  if (grid > 1024) grid = 1024;   // 16 waves per compute unit, each with its next row already requested
  if (d <= 256) layernorm_fwd_wave_kernel<T, 1><<<grid, kLnThreads, 0, s>>>(x, g, b, y, mean, rstd, N, d);
  else if (d <= 512) layernorm_fwd_wave_kernel<T, 2><<<grid, kLnThreads, 0, s>>>(x, g, b, y, mean, rstd, N, d);
  else if (d <= 1024) layernorm_fwd_wave_kernel<T, 4><<<grid, kLnThreads, 0, s>>>(x, g, b, y, mean, rstd, N, d);
  else layernorm_fwd_wave_kernel<T, 8><<<grid, kLnThreads, 0, s>>>(x, g, b, y, mean, rstd, N, d);
}

hipError_t launch_layernorm_fwd(hipStream_t s, int dtype, const float* x, const float* g, const float* b, void* y,
                                float* mean, float* rstd, int N, int d) {
  if (!x || !g || !b || !y || !mean || !rstd || N < 0 || d <= 0) return hipErrorInvalidValue;
  if (d % 4 || d > kLnThreads * 4 * kLnMaxVec) return hipErrorInvalidValue;
  if (((uintptr_t)x | (uintptr_t)g | (uintptr_t)b) & 15) return hipErrorInvalidValue;
  if ((uintptr_t)y & (dtype == kBF16 ? 7 : 15)) return hipErrorInvalidValue;
  if (N == 0) return hipSuccess;
  if (dtype != kF32 && dtype != kBF16) return hipErrorInvalidValue;
  if (d <= kLnWaveMaxD) {
    if (dtype == kF32) launch_ln_fwd_wave<float>(s, x, g, b, (float*)y, mean, rstd, N, d);
    else launch_ln_fwd_wave<bf16>(s, x, g, b, (bf16*)y, mean, rstd, N, d);
    return hipGetLastError();
  }
  const int grid = N < 8192 ? N : 8192;
  if (dtype == kF32)
    layernorm_fwd_kernel<float><<<grid, kLnThreads, 0, s>>>(x, g, b, (float*)y, mean, rstd, N, d);
  else if (dtype == kBF16)
    layernorm_fwd_kernel<bf16><<<grid, kLnThreads, 0, s>>>(x, g, b, (bf16*)y, mean, rstd, N, d);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

// ---- backward -----------------------------------------------------------------------------------
// dx = dres + rstd (gg - mean(gg) - xh mean(gg xh)), gg = dy gamma, xh = (x - mean) rstd.  Next to dx every
// thread keeps running sums, over the rows it sees, of dy*xh (-> dgamma), dy (-> dbeta) and, if asked for,
// of dx itself (-> the bias gradient of the linear layer whose output gradient dx is).  Each block writes
// its sums to ws[set][block][:]; a second kernel adds the blocks in index order, so results are the same
// bits on every run.
constexpr int kLnBwdMaxBlocks = 512;

static inline int ln_bwd_blocks(int N) { return N < kLnBwdMaxBlocks ? (N < 1 ? 1 : N) : kLnBwdMaxBlocks; }
int64_t layernorm_bwd_ws_floats(int N, int d) { return 3LL * ln_bwd_blocks(N) * d; }

__device__ __forceinline__ void add4(float4& a, const float4& b) { a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w; }

// Wide rows (d > 2048): block b handles rows b, b+G, ...; two block sums per row.
template <class T>
__global__ __launch_bounds__(kLnThreads) void layernorm_bwd_kernel(const T* __restrict__ dy, const float* __restrict__ x,
                                                                   const float* __restrict__ g,
                                                                   const float* __restrict__ mean,
                                                                   const float* __restrict__ rstd,
                                                                   const float* __restrict__ dres, float* __restrict__ dx,
                                                                   T* __restrict__ dx_lp, float* __restrict__ ws, int N,
                                                                   int d, int want_dsum) {
  __shared__ float red[kLnThreads / 64];
  const int d4 = d >> 2;
  float4 accg[kLnMaxVec], accb[kLnMaxVec], accd[kLnMaxVec];
#pragma unroll
  for (int i = 0; i < kLnMaxVec; ++i) accg[i] = accb[i] = accd[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int n = blockIdx.x; n < N; n += gridDim.x) {
    const float mu = mean[n], rs = rstd[n];
    float4 xh[kLnMaxVec], gg[kLnMaxVec];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < kLnMaxVec; ++i) {
      const int c4 = threadIdx.x + i * kLnThreads;
      if (c4 < d4) {
        const float4 xv = reinterpret_cast<const float4*>(x + (size_t)n * d)[c4];
        const float4 dv = load4<T>(dy + (size_t)n * d + 4 * c4);
        const float4 gv = reinterpret_cast<const float4*>(g)[c4];
        xh[i] = make_float4((xv.x - mu) * rs, (xv.y - mu) * rs, (xv.z - mu) * rs, (xv.w - mu) * rs);
        gg[i] = make_float4(dv.x * gv.x, dv.y * gv.y, dv.z * gv.z, dv.w * gv.w);
        s1 += (gg[i].x + gg[i].y) + (gg[i].z + gg[i].w);
        s2 += (gg[i].x * xh[i].x + gg[i].y * xh[i].y) + (gg[i].z * xh[i].z + gg[i].w * xh[i].w);
        accg[i].x += dv.x * xh[i].x; accg[i].y += dv.y * xh[i].y; accg[i].z += dv.z * xh[i].z; accg[i].w += dv.w * xh[i].w;
        add4(accb[i], dv);
      }
    }
    const float m1 = block_sum(s1, red) / (float)d;
    const float m2 = block_sum(s2, red) / (float)d;
#pragma unroll
    for (int i = 0; i < kLnMaxVec; ++i) {
      const int c4 = threadIdx.x + i * kLnThreads;
      if (c4 < d4) {
        float4 o = make_float4(rs * (gg[i].x - m1 - xh[i].x * m2), rs * (gg[i].y - m1 - xh[i].y * m2),
                               rs * (gg[i].z - m1 - xh[i].z * m2), rs * (gg[i].w - m1 - xh[i].w * m2));
        if (dres) add4(o, reinterpret_cast<const float4*>(dres + (size_t)n * d)[c4]);
        reinterpret_cast<float4*>(dx + (size_t)n * d)[c4] = o;
        if (dx_lp) store4<T>(dx_lp + (size_t)n * d + 4 * c4, o.x, o.y, o.z, o.w);
        add4(accd[i], o);
      }
    }
  }
  float* w0 = ws + (size_t)blockIdx.x * d;
  const size_t set = (size_t)gridDim.x * d;
#pragma unroll
  for (int i = 0; i < kLnMaxVec; ++i) {
    const int c4 = threadIdx.x + i * kLnThreads;
    if (c4 < d4) {
      reinterpret_cast<float4*>(w0)[c4] = accg[i];
      reinterpret_cast<float4*>(w0 + set)[c4] = accb[i];
      if (want_dsum) reinterpret_cast<float4*>(w0 + 2 * set)[c4] = accd[i];
    }
  }
}

// Rows of up to 2048 columns: one wave per row (wave w of the grid handles rows w, w + W, ...), lane l owns
// float4 columns l, l + 64, ...  At the end the four waves of a block add their sums through LDS in wave order.
template <class T, int VEC>
__global__ __launch_bounds__(kLnThreads) void layernorm_bwd_wave_kernel(const T* __restrict__ dy, const float* __restrict__ x,
                                                                        const float* __restrict__ g,
                                                                        const float* __restrict__ mean,
                                                                        const float* __restrict__ rstd,
                                                                        const float* __restrict__ dres,
                                                                        float* __restrict__ dx, T* __restrict__ dx_lp,
                                                                        float* __restrict__ ws, int N, int d,
                                                                        int want_dsum) {
  constexpr int kWaves = kLnThreads / 64;
  __shared__ float4 part[kWaves][VEC * 64];
  const int d4 = d >> 2, lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
  const int wave = blockIdx.x * kWaves + wib, nwaves = gridDim.x * kWaves;
  const float4* g4 = reinterpret_cast<const float4*>(g);
  float4 acc[3][VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) acc[0][i] = acc[1][i] = acc[2][i] = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int n = wave; n < N; n += nwaves) {
    const float mu = mean[n], rs = rstd[n];
    float4 xh[VEC], dv[VEC], rv[VEC];
    float s1 = 0.f, s2 = 0.f;
    // the residual gradient is fetched together with the other inputs, not after the row reductions
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
      const int c4 = lane + i * 64;
      rv[i] = (dres && c4 < d4) ? reinterpret_cast<const float4*>(dres + (size_t)n * d)[c4] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
      const int c4 = lane + i * 64;
      if (c4 < d4) {
        const float4 xv = reinterpret_cast<const float4*>(x + (size_t)n * d)[c4];
        dv[i] = load4<T>(dy + (size_t)n * d + 4 * c4);
        const float4 gv = g4[c4];
        xh[i] = make_float4((xv.x - mu) * rs, (xv.y - mu) * rs, (xv.z - mu) * rs, (xv.w - mu) * rs);
        const float4 gg = make_float4(dv[i].x * gv.x, dv[i].y * gv.y, dv[i].z * gv.z, dv[i].w * gv.w);
        s1 += (gg.x + gg.y) + (gg.z + gg.w);
        s2 += (gg.x * xh[i].x + gg.y * xh[i].y) + (gg.z * xh[i].z + gg.w * xh[i].w);
        acc[0][i].x += dv[i].x * xh[i].x; acc[0][i].y += dv[i].y * xh[i].y;
        acc[0][i].z += dv[i].z * xh[i].z; acc[0][i].w += dv[i].w * xh[i].w;
        add4(acc[1][i], dv[i]);
      }
    }
    const float m1 = wave_sum(s1) / (float)d;
    const float m2 = wave_sum(s2) / (float)d;
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
      const int c4 = lane + i * 64;
      if (c4 < d4) {
        const float4 gv = g4[c4];
        float4 o = make_float4(rs * (dv[i].x * gv.x - m1 - xh[i].x * m2), rs * (dv[i].y * gv.y - m1 - xh[i].y * m2),
                               rs * (dv[i].z * gv.z - m1 - xh[i].z * m2), rs * (dv[i].w * gv.w - m1 - xh[i].w * m2));
        add4(o, rv[i]);
        reinterpret_cast<float4*>(dx + (size_t)n * d)[c4] = o;
        if (dx_lp) store4<T>(dx_lp + (size_t)n * d + 4 * c4, o.x, o.y, o.z, o.w);
        add4(acc[2][i], o);
      }
    }
  }
  const size_t set = (size_t)gridDim.x * d;
  auto flush = [&](int k, const float4 (&a)[VEC]) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < VEC; ++i)
      if (lane + i * 64 < d4) part[wib][lane + i * 64] = a[i];
    __syncthreads();
    float* out = ws + k * set + (size_t)blockIdx.x * d;
    for (int c4 = threadIdx.x; c4 < d4; c4 += kLnThreads) {
      float4 t = part[0][c4];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) add4(t, part[w][c4]);
      reinterpret_cast<float4*>(out)[c4] = t;
    }
  };
  flush(0, acc[0]);
  flush(1, acc[1]);
  if (want_dsum) flush(2, acc[2]);   // uniform over the grid
}

template <class T>
static void launch_ln_bwd_wave(hipStream_t s, int G, const T* dy, const float* x, const float* g, const float* mean,
                               const float* rstd, const float* dres, float* dx, T* dx_lp, float* ws, int N, int d, int want) {
  if (d <= 256) layernorm_bwd_wave_kernel<T, 1><<<G, kLnThreads, 0, s>>>(dy, x, g, mean, rstd, dres, dx, dx_lp, ws, N, d, want);
  else if (d <= 512) layernorm_bwd_wave_kernel<T, 2><<<G, kLnThreads, 0, s>>>(dy, x, g, mean, rstd, dres, dx, dx_lp, ws, N, d, want);
  else if (d <= 1024) layernorm_bwd_wave_kernel<T, 4><<<G, kLnThreads, 0, s>>>(dy, x, g, mean, rstd, dres, dx, dx_lp, ws, N, d, want);
  else layernorm_bwd_wave_kernel<T, 8><<<G, kLnThreads, 0, s>>>(dy, x, g, mean, rstd, dres, dx, dx_lp, ws, N, d, want);
}

// out[c] (=|+=) sum_{p < parts} ws[p*stride + c].  Block = 32 columns x 32 part-groups: group j adds parts
// j, j+32, ... in order, then the 32 group sums are added in group order: a fixed tree, same bits every run.
constexpr int kRpCols = 32, kRpGroups = 32;
__global__ __launch_bounds__(kRpCols * kRpGroups) void reduce_parts_kernel(const float* __restrict__ ws,
                                                                           float* __restrict__ out, int parts,
                                                                           int64_t stride, int64_t cols, int accumulate) {
  __shared__ float part[kRpGroups][kRpCols + 1];
  const int tx = threadIdx.x % kRpCols, ty = threadIdx.x / kRpCols;
  const int64_t c = (int64_t)blockIdx.x * kRpCols + tx;
  float s = 0.f;
  if (c < cols)
    for (int p = ty; p < parts; p += kRpGroups) s += ws[(size_t)p * stride + c];
  part[ty][tx] = s;
  __syncthreads();
  if (ty == 0 && c < cols) {
    float t = 0.f;
#pragma unroll
    for (int j = 0; j < kRpGroups; ++j) t += part[j][tx];
    out[c] = accumulate ? out[c] + t : t;
  }
}
// Up to three independent reductions in one launch: blockIdx.y picks (ws + y * set_stride) -> out[y].
struct ReduceOuts { float* out[3]; };
__global__ __launch_bounds__(kRpCols * kRpGroups) void reduce_parts_multi_kernel(const float* __restrict__ ws, ReduceOuts o,
                                                                                 int parts, int64_t set_stride,
                                                                                 int64_t cols, int accumulate) {
  __shared__ float part[kRpGroups][kRpCols + 1];
  const int tx = threadIdx.x % kRpCols, ty = threadIdx.x / kRpCols;
  const int64_t c = (int64_t)blockIdx.x * kRpCols + tx;
  const float* src = ws + (size_t)blockIdx.y * set_stride;
  float* out = blockIdx.y == 0 ? o.out[0] : blockIdx.y == 1 ? o.out[1] : o.out[2];
  float s = 0.f;
  if (c < cols)
    for (int p = ty; p < parts; p += kRpGroups) s += src[(size_t)p * cols + c];
  part[ty][tx] = s;
  __syncthreads();
  if (ty == 0 && c < cols) {
    float t = 0.f;
#pragma unroll
    for (int j = 0; j < kRpGroups; ++j) t += part[j][tx];
    out[c] = accumulate ? out[c] + t : t;
  }
}
static inline void launch_reduce_parts(hipStream_t s, const float* ws, float* out, int parts, int64_t stride, int64_t cols,
                                       int accumulate) {
  reduce_parts_kernel<<<(unsigned)((cols + kRpCols - 1) / kRpCols), kRpCols * kRpGroups, 0, s>>>(ws, out, parts, stride, cols, accumulate);
}

hipError_t launch_layernorm_bwd(hipStream_t s, int dtype, const void* dy, const float* x, const float* g,
                                const float* mean, const float* rstd, const float* dres, float* dx, void* dx_lp,
                                float* dg, float* db, float* dsum, float* ws, int N, int d, int accumulate) {
  if (!dy || !x || !g || !mean || !rstd || !dx || !dg || !db || !ws || N < 0 || d <= 0) return hipErrorInvalidValue;
  if (d % 4 || d > kLnThreads * 4 * kLnMaxVec) return hipErrorInvalidValue;
  if (dtype != kF32 && dtype != kBF16) return hipErrorInvalidValue;
  if (((uintptr_t)x | (uintptr_t)g | (uintptr_t)dx | (uintptr_t)ws | (uintptr_t)dres) & 15) return hipErrorInvalidValue;
  const uintptr_t lp_mask = dtype == kBF16 ? 7 : 15;
  if (((uintptr_t)dy | (uintptr_t)dx_lp) & lp_mask) return hipErrorInvalidValue;
  if (dtype == kF32 && dx_lp == (void*)dx) dx_lp = nullptr;   // the fp32 copy is dx itself
  const int want = dsum != nullptr;
  int G = ln_bwd_blocks(N);
  if (N > 0) {
    if (d <= kLnWaveMaxD) {
      const int by_rows = (N + kLnThreads / 64 - 1) / (kLnThreads / 64);
      if (by_rows < G) G = by_rows;
      if (dtype == kF32)
        launch_ln_bwd_wave<float>(s, G, (const float*)dy, x, g, mean, rstd, dres, dx, (float*)dx_lp, ws, N, d, want);
      else
        launch_ln_bwd_wave<bf16>(s, G, (const bf16*)dy, x, g, mean, rstd, dres, dx, (bf16*)dx_lp, ws, N, d, want);
    } else if (dtype == kF32) {
      layernorm_bwd_kernel<float><<<G, kLnThreads, 0, s>>>((const float*)dy, x, g, mean, rstd, dres, dx, (float*)dx_lp, ws, N, d, want);
    } else {
      layernorm_bwd_kernel<bf16><<<G, kLnThreads, 0, s>>>((const bf16*)dy, x, g, mean, rstd, dres, dx, (bf16*)dx_lp, ws, N, d, want);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const int parts = N > 0 ? G : 0;
  ReduceOuts outs{{dg, db, dsum}};
  reduce_parts_multi_kernel<<<dim3((unsigned)((d + kRpCols - 1) / kRpCols), want ? 3 : 2), kRpCols * kRpGroups, 0, s>>>(
      ws, outs, parts, (int64_t)G * d, d, accumulate);
  return hipGetLastError();
}

// ---- LayerNorm backward for callers that cannot allocate ----------------------------------------------
// The same kernels with the block sums in a fixed array of the code object instead of a caller workspace.  Each GPU
// that loads the library holds its own copy of the array, at its own address, until the process ends.  In host code
// the array's name is only a handle for hipGetSymbolAddress: the address the kernels get is the one looked up below,
// once per device with that device current.
constexpr int64_t kLnScratchFloats = 3LL * kLnBwdMaxBlocks * kLnWaveMaxD;   // 3 x 512 x 2048 floats = 12 MiB
static __device__ __align__(256) float scratch[kLnScratchFloats];

constexpr int kMaxDevices = 64;
static float* g_scratch_ptr[kMaxDevices] = {nullptr};

int64_t layernorm_bwd_static_max_ws_floats() { return kLnScratchFloats; }

hipError_t layernorm_bwd_static_init(int device) {
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  if (g_scratch_ptr[device]) return hipSuccess;
  int cur = -1;
  hipError_t e = hipGetDevice(&cur);
  if (e != hipSuccess) return e;
  if (cur != device) return hipErrorInvalidDevice;   // the lookup below answers for the current device
  float* p = nullptr;
  e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
  if (e != hipSuccess) return e;
  if (!p) return hipErrorInvalidSymbol;
  g_scratch_ptr[device] = p;
  return hipSuccess;
}

hipError_t launch_layernorm_bwd_static(hipStream_t s, int device, int dtype, const void* dy, const float* x, const float* g,
                                       const float* mean, const float* rstd, const float* dres, float* dx, void* dx_lp,
                                       float* dg, float* db, float* dsum, int N, int d, int accumulate) {
  if (device < 0 || device >= kMaxDevices || !g_scratch_ptr[device]) return hipErrorNotInitialized;
  if (N < 0 || d <= 0) return hipErrorInvalidValue;
  if (layernorm_bwd_ws_floats(N, d) > kLnScratchFloats) return hipErrorNotSupported;
  // Every block of the first kernel overwrites its slots of the array and the second kernel reads exactly those
  // slots, so nothing has to be cleared between calls; two calls in flight at once on one GPU would share the slots.
  return launch_layernorm_bwd(s, dtype, dy, x, g, mean, rstd, dres, dx, dx_lp, dg, db, dsum, g_scratch_ptr[device], N, d,
                              accumulate);
}

// ---- column sums --------------------------------------------------------------------------------
// Grid (column blocks, row slabs).  Each thread owns kVec adjacent columns and walks its slab's rows;
// partial sums land in ws[slab][cols]; reduce_parts_kernel adds the slabs in order.
constexpr int kCsThreads = 256;
static inline int colsum_slabs(int64_t rows) {
  int64_t s = (rows + 31) / 32;   // at least 32 rows per slab
  if (s > 256) s = 256;
  if (s < 1) s = 1;
  return (int)s;
}
int64_t colsum_ws_floats(int64_t rows, int64_t cols) { return (int64_t)colsum_slabs(rows) * cols; }

template <class T>
__global__ __launch_bounds__(kCsThreads) void colsum_kernel(const T* __restrict__ in, float* __restrict__ ws,
                                                            int64_t rows, int64_t cols) {
  const int64_t c0 = ((int64_t)blockIdx.x * kCsThreads + threadIdx.x) * 4;
  if (c0 >= cols) return;
  const int slabs = gridDim.y;
  const int64_t per = (rows + slabs - 1) / slabs;
  const int64_t r0 = (int64_t)blockIdx.y * per;
  const int64_t r1 = r0 + per < rows ? r0 + per : rows;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int64_t r = r0; r < r1; ++r) {
    const float4 v = load4<T>(in + (size_t)r * cols + c0);
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  *reinterpret_cast<float4*>(ws + (size_t)blockIdx.y * cols + c0) = acc;
}

hipError_t launch_colsum(hipStream_t s, int dtype, const void* in, float* out, float* ws, int64_t rows, int64_t cols,
                         int accumulate) {
  if (!in || !out || !ws || rows < 0 || cols <= 0 || cols % 4) return hipErrorInvalidValue;
  if (((uintptr_t)ws & 15) || ((uintptr_t)in & (dtype == kBF16 ? 7 : 15))) return hipErrorInvalidValue;
  const int slabs = colsum_slabs(rows);
  if (rows > 0) {
    dim3 grid((unsigned)((cols / 4 + kCsThreads - 1) / kCsThreads), (unsigned)slabs);
    if (dtype == kF32)
      colsum_kernel<float><<<grid, kCsThreads, 0, s>>>((const float*)in, ws, rows, cols);
    else if (dtype == kBF16)
      colsum_kernel<bf16><<<grid, kCsThreads, 0, s>>>((const bf16*)in, ws, rows, cols);
    else
      return hipErrorInvalidValue;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  launch_reduce_parts(s, ws, out, rows > 0 ? slabs : 0, cols, cols, accumulate);
  return hipGetLastError();
}

}  // namespace pw
