// LayerNorm forward / backward and column sums (bias gradients).  HBM-bound: every row is read once
// from memory with 16-byte accesses, held in registers, and reduced with wave64 shuffles.
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

hipError_t launch_layernorm_fwd(hipStream_t s, int dtype, const float* x, const float* g, const float* b, void* y,
                                float* mean, float* rstd, int N, int d) {
  if (!x || !g || !b || !y || !mean || !rstd || N < 0 || d <= 0) return hipErrorInvalidValue;
  if (d % 4 || d > kLnThreads * 4 * kLnMaxVec) return hipErrorInvalidValue;
  if (((uintptr_t)x | (uintptr_t)g | (uintptr_t)b) & 15) return hipErrorInvalidValue;
  if ((uintptr_t)y & (dtype == kBF16 ? 7 : 15)) return hipErrorInvalidValue;
  if (N == 0) return hipSuccess;
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
// Block b handles rows b, b+G, ...; per row two block sums give mean(gg) and mean(gg xh); each thread
// keeps running sums of dy*xh and dy for the columns it owns and writes them to ws[b] at the end.  A
// second kernel adds the G partial rows in index order, so results are the same bits on every run.
constexpr int kLnBwdMaxBlocks = 512;

static inline int ln_bwd_blocks(int N) { return N < kLnBwdMaxBlocks ? (N < 1 ? 1 : N) : kLnBwdMaxBlocks; }
int64_t layernorm_bwd_ws_floats(int N, int d) { return 2LL * ln_bwd_blocks(N) * d; }

template <class T>
__global__ __launch_bounds__(kLnThreads) void layernorm_bwd_kernel(const T* __restrict__ dy, const float* __restrict__ x,
                                                                   const float* __restrict__ g,
                                                                   const float* __restrict__ mean,
                                                                   const float* __restrict__ rstd,
                                                                   const float* __restrict__ dres, float* __restrict__ dx,
                                                                   T* __restrict__ dx_lp, float* __restrict__ ws, int N,
                                                                   int d) {
  __shared__ float red[kLnThreads / 64];
  const int d4 = d >> 2;
  float4 accg[kLnMaxVec], accb[kLnMaxVec], gv[kLnMaxVec];
#pragma unroll
  for (int i = 0; i < kLnMaxVec; ++i) {
    accg[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    accb[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    const int c4 = threadIdx.x + i * kLnThreads;
    gv[i] = c4 < d4 ? reinterpret_cast<const float4*>(g)[c4] : make_float4(0.f, 0.f, 0.f, 0.f);
  }
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
        xh[i] = make_float4((xv.x - mu) * rs, (xv.y - mu) * rs, (xv.z - mu) * rs, (xv.w - mu) * rs);
        gg[i] = make_float4(dv.x * gv[i].x, dv.y * gv[i].y, dv.z * gv[i].z, dv.w * gv[i].w);
        s1 += (gg[i].x + gg[i].y) + (gg[i].z + gg[i].w);
        s2 += (gg[i].x * xh[i].x + gg[i].y * xh[i].y) + (gg[i].z * xh[i].z + gg[i].w * xh[i].w);
        accg[i].x += dv.x * xh[i].x; accg[i].y += dv.y * xh[i].y; accg[i].z += dv.z * xh[i].z; accg[i].w += dv.w * xh[i].w;
        accb[i].x += dv.x; accb[i].y += dv.y; accb[i].z += dv.z; accb[i].w += dv.w;
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
        if (dres) {
          const float4 r = reinterpret_cast<const float4*>(dres + (size_t)n * d)[c4];
          o.x += r.x; o.y += r.y; o.z += r.z; o.w += r.w;
        }
        reinterpret_cast<float4*>(dx + (size_t)n * d)[c4] = o;
        if (dx_lp) store4<T>(dx_lp + (size_t)n * d + 4 * c4, o.x, o.y, o.z, o.w);
      }
    }
  }
  float* wg = ws + (size_t)blockIdx.x * d;
  float* wb = ws + (size_t)(gridDim.x + blockIdx.x) * d;
#pragma unroll
  for (int i = 0; i < kLnMaxVec; ++i) {
    const int c4 = threadIdx.x + i * kLnThreads;
    if (c4 < d4) {
      reinterpret_cast<float4*>(wg)[c4] = accg[i];
      reinterpret_cast<float4*>(wb)[c4] = accb[i];
    }
  }
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
static inline void launch_reduce_parts(hipStream_t s, const float* ws, float* out, int parts, int64_t stride, int64_t cols,
                                       int accumulate) {
  reduce_parts_kernel<<<(unsigned)((cols + kRpCols - 1) / kRpCols), kRpCols * kRpGroups, 0, s>>>(ws, out, parts, stride, cols, accumulate);
}

hipError_t launch_layernorm_bwd(hipStream_t s, int dtype, const void* dy, const float* x, const float* g,
                                const float* mean, const float* rstd, const float* dres, float* dx, void* dx_lp,
                                float* dg, float* db, float* ws, int N, int d, int accumulate) {
  if (!dy || !x || !g || !mean || !rstd || !dx || !dg || !db || !ws || N < 0 || d <= 0) return hipErrorInvalidValue;
  if (d % 4 || d > kLnThreads * 4 * kLnMaxVec) return hipErrorInvalidValue;
  if (((uintptr_t)x | (uintptr_t)g | (uintptr_t)dx | (uintptr_t)ws | (uintptr_t)dres) & 15) return hipErrorInvalidValue;
  const uintptr_t lp_mask = dtype == kBF16 ? 7 : 15;
  if (((uintptr_t)dy | (uintptr_t)dx_lp) & lp_mask) return hipErrorInvalidValue;
  if (dtype == kF32 && dx_lp == (void*)dx) dx_lp = nullptr;   // the fp32 copy is dx itself
  const int G = ln_bwd_blocks(N);
  if (N > 0) {
    if (dtype == kF32)
      layernorm_bwd_kernel<float><<<G, kLnThreads, 0, s>>>((const float*)dy, x, g, mean, rstd, dres, dx, (float*)dx_lp, ws, N, d);
    else if (dtype == kBF16)
      layernorm_bwd_kernel<bf16><<<G, kLnThreads, 0, s>>>((const bf16*)dy, x, g, mean, rstd, dres, dx, (bf16*)dx_lp, ws, N, d);
    else
      return hipErrorInvalidValue;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const int parts = N > 0 ? G : 0;
  launch_reduce_parts(s, ws, dg, parts, d, d, accumulate);
  launch_reduce_parts(s, ws + (size_t)G * d, db, parts, d, d, accumulate);
  return hipGetLastError();
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
