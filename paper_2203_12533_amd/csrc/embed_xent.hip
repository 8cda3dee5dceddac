// Embedding lookup (forward, backward) and fused softmax cross-entropy.  HBM-bound kernels.
#include "common.hpp"
#include "kernels.hpp"

namespace pw {

// Token id of flat position p = b*T + t in a token array whose rows are `stride` ids apart (T+1 for the
// [B, T+1] arrays that carry inputs and next-token targets together), clamped into [0, V) so that a bad id
// can never index outside the tables (forward and backward clamp identically).
__device__ __forceinline__ int token_at(const int32_t* __restrict__ tokens, int p, int T, int stride, int V, int shift = 0) {
  const int b = p / T, t = p - b * T;
  const int id = tokens[(size_t)b * stride + t + shift];
  return id < 0 ? 0 : (id >= V ? V - 1 : id);
}

// ---- embedding forward: x[b*T+t,:] = wte[tok[b,t],:] + wpe[t,:] (one fp32 add per element: exact) ----
__global__ void embedding_fwd_kernel(const int32_t* __restrict__ tokens, const float* __restrict__ wte,
                                     const float* __restrict__ wpe, float* __restrict__ x, int B, int T, int d, int V,
                                     int stride) {
  const int n = blockIdx.x;
  const int t = n % T;
  const int id = token_at(tokens, n, T, stride, V);
  const float4* we = reinterpret_cast<const float4*>(wte + (size_t)id * d);
  const float4* pe = reinterpret_cast<const float4*>(wpe + (size_t)t * d);
  float4* xo = reinterpret_cast<float4*>(x + (size_t)n * d);
  for (int c = threadIdx.x; c < (d >> 2); c += blockDim.x) {
    const float4 a = we[c], p = pe[c];
    xo[c] = make_float4(a.x + p.x, a.y + p.y, a.z + p.z, a.w + p.w);
  }
}

hipError_t launch_embedding_fwd(hipStream_t s, const int32_t* tokens, const float* wte, const float* wpe, float* x,
                                int B, int T, int d, int V, int tok_stride) {
  const int stride = tok_stride > 0 ? tok_stride : T + 1;
  if (stride < T) return hipErrorInvalidValue;
  if (!tokens || !wte || !wpe || !x || B < 0 || T <= 0 || d <= 0 || d % 4 || V <= 0) return hipErrorInvalidValue;
  if (((uintptr_t)wte | (uintptr_t)wpe | (uintptr_t)x) & 15) return hipErrorInvalidValue;
  if (B == 0) return hipSuccess;
  embedding_fwd_kernel<<<B * T, 256, 0, s>>>(tokens, wte, wpe, x, B, T, d, V, stride);
  return hipGetLastError();
}

// ---- embedding backward -------------------------------------------------------------------------------
// dwte is a scatter-add with repeated ids.  To get the same bits on every run without atomics, the
// block of position n first looks for an earlier position with the same id: if there is one it has
// nothing to do.  Otherwise it owns that id: it lists every position holding the id in ascending order
// and adds their dx rows in that order.  Rows of ids that never occur are zeroed by a fill beforehand.
constexpr int kEbThreads = 256;
constexpr int kEbList = 2048;

__global__ __launch_bounds__(kEbThreads) void embedding_bwd_wte_kernel(const int32_t* __restrict__ tokens,
                                                                       const float* __restrict__ dx,
                                                                       float* __restrict__ dwte, int B, int T, int d, int V,
                                                                       int stride) {
  __shared__ int list[kEbList];
  __shared__ int wave_cnt[kEbThreads / 64];
  __shared__ int s_found_earlier;
  const int N = B * T;
  const int n = blockIdx.x;
  const int my = token_at(tokens, n, T, stride, V);
  if (threadIdx.x == 0) s_found_earlier = 0;
  __syncthreads();
  int found = 0;
  for (int p = threadIdx.x; p < n; p += kEbThreads)
    if (token_at(tokens, p, T, stride, V) == my) found = 1;
  if (found) s_found_earlier = 1;   // benign race: every writer stores 1
  __syncthreads();
  if (s_found_earlier) return;

  const int d4 = d >> 2;
  constexpr int kMaxVec = 8;        // d <= 256*4*8
  float4 acc[kMaxVec];
#pragma unroll
  for (int i = 0; i < kMaxVec; ++i) acc[i] = make_float4(0.f, 0.f, 0.f, 0.f);

  int start = n;
  while (start < N) {
    // fill the list with matching positions in [start, N), ascending, until it is full
    int count = 0;
    int next_start = N;
    for (int base = start; base < N; base += kEbThreads) {
      const int p = base + threadIdx.x;
      const bool hit = p < N && token_at(tokens, p, T, stride, V) == my;
      const uint64_t mask = __ballot(hit);
      const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
      if (lane == 0) wave_cnt[w] = __popcll(mask);
      __syncthreads();
      int before = 0, total = 0;
      for (int i = 0; i < kEbThreads / 64; ++i) {
        if (i < w) before += wave_cnt[i];
        total += wave_cnt[i];
      }
      if (count + total > kEbList) {   // would overflow: stop before this chunk (uniform decision)
        next_start = base;
        __syncthreads();
        break;
      }
      if (hit) list[count + before + __popcll(mask & ((1ull << lane) - 1))] = p;
      count += total;
      __syncthreads();
    }
    // add the rows in list order
    for (int k = 0; k < count; ++k) {
      const float* row = dx + (size_t)list[k] * d;
#pragma unroll
      for (int i = 0; i < kMaxVec; ++i) {
        const int c4 = threadIdx.x + i * kEbThreads;
        if (c4 < d4) {
          const float4 v = reinterpret_cast<const float4*>(row)[c4];
          acc[i].x += v.x; acc[i].y += v.y; acc[i].z += v.z; acc[i].w += v.w;
        }
      }
    }
    __syncthreads();
    start = next_start;
  }
#pragma unroll
  for (int i = 0; i < kMaxVec; ++i) {
    const int c4 = threadIdx.x + i * kEbThreads;
    if (c4 < d4) reinterpret_cast<float4*>(dwte + (size_t)my * d)[c4] = acc[i];
  }
}

__global__ void embedding_bwd_wpe_kernel(const float* __restrict__ dx, float* __restrict__ dwpe, int B, int T, int d) {
  const int t = blockIdx.x;
  for (int c = threadIdx.x; c < (d >> 2); c += blockDim.x) {
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int b = 0; b < B; ++b) {
      const float4 v = reinterpret_cast<const float4*>(dx + ((size_t)b * T + t) * d)[c];
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    reinterpret_cast<float4*>(dwpe + (size_t)t * d)[c] = acc;
  }
}

hipError_t launch_embedding_bwd(hipStream_t s, const int32_t* tokens, const float* dx, float* dwte, float* dwpe,
                                int B, int T, int d, int V, int tok_stride) {
  const int stride = tok_stride > 0 ? tok_stride : T + 1;
  if (stride < T) return hipErrorInvalidValue;
  if (!tokens || !dx || !dwte || !dwpe || B < 0 || T <= 0 || d <= 0 || d % 4 || d > kEbThreads * 4 * 8 || V <= 0)
    return hipErrorInvalidValue;
  if (((uintptr_t)dx | (uintptr_t)dwte | (uintptr_t)dwpe) & 15) return hipErrorInvalidValue;
  hipError_t e = launch_fill_f32(s, dwte, (int64_t)V * d, 0.f);
  if (e != hipSuccess) return e;
  if (B == 0) return launch_fill_f32(s, dwpe, (int64_t)T * d, 0.f);
  embedding_bwd_wte_kernel<<<B * T, kEbThreads, 0, s>>>(tokens, dx, dwte, B, T, d, V, stride);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  embedding_bwd_wpe_kernel<<<T, 256, 0, s>>>(dx, dwpe, B, T, d);
  return hipGetLastError();
}

// ---- softmax cross-entropy ----------------------------------------------------------------------------
// One block per row of logits.  Pass 1 keeps a running (max, sum of exp) per thread and merges them
// across the block; pass 2 re-reads the row (it is still in L2: 64 KiB at V = 32768) and overwrites it
// with (softmax - onehot)/N.  Row losses are added in index order by a one-block kernel.
constexpr int kXeThreads = 512;

template <class T> struct Vec8;
template <> struct Vec8<bf16> {
  static constexpr int n = 8;
  static __device__ __forceinline__ void load(const bf16* p, float* o) {
    const bf16x8 v = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (float)v[i];
  }
  static __device__ __forceinline__ void store(bf16* p, const float* o) {
    bf16x8 v;
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (bf16)o[i];
    *reinterpret_cast<bf16x8*>(p) = v;
  }
};
template <> struct Vec8<float> {
  static constexpr int n = 4;
  static __device__ __forceinline__ void load(const float* p, float* o) {
    const float4 v = *reinterpret_cast<const float4*>(p);
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
  }
  static __device__ __forceinline__ void store(float* p, const float* o) {
    *reinterpret_cast<float4*>(p) = make_float4(o[0], o[1], o[2], o[3]);
  }
};

template <class T>
__global__ __launch_bounds__(kXeThreads) void softmax_xent_kernel(T* __restrict__ z, const int32_t* __restrict__ tokens,
                                                                  float* __restrict__ row_loss, int T_, int V, float inv_n) {
  __shared__ float red[kXeThreads / 64];
  constexpr int W = Vec8<T>::n;
  const int n = blockIdx.x;
  const int tgt = token_at(tokens, n, T_, T_ + 1, V, 1);
  T* zr = z + (size_t)n * V;
  float m = -INFINITY, l = 0.f;
  for (int c = threadIdx.x * W; c < V; c += kXeThreads * W) {
    float v[W];
    Vec8<T>::load(zr + c, v);
    float cm = v[0];
#pragma unroll
    for (int i = 1; i < W; ++i) cm = fmaxf(cm, v[i]);
    const float nm = fmaxf(m, cm);
    float add = 0.f;
#pragma unroll
    for (int i = 0; i < W; ++i) add += __expf(v[i] - nm);
    l = l * __expf(m - nm) + add;
    m = nm;
  }
  const float gm = block_max(m, red);
  const float gl = block_sum(l * __expf(m - gm), red);   // threads with no column have l = 0, m = -inf: exp(-inf) = 0
  const float lse = gm + logf(gl);
  if (threadIdx.x == 0) row_loss[n] = lse - to_f32(zr[tgt]);
  __syncthreads();   // zr[tgt] was read before anyone overwrites the row
  for (int c = threadIdx.x * W; c < V; c += kXeThreads * W) {
    float v[W];
    Vec8<T>::load(zr + c, v);
#pragma unroll
    for (int i = 0; i < W; ++i) v[i] = (__expf(v[i] - lse) - (c + i == tgt ? 1.f : 0.f)) * inv_n;
    Vec8<T>::store(zr + c, v);
  }
}

__global__ void mean_rows_kernel(const float* __restrict__ row_loss, float* __restrict__ loss, int N) {
  __shared__ float part[256];
  // thread i adds rows i, i+256, ... in order; then thread 0 adds the 256 partials in order
  float s = 0.f;
  for (int n = threadIdx.x; n < N; n += 256) s += row_loss[n];
  part[threadIdx.x] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    float tot = 0.f;
    for (int i = 0; i < 256; ++i) tot += part[i];
    *loss = tot / (float)N;
  }
}

// Loss from the per-group statistics that the LM-head GEMM's kEpiXentStats epilogue leaves (the logits themselves
// were never stored): one wave per row merges the (max, sum exp(z - max)) pairs of the row's 64-column groups.
__global__ __launch_bounds__(256) void xent_from_stats_kernel(const float* __restrict__ part, const float* __restrict__ zt,
                                                               float* __restrict__ lse, float* __restrict__ row_loss,
                                                               int N, int groups) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= N) return;   // whole waves leave together
  const float2* pr = reinterpret_cast<const float2*>(part) + (size_t)r * groups;
  float m = -INFINITY, l = 0.f;
  for (int g = lane; g < groups; g += 64) {
    const float2 p = pr[g];
    const float nm = fmaxf(m, p.x);
    l = l * __expf(m - nm) + p.y * __expf(p.x - nm);
    m = nm;
  }
  const float gm = wave_max(m);
  const float gl = wave_sum(l * __expf(m - gm));   // lanes without a group: l = 0, exp(-inf) = 0
  if (lane == 0) {
    const float v = gm + logf(gl);
    lse[r] = v;
    row_loss[r] = v - zt[r];
  }
}

hipError_t launch_xent_from_stats(hipStream_t s, const float* part, const float* zt, float* lse, float* row_loss,
                                  float* loss, int N, int groups) {
  if (!part || !zt || !lse || !row_loss || !loss || N <= 0 || groups <= 0 || ((uintptr_t)part & 7)) return hipErrorInvalidValue;
  xent_from_stats_kernel<<<(N + 3) / 4, 256, 0, s>>>(part, zt, lse, row_loss, N, groups);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  mean_rows_kernel<<<1, 256, 0, s>>>(row_loss, loss, N);
  return hipGetLastError();
}

hipError_t launch_softmax_xent(hipStream_t s, int dtype, void* z, const int32_t* tokens, float* loss, float* row_loss,
                               int B, int T, int V) {
  if (!z || !tokens || !loss || !row_loss || B <= 0 || T <= 0 || V <= 0) return hipErrorInvalidValue;
  const int W = dtype == kBF16 ? 8 : 4;
  if (V % W || ((uintptr_t)z & 15)) return hipErrorInvalidValue;
  const int N = B * T;
  if (dtype == kF32)
    softmax_xent_kernel<float><<<N, kXeThreads, 0, s>>>((float*)z, tokens, row_loss, T, V, 1.f / (float)N);
  else if (dtype == kBF16)
    softmax_xent_kernel<bf16><<<N, kXeThreads, 0, s>>>((bf16*)z, tokens, row_loss, T, V, 1.f / (float)N);
  else
    return hipErrorInvalidValue;
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  mean_rows_kernel<<<1, 256, 0, s>>>(row_loss, loss, N);
  return hipGetLastError();
}

}  // namespace pw
