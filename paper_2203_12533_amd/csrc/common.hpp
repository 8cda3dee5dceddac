// Shared device helpers for the gfx950 kernels: bf16 storage type, wave64 reductions, vector types.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pw {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kWave = 64;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return (float)v; }
template <class T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }   // v_cvt_pk_bf16_f32: RNE

// Sum / max over the 64 lanes of a wave; every lane gets the result.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Block-wide sum in a fixed order (lane tree, then waves in index order): same bits every run.
// `red` is shared scratch of at least blockDim.x/64 floats.  All threads must call.
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += red[i];
  return t;
}
__device__ __forceinline__ float block_max(float v, float* red) {
  v = wave_max(v);
  const int w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float t = red[0];
  for (int i = 1; i < nw; ++i) t = fmaxf(t, red[i]);
  return t;
}

// tanh-form GELU and its derivative, fp32, written through the logistic function: with z = c (u + 0.044715 u^3),
// 0.5 (1 + tanh z) = s = 1 / (1 + exp(-2z)), so gelu(u) = u s and gelu'(u) = s + u s (1 - s) 2 dz/du.  Six plain
// operations and two transcendentals for gelu, three more operations for the derivative on top.
struct GeluSig { float s, dz2; };   // s as above; dz2 = 2 dz/du = 2c (1 + 3 * 0.044715 u^2)
__device__ __forceinline__ GeluSig gelu_sigmoid(float u) {
  constexpr float c2 = 2.f * 0.7978845608028654f;            // 2 sqrt(2/pi)
  constexpr float ka = -c2 * 1.4426950408889634f;            // exp(-2z) = exp2(u (ka + kb u^2))
  constexpr float kb = ka * 0.044715f;
  const float u2 = u * u;
  const float e = __builtin_amdgcn_exp2f(u * __builtin_fmaf(kb, u2, ka));
  return {__builtin_amdgcn_rcpf(1.f + e), __builtin_fmaf(c2 * 3.f * 0.044715f, u2, c2)};
}
__device__ __forceinline__ float gelu_f(float u) { return u * gelu_sigmoid(u).s; }
__device__ __forceinline__ float gelu_grad_f(float u) {
  const GeluSig g = gelu_sigmoid(u);
  const float h = u * g.s;
  return __builtin_fmaf(__builtin_fmaf(-h, g.s, h), g.dz2, g.s);
}

// One Adam update with bias corrections inv_c1 = 1 / (1 - beta1^t), inv_c2 = 1 / (1 - beta2^t).
__device__ __forceinline__ void adam_one(float& w, float& m, float& v, float g, float lr, float b1, float b2,
                                         float eps, float inv_c1, float inv_c2) {
  m = b1 * m + (1.f - b1) * g;
  v = b2 * v + (1.f - b2) * g * g;
  w -= lr * (m * inv_c1) / (sqrtf(v * inv_c2) + eps);
}

}  // namespace pw
