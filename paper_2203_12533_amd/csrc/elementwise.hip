// Elementwise / optimiser / dispatch-support kernels (HBM- or latency-bound; no contraction).
#include "common.hpp"
#include "kernels.hpp"

namespace pw {

// Every kernel here strides over its input, so any grid is correct; one work item per thread (no cap short of the
// launch limit) is what the HBM-bound ones measured fastest with.
static inline int grid_for(int64_t work_items, int block, int max_blocks = 1 << 30) {
  int64_t g = (work_items + block - 1) / block;
  if (g < 1) g = 1;
  if (g > max_blocks) g = max_blocks;
  return (int)g;
}

// ---- trivial compiled functions of the dispatch micro-benchmark -------------------------------------
// kind 1: x + c, 2: x * c, 3: x / c, 4: x + c after a bounded spin of busy_ticks (100 MHz wall clock),
// 5: kind 4 applied `reps` times in a row inside one launch (a chain of computations fused into one node).
// done (optional, one-block launches only): a word in pinned host memory that receives `token` once every element has
// been written - a completion signal the host can poll without going through the stream's end-of-kernel event.
__global__ void scalar_fn_kernel(int kind, const float* __restrict__ x, float* __restrict__ y, int64_t n, float c,
                                 uint64_t busy_ticks, int reps, uint32_t* done, uint32_t token) {
  if (kind < 5) {
    if (kind == 4 && busy_ticks) {
      const uint64_t t0 = wall_clock64();
      while (wall_clock64() - t0 < busy_ticks) __builtin_amdgcn_s_sleep(8);
    }
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
      const float v = x[i];
      y[i] = kind == 2 ? v * c : kind == 3 ? v / c : v + c;
    }
  } else {
    // Every thread owns its elements through all repetitions, so no synchronisation is needed between them; each
    // repetition is one fp32 addition rounded to nearest, exactly as in a chain of separate functions.
    for (int r = 0; r < reps; ++r) {
      if (busy_ticks) {
        const uint64_t t0 = wall_clock64();
        while (wall_clock64() - t0 < busy_ticks) __builtin_amdgcn_s_sleep(8);
      }
      for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const float v = r == 0 ? x[i] : y[i];
        y[i] = __fadd_rn(v, c);
      }
    }
  }
  if (done) {   // uniform over the (single) block
    __threadfence_system();
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_store(done, token, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
  }
}

static inline int scalar_fn_block(int64_t n) { return n <= 128 ? 128 : 256; }
bool scalar_fn_one_block(int64_t n) { return n > 0 && grid_for(n, scalar_fn_block(n)) == 1; }

hipError_t launch_scalar_fn(hipStream_t s, int kind, const float* x, float* y, int64_t n, float c, float busy_us, int reps,
                            uint32_t* done, uint32_t token) {
  if (kind < 1 || kind > 5 || !x || !y || n < 0 || reps < 1 || reps > 65536) return hipErrorInvalidValue;
  if (busy_us < 0.f || busy_us > 1e6f) return hipErrorInvalidValue;   // at most one second of spin per repetition
  if ((double)busy_us * reps > 1e7) return hipErrorInvalidValue;       // and ten seconds per launch
  if (done && !scalar_fn_one_block(n)) return hipErrorInvalidValue;   // one block signals; several would need a count
  if (n == 0) return hipSuccess;
  const int block = scalar_fn_block(n);
  scalar_fn_kernel<<<grid_for(n, block), block, 0, s>>>(kind, x, y, n, c, (uint64_t)(busy_us * 100.f), reps, done, token);
  return hipGetLastError();
}

// y = a + b, the two-input node of dataflow programs with fan-in.
__global__ void add2_kernel(const float* __restrict__ a, const float* __restrict__ b, float* __restrict__ y, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    y[i] = __fadd_rn(a[i], b[i]);
}
hipError_t launch_add2(hipStream_t s, const float* a, const float* b, float* y, int64_t n) {
  if (!a || !b || !y || n < 0) return hipErrorInvalidValue;
  if (n == 0) return hipSuccess;
  const int block = n <= 128 ? 128 : 256;
  add2_kernel<<<grid_for(n, block), block, 0, s>>>(a, b, y, n);
  return hipGetLastError();
}

// ---- fills, conversions, copies -----------------------------------------------------------------------
__global__ void fill_f32_kernel(float* __restrict__ p, int64_t n, float v) {
  const int64_t n4 = n >> 2;
  float4* p4 = reinterpret_cast<float4*>(p);
  const float4 v4 = make_float4(v, v, v, v);
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (int64_t)gridDim.x * blockDim.x) p4[i] = v4;
  for (int64_t i = (n4 << 2) + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}
hipError_t launch_fill_f32(hipStream_t s, float* p, int64_t n, float v) {
  if (!p || n < 0 || ((uintptr_t)p & 15)) return hipErrorInvalidValue;
  if (n == 0) return hipSuccess;
  fill_f32_kernel<<<grid_for((n + 3) / 4, 256), 256, 0, s>>>(p, n, v);
  return hipGetLastError();
}

__global__ void f32_to_bf16_kernel(const float* __restrict__ src, bf16* __restrict__ dst, int64_t n) {
  const int64_t n4 = n >> 2;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (int64_t)gridDim.x * blockDim.x) {
    const float4 v = reinterpret_cast<const float4*>(src)[i];
    bf16x4 o = {(bf16)v.x, (bf16)v.y, (bf16)v.z, (bf16)v.w};
    reinterpret_cast<bf16x4*>(dst)[i] = o;
  }
  for (int64_t i = (n4 << 2) + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    dst[i] = (bf16)src[i];
}
hipError_t launch_f32_to_bf16(hipStream_t s, const float* src, void* dst, int64_t n) {
  if (!src || !dst || n < 0 || ((uintptr_t)src & 15) || ((uintptr_t)dst & 7)) return hipErrorInvalidValue;
  if (n == 0) return hipSuccess;
  f32_to_bf16_kernel<<<grid_for((n + 3) / 4, 256), 256, 0, s>>>(src, (bf16*)dst, n);
  return hipGetLastError();
}

__global__ void bf16_to_f32_kernel(const bf16* __restrict__ src, float* __restrict__ dst, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    dst[i] = (float)src[i];
}
hipError_t launch_bf16_to_f32(hipStream_t s, const void* src, float* dst, int64_t n) {
  if (!src || !dst || n < 0) return hipErrorInvalidValue;
  if (n == 0) return hipSuccess;
  bf16_to_f32_kernel<<<grid_for(n, 256), 256, 0, s>>>((const bf16*)src, dst, n);
  return hipGetLastError();
}

__global__ void copy_bytes_kernel(const uint8_t* __restrict__ src, uint8_t* __restrict__ dst, int64_t bytes) {
  const int64_t n16 = bytes >> 4;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (int64_t)gridDim.x * blockDim.x)
    reinterpret_cast<uint4*>(dst)[i] = reinterpret_cast<const uint4*>(src)[i];
  for (int64_t i = (n16 << 4) + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < bytes; i += (int64_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}
hipError_t launch_copy_bytes(hipStream_t s, const void* src, void* dst, int64_t bytes) {
  if (!src || !dst || bytes < 0 || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return hipErrorInvalidValue;
  if (bytes == 0) return hipSuccess;
  copy_bytes_kernel<<<grid_for((bytes + 15) / 16, 256), 256, 0, s>>>((const uint8_t*)src, (uint8_t*)dst, bytes);
  return hipGetLastError();
}

// ---- gate: device-side wait on a host-resolved future -----------------------------------------------
// One lane polls a word in pinned host memory.  The wait is bounded: after timeout_ticks the kernel
// gives up and raises *poison, so the grid always drains even if the host never resolves.
__global__ void gate_kernel(const uint32_t* flag, uint32_t* poison, uint64_t timeout_ticks) {
  if (threadIdx.x != 0) return;
  const uint64_t t0 = wall_clock64();
  uint32_t v = 0;
  for (;;) {
    v = __hip_atomic_load(flag, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_SYSTEM);
    if (v != 0) break;
    if (wall_clock64() - t0 >= timeout_ticks) break;
    __builtin_amdgcn_s_sleep(32);
  }
  if (v != 1) __hip_atomic_store(poison, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}
hipError_t launch_gate(hipStream_t s, const uint32_t* flag, uint32_t* poison, uint64_t timeout_ticks) {
  if (!flag || !poison || timeout_ticks == 0) return hipErrorInvalidValue;
  gate_kernel<<<1, 64, 0, s>>>(flag, poison, timeout_ticks);
  return hipGetLastError();
}

// ---- optimisers -------------------------------------------------------------------------------------
__global__ void sgd_kernel(float* __restrict__ w, const float* __restrict__ g, int64_t n, float lr) {
  const int64_t n4 = n >> 2;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (int64_t)gridDim.x * blockDim.x) {
    float4 wv = reinterpret_cast<float4*>(w)[i];
    const float4 gv = reinterpret_cast<const float4*>(g)[i];
    wv.x -= lr * gv.x; wv.y -= lr * gv.y; wv.z -= lr * gv.z; wv.w -= lr * gv.w;
    reinterpret_cast<float4*>(w)[i] = wv;
  }
  for (int64_t i = (n4 << 2) + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    w[i] -= lr * g[i];
}
hipError_t launch_sgd(hipStream_t s, float* w, const float* g, int64_t n, float lr) {
  if (!w || !g || n < 0 || ((uintptr_t)w & 15) || ((uintptr_t)g & 15)) return hipErrorInvalidValue;
  if (n == 0) return hipSuccess;
  sgd_kernel<<<grid_for((n + 3) / 4, 256), 256, 0, s>>>(w, g, n, lr);
  return hipGetLastError();
}

// Adam over a flat fp32 arena: 16 B read of g, w, m, v and 16 B write of w, m, v per 4 elements, plus the
// bf16 compute copy (8 B): 30 B per parameter, all fully coalesced.  The step number comes from t_dev
// when non-null (so that a captured graph can be replayed across steps), else from t.
__global__ void adam_kernel(float* __restrict__ w, float* __restrict__ m, float* __restrict__ v,
                            const float* __restrict__ g, bf16* __restrict__ wlp, int64_t n, float lr, float b1,
                            float b2, float eps, int t, const int* __restrict__ t_dev) {
  const int step = t_dev ? *t_dev : t;
  const float inv_c1 = 1.f / (1.f - powf(b1, (float)step));
  const float inv_c2 = 1.f / (1.f - powf(b2, (float)step));
  const int64_t n4 = n >> 2;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (int64_t)gridDim.x * blockDim.x) {
    float4 wv = reinterpret_cast<float4*>(w)[i];
    float4 mv = reinterpret_cast<float4*>(m)[i];
    float4 vv = reinterpret_cast<float4*>(v)[i];
    const float4 gv = reinterpret_cast<const float4*>(g)[i];
    adam_one(wv.x, mv.x, vv.x, gv.x, lr, b1, b2, eps, inv_c1, inv_c2);
    adam_one(wv.y, mv.y, vv.y, gv.y, lr, b1, b2, eps, inv_c1, inv_c2);
    adam_one(wv.z, mv.z, vv.z, gv.z, lr, b1, b2, eps, inv_c1, inv_c2);
    adam_one(wv.w, mv.w, vv.w, gv.w, lr, b1, b2, eps, inv_c1, inv_c2);
    reinterpret_cast<float4*>(w)[i] = wv;
    reinterpret_cast<float4*>(m)[i] = mv;
    reinterpret_cast<float4*>(v)[i] = vv;
    if (wlp) {
      bf16x4 o = {(bf16)wv.x, (bf16)wv.y, (bf16)wv.z, (bf16)wv.w};
      reinterpret_cast<bf16x4*>(wlp)[i] = o;
    }
  }
  for (int64_t i = (n4 << 2) + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
    float wv = w[i], mv = m[i], vv = v[i];
    adam_one(wv, mv, vv, g[i], lr, b1, b2, eps, inv_c1, inv_c2);
    w[i] = wv; m[i] = mv; v[i] = vv;
    if (wlp) wlp[i] = (bf16)wv;
  }
}
hipError_t launch_adam(hipStream_t s, float* w, float* m, float* v, const float* g, void* w_bf16, int64_t n,
                       float lr, float b1, float b2, float eps, int t, const int* t_dev) {
  if (!w || !m || !v || !g || n < 0 || (!t_dev && t < 1)) return hipErrorInvalidValue;
  if (((uintptr_t)w | (uintptr_t)m | (uintptr_t)v | (uintptr_t)g) & 15) return hipErrorInvalidValue;
  if (w_bf16 && ((uintptr_t)w_bf16 & 7)) return hipErrorInvalidValue;
  if (n == 0) return hipSuccess;
  // One float4 per thread and as many workgroups as that takes: measured 13 % faster on 740 M parameters
  // (5.5 TB/s) than a grid of 8192 workgroups striding through the arrays.
  adam_kernel<<<grid_for((n + 3) / 4, 256), 256, 0, s>>>(w, m, v, g, (bf16*)w_bf16, n, lr, b1, b2, eps, t, t_dev);
  return hipGetLastError();
}

__global__ void increment_kernel(int* c) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *c += 1;
}
hipError_t launch_increment(hipStream_t s, int* counter) {
  if (!counter) return hipErrorInvalidValue;
  increment_kernel<<<1, 64, 0, s>>>(counter);
  return hipGetLastError();
}

__global__ void adam_step_kernel(int* state, int set_to, float b1, float b2) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  const int t = set_to > 0 ? set_to : state[0] + 1;
  state[0] = t;
  float* c = reinterpret_cast<float*>(state);
  c[4] = 1.f / (1.f - powf(b1, (float)t));     // the expressions of adam_kernel: same bits
  c[5] = 1.f / (1.f - powf(b2, (float)t));
}
hipError_t launch_adam_step(hipStream_t s, int* state, int set_to, float b1, float b2) {
  if (!state || set_to < 0) return hipErrorInvalidValue;
  adam_step_kernel<<<1, 64, 0, s>>>(state, set_to, b1, b2);
  return hipGetLastError();
}

}  // namespace pw
