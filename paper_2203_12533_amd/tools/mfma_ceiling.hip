// Ceiling of the GEMM's inner loop on this chip, with no global memory involved: the instruction mix of
// gemm_bf16_kernel's k-loop (8 waves, 4 + 2 LDS fragment reads per 8 MFMAs, optional barrier per 32 MFMAs),
// on near-constant or on random bf16 operands.  The clock falls with operand activity, so the random-data
// figure is the practical roofline of that loop.  Everything stays in bounds; loops are bounded.
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -o /tmp/mfma_ceiling paper_2203_12533_amd/tools/mfma_ceiling.hip && /tmp/mfma_ceiling
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("err %s line %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)

// MODE 0: pure MFMA (8 independent accumulators).  MODE 1: + LDS fragment reads as in the GEMM (6 per 8 MFMAs).
// MODE 2: MODE 1 + one barrier per 32 MFMAs.
template <int MODE, int NT, int RANDOM>
__global__ __launch_bounds__(NT) void k(float* out, int iters) {
  extern __shared__ __attribute__((aligned(16))) __bf16 smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i = threadIdx.x; i < 512 * 72; i += NT) {
    unsigned h = (unsigned)i * 2654435761u + blockIdx.x * 40503u; h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    smem[i] = RANDOM ? (__bf16)(((int)(h & 0xFFFF) - 32768) * (1.0f / 32768.f)) : (__bf16)(0.001f * (i & 15));
  }
  __syncthreads();
  f32x16 acc[8];
  for (int a = 0; a < 8; ++a) for (int r = 0; r < 16; ++r) acc[a][r] = 0.f;
  bf16x8 af[4], bf[2];
  for (int i = 0; i < 4; ++i) for (int e = 0; e < 8; ++e) af[i][e] = (__bf16)(0.01f * (lane + i));
  for (int i = 0; i < 2; ++i) for (int e = 0; e < 8; ++e) bf[i][e] = (__bf16)(0.02f * (lane + i));
  const __bf16* a_tile = smem + ((wave / 4) * 128 + (lane & 31)) * 72 + (lane >> 5) * 8;
  const __bf16* b_tile = smem + 256 * 72 + ((wave % 4) * 64 + (lane & 31)) * 72 + (lane >> 5) * 8;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      if (MODE >= 1) {
#pragma unroll
        for (int i = 0; i < 4; ++i) af[i] = *reinterpret_cast<const bf16x8*>(a_tile + i * 32 * 72 + kk * 16);
#pragma unroll
        for (int j = 0; j < 2; ++j) bf[j] = *reinterpret_cast<const bf16x8*>(b_tile + j * 32 * 72 + kk * 16);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i * 2 + j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[j], af[i], acc[i * 2 + j], 0, 0, 0);
    }
    if (MODE == 2) __syncthreads();
  }
  float s = 0.f;
  for (int a = 0; a < 8; ++a) for (int r = 0; r < 16; ++r) s += acc[a][r];
  out[blockIdx.x * NT + threadIdx.x] = s;
}

template <int MODE, int NT, int RANDOM>
void run(const char* name, int blocks_per_cu, int iters) {
  const int blocks = 256 * blocks_per_cu;
  float* out; CK(hipMalloc(&out, (size_t)blocks * NT * 4));
  const size_t smem = 512 * 72 * 2;
  CK(hipFuncSetAttribute((const void*)k<MODE, NT, RANDOM>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
  hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
  k<MODE, NT, RANDOM><<<blocks, NT, smem>>>(out, 10); CK(hipDeviceSynchronize());
  CK(hipEventRecord(a)); k<MODE, NT, RANDOM><<<blocks, NT, smem>>>(out, iters); CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
  float ms; CK(hipEventElapsedTime(&ms, a, b));
  const double flops = (double)blocks * (NT / 64) * iters * 32.0 * 32768.0;
  printf("%-30s rnd=%d NT=%d blocks/CU=%d iters=%d: %8.3f ms  %8.1f TFLOP/s\n", name, RANDOM, NT, blocks_per_cu, iters, ms, flops / ms / 1e9); fflush(stdout);
  CK(hipFree(out));
}
int main() {
  run<2, 512, 0>("MFMA + LDS reads + barrier", 1, 2000);
  run<2, 512, 0>("MFMA + LDS reads + barrier", 1, 20000);
  run<2, 512, 1>("MFMA + LDS reads + barrier", 1, 2000);
  run<2, 512, 1>("MFMA + LDS reads + barrier", 1, 20000);
  run<1, 512, 1>("MFMA + LDS reads", 1, 20000);
  run<1, 256, 1>("MFMA + LDS reads", 1, 20000);
  run<0, 512, 0>("pure MFMA", 1, 20000);
  return 0;
}
