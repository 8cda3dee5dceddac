// Ceiling of the GEMM's inner loop on this chip, with no global memory involved, and what sets it: the board
// power limit.  One workgroup of 8 waves per compute unit runs the instruction mix of the ring GEMM's k-loop
// (128 x 64 wave tiles; per 64-deep k-tile 24 LDS fragment reads of 16 bytes and the MFMAs that consume them)
// for a few seconds while a host thread samples the engine clock and the board power from sysfs.  Variants:
// the two bf16 MFMA shapes (same flops, same LDS bytes), the order in which a wave walks its accumulator
// blocks, constant against random operands, with and without one barrier per k-tile.
// Everything stays in bounds; every loop is bounded.
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -o /tmp/mfma_ceiling paper_2203_12533_amd/tools/mfma_ceiling.hip && /tmp/mfma_ceiling
#include <hip/hip_runtime.h>
#include <glob.h>

#include <atomic>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <thread>
#include <vector>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("err %s line %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)

constexpr int kNT = 512;             // 8 waves: 2 (rows) x 4 (columns) wave tiles of 128 x 64
constexpr int kLd = 72;              // LDS row of 64 k-values + padding
constexpr int kLdsElems = 512 * kLd; // A tile (256 rows) then B tile (256 rows)

// Operands: activation-like small values with random mantissas, or a constant pattern.
__device__ inline void fill(__bf16* smem, int rnd) {
  for (int i = threadIdx.x; i < kLdsElems; i += kNT) {
    unsigned h = (unsigned)i * 2654435761u + blockIdx.x * 40503u; h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    const float u = ((h & 255) + ((h >> 8) & 255) + ((h >> 16) & 255) + ((h >> 24) & 255) - 510.f) * (0.05f / 148.f);
    smem[i] = rnd ? (__bf16)u : (__bf16)(0.001f * (i & 15));
  }
}

// v_mfma_f32_32x32x16_bf16: 4 x 2 accumulator blocks per wave, four 16-deep k-steps per k-tile.
template <int BARRIER>
__global__ __launch_bounds__(kNT) void loop_32x32x16(float* out, int iters, int rnd) {
  extern __shared__ __attribute__((aligned(16))) __bf16 smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  fill(smem, rnd);
  __syncthreads();
  constexpr int FM = 4, FN = 2;
  f32x16 acc[FM * FN];
  for (int a = 0; a < FM * FN; ++a) for (int r = 0; r < 16; ++r) acc[a][r] = 0.f;
  bf16x8 af[FM], bf[FN];
  const __bf16* a_tile = smem + ((wave & 1) * 128 + (lane & 31)) * kLd + (lane >> 5) * 8;
  const __bf16* b_tile = smem + 256 * kLd + ((wave >> 1) * 64 + (lane & 31)) * kLd + (lane >> 5) * 8;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
      for (int i = 0; i < FM; ++i) af[i] = *reinterpret_cast<const bf16x8*>(a_tile + i * 32 * kLd + kk * 16);
#pragma unroll
      for (int j = 0; j < FN; ++j) bf[j] = *reinterpret_cast<const bf16x8*>(b_tile + j * 32 * kLd + kk * 16);
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i * FN + j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[j], af[i], acc[i * FN + j], 0, 0, 0);
    }
    if (BARRIER) __syncthreads();
  }
  float s = 0.f;
  for (int a = 0; a < FM * FN; ++a) for (int r = 0; r < 16; ++r) s += acc[a][r];
  out[blockIdx.x * kNT + threadIdx.x] = s;
}

// v_mfma_f32_16x16x32_bf16: 8 x 4 accumulator blocks per wave, two 32-deep k-steps per k-tile.
// ORDER 0: row block outer, column block inner, always ascending.  ORDER 1: columns back and forth, so that every
// MFMA shares one operand with the one before it.
template <int ORDER, int BARRIER>
__global__ __launch_bounds__(kNT) void loop_16x16x32(float* out, int iters, int rnd) {
  extern __shared__ __attribute__((aligned(16))) __bf16 smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  fill(smem, rnd);
  __syncthreads();
  constexpr int FM = 8, FN = 4;
  f32x4 acc[FM * FN];
  for (int a = 0; a < FM * FN; ++a) for (int r = 0; r < 4; ++r) acc[a][r] = 0.f;
  bf16x8 af[FM], bf[FN];
  const __bf16* a_tile = smem + ((wave & 1) * 128 + (lane & 15)) * kLd + (lane >> 4) * 8;
  const __bf16* b_tile = smem + 256 * kLd + ((wave >> 1) * 64 + (lane & 15)) * kLd + (lane >> 4) * 8;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
      for (int i = 0; i < FM; ++i) af[i] = *reinterpret_cast<const bf16x8*>(a_tile + i * 16 * kLd + kk * 32);
#pragma unroll
      for (int j = 0; j < FN; ++j) bf[j] = *reinterpret_cast<const bf16x8*>(b_tile + j * 16 * kLd + kk * 32);
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int jj = 0; jj < FN; ++jj) {
          const int j = (ORDER == 1 && (i & 1)) ? FN - 1 - jj : jj;
          acc[i * FN + j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bf[j], af[i], acc[i * FN + j], 0, 0, 0);
        }
    }
    if (BARRIER) __syncthreads();
  }
  float s = 0.f;
  for (int a = 0; a < FM * FN; ++a) for (int r = 0; r < 4; ++r) s += acc[a][r];
  out[blockIdx.x * kNT + threadIdx.x] = s;
}

// The same loop laid out as the ring GEMM does it: fragments double-buffered in registers - the reads of a k-step
// are issued under the MFMAs of the step before - and, with BARRIER, one bare s_barrier per k-tile placed in front
// of the last eight MFMAs of the tile, the next tile's first fragment reads right behind it.  (The plain variant
// above waits for its fragments at the top of every k-step and, with its barrier, drains the matrix pipe once per
// k-tile: its cost is that of the drain, not of the barrier instruction.)
template <int BARRIER>
__global__ __launch_bounds__(kNT) void loop_16x16x32_pipelined(float* out, int iters, int rnd) {
  extern __shared__ __attribute__((aligned(16))) __bf16 smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  fill(smem, rnd);
  __syncthreads();
  constexpr int FM = 8, FN = 4;
  f32x4 acc[FM * FN];
  for (int a = 0; a < FM * FN; ++a) for (int r = 0; r < 4; ++r) acc[a][r] = 0.f;
  bf16x8 af[2][FM], bf[2][FN];
  const __bf16* a_tile = smem + ((wave & 1) * 128 + (lane & 15)) * kLd + (lane >> 4) * 8;
  const __bf16* b_tile = smem + 256 * kLd + ((wave >> 1) * 64 + (lane & 15)) * kLd + (lane >> 4) * 8;
  auto read = [&](int kk) {
#pragma unroll
    for (int i = 0; i < FM; ++i) af[kk][i] = *reinterpret_cast<const bf16x8*>(a_tile + i * 16 * kLd + kk * 32);
#pragma unroll
    for (int j = 0; j < FN; ++j) bf[kk][j] = *reinterpret_cast<const bf16x8*>(b_tile + j * 16 * kLd + kk * 32);
  };
  auto rows = [&](int kk, int i0, int i1) {
#pragma unroll
    for (int i = i0; i < i1; ++i)
#pragma unroll
      for (int jj = 0; jj < FN; ++jj) {
        const int j = (i & 1) ? FN - 1 - jj : jj;
        acc[i * FN + j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bf[kk][j], af[kk][i], acc[i * FN + j], 0, 0, 0);
      }
  };
  read(0);
  for (int it = 0; it < iters; ++it) {
    read(1);
    rows(0, 0, FM);
    rows(1, 0, FM - 2);
    if (BARRIER) __builtin_amdgcn_s_barrier();
    read(0);
    rows(1, FM - 2, FM);
  }
  float s = 0.f;
  for (int a = 0; a < FM * FN; ++a) for (int r = 0; r < 4; ++r) s += acc[a][r];
  out[blockIdx.x * kNT + threadIdx.x] = s;
}

// Host-side sampler of engine clock (the starred level of pp_dpm_sclk) and board power (hwmon power1_input).
struct Sampler {
  std::string sclk_path, power_path;
  std::atomic<bool> stop{false};
  std::vector<int> mhz;
  std::vector<double> watts;
  std::thread th;
  static std::string first_match(const char* pattern) {
    glob_t g;
    std::string r;
    if (glob(pattern, 0, nullptr, &g) == 0 && g.gl_pathc > 0) r = g.gl_pathv[0];
    globfree(&g);
    return r;
  }
  Sampler() {
    sclk_path = first_match("/sys/class/drm/card*/device/pp_dpm_sclk");
    power_path = first_match("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input");
  }
  void start() {
    th = std::thread([this] {
      while (!stop.load()) {
        if (FILE* f = sclk_path.empty() ? nullptr : fopen(sclk_path.c_str(), "r")) {
          char line[128];
          while (fgets(line, sizeof line, f))
            if (strchr(line, '*')) {
              const char* c = strchr(line, ':');
              if (c) mhz.push_back(atoi(c + 1));
            }
          fclose(f);
        }
        if (FILE* f = power_path.empty() ? nullptr : fopen(power_path.c_str(), "r")) {
          long long uw = 0;
          if (fscanf(f, "%lld", &uw) == 1) watts.push_back(uw / 1e6);
          fclose(f);
        }
        std::this_thread::sleep_for(std::chrono::milliseconds(50));
      }
    });
  }
  void finish(double* mean_mhz, double* mean_w) {
    stop.store(true);
    th.join();
    double a = 0, b = 0;
    for (int v : mhz) a += v;
    for (double v : watts) b += v;
    *mean_mhz = mhz.empty() ? 0 : a / mhz.size();
    *mean_w = watts.empty() ? 0 : b / watts.size();
  }
};

// Launches of 4000 k-tiles each for `secs` seconds; the rate, the clock and the power are those of the second half.
template <typename K>
void run(const char* name, K kern, int rnd, double secs) {
  const int blocks = 256, iters = 4000;
  float* out; CK(hipMalloc(&out, (size_t)blocks * kNT * 4));
  const size_t smem = (size_t)kLdsElems * 2;
  CK(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
  hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
  kern<<<blocks, kNT, smem>>>(out, 10, rnd); CK(hipDeviceSynchronize());
  CK(hipEventRecord(a)); kern<<<blocks, kNT, smem>>>(out, iters, rnd); CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
  float ms; CK(hipEventElapsedTime(&ms, a, b));
  const int n = (int)(secs * 1e3 / ms) + 2, warm = n / 2;
  for (int i = 0; i < warm; ++i) kern<<<blocks, kNT, smem>>>(out, iters, rnd);
  CK(hipDeviceSynchronize());
  Sampler s; s.start();
  CK(hipEventRecord(a));
  for (int i = 0; i < n - warm; ++i) kern<<<blocks, kNT, smem>>>(out, iters, rnd);
  CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
  double mhz, w; s.finish(&mhz, &w);
  CK(hipEventElapsedTime(&ms, a, b));
  const double flops = 2.0 * 128 * 64 * 64 * 8 * (double)iters * blocks * (n - warm);   // per k-tile and wave: 128 x 64 x 64
  printf("%-46s %-8s %8.1f TFLOP/s   %5.0f MHz  %5.0f W\n", name, rnd ? "random" : "constant", flops / (ms * 1e-3) / 1e12, mhz, w);
  fflush(stdout);
  CK(hipFree(out));
  std::this_thread::sleep_for(std::chrono::milliseconds(1000));
}

int main() {
  const double secs = 2.5;
  printf("%-46s %-8s %17s %10s %8s\n", "loop (8 waves per CU, 256 CUs, LDS reads)", "operands", "sustained", "clock", "power");
  run("32x32x16", loop_32x32x16<0>, 1, secs);
  run("16x16x32, ascending columns", loop_16x16x32<0, 0>, 1, secs);
  run("16x16x32, columns back and forth", loop_16x16x32<1, 0>, 1, secs);
  run("16x16x32, back and forth, barrier per k-tile", loop_16x16x32<1, 1>, 1, secs);
  run("16x16x32, b&f, fragments double-buffered", loop_16x16x32_pipelined<0>, 1, secs);
  run("16x16x32, b&f, double-buffered, bare barrier", loop_16x16x32_pipelined<1>, 1, secs);
  run("32x32x16", loop_32x32x16<0>, 0, secs);
  run("16x16x32, columns back and forth", loop_16x16x32<1, 0>, 0, secs);
  return 0;
}
