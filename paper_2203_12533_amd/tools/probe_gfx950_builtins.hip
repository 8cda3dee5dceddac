// In-bounds probes of two gfx950 builtins: lane layout of ds_read_tr16_b64 and LDS placement of global_load_lds (16 B).
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("err %s line %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)
typedef short short4v __attribute__((ext_vector_type(4)));

__global__ void probe_tr(short* out) {
  __shared__ __attribute__((aligned(16))) short lds[1024];
  for (int i = threadIdx.x; i < 1024; i += 64) lds[i] = (short)i;
  __syncthreads();
  // lane L points at elements 4L .. 4L+3
  short4v v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)(lds + threadIdx.x * 4));
  for (int e = 0; e < 4; ++e) out[threadIdx.x * 4 + e] = v[e];
}

__global__ void probe_gl(const short* src, short* out) {
  __shared__ __attribute__((aligned(16))) short lds[2048];
  for (int i = threadIdx.x; i < 2048; i += 64) lds[i] = (short)-1;
  __syncthreads();
  // lane L fetches 16 bytes = elements 8*(63-L) .. +7 of src; destination base is lds + 256 elements (wave-uniform)
  const short* g = src + 8 * (63 - threadIdx.x);
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                   (__attribute__((address_space(3))) void*)(lds + 256), 16, 0, 0);
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  for (int i = threadIdx.x; i < 2048; i += 64) out[i] = lds[i];
}

int main() {
  short *d_out, *d_src; CK(hipMalloc(&d_out, 4096 * 2)); CK(hipMalloc(&d_src, 1024 * 2));
  short h[2048], src[1024];
  for (int i = 0; i < 1024; ++i) src[i] = (short)(1000 + i);
  CK(hipMemcpy(d_src, src, sizeof src, hipMemcpyHostToDevice));
  probe_tr<<<1, 64>>>(d_out); CK(hipDeviceSynchronize());
  CK(hipMemcpy(h, d_out, 256 * 2, hipMemcpyDeviceToHost));
  printf("ds_read_tr16_b64: lane: 4 source element indices (source lane = idx/4, element = idx%%4)\n");
  for (int l = 0; l < 64; ++l) { printf("L%02d: %4d %4d %4d %4d   ", l, h[l*4], h[l*4+1], h[l*4+2], h[l*4+3]); if (l % 4 == 3) printf("\n"); }
  probe_gl<<<1, 64>>>(d_src, d_out); CK(hipDeviceSynchronize());
  CK(hipMemcpy(h, d_out, 2048 * 2, hipMemcpyDeviceToHost));
  printf("global_load_lds 16B: first LDS element written per 8-element slot (slot: src element)\n");
  for (int s = 0; s < 256; ++s) if (h[s*8] != -1) printf("slot%03d:%d ", s, h[s*8]);
  printf("\n");
  return 0;
}
