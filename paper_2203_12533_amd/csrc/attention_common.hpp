// Helpers shared by the MFMA attention kernels (register-layout bookkeeping; see attention_mfma.hip).
#pragma once
#include "common.hpp"

namespace pw {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Linear workgroup id -> (problem = batch*H + head, block index inside the problem).  The hardware deals
// consecutive workgroup ids round-robin over the 8 XCDs, each with an L2 of its own; the n_inner blocks of one
// problem all stream the same K/V (or Q/dO) rows, so they are given ids that land on ONE XCD, close together:
// XCD x owns a contiguous range of (problem, block) pairs.  A bijection for any grid size.
// With a causal mask the blocks of a problem differ in length (inner = 0 is the longest).  Workgroups start in id
// order as compute units free up, so problems are taken `group` at a time and inside a group all blocks of rank 0
// come first, then rank 1, ...: with group * n_inner at or above the number of workgroups an XCD holds at once
// this is longest-first scheduling and every compute unit ends at the same time (problem after problem it left
// the last long blocks to start late: 44 against 36 units of time for the dK/dV kernel at 8 blocks per problem).
__device__ __forceinline__ void xcd_block_map(int pid, int nblk, int n_inner, int group, int& problem, int& inner) {
  constexpr int kXcd = 8;
  const int q = nblk / kXcd, r = nblk % kXcd;
  const int xcd = pid % kXcd, j = pid / kXcd;
  const int logical = xcd * q + (xcd < r ? xcd : r) + j;
  const int per_group = group * n_inner;
  const int g = logical / per_group, within = logical - g * per_group;
  const int first = g * group, left = nblk / n_inner - first;
  const int members = left < group ? left : group;       // the last group may be smaller
  inner = within / members;
  problem = first + within - inner * members;
}

// Problems per group for xcd_block_map under a causal mask: enough that one group fills the `resident` workgroups
// an XCD holds at once (32 compute units x workgroups per unit).
__device__ __forceinline__ int causal_group(int n_inner, int resident) { return (resident + n_inner - 1) / n_inner; }

// max of three in one instruction.  (Scores are never signalling NaNs, so the quieting pass the compiler puts
// in front of every fmaxf on values it cannot trace is not needed.)
__device__ __forceinline__ float max3(float a, float b, float c) {
  float d;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
  return d;
}

__device__ __forceinline__ int perm_row(int i) {   // [0-3, 8-11, 4-7, 12-15] within each 16
  const int j = i & 15;
  const int p = (j & 3) | ((j & 4) << 1) | ((j & 8) >> 1);
  return (i & ~15) | p;
}


// Fragments of 32 rows x HD features held in registers as the B operand of a first product:
// lane l holds row (row0 + l%32), features kk*16 + 8*(l/32) .. +7 for every kk.  Rows >= limit read as zero.
template <int HD>
__device__ __forceinline__ void load_row_frags(const bf16* __restrict__ src, int64_t ld, int row0, int limit, bf16x8* frag) {
  const int lane = threadIdx.x & 63;
  const int row = row0 + (lane & 31);
  const bf16* p = src + (int64_t)row * ld + (lane >> 5) * 8;
#pragma unroll
  for (int kk = 0; kk < HD / 16; ++kk) {
    if (row < limit) {
      frag[kk] = *reinterpret_cast<const bf16x8*>(p + kk * 16);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) frag[kk][e] = (bf16)0.f;
    }
  }
}


__device__ __forceinline__ bf16x8 pack8(const f32x16& v, int first) {
  bf16x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = (bf16)v[first + e];
  return o;
}


// Tile-local row index that register r of this lane's D column stands for (see file header).
__device__ __forceinline__ int reg_row(int r, int half) { return 16 * (r >> 3) + 8 * half + (r & 7); }

// Writes acc (feature-major: register r of block cb = feature cb*32 + 8*(r/4) + 4*half + r%4) for this lane's
// row to dst (row pointer, feature 0), scaled.
template <int HD>
__device__ __forceinline__ void store_row(bf16* __restrict__ dst, const f32x16* acc, float scale) {
  const int half = (threadIdx.x & 63) >> 5;
#pragma unroll
  for (int cb = 0; cb < HD / 32; ++cb)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      bf16x4 o = {(bf16)(acc[cb][q * 4] * scale), (bf16)(acc[cb][q * 4 + 1] * scale), (bf16)(acc[cb][q * 4 + 2] * scale),
                  (bf16)(acc[cb][q * 4 + 3] * scale)};
      *reinterpret_cast<bf16x4*>(dst + cb * 32 + q * 8 + half * 4) = o;
    }
}


// The same, plus what the rounding left over to a second row (lo): value ~ bf16(dst) + bf16(lo).
template <int HD>
__device__ __forceinline__ void store_row_split(bf16* __restrict__ dst, bf16* __restrict__ lo, const f32x16* acc, float scale) {
  const int half = (threadIdx.x & 63) >> 5;
#pragma unroll
  for (int cb = 0; cb < HD / 32; ++cb)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      bf16x4 o, r;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float v = acc[cb][q * 4 + e] * scale;
        o[e] = (bf16)v;
        r[e] = (bf16)(v - (float)o[e]);
      }
      *reinterpret_cast<bf16x4*>(dst + cb * 32 + q * 8 + half * 4) = o;
      *reinterpret_cast<bf16x4*>(lo + cb * 32 + q * 8 + half * 4) = r;
    }
}

}  // namespace pw
