// bf16 MFMA attention for head_dim 128 with direct global->LDS loads and transposing LDS reads.
//
// Same register-layout scheme as attention_mfma.hip (softmax row on the lane; first product's A rows read
// permuted so that P / dS feed the second product from the accumulator registers).  What changes is how
// operands travel:
//  * every tile (K, V, or Q, dO) is brought into LDS once, in its natural [row][128] layout, by
//    global_load_lds_dwordx4 (each wave instruction deposits 4 rows = 1 KiB; no staging registers, no LDS
//    store instructions), double-buffered so the next tile is in flight while one is consumed;
//  * the second product needs the tile as [feature][row]; instead of keeping a transposed copy it is read
//    with ds_read_b64_tr_b16 (lane L of each 16-lane group points at [k0 + L/4][c0 + 4*(L%4)], lane i
//    receives rows k0..k0+3 of feature c0 + i).
// LDS swizzle, one rule for both access patterns: chunk c (8 features = 16 bytes) of row r sits at
// position c ^ (((r & 3) << 2) | ((r >> 2) & 3)).  16 consecutive (or permuted-within-16) rows of one chunk
// then hit 16 distinct 16-byte bank groups, and the 4 rows touched by one transposing read fall into 4
// different 64-byte windows.
// Rows past the end of a sequence are fetched from its last valid row (always in bounds); every use of such
// a row is masked (causality, or the explicit key-index mask of the unmasked variant) or multiplied by an exact
// zero (P = exp2(-inf)).
// Queries, keys and values come with their own pointers, row strides and lengths (MhaDev), so one set of kernels
// serves the packed causal self-attention of a decoder, the unmasked self-attention of an encoder and attention
// of decoder queries over encoder keys; CAUSAL is a template parameter (it decides which tiles are visited).
#include <type_traits>

#include "attention_common.hpp"
#include "common.hpp"
#include "kernels.hpp"

namespace pw {

namespace {

constexpr int HD = 128;
constexpr int kNT = 256;                 // 4 waves
constexpr int kRowBytes = HD * 2;        // 256
typedef __attribute__((address_space(3))) void* lds_ptr;
typedef short short4v __attribute__((ext_vector_type(4)));

// q, k, v: element (batch 0, row 0, feature 0); rows ldq / ldkv elements apart; batch b starts at row b*Tq / b*Tk.
struct MhaDev {
  const bf16 *q, *k, *v;
  int64_t ldq, ldkv;
  int Tq, Tk, H;
};

__device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

__device__ __forceinline__ void dma16(const bf16* g, uint32_t lds_off) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(g), "s"(lds_off) : "memory", "m0");
}

// 4 bytes per lane straight into LDS at lds_off + 4*lane (per-row statistics of a tile).
__device__ __forceinline__ void dma4(const float* g, uint32_t lds_off) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off" : : "v"(g), "s"(lds_off) : "memory", "m0");
}

// Same with a wave-uniform base pointer in scalar registers and a 32-bit per-lane byte offset.
__device__ __forceinline__ void dma16_s(const bf16* base, uint32_t voff, uint32_t lds_off) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(voff), "s"(base), "s"(lds_off) : "memory", "m0");
}

// Direct loads of a ROWS x 128 tile, ROWS/16 instructions of 1 KiB per wave (4 waves).  Instruction j of wave w
// covers tile rows 4 (w ROWS/16 + j) .. +3; lane l fetches chunk (l%16) ^ swz(row) of row l/16 of those.
// TileOffsets holds this lane's byte offsets inside a tile whose first row is row 0 (they do not depend on the
// tile), so a tile that lies fully inside the sequence costs no vector arithmetic: base + rows*ld is scalar.
template <int ROWS>
struct TileOffsets {
  static constexpr int kPerWave = ROWS / 16;
  uint32_t off[kPerWave];
  __device__ __forceinline__ void init(int64_t ld, int wave, int lane) {
#pragma unroll
    for (int j = 0; j < kPerWave; ++j) {
      const int r = (wave * kPerWave + j) * 4 + (lane >> 4);
      off[j] = (uint32_t)((r * ld + (((lane & 15) ^ swz(r)) << 3)) * 2);
    }
  }
};
// src: element (row 0 of the sequence, feature 0); tile rows row0 .. row0+ROWS-1; rows past `last` are fetched
// from row `last` (the slow path, only for the one tile that straddles the end of the sequence).
template <int ROWS>
__device__ __forceinline__ void issue_tile(const bf16* __restrict__ src, int64_t ld, int row0, int last,
                                           const TileOffsets<ROWS>& to, uint32_t lds_off, int wave, int lane) {
  constexpr int kPerWave = ROWS / 16;
  if (row0 + ROWS - 1 <= last) {
    const bf16* base = src + (int64_t)row0 * ld;
#pragma unroll
    for (int j = 0; j < kPerWave; ++j) dma16_s(base, to.off[j], lds_off + (wave * kPerWave + j) * 1024);
  } else {
#pragma unroll
    for (int j = 0; j < kPerWave; ++j) {
      const int instr = wave * kPerWave + j;
      const int r = instr * 4 + (lane >> 4);
      const int c = (lane & 15) ^ swz(r);
      const int row = min(row0 + r, last);
      dma16(src + (int64_t)row * ld + c * 8, lds_off + instr * 1024);
    }
  }
}

// 32x32 block of a first product: A rows (permuted) from a swizzled natural LDS tile, B from register fragments.
// The A fragments are fetched kDepth MFMAs ahead of their use (left alone the compiler fetches each one right
// before the MFMA that needs it, and every MFMA of the chain then waits out a full LDS round trip).
__device__ __forceinline__ f32x16 first_product(const bf16* __restrict__ tile, int row_base, const bf16x8* bfrag) {
  constexpr int kDepth = 3, KK = HD / 16;   // 2 and 4 measured the same
  const int lane = threadIdx.x & 63;
  const int row = row_base + perm_row(lane & 31);
  const int t = (lane >> 5) ^ swz(row);                 // chunk (2 kk + half) ^ swz = (2 kk) ^ t
  const bf16* a = tile + row * HD;
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  bf16x8 af[kDepth];
#pragma unroll
  for (int kk = 0; kk < kDepth; ++kk) af[kk] = *reinterpret_cast<const bf16x8*>(a + ((2 * kk) ^ t) * 8);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk % kDepth], bfrag[kk], acc, 0, 0, 0);
    if (kk + kDepth < KK) af[kk % kDepth] = *reinterpret_cast<const bf16x8*>(a + ((2 * (kk + kDepth)) ^ t) * 8);
    __builtin_amdgcn_sched_barrier(0);
  }
  return acc;
}

// acc[cb] += Tile^T[features cb*32 ..][rows row_base .. row_base+15] . frag, the tile read transposed.
__device__ __forceinline__ void second_product(const bf16* __restrict__ tile, int row_base, const bf16x8& frag, f32x16* acc) {
  const int lane = threadIdx.x & 63;
  const int grp = lane >> 4, L = lane & 15;
  const int row0 = row_base + 8 * (grp >> 1) + (L >> 2);          // tile row this lane points at for t = 0
  const int f0 = 16 * (grp & 1) + 4 * (L & 3);                    // first of its 4 features inside a 32-feature block
#pragma unroll
  for (int cb = 0; cb < HD / 32; ++cb) {
    union { bf16x8 v; short4v h[2]; } u;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int row = row0 + 4 * t;
      const int chunk = (cb * 32 + f0) >> 3;
      const bf16* p = tile + row * HD + ((chunk ^ swz(row)) << 3) + (f0 & 7);
      u.h[t] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)p);
    }
    acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u.v, frag, acc[cb], 0, 0, 0);
  }
}

__device__ __forceinline__ void wait_and_sync() {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's share of the tile in flight has landed
  __builtin_amdgcn_s_barrier();                      // ... and so has everyone else's; the other stage is free again
  asm volatile("" ::: "memory");
}

// ===================================================================================================
// forward: block = 128 queries of one (batch, head); wave = 32 queries; key/value tiles of 64
// ===================================================================================================
template <bool CAUSAL>
__global__ __launch_bounds__(kNT, 2) void attn_fwd_dma_kernel(MhaDev a, bf16* __restrict__ o, bf16* __restrict__ o_lo,
                                                              float* __restrict__ lse) {
  constexpr int BKV = 64;
  constexpr int kTile = BKV * HD;                       // elements per K (or V) tile
  extern __shared__ __attribute__((aligned(1024))) bf16 smem[];         // [stage][K | V], 64 KiB
  const int Tq = a.Tq, Tk = a.Tk, H = a.H;
  const int d = H * HD;
  const int64_t ld = a.ldkv;
  const int nq = (Tq + 127) / 128;
  int bh, qi;
  xcd_block_map(blockIdx.x, gridDim.x, nq, CAUSAL ? causal_group(nq, 64) : 1, bh, qi);
  const int b = bh / H, h = bh - b * H;
  const int qblk = CAUSAL ? nq - 1 - qi : qi;           // causal: longest blocks of a problem first
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, half = lane >> 5;
  const int q0 = qblk * 128 + wave * 32;
  const int query = q0 + (lane & 31);
  const bf16* qbase = a.q + (int64_t)b * Tq * a.ldq + h * HD;
  const bf16* kbase = a.k + (int64_t)b * Tk * ld + h * HD;
  const bf16* vbase = a.v + (int64_t)b * Tk * ld + h * HD;
  const float c2 = kLog2e / sqrtf((float)HD);
  const uint32_t smem_off = (uint32_t)(uintptr_t)(lds_ptr)smem;

  bf16x8 qf[HD / 16];
  load_row_frags<HD>(qbase, a.ldq, q0, Tq, qf);
  f32x16 acc[HD / 32];
#pragma unroll
  for (int cb = 0; cb < HD / 32; ++cb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[cb][r] = 0.f;
  float m = -INFINITY, l = 0.f;

  const int last_q = min(Tq, (qblk + 1) * 128) - 1;
  const int n_tiles = CAUSAL ? last_q / BKV + 1 : (Tk + BKV - 1) / BKV;
  TileOffsets<BKV> to;
  to.init(ld, wave, lane);
  auto issue = [&](int t) {
    const uint32_t st = smem_off + (uint32_t)(t & 1) * (2 * kTile * 2);
    issue_tile<BKV>(kbase, ld, t * BKV, Tk - 1, to, st, wave, lane);
    issue_tile<BKV>(vbase, ld, t * BKV, Tk - 1, to, st + kTile * 2, wave, lane);
  };
  issue(0);
  for (int t = 0; t < n_tiles; ++t) {
    const int j0 = t * BKV;
    wait_and_sync();
    if (t + 1 < n_tiles) issue(t + 1);
    if (CAUSAL && j0 > q0 + 31) continue;   // every key of the tile lies in this wave's future
    const bf16* Ks = smem + (t & 1) * (2 * kTile);
    const bf16* Vs = Ks + kTile;
    f32x16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) s[kb] = first_product(Ks, kb * 32, qf);
    // last visible key of this lane's query: itself (causal), else the last key there is
    const int last_key = CAUSAL ? query : Tk - 1;
    if (CAUSAL ? j0 + BKV - 1 > q0 : j0 + BKV > Tk) {   // the tile straddles the diagonal / the end of the keys
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (j0 + kb * 32 + reg_row(r, half) > last_key) s[kb][r] = -INFINITY;
    }
    float mx = max3(s[0][0], s[1][0], s[0][1]);
#pragma unroll
    for (int r = 1; r < 15; ++r) mx = max3(mx, s[1][r], s[0][r + 1]);
    mx = max3(mx, s[1][15], s[1][15]);
    const float other = __shfl_xor(mx, 32, 64);
    mx = max3(mx, other, other) * c2;
    // lazy rescaling: the reference m only has to bound the exponents (see attention_mfma.hip)
    if (__builtin_amdgcn_ballot_w64(mx > m + 8.f) != 0) {
      const float m_new = fmaxf(m, mx);
      const float alpha = __builtin_amdgcn_exp2f(m - m_new);
      m = m_new;
      l *= alpha;
#pragma unroll
      for (int cb = 0; cb < HD / 32; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[cb][r] *= alpha;
    }
    float sum = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = __builtin_amdgcn_exp2f(fmaf(s[kb][r], c2, -m));
        s[kb][r] = p;
        sum += p;
      }
    l += sum;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int b2 = 0; b2 < 2; ++b2) second_product(Vs, kb * 32 + b2 * 16, pack8(s[kb], b2 * 8), acc);
  }
  l += __shfl_xor(l, 32, 64);
  if (query < Tq) {
    const int64_t row = ((int64_t)b * Tq + query) * d + h * HD;
    if (o_lo)
      store_row_split<HD>(o + row, o_lo + row, acc, 1.f / l);
    else
      store_row<HD>(o + row, acc, 1.f / l);
    if (half == 0) lse[(int64_t)bh * Tq + query] = (m + __builtin_amdgcn_logf(l)) * kLn2;
  }
}

// ===================================================================================================
// dQ: same tiling as the forward.  dQ_i = scale * sum_j dS_ij K_j, dS = P (dP - delta)
// ===================================================================================================
// It also produces delta_i = sum_c dO_ic O_ic for its queries (each wave has the dO fragments of its 32 rows in
// registers anyway; O, plus the optional rounding remainder o_lo, is read the same way once) and leaves it in
// `delta` for the dK/dV kernel, which is launched behind this one.
template <bool CAUSAL>
__global__ __launch_bounds__(kNT, 2) void attn_dq_dma_kernel(MhaDev a, const bf16* __restrict__ o, const bf16* __restrict__ o_lo,
                                                             const bf16* __restrict__ dout, const float* __restrict__ lse,
                                                             float* __restrict__ delta, bf16* __restrict__ dq, int64_t lddq) {
  constexpr int BKV = 64;
  constexpr int kTile = BKV * HD;
  extern __shared__ __attribute__((aligned(1024))) bf16 smem[];
  const int Tq = a.Tq, Tk = a.Tk, H = a.H;
  const int d = H * HD;
  const int64_t ld = a.ldkv;
  const int nq = (Tq + 127) / 128;
  int bh, qi;
  xcd_block_map(blockIdx.x, gridDim.x, nq, CAUSAL ? causal_group(nq, 64) : 1, bh, qi);
  const int b = bh / H, h = bh - b * H;
  const int qblk = CAUSAL ? nq - 1 - qi : qi;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, half = lane >> 5;
  const int q0 = qblk * 128 + wave * 32;
  const int query = q0 + (lane & 31);
  const bf16* qbase = a.q + (int64_t)b * Tq * a.ldq + h * HD;
  const bf16* kbase = a.k + (int64_t)b * Tk * ld + h * HD;
  const bf16* vbase = a.v + (int64_t)b * Tk * ld + h * HD;
  const float scale = 1.f / sqrtf((float)HD);
  const float c2 = kLog2e * scale;
  const uint32_t smem_off = (uint32_t)(uintptr_t)(lds_ptr)smem;

  bf16x8 qf[HD / 16], gf[HD / 16];
  load_row_frags<HD>(qbase, a.ldq, q0, Tq, qf);
  load_row_frags<HD>(dout + (int64_t)b * Tq * d + h * HD, d, q0, Tq, gf);
  const float lse2 = query < Tq ? lse[(int64_t)bh * Tq + query] * kLog2e : INFINITY;   // +inf: P = 0 for rows past the end
  float dl;
  {
    bf16x8 of[HD / 16];
    load_row_frags<HD>(o + (int64_t)b * Tq * d + h * HD, d, q0, Tq, of);
    float part = 0.f;
    if (o_lo) {
      bf16x8 lf[HD / 16];
      load_row_frags<HD>(o_lo + (int64_t)b * Tq * d + h * HD, d, q0, Tq, lf);
#pragma unroll
      for (int kk = 0; kk < HD / 16; ++kk)
#pragma unroll
        for (int e = 0; e < 8; ++e) part += ((float)of[kk][e] + (float)lf[kk][e]) * (float)gf[kk][e];
    } else {
#pragma unroll
      for (int kk = 0; kk < HD / 16; ++kk)
#pragma unroll
        for (int e = 0; e < 8; ++e) part += (float)of[kk][e] * (float)gf[kk][e];
    }
    dl = part + __shfl_xor(part, 32, 64);            // the two halves of the row's features
    if (half == 0 && query < Tq) delta[(int64_t)bh * Tq + query] = dl;
  }
  f32x16 acc[HD / 32];
#pragma unroll
  for (int cb = 0; cb < HD / 32; ++cb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[cb][r] = 0.f;

  const int last_q = min(Tq, (qblk + 1) * 128) - 1;
  const int n_tiles = CAUSAL ? last_q / BKV + 1 : (Tk + BKV - 1) / BKV;
  const int last_key = CAUSAL ? query : Tk - 1;
  TileOffsets<BKV> to;
  to.init(ld, wave, lane);
  auto issue = [&](int t) {
    const uint32_t st = smem_off + (uint32_t)(t & 1) * (2 * kTile * 2);
    issue_tile<BKV>(kbase, ld, t * BKV, Tk - 1, to, st, wave, lane);
    issue_tile<BKV>(vbase, ld, t * BKV, Tk - 1, to, st + kTile * 2, wave, lane);
  };
  issue(0);
  for (int t = 0; t < n_tiles; ++t) {
    const int j0 = t * BKV;
    wait_and_sync();
    if (t + 1 < n_tiles) issue(t + 1);
    if (CAUSAL && j0 > q0 + 31) continue;
    const bf16* Ks = smem + (t & 1) * (2 * kTile);
    const bf16* Vs = Ks + kTile;
    const bool diag = CAUSAL ? j0 + BKV - 1 > q0 : j0 + BKV > Tk;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      f32x16 s = first_product(Ks, kb * 32, qf);      // S^T
      f32x16 dp = first_product(Vs, kb * 32, gf);     // dP^T = V . dO^T
      if (diag) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (j0 + kb * 32 + reg_row(r, half) > last_key) s[r] = -INFINITY;
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = __builtin_amdgcn_exp2f(fmaf(s[r], c2, -lse2)) * (dp[r] - dl);
#pragma unroll
      for (int b2 = 0; b2 < 2; ++b2) second_product(Ks, kb * 32 + b2 * 16, pack8(s, b2 * 8), acc);   // dQ^T += K^T . dS^T
    }
  }
  if (query < Tq) store_row<HD>(dq + ((int64_t)b * Tq + query) * lddq + h * HD, acc, scale);
}

// ===================================================================================================
// dK, dV: block = 128 keys of one (batch, head); wave = 32 keys; query tiles of 64 as two 32-query blocks.
// Software-pipelined: the four phases of a block - first products S and dP, softmax / dS arithmetic on the
// vector ALU, second products into dV and dK - no longer run one after the other.  A wave has one SIMD to itself
// here (its two output accumulators, the K / V fragments and the scores leave no room for a second wave), so
// nothing else hides the latencies: the first products of block n+1 are issued between the vector instructions
// of block n (one score element per MFMA: about as many vector cycles as the MFMA occupies the matrix pipe), and
// the transposed LDS reads of the second products run two MFMAs ahead.  Three tiles are resident (ring of
// three stages): the first products of the next tile start while the second products of the current one still
// read theirs.
// ===================================================================================================
struct DkvStats { float lq[16], dq[16]; };

// This lane's log-sum-exp (scaled for exp2) and delta of the 16 queries its score registers stand for (block hb of
// the tile).
// (Raw values: the scaling of the log-sum-exp is left to the user, so that the reads can be issued a phase early.)
__device__ __forceinline__ void load_stats(const float* Ls, const float* Ds, int hb, int half, DkvStats& st) {
#pragma unroll
  for (int g = 0; g < 2; ++g)
#pragma unroll
    for (int v4 = 0; v4 < 2; ++v4) {
      const int base = hb * 32 + 16 * g + 8 * half + 4 * v4;
      const float4 l = *reinterpret_cast<const float4*>(Ls + base);
      const float4 d = *reinterpret_cast<const float4*>(Ds + base);
      const int r = 8 * g + 4 * v4;
      st.lq[r] = l.x; st.lq[r + 1] = l.y; st.lq[r + 2] = l.z; st.lq[r + 3] = l.w;
      st.dq[r] = d.x; st.dq[r + 1] = d.y; st.dq[r + 2] = d.z; st.dq[r + 3] = d.w;
    }
}

// First products of block `next` (sn = S, dpn = dP against the tile rows rbn .. rbn+31 of Qn / Gn), with - when
// HAVE_CUR - the arithmetic of block `cur` between the MFMAs: s becomes P = exp2(S c2 - lse), ds = P (dP - delta).
// (Masked scores are handled through the statistics: a log-sum-exp of +inf makes P an exact zero.)
template <bool HAVE_NEXT, bool HAVE_CUR>
__device__ __forceinline__ void dkv_front(const bf16* __restrict__ Qn, const bf16* __restrict__ Gn, int rbn,
                                          const bf16x8* kf, const bf16x8* vf, f32x16& sn, f32x16& dpn, f32x16& s,
                                          const f32x16& dp, const DkvStats& st, float c2, bf16x8* pf, bf16x8* dsf) {
  constexpr int kDepth = 3, KK = HD / 16;
  const int lane = threadIdx.x & 63;
  const int row = rbn + perm_row(lane & 31);
  const int t = (lane >> 5) ^ swz(row);
  const bf16* aq = Qn + row * HD;
  const bf16* ag = Gn + row * HD;
  bf16x8 fq[kDepth], fg[kDepth];
  if (HAVE_NEXT) {
#pragma unroll
    for (int r = 0; r < 16; ++r) sn[r] = dpn[r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < kDepth; ++kk) {
      fq[kk] = *reinterpret_cast<const bf16x8*>(aq + ((2 * kk) ^ t) * 8);
      fg[kk] = *reinterpret_cast<const bf16x8*>(ag + ((2 * kk) ^ t) * 8);
    }
  }
  f32x16 ds;
  auto element = [&](int r) {
    if (HAVE_CUR) {
      const float p = __builtin_amdgcn_exp2f(fmaf(s[r], c2, -st.lq[r]));
      s[r] = p;
      ds[r] = p * (dp[r] - st.dq[r]);
    }
  };
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    if (HAVE_NEXT) {
      sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[kk % kDepth], kf[kk], sn, 0, 0, 0);
      if (kk + kDepth < KK) fq[kk % kDepth] = *reinterpret_cast<const bf16x8*>(aq + ((2 * (kk + kDepth)) ^ t) * 8);
    }
    element(2 * kk);
    __builtin_amdgcn_sched_barrier(0);
    if (HAVE_NEXT) {
      dpn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fg[kk % kDepth], vf[kk], dpn, 0, 0, 0);
      if (kk + kDepth < KK) fg[kk % kDepth] = *reinterpret_cast<const bf16x8*>(ag + ((2 * (kk + kDepth)) ^ t) * 8);
    }
    element(2 * kk + 1);
    __builtin_amdgcn_sched_barrier(0);
  }
  if (HAVE_CUR) {
#pragma unroll
    for (int b2 = 0; b2 < 2; ++b2) {
      pf[b2] = pack8(s, b2 * 8);
      dsf[b2] = pack8(ds, b2 * 8);
    }
  }
}

// Second products of a block: dv += Gs^T . P and dk += Qs^T . dS over the 32 queries at tile rows rb .. rb+31,
// 16 MFMAs whose transposed operand reads run kAhead steps ahead.
__device__ __forceinline__ void dkv_back(const bf16* __restrict__ Qs, const bf16* __restrict__ Gs, int rb, const bf16x8* pf,
                                         const bf16x8* dsf, f32x16* dk, f32x16* dv) {
  constexpr int kAhead = 2, kSteps = 16;
  const int lane = threadIdx.x & 63;
  const int grp = lane >> 4, L = lane & 15;
  const int f0 = 16 * (grp & 1) + 4 * (L & 3);
  // step j: b2 = j / 8 (16-query half of the block), mat = (j / 4) % 2 (0: dO -> dV, 1: Q -> dK), cb = j % 4
  auto read = [&](int j) {
    const int b2 = j >> 3, mat = (j >> 2) & 1, cb = j & 3;
    const bf16* tile = mat ? Qs : Gs;
    const int row0 = rb + b2 * 16 + 8 * (grp >> 1) + (L >> 2);
    union { bf16x8 v; short4v h[2]; } u;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int row = row0 + 4 * t;
      const int chunk = (cb * 32 + f0) >> 3;
      const bf16* p = tile + row * HD + ((chunk ^ swz(row)) << 3) + (f0 & 7);
      u.h[t] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)p);
    }
    return u.v;
  };
  bf16x8 fr[kAhead + 1];
#pragma unroll
  for (int j = 0; j < kAhead; ++j) fr[j] = read(j);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int j = 0; j < kSteps; ++j) {
    if (j + kAhead < kSteps) fr[(j + kAhead) % (kAhead + 1)] = read(j + kAhead);
    const int b2 = j >> 3, mat = (j >> 2) & 1, cb = j & 3;
    if (mat) dk[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j % (kAhead + 1)], dsf[b2], dk[cb], 0, 0, 0);
    else dv[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j % (kAhead + 1)], pf[b2], dv[cb], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
}

template <bool CAUSAL>
__global__ __launch_bounds__(kNT) void attn_dkv_dma_kernel(MhaDev a, const bf16* __restrict__ dout,
                                                            const float* __restrict__ lse, const float* __restrict__ delta,
                                                            bf16* __restrict__ dk_out, bf16* __restrict__ dv_out, int64_t lddkv) {
  constexpr int BQ = 64, kStages = 3;
  constexpr int kTile = BQ * HD;
  extern __shared__ __attribute__((aligned(1024))) bf16 smem[];          // [stage][Q | dO], then the statistics
  float (*Ls)[BQ] = reinterpret_cast<float (*)[BQ]>(smem + kStages * 2 * kTile);
  float (*Ds)[BQ] = Ls + kStages;
  const int T = a.Tq, Tk = a.Tk, H = a.H;
  const int d = H * HD;
  const int64_t ld = a.ldq;
  int bh, kblk;                                         // causal: first key blocks see the most queries, they come first
  xcd_block_map(blockIdx.x, gridDim.x, (Tk + 127) / 128, CAUSAL ? causal_group((Tk + 127) / 128, 32) : 1, bh, kblk);
  const int b = bh / H, h = bh - b * H;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, half = lane >> 5;
  const int k0 = kblk * 128 + wave * 32;
  const int key = k0 + (lane & 31);
  const bf16* qbase = a.q + (int64_t)b * T * ld + h * HD;
  const bf16* gbase = dout + (int64_t)b * T * d + h * HD;
  const float scale = 1.f / sqrtf((float)HD);
  const float c2 = kLog2e * scale;
  const uint32_t smem_off = (uint32_t)(uintptr_t)(lds_ptr)smem;

  TileOffsets<BQ> to_q, to_g;
  to_q.init(ld, wave, lane);
  to_g.init(d, wave, lane);
  bf16x8 kf[HD / 16], vf[HD / 16];
  load_row_frags<HD>(a.k + (int64_t)b * Tk * a.ldkv + h * HD, a.ldkv, k0, Tk, kf);
  load_row_frags<HD>(a.v + (int64_t)b * Tk * a.ldkv + h * HD, a.ldkv, k0, Tk, vf);
  f32x16 dk[HD / 32], dv[HD / 32];
#pragma unroll
  for (int cb = 0; cb < HD / 32; ++cb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      dk[cb][r] = 0.f;
      dv[cb][r] = 0.f;
    }

  const int first_tile = CAUSAL ? (kblk * 128) / BQ : 0;
  const int n_tiles = (T + BQ - 1) / BQ;
  // A tile = 64 rows of Q and of dO plus the 64 queries' log-sum-exp and delta; all of it travels global -> LDS
  // directly (no destination registers: the compiler then has no pending load to wait for in the middle of the
  // pipeline, and the loads stay in flight until the explicit wait in front of the tile's barrier).  Statistics of
  // rows past the end are fetched from the last row and masked where they are used.
  const float* lse_bh = lse + (int64_t)bh * T;
  const float* delta_bh = delta + (int64_t)bh * T;
  const uint32_t stats_off = smem_off + kStages * 2 * kTile * 2;
  auto issue = [&](int t) {
    const uint32_t st = smem_off + (uint32_t)(t % kStages) * (2 * kTile * 2);
    issue_tile<BQ>(qbase, ld, t * BQ, T - 1, to_q, st, wave, lane);
    issue_tile<BQ>(gbase, d, t * BQ, T - 1, to_g, st + kTile * 2, wave, lane);
    if (wave == 0) {
      const int i = min(t * BQ + lane, T - 1);
      dma4(lse_bh + i, stats_off + (uint32_t)(t % kStages) * (BQ * 4));
      dma4(delta_bh + i, stats_off + (uint32_t)(kStages + t % kStages) * (BQ * 4));
    }
  };
  // Block n = 2 t + hb covers queries 32 n .. 32 n + 31.  Under the causal mask this wave's keys see the blocks from
  // k0 / 32 on; it starts with the tile that holds that block (waves 2 and 3 of a workgroup one tile after waves 0
  // and 1) and from there on runs every block - an odd first block's even neighbour is computed fully masked, which
  // keeps the pipeline below free of per-wave branches.
  auto tile_q = [&](int n) { return smem + ((n >> 1) % kStages) * (2 * kTile); };
  // What happens between the two blocks of tile t: tile t + 1 has to have landed, for every wave; behind the barrier
  // nobody reads tile t - 1 any more, so its stage takes tile t + 2.
  auto advance = [&](int t) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (t + 2 < n_tiles) issue(t + 2);
  };

  issue(first_tile);
  if (first_tile + 1 < n_tiles) {
    issue(first_tile + 1);
    // all but the second tile: 2 x 4 direct loads per wave, two more (the statistics) in wave 0
    if (wave == 0) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * (BQ / 16) + 2) : "memory");
    else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * (BQ / 16)) : "memory");
  } else {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");

  // Two sets of score registers: the even block of a tile lives in (s0, dp0), the odd one in (s1, dp1), so nothing is
  // ever copied from "next" to "current".
  f32x16 s0, dp0, s1, dp1;
  bf16x8 pf[2], dsf[2];
  DkvStats st;
  // One step of the pipeline: the arithmetic of block n (scores in s, dp) between the first products of block n + 1
  // (into sn, dpn; NEXT: there is one), then the second products of block n.
  auto step = [&](int n, auto next, f32x16& s, f32x16& dp, f32x16& sn, f32x16& dpn) {
    constexpr bool NEXT = decltype(next)::value;
    const int hb = n & 1, t = n >> 1;
    const bf16* Qs = tile_q(n);
    const bf16* Qn = tile_q(n + 1);
    // st holds the block's raw statistics, read from LDS during the previous step
#pragma unroll
    for (int r = 0; r < 16; ++r) st.lq[r] *= kLog2e;
    const int ib = 32 * n;
    // (The empty volatile statements tie the values to the rare branches below: without them the compiler turns the
    // two fix-ups into selects that every block pays for - some 130 vector instructions with their wait states.)
    if (CAUSAL && ib < k0 + 31) {        // a block on (or before) the diagonal: register r stands for query ib + reg_row(r, half)
      const int thr = key - ib - 8 * half;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (16 * (r >> 3) + (r & 7) < thr) st.lq[r] = INFINITY;     // the key may not see this earlier query: P = 0
        asm volatile("" : "+v"(st.lq[r]));
      }
    }
    if (ib + 31 >= T) {                  // the block straddles the end of the queries
      const int thr = T - ib - 8 * half;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (16 * (r >> 3) + (r & 7) >= thr) st.lq[r] = INFINITY;    // no such query: P = 0
        asm volatile("" : "+v"(st.lq[r]));
      }
    }
    dkv_front<NEXT, true>(Qn, Qn + kTile, (hb ^ 1) * 32, kf, vf, sn, dpn, s, dp, st, c2, pf, dsf);
    // the next block's statistics travel to registers under the second products (its tile is resident: see advance)
    if (NEXT) load_stats(Ls[((n + 1) >> 1) % kStages], Ds[((n + 1) >> 1) % kStages], hb ^ 1, half, st);
    dkv_back(Qs, Qs + kTile, hb * 32, pf, dsf, dk, dv);
    // Register classes: the output accumulators and the K / V fragments are only ever touched by MFMAs and live in
    // the accumulation registers; the scores are worked on by the vector ALU and stay in ordinary registers, so no
    // MFMA result has to be copied across (with the wait states that costs).
#pragma unroll
    for (int cb = 0; cb < HD / 32; ++cb) asm volatile("" : "+a"(dk[cb]), "+a"(dv[cb]));
#pragma unroll
    for (int kk = 0; kk < HD / 16; ++kk) asm volatile("" : "+v"(kf[kk]), "+v"(vf[kk]));
  };
  using yes = std::integral_constant<bool, true>;
  using no = std::integral_constant<bool, false>;
  int t0 = first_tile;
  bool any = true;
  if (CAUSAL && wave >= 2) {             // this wave's first tile is the next one
    any = first_tile + 1 < n_tiles;
    if (any) advance(first_tile);
    t0 = first_tile + 1;
  }
  if (any) {
    load_stats(Ls[t0 % kStages], Ds[t0 % kStages], 0, half, st);
    dkv_front<true, false>(tile_q(2 * t0), tile_q(2 * t0) + kTile, 0, kf, vf, s0, dp0, s0, dp0, st, c2, pf, dsf);
    for (int t = t0; t + 1 < n_tiles; ++t) {
      step(2 * t, yes{}, s0, dp0, s1, dp1);
      advance(t);
      step(2 * t + 1, yes{}, s1, dp1, s0, dp0);
    }
    step(2 * (n_tiles - 1), yes{}, s0, dp0, s1, dp1);
    step(2 * (n_tiles - 1) + 1, no{}, s1, dp1, s0, dp0);
  }
  if (key < Tk) {
    const int64_t row = ((int64_t)b * Tk + key) * lddkv + h * HD;
    store_row<HD>(dk_out + row, dk, scale);
    store_row<HD>(dv_out + row, dv, 1.f);
  }
}

}  // namespace

constexpr int kSmemTiles = 2 * 2 * 64 * HD * 2;          // two stages of two 64 x 128 bf16 tiles: 64 KiB
constexpr int kSmemDkv = 3 * 2 * 64 * HD * 2 + 6 * 64 * 4;   // dK/dV: three stages and their statistics: 97.5 KiB

// Raises the dynamic-LDS limit of the kernels (once; called at context creation, never inside a capture).
hipError_t attention_dma_init() {
  static bool done = false;
  if (done) return hipSuccess;
  const struct { const void* fn; int bytes; } all[] = {
      {reinterpret_cast<const void*>(attn_fwd_dma_kernel<true>), kSmemTiles},
      {reinterpret_cast<const void*>(attn_fwd_dma_kernel<false>), kSmemTiles},
      {reinterpret_cast<const void*>(attn_dq_dma_kernel<true>), kSmemTiles},
      {reinterpret_cast<const void*>(attn_dq_dma_kernel<false>), kSmemTiles},
      {reinterpret_cast<const void*>(attn_dkv_dma_kernel<true>), kSmemDkv},
      {reinterpret_cast<const void*>(attn_dkv_dma_kernel<false>), kSmemDkv}};
  for (const auto& k : all) {
    const hipError_t e = hipFuncSetAttribute(k.fn, hipFuncAttributeMaxDynamicSharedMemorySize, k.bytes);
    if (e != hipSuccess) return e;
  }
  done = true;
  return hipSuccess;
}

static MhaDev dev_of(const MhaArgs& a) {
  return MhaDev{(const bf16*)a.q, (const bf16*)a.k, (const bf16*)a.v, a.ldq, a.ldkv, a.Tq, a.Tk, a.H};
}

// Whether the kernels of this file take the problem: bf16, head_dim 128, 16-byte aligned rows.
bool mha_dma_supported(const MhaArgs& a) {
  if (a.dtype != kBF16 || a.hd != HD) return false;
  if (((uintptr_t)a.q | (uintptr_t)a.k | (uintptr_t)a.v) & 15) return false;
  return a.ldq % 8 == 0 && a.ldkv % 8 == 0;
}

hipError_t launch_mha_fwd_dma(hipStream_t s, const MhaArgs& a, void* o, void* o_lo, float* lse) {
  hipError_t e = attention_dma_init();
  if (e != hipSuccess) return e;
  const int grid = ((a.Tq + 127) / 128) * a.B * a.H;          // (problem, block) pairs, see xcd_block_map
  if (a.causal)
    attn_fwd_dma_kernel<true><<<grid, kNT, kSmemTiles, s>>>(dev_of(a), (bf16*)o, (bf16*)o_lo, lse);
  else
    attn_fwd_dma_kernel<false><<<grid, kNT, kSmemTiles, s>>>(dev_of(a), (bf16*)o, (bf16*)o_lo, lse);
  return hipGetLastError();
}

hipError_t launch_mha_dq_dkv_dma(hipStream_t s, const MhaArgs& a, const void* o, const void* o_lo, const void* dout,
                                 const float* lse, float* delta, void* dq, int64_t lddq, void* dk, void* dv, int64_t lddkv) {
  hipError_t e = attention_dma_init();
  if (e != hipSuccess) return e;
  if ((((uintptr_t)dq | (uintptr_t)dk | (uintptr_t)dv) & 7) || lddq % 4 || lddkv % 4) return hipErrorInvalidValue;
  const int grid_q = ((a.Tq + 127) / 128) * a.B * a.H, grid_k = ((a.Tk + 127) / 128) * a.B * a.H;
  const MhaDev dv_ = dev_of(a);
  if (a.causal) {
    attn_dq_dma_kernel<true><<<grid_q, kNT, kSmemTiles, s>>>(dv_, (const bf16*)o, (const bf16*)o_lo, (const bf16*)dout, lse, delta, (bf16*)dq, lddq);
    attn_dkv_dma_kernel<true><<<grid_k, kNT, kSmemDkv, s>>>(dv_, (const bf16*)dout, lse, delta, (bf16*)dk, (bf16*)dv, lddkv);
  } else {
    attn_dq_dma_kernel<false><<<grid_q, kNT, kSmemTiles, s>>>(dv_, (const bf16*)o, (const bf16*)o_lo, (const bf16*)dout, lse, delta, (bf16*)dq, lddq);
    attn_dkv_dma_kernel<false><<<grid_k, kNT, kSmemDkv, s>>>(dv_, (const bf16*)dout, lse, delta, (bf16*)dk, (bf16*)dv, lddkv);
  }
  return hipGetLastError();
}

}  // namespace pw
