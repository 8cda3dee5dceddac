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
// dK, dV: block = 128 keys of one (batch, head); wave = 32 keys; query tiles of 64 (two 32-row halves)
// ===================================================================================================
template <bool CAUSAL>
__global__ __launch_bounds__(kNT) void attn_dkv_dma_kernel(MhaDev a, const bf16* __restrict__ dout,
                                                           const float* __restrict__ lse, const float* __restrict__ delta,
                                                           bf16* __restrict__ dk_out, bf16* __restrict__ dv_out, int64_t lddkv) {
  constexpr int BQ = 64;
  constexpr int kTile = BQ * HD;
  extern __shared__ __attribute__((aligned(1024))) bf16 smem[];          // [stage][Q | dO], then the statistics
  float (*Ls)[BQ] = reinterpret_cast<float (*)[BQ]>(smem + 2 * 2 * kTile);
  float (*Ds)[BQ] = Ls + 2;
  const int T = a.Tq, Tk = a.Tk, H = a.H;               // T: number of queries (the streamed side)
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
  TileOffsets<BQ> to_q, to_g;
  to_q.init(ld, wave, lane);
  to_g.init(d, wave, lane);
  auto issue = [&](int t) {
    const uint32_t st = smem_off + (uint32_t)(t & 1) * (2 * kTile * 2);
    issue_tile<BQ>(qbase, ld, t * BQ, T - 1, to_q, st, wave, lane);
    issue_tile<BQ>(gbase, d, t * BQ, T - 1, to_g, st + kTile * 2, wave, lane);
  };
  // per-query statistics of a tile: fetched one tile ahead into registers by the first 64 threads
  float l_next = 0.f, d_next = 0.f;
  auto fetch_stats = [&](int t) {
    if (threadIdx.x < BQ) {
      const int i = t * BQ + threadIdx.x;
      l_next = i < T ? lse[(int64_t)bh * T + i] * kLog2e : INFINITY;   // +inf: P = 0 for queries past the end
      d_next = i < T ? delta[(int64_t)bh * T + i] : 0.f;
    }
  };
  fetch_stats(first_tile);
  issue(first_tile);
  for (int t = first_tile; t < n_tiles; ++t) {
    const int i0 = t * BQ;
    if (threadIdx.x < BQ) {          // stage t&1 of the statistics was last read two tiles ago
      Ls[t & 1][threadIdx.x] = l_next;
      Ds[t & 1][threadIdx.x] = d_next;
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the two LDS stores above are done before the barrier
    wait_and_sync();
    if (t + 1 < n_tiles) {
      issue(t + 1);
      fetch_stats(t + 1);
    }
    const bf16* Qs = smem + (t & 1) * (2 * kTile);
    const bf16* Gs = Qs + kTile;
#pragma unroll
    for (int hb = 0; hb < 2; ++hb) {                     // the two 32-query halves of the tile
      const int ib = i0 + hb * 32;
      if (CAUSAL && ib + 31 < k0) continue;              // every query of this half precedes this wave's keys
      f32x16 s = first_product(Qs, hb * 32, kf);         // S[query][key]
      f32x16 dp = first_product(Gs, hb * 32, vf);        // dP = dO . V^T
      if (CAUSAL && ib < k0 + 31) {                      // diagonal: a key may not see an earlier query
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (key > ib + reg_row(r, half)) s[r] = -INFINITY;
      }
      f32x16 ds;
#pragma unroll
      for (int g = 0; g < 2; ++g)
#pragma unroll
        for (int v4 = 0; v4 < 2; ++v4) {
          const int base = hb * 32 + 16 * g + 8 * half + 4 * v4;
          const float4 lq = *reinterpret_cast<const float4*>(&Ls[t & 1][base]);
          const float4 dq = *reinterpret_cast<const float4*>(&Ds[t & 1][base]);
          const float lqa[4] = {lq.x, lq.y, lq.z, lq.w}, dqa[4] = {dq.x, dq.y, dq.z, dq.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int r = 8 * g + 4 * v4 + e;
            const float p = __builtin_amdgcn_exp2f(fmaf(s[r], c2, -lqa[e]));
            s[r] = p;
            ds[r] = p * (dp[r] - dqa[e]);
          }
        }
#pragma unroll
      for (int b2 = 0; b2 < 2; ++b2) {
        second_product(Gs, hb * 32 + b2 * 16, pack8(s, b2 * 8), dv);    // dV^T += dO^T . P
        second_product(Qs, hb * 32 + b2 * 16, pack8(ds, b2 * 8), dk);   // dK^T += Q^T . dS
      }
      // Register classes: the two output accumulators are only ever touched by MFMAs, so they belong in the
      // accumulation registers; the K/V fragments feed MFMAs as ordinary operands.  Without the hint the
      // allocator parks the fragments and the score accumulators there and copies them back and forth.
#pragma unroll
      for (int cb = 0; cb < HD / 32; ++cb) asm volatile("" : "+a"(dk[cb]), "+a"(dv[cb]));
#pragma unroll
      for (int kk = 0; kk < HD / 16; ++kk) asm volatile("" : "+v"(kf[kk]), "+v"(vf[kk]));
    }
  }
  if (key < Tk) {
    const int64_t row = ((int64_t)b * Tk + key) * lddkv + h * HD;
    store_row<HD>(dk_out + row, dk, scale);
    store_row<HD>(dv_out + row, dv, 1.f);
  }
}

}  // namespace

constexpr int kSmemTiles = 2 * 2 * 64 * HD * 2;          // two stages of two 64 x 128 bf16 tiles: 64 KiB
constexpr int kSmemDkv = kSmemTiles + 4 * 64 * 4;        // + log-sum-exp and delta of two query tiles

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
