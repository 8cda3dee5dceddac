// bf16 MFMA attention: forward, dQ, and dK/dV kernels (v_mfma_f32_32x32x16_bf16, wave64).
//
// Register-layout facts everything below rests on (D = A.B, 32x32 output, k = 16 per instruction):
//   A operand: lane l supplies row l%32, k-slots 8*(l/32) .. +7        (8 bf16)
//   B operand: lane l supplies column l%32, the same k-slots
//   D:         lane l holds column l%32; register r holds row 8*(r/4) + 4*(l/32) + r%4
// The contraction only needs A and B to agree on what k-slot (half h, element e) means.
//
// All three kernels put the softmax row index on the D *column*, i.e. on the lane, so that row
// statistics (max, sum, log-sum-exp, delta) are one value per lane and never need a transpose:
//   forward / dQ :  S^T[key][query] = K . Q^T      (A = K tile from LDS, B = Q fragments in registers)
//   dK/dV        :  S[query][key]   = Q . K^T      (A = Q tile from LDS, B = K fragments in registers)
// The second product consumes P (or dS) straight from the D registers as its B operand.  For that the 16
// rows a lane holds in registers 0..7 / 8..15 must be the 8 k-slots of its half for the first / second
// k=16 step.  That is arranged by reading the A tile of the FIRST product with permuted rows: MFMA row i
// is fed tile row perm(i), perm = [0-3, 8-11, 4-7, 12-15] within every 16, so that register r of half h
// corresponds to tile row 16*(r/8) + 8*h + r%8.  LDS reads are lane-addressed, so this costs nothing.
// The second product's A operand needs the tile transposed ([feature][row], rows contiguous); tiles are
// written to LDS in both forms from one set of global loads (4 rows x 8 features per thread, regrouped
// with v_perm_b32).
//
// Determinism: no atomics.  dQ is accumulated by the block that owns the queries, dK/dV by the block that
// owns the keys, each over its tiles in ascending order (two kernels, S recomputed in both).
#include "attention_common.hpp"
#include "common.hpp"
#include "kernels.hpp"

#include <cstdlib>

namespace pw {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kNT = 256;           // threads per block: 4 waves

// One tile of ROWS rows x HD features, fetched as 4-row x 8-feature pieces.
template <int ROWS, int HD>
struct Tile {
  static constexpr int kPieces = (ROWS / 4) * (HD / 8);
  static constexpr int CNT = (kPieces + kNT - 1) / kNT;
  static constexpr int kLdNat = HD + 8;     // [row][feature] layout
  static constexpr int kLdTr = ROWS + 8;    // [feature][row] layout
  u32x4 reg[CNT][4];

  // Which 8-feature chunk (fc) and which 4-row group (rq) piece p covers.  A 32-lane half-wave gets two
  // adjacent feature chunks x the row groups: its 8-byte transposed LDS stores then fall on distinct banks
  // (the bank depends on fc only through its parity).
  static constexpr int kRqBits = ROWS == 64 ? 4 : 3;
  static_assert(ROWS == 64 || ROWS == 32, "tile heights used by the kernels");
  static __device__ __forceinline__ int piece_fc(int p) { return (p & 1) | ((p >> (1 + kRqBits)) << 1); }
  static __device__ __forceinline__ int piece_rq(int p) { return (p >> 1) & (ROWS / 4 - 1); }

  // src: element (row 0, feature 0); ld: row stride in elements; rows at or past `limit` read as zero.
  __device__ __forceinline__ void load(const bf16* __restrict__ src, int64_t ld, int row0, int limit) {
#pragma unroll
    for (int i = 0; i < CNT; ++i) {
      const int p = threadIdx.x + i * kNT;
      const int fc = piece_fc(p), rq = piece_rq(p);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int row = row0 + rq * 4 + j;
        if ((kPieces % kNT == 0 || p < kPieces) && row < limit)
          reg[i][j] = *reinterpret_cast<const u32x4*>(src + (int64_t)row * ld + fc * 8);
        else
          reg[i][j] = u32x4{0, 0, 0, 0};
      }
    }
  }
  __device__ __forceinline__ void store_nat(bf16* __restrict__ lds) const {
#pragma unroll
    for (int i = 0; i < CNT; ++i) {
      const int p = threadIdx.x + i * kNT;
      if (kPieces % kNT != 0 && p >= kPieces) continue;
      const int fc = piece_fc(p), rq = piece_rq(p);
#pragma unroll
      for (int j = 0; j < 4; ++j) *reinterpret_cast<u32x4*>(lds + (rq * 4 + j) * kLdNat + fc * 8) = reg[i][j];
    }
  }
  __device__ __forceinline__ void store_tr(bf16* __restrict__ lds) const {
#pragma unroll
    for (int i = 0; i < CNT; ++i) {
      const int p = threadIdx.x + i * kNT;
      if (kPieces % kNT != 0 && p >= kPieces) continue;
      const int fc = piece_fc(p), rq = piece_rq(p);
      const u32x4 w0 = reg[i][0], w1 = reg[i][1], w2 = reg[i][2], w3 = reg[i][3];
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) {
        u32x2 lo, hi;   // features 2*e2 and 2*e2+1 of the piece, 4 consecutive rows each
        lo.x = __builtin_amdgcn_perm(w1[e2], w0[e2], 0x05040100u);
        lo.y = __builtin_amdgcn_perm(w3[e2], w2[e2], 0x05040100u);
        hi.x = __builtin_amdgcn_perm(w1[e2], w0[e2], 0x07060302u);
        hi.y = __builtin_amdgcn_perm(w3[e2], w2[e2], 0x07060302u);
        *reinterpret_cast<u32x2*>(lds + (fc * 8 + 2 * e2) * kLdTr + rq * 4) = lo;
        *reinterpret_cast<u32x2*>(lds + (fc * 8 + 2 * e2 + 1) * kLdTr + rq * 4) = hi;
      }
    }
  }
};

// 32x32 block of a first product: A rows from a natural-layout LDS tile (permuted), B from register fragments.
template <int HD, int LDN>
__device__ __forceinline__ f32x16 first_product(const bf16* __restrict__ tile, int row_base, const bf16x8* bfrag) {
  const int lane = threadIdx.x & 63;
  const bf16* a = tile + (row_base + perm_row(lane & 31)) * LDN + (lane >> 5) * 8;
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
  for (int kk = 0; kk < HD / 16; ++kk)
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(a + kk * 16), bfrag[kk], acc, 0, 0, 0);
  return acc;
}

// acc[cb] += T^T[feature block cb][rows kb*32 + 16 b ..] . frag   for a transposed LDS tile (ld = LDT)
template <int HD, int LDT>
__device__ __forceinline__ void second_product(const bf16* __restrict__ tile_tr, int row_base, const bf16x8& frag, f32x16* acc) {
  const int lane = threadIdx.x & 63;
  const bf16* a = tile_tr + (lane & 31) * LDT + row_base + (lane >> 5) * 8;
#pragma unroll
  for (int cb = 0; cb < HD / 32; ++cb)
    acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(a + cb * 32 * LDT), frag, acc[cb], 0, 0, 0);
}

// ===================================================================================================
// forward: block = 128 queries of one (batch, head); wave = 32 queries; key/value tiles of 64
// ===================================================================================================
template <int HD>
__global__ __launch_bounds__(kNT, 2) void attn_fwd_kernel(const bf16* __restrict__ qkv, bf16* __restrict__ o,
                                                       float* __restrict__ lse, int T, int H) {
  constexpr int BKV = 64;
  using KT = Tile<BKV, HD>;
  __shared__ __attribute__((aligned(16))) bf16 Ks[BKV * KT::kLdNat];
  __shared__ __attribute__((aligned(16))) bf16 Vt[HD * KT::kLdTr];
  const int d = H * HD;
  const int64_t ld = 3 * (int64_t)d;
  const int bh = blockIdx.y, b = bh / H, h = bh - b * H;
  const int qblk = gridDim.x - 1 - blockIdx.x;          // longest blocks first
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5;
  const int q0 = qblk * 128 + wave * 32;
  const int query = q0 + (lane & 31);
  const bf16* qbase = qkv + (int64_t)b * T * ld + h * HD;
  const bf16* kbase = qbase + d;
  const bf16* vbase = qbase + 2 * d;
  const float c2 = kLog2e / sqrtf((float)HD);

  bf16x8 qf[HD / 16];
  load_row_frags<HD>(qbase, ld, q0, T, qf);
  f32x16 acc[HD / 32];
#pragma unroll
  for (int cb = 0; cb < HD / 32; ++cb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[cb][r] = 0.f;
  float m = -INFINITY, l = 0.f;

  const int last_q = min(T, (qblk + 1) * 128) - 1;
  const int n_tiles = last_q / BKV + 1;
  KT kt, vt;
  kt.load(kbase, ld, 0, T);
  vt.load(vbase, ld, 0, T);
  for (int t = 0; t < n_tiles; ++t) {
    const int j0 = t * BKV;
    __syncthreads();            // everyone is done with the previous tile
    kt.store_nat(Ks);
    vt.store_tr(Vt);
    __syncthreads();
    if (t + 1 < n_tiles) {
      kt.load(kbase, ld, j0 + BKV, T);
      vt.load(vbase, ld, j0 + BKV, T);
    }
    if (j0 > q0 + 31) continue;   // every key of the tile lies in this wave's future
    f32x16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) s[kb] = first_product<HD, KT::kLdNat>(Ks, kb * 32, qf);
    if (j0 + BKV - 1 > q0) {        // the tile straddles the diagonal for this wave: mask key > query
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (j0 + kb * 32 + reg_row(r, half) > query) s[kb][r] = -INFINITY;
    }
    // row maximum of the raw scores (the scale is positive, so it commutes with max)
    float mx = fmaxf(s[0][0], s[1][0]);
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, fmaxf(s[0][r], s[1][r]));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * c2;
    // Lazy rescaling: the running reference m only has to bound the exponents, not equal the maximum.  It is
    // moved (and the accumulators rescaled) only when some row's maximum grew by more than 2^8; otherwise
    // exp2(s - m) <= 256 and nothing can overflow.  Same mathematics, far fewer multiplies.
    if (__builtin_amdgcn_ballot_w64(mx > m + 8.f) != 0) {
      const float m_new = fmaxf(m, mx);
      const float alpha = __builtin_amdgcn_exp2f(m - m_new);      // m = -inf on the first tile: exp2(-inf) = 0
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
      for (int b2 = 0; b2 < 2; ++b2) second_product<HD, KT::kLdTr>(Vt, kb * 32 + b2 * 16, pack8(s[kb], b2 * 8), acc);
  }
  l += __shfl_xor(l, 32, 64);
  if (query < T) {
    store_row<HD>(o + ((int64_t)b * T + query) * d + h * HD, acc, 1.f / l);
    if (half == 0) lse[(int64_t)bh * T + query] = (m + __builtin_amdgcn_logf(l)) * kLn2;   // v_log_f32 is log2
  }
}

// ===================================================================================================
// dQ: same tiling as the forward.  dQ_i = scale * sum_j dS_ij K_j, dS = P (dP - delta)
// ===================================================================================================
template <int HD>
__global__ __launch_bounds__(kNT, 2) void attn_dq_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ dout,
                                                      const float* __restrict__ lse, const float* __restrict__ delta,
                                                      bf16* __restrict__ dqkv, int T, int H) {
  constexpr int BKV = 64;
  using KT = Tile<BKV, HD>;
  __shared__ __attribute__((aligned(16))) bf16 Ks[BKV * KT::kLdNat];
  __shared__ __attribute__((aligned(16))) bf16 Vs[BKV * KT::kLdNat];
  __shared__ __attribute__((aligned(16))) bf16 Kt[HD * KT::kLdTr];
  const int d = H * HD;
  const int64_t ld = 3 * (int64_t)d;
  const int bh = blockIdx.y, b = bh / H, h = bh - b * H;
  const int qblk = gridDim.x - 1 - blockIdx.x;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5;
  const int q0 = qblk * 128 + wave * 32;
  const int query = q0 + (lane & 31);
  const bf16* qbase = qkv + (int64_t)b * T * ld + h * HD;
  const bf16* kbase = qbase + d;
  const bf16* vbase = qbase + 2 * d;
  const float scale = 1.f / sqrtf((float)HD);
  const float c2 = kLog2e * scale;

  bf16x8 qf[HD / 16], gf[HD / 16];
  load_row_frags<HD>(qbase, ld, q0, T, qf);
  load_row_frags<HD>(dout + (int64_t)b * T * d + h * HD, d, q0, T, gf);
  const float lse2 = query < T ? lse[(int64_t)bh * T + query] * kLog2e : INFINITY;   // +inf: P = 0 for rows past the end
  const float dl = query < T ? delta[(int64_t)bh * T + query] : 0.f;
  f32x16 acc[HD / 32];
#pragma unroll
  for (int cb = 0; cb < HD / 32; ++cb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[cb][r] = 0.f;

  const int last_q = min(T, (qblk + 1) * 128) - 1;
  const int n_tiles = last_q / BKV + 1;
  KT kt, vt;
  kt.load(kbase, ld, 0, T);
  vt.load(vbase, ld, 0, T);
  for (int t = 0; t < n_tiles; ++t) {
    const int j0 = t * BKV;
    __syncthreads();
    kt.store_nat(Ks);
    kt.store_tr(Kt);
    vt.store_nat(Vs);
    __syncthreads();
    if (t + 1 < n_tiles) {
      kt.load(kbase, ld, j0 + BKV, T);
      vt.load(vbase, ld, j0 + BKV, T);
    }
    if (j0 > q0 + 31) continue;
    const bool diag = j0 + BKV - 1 > q0;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      f32x16 s = first_product<HD, KT::kLdNat>(Ks, kb * 32, qf);      // S^T
      f32x16 dp = first_product<HD, KT::kLdNat>(Vs, kb * 32, gf);     // dP^T = V . dO^T
      if (diag) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (j0 + kb * 32 + reg_row(r, half) > query) s[r] = -INFINITY;      // exp2(-inf) = 0
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = __builtin_amdgcn_exp2f(fmaf(s[r], c2, -lse2)) * (dp[r] - dl);
#pragma unroll
      for (int b2 = 0; b2 < 2; ++b2) second_product<HD, KT::kLdTr>(Kt, kb * 32 + b2 * 16, pack8(s, b2 * 8), acc);
    }
  }
  if (query < T) store_row<HD>(dqkv + ((int64_t)b * T + query) * ld + h * HD, acc, scale);
}

// ===================================================================================================
// dK, dV: block = 128 keys of one (batch, head); wave = 32 keys; query tiles of 32
// ===================================================================================================
template <int HD>
__global__ __launch_bounds__(kNT, HD == 64 ? 2 : 1) void attn_dkv_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ dout,
                                                       const float* __restrict__ lse, const float* __restrict__ delta,
                                                       bf16* __restrict__ dqkv, int T, int H) {
  constexpr int BQ = 32;
  using QT = Tile<BQ, HD>;
  __shared__ __attribute__((aligned(16))) bf16 Qs[BQ * QT::kLdNat];
  __shared__ __attribute__((aligned(16))) bf16 Gs[BQ * QT::kLdNat];
  __shared__ __attribute__((aligned(16))) bf16 Qt[HD * QT::kLdTr];
  __shared__ __attribute__((aligned(16))) bf16 Gt[HD * QT::kLdTr];
  __shared__ __attribute__((aligned(16))) float Ls[BQ];
  __shared__ __attribute__((aligned(16))) float Ds[BQ];
  const int d = H * HD;
  const int64_t ld = 3 * (int64_t)d;
  const int bh = blockIdx.y, b = bh / H, h = bh - b * H;
  const int kblk = blockIdx.x;                          // first key blocks see the most queries: they come first
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5;
  const int k0 = kblk * 128 + wave * 32;
  const int key = k0 + (lane & 31);
  const bf16* qbase = qkv + (int64_t)b * T * ld + h * HD;
  const bf16* gbase = dout + (int64_t)b * T * d + h * HD;
  const float scale = 1.f / sqrtf((float)HD);
  const float c2 = kLog2e * scale;

  bf16x8 kf[HD / 16], vf[HD / 16];
  load_row_frags<HD>(qbase + d, ld, k0, T, kf);
  load_row_frags<HD>(qbase + 2 * d, ld, k0, T, vf);
  f32x16 dk[HD / 32], dv[HD / 32];
#pragma unroll
  for (int cb = 0; cb < HD / 32; ++cb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      dk[cb][r] = 0.f;
      dv[cb][r] = 0.f;
    }

  const int first_tile = (kblk * 128) / BQ;
  const int n_tiles = (T + BQ - 1) / BQ;
  QT qt, gt;
  float l_next = 0.f, d_next = 0.f;
  auto fetch = [&](int i0) {
    qt.load(qbase, ld, i0, T);
    gt.load(gbase, d, i0, T);
    if (threadIdx.x < BQ) {
      const int i = i0 + threadIdx.x;
      l_next = i < T ? lse[(int64_t)bh * T + i] * kLog2e : INFINITY;
      d_next = i < T ? delta[(int64_t)bh * T + i] : 0.f;
    }
  };
  fetch(first_tile * BQ);
  for (int t = first_tile; t < n_tiles; ++t) {
    const int i0 = t * BQ;
    __syncthreads();
    qt.store_nat(Qs);
    qt.store_tr(Qt);
    gt.store_nat(Gs);
    gt.store_tr(Gt);
    if (threadIdx.x < BQ) {
      Ls[threadIdx.x] = l_next;
      Ds[threadIdx.x] = d_next;
    }
    __syncthreads();
    if (t + 1 < n_tiles) fetch(i0 + BQ);
    if (i0 + BQ - 1 < k0) continue;        // every query of the tile precedes this wave's keys
    f32x16 s = first_product<HD, QT::kLdNat>(Qs, 0, kf);       // S[query][key]
    f32x16 dp = first_product<HD, QT::kLdNat>(Gs, 0, vf);      // dP = dO . V^T
    // statistics of the 16 queries this lane's registers stand for: rows 8h..8h+7 and 16+8h..16+8h+7
    float lq[16], dq[16];
#pragma unroll
    for (int g = 0; g < 2; ++g)
#pragma unroll
      for (int v4 = 0; v4 < 2; ++v4) {
        const float4 a = *reinterpret_cast<const float4*>(&Ls[16 * g + 8 * half + 4 * v4]);
        const float4 c = *reinterpret_cast<const float4*>(&Ds[16 * g + 8 * half + 4 * v4]);
        lq[8 * g + 4 * v4] = a.x; lq[8 * g + 4 * v4 + 1] = a.y; lq[8 * g + 4 * v4 + 2] = a.z; lq[8 * g + 4 * v4 + 3] = a.w;
        dq[8 * g + 4 * v4] = c.x; dq[8 * g + 4 * v4 + 1] = c.y; dq[8 * g + 4 * v4 + 2] = c.z; dq[8 * g + 4 * v4 + 3] = c.w;
      }
    if (i0 < k0 + 31) {              // diagonal tile: a key may not see an earlier query
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (key > i0 + reg_row(r, half)) s[r] = -INFINITY;
    }
    f32x16 ds;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float p = __builtin_amdgcn_exp2f(fmaf(s[r], c2, -lq[r]));
      s[r] = p;
      ds[r] = p * (dp[r] - dq[r]);
    }
#pragma unroll
    for (int b2 = 0; b2 < 2; ++b2) {
      second_product<HD, QT::kLdTr>(Gt, b2 * 16, pack8(s, b2 * 8), dv);    // dV^T += dO^T . P
      second_product<HD, QT::kLdTr>(Qt, b2 * 16, pack8(ds, b2 * 8), dk);   // dK^T += Q^T . dS
    }
  }
  if (key < T) {
    bf16* row = dqkv + ((int64_t)b * T + key) * ld + h * HD;
    store_row<HD>(row + d, dk, scale);
    store_row<HD>(row + 2 * d, dv, 1.f);
  }
}

// delta[b,h,i] = sum_c dO[i,c] O[i,c].  16 lanes share one (token, head) row of 128 (8 lanes for 64).
template <int HD>
__global__ void attn_delta_kernel(const bf16* __restrict__ o, const bf16* __restrict__ dout, float* __restrict__ delta,
                                  int T, int H, int64_t rows) {
  constexpr int LPR = HD / 8;                       // lanes per row
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t row = gid / LPR;                    // (token n, head h) flattened: n*H + h
  const int part = (int)(gid % LPR);
  float s = 0.f;
  if (row < rows) {
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(o + row * HD + part * 8);
    const bf16x8 g = *reinterpret_cast<const bf16x8*>(dout + row * HD + part * 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) s += (float)a[e] * (float)g[e];
  }
#pragma unroll
  for (int off = LPR / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
  if (row < rows && part == 0) {
    const int64_t n = row / H;
    const int hh = (int)(row - n * H);
    const int64_t bb = n / T, t = n - bb * T;
    delta[(bb * H + hh) * T + t] = s;
  }
}

}  // namespace

bool attention_mfma_supported(int T, int hd) { return T >= 1 && (hd == 64 || hd == 128); }

hipError_t launch_attention_fwd_mfma(hipStream_t s, const void* qkv, void* o, float* lse, int B, int T, int H, int hd) {
  if (!qkv || !o || !lse || B <= 0 || T <= 0 || H <= 0 || (int64_t)B * H > 65535) return hipErrorInvalidValue;
  if (((uintptr_t)qkv | (uintptr_t)o) & 15) return hipErrorInvalidValue;
  dim3 grid((T + 127) / 128, B * H);
  if (hd == 128)
    attn_fwd_kernel<128><<<grid, kNT, 0, s>>>((const bf16*)qkv, (bf16*)o, lse, T, H);
  else if (hd == 64)
    attn_fwd_kernel<64><<<grid, kNT, 0, s>>>((const bf16*)qkv, (bf16*)o, lse, T, H);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_attention_bwd_mfma(hipStream_t s, const void* qkv, const void* o, const void* dout, const float* lse,
                                     float* delta, void* dqkv, int B, int T, int H, int hd) {
  if (!qkv || !o || !dout || !lse || !delta || !dqkv || B <= 0 || T <= 0 || H <= 0 || (int64_t)B * H > 65535)
    return hipErrorInvalidValue;
  if (((uintptr_t)qkv | (uintptr_t)o | (uintptr_t)dout | (uintptr_t)dqkv) & 15) return hipErrorInvalidValue;
  if (hd != 64 && hd != 128) return hipErrorInvalidValue;
  const int64_t rows = (int64_t)B * T * H;
  const int64_t threads = rows * (hd / 8);
  dim3 grid((T + 127) / 128, B * H);
  if (hd == 128) {
    attn_delta_kernel<128><<<(unsigned)((threads + 255) / 256), 256, 0, s>>>((const bf16*)o, (const bf16*)dout, delta, T, H, rows);
    attn_dq_kernel<128><<<grid, kNT, 0, s>>>((const bf16*)qkv, (const bf16*)dout, lse, delta, (bf16*)dqkv, T, H);
    attn_dkv_kernel<128><<<grid, kNT, 0, s>>>((const bf16*)qkv, (const bf16*)dout, lse, delta, (bf16*)dqkv, T, H);
  } else {
    attn_delta_kernel<64><<<(unsigned)((threads + 255) / 256), 256, 0, s>>>((const bf16*)o, (const bf16*)dout, delta, T, H, rows);
    attn_dq_kernel<64><<<grid, kNT, 0, s>>>((const bf16*)qkv, (const bf16*)dout, lse, delta, (bf16*)dqkv, T, H);
    attn_dkv_kernel<64><<<grid, kNT, 0, s>>>((const bf16*)qkv, (const bf16*)dout, lse, delta, (bf16*)dqkv, T, H);
  }
  return hipGetLastError();
}

}  // namespace pw
