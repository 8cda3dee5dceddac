// Pieces shared by the GEMM kernels: epilogue parameters and functions, tile mapping.
#pragma once
#include "common.hpp"
#include "kernels.hpp"

namespace pw {

struct EpiParams {
  int mode, out_bf16, accumulate;
  const float* bias;
  const void* aux;
  void* C;
  void* C2;
  int64_t ldc;
  // kEpiAdam (see AdamEpi): arrays laid out like C; ad_c: device pointer to the two bias corrections, or null
  // (then ad_ic1, ad_ic2 hold them)
  float *ad_w, *ad_m, *ad_v;
  bf16* ad_wlp;
  const float* ad_c;
  float ad_lr, ad_b1, ad_b2, ad_eps, ad_ic1, ad_ic2;
  // kEpiXentStats / kEpiXentGrad (see XentEpi); xe_groups = N / 64
  const int32_t* xe_tokens;
  float* xe_part;
  float* xe_zt;
  const float* xe_lse;
  float xe_inv_n;
  int xe_T, xe_V, xe_groups;
};

__device__ __forceinline__ bool epi_has_bias(int mode) {
  return mode == kEpiBias || mode == kEpiBiasResidual || mode == kEpiBiasGelu;
}

// Epilogue on 4 consecutive columns n0..n0+3 of row m.  AUXT: element type of aux for kEpiGeluBwd / of the
// outputs when out_bf16 (the activation type).
template <bool BF16ACT>
__device__ __forceinline__ void epilogue4(const EpiParams& e, int64_t m, int64_t n0, float v0, float v1, float v2, float v3) {
  const int64_t off = m * e.ldc + n0;
  if (epi_has_bias(e.mode) && e.bias) {
    const float4 b = *reinterpret_cast<const float4*>(e.bias + n0);
    v0 += b.x; v1 += b.y; v2 += b.z; v3 += b.w;
  }
  float h0 = 0.f, h1 = 0.f, h2 = 0.f, h3 = 0.f;
  const bool two = e.mode == kEpiBiasGelu;
  if (two) {
    h0 = gelu_f(v0); h1 = gelu_f(v1); h2 = gelu_f(v2); h3 = gelu_f(v3);
  }
  if (e.mode == kEpiBiasResidual) {
    const float4 r = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(e.aux) + off);
    v0 += r.x; v1 += r.y; v2 += r.z; v3 += r.w;
  } else if (e.mode == kEpiGeluBwd) {
    float u0, u1, u2, u3;
    if (BF16ACT) {
      const bf16x4 u = *reinterpret_cast<const bf16x4*>(reinterpret_cast<const bf16*>(e.aux) + off);
      u0 = (float)u[0]; u1 = (float)u[1]; u2 = (float)u[2]; u3 = (float)u[3];
    } else {
      const float4 u = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(e.aux) + off);
      u0 = u.x; u1 = u.y; u2 = u.z; u3 = u.w;
    }
    v0 *= gelu_grad_f(u0); v1 *= gelu_grad_f(u1); v2 *= gelu_grad_f(u2); v3 *= gelu_grad_f(u3);
  }
  if (e.out_bf16) {
    bf16x4 o = {(bf16)v0, (bf16)v1, (bf16)v2, (bf16)v3};
    *reinterpret_cast<bf16x4*>(reinterpret_cast<bf16*>(e.C) + off) = o;
    if (two) {
      bf16x4 h = {(bf16)h0, (bf16)h1, (bf16)h2, (bf16)h3};
      *reinterpret_cast<bf16x4*>(reinterpret_cast<bf16*>(e.C2) + off) = h;
    }
  } else {
    float* c = reinterpret_cast<float*>(e.C) + off;
    if (e.accumulate) {
      const float4 old = *reinterpret_cast<const float4*>(c);
      v0 += old.x; v1 += old.y; v2 += old.z; v3 += old.w;
    }
    *reinterpret_cast<float4*>(c) = make_float4(v0, v1, v2, v3);
    if (two) *reinterpret_cast<float4*>(reinterpret_cast<float*>(e.C2) + off) = make_float4(h0, h1, h2, h3);
  }
}

// Same, one element (ragged right edge).
template <bool BF16ACT>
__device__ __forceinline__ void epilogue1(const EpiParams& e, int64_t m, int64_t n, float v) {
  const int64_t off = m * e.ldc + n;
  if (epi_has_bias(e.mode) && e.bias) v += e.bias[n];
  if (e.mode == kEpiBiasResidual) v += reinterpret_cast<const float*>(e.aux)[off];
  if (e.mode == kEpiGeluBwd) {
    const float u = BF16ACT ? (float)reinterpret_cast<const bf16*>(e.aux)[off] : reinterpret_cast<const float*>(e.aux)[off];
    v *= gelu_grad_f(u);
  }
  float h = 0.f;
  const bool two = e.mode == kEpiBiasGelu;
  if (two) h = gelu_f(v);
  if (e.out_bf16) {
    reinterpret_cast<bf16*>(e.C)[off] = (bf16)v;
    if (two) reinterpret_cast<bf16*>(e.C2)[off] = (bf16)h;
  } else {
    float* c = reinterpret_cast<float*>(e.C) + off;
    if (e.accumulate) v += *c;
    *c = v;
    if (two) reinterpret_cast<float*>(e.C2)[off] = h;
  }
}

// What epilogue8 reads from global memory besides the bias: 16 bytes of bf16 aux, 32 bytes of fp32 residual, or the
// 32 bytes of fp32 output it accumulates into.  The staged epilogue fetches these a few row segments ahead of their
// use, so that a wave has several such loads in flight instead of one round trip per row segment.
struct EpiExtra { uint4 lo, hi; };
enum { kExtraNone = 0, kExtraAuxBf16, kExtraAuxF32, kExtraOldC, kExtraAdam, kExtraXentStats, kExtraXentGrad };
__device__ __forceinline__ int epi_extra_kind(const EpiParams& e) {
  if (e.mode == kEpiAdam) return kExtraAdam;
  if (e.mode == kEpiXentStats) return kExtraXentStats;
  if (e.mode == kEpiXentGrad) return kExtraXentGrad;
  if (e.mode == kEpiBiasResidual) return kExtraAuxF32;
  if (e.mode == kEpiGeluBwd) return kExtraAuxBf16;
  return (!e.out_bf16 && e.accumulate) ? kExtraOldC : kExtraNone;
}
// src: e.aux for the two aux kinds, e.C for kExtraOldC.
__device__ __forceinline__ const void* epi_extra_src(const EpiParams& e, int kind) {
  return kind == kExtraOldC ? e.C : e.aux;
}
__device__ __forceinline__ void epi_extra_load(int kind, const void* src, int64_t off, EpiExtra& x) {
  if (kind == kExtraAuxBf16) {
    x.lo = *reinterpret_cast<const uint4*>(reinterpret_cast<const bf16*>(src) + off);
  } else if (kind != kExtraNone) {
    const uint4* s4 = reinterpret_cast<const uint4*>(reinterpret_cast<const float*>(src) + off);
    x.lo = s4[0];
    x.hi = s4[1];
  }
}
__device__ __forceinline__ void add8(float* v, const uint4& lo, const uint4& hi) {
  v[0] += __uint_as_float(lo.x); v[1] += __uint_as_float(lo.y); v[2] += __uint_as_float(lo.z); v[3] += __uint_as_float(lo.w);
  v[4] += __uint_as_float(hi.x); v[5] += __uint_as_float(hi.y); v[6] += __uint_as_float(hi.z); v[7] += __uint_as_float(hi.w);
}

// Epilogue on 8 consecutive columns n0..n0+7 of row m (bf16-activation kernels; all accesses 16-byte vectors).
// x holds what epi_extra_load(kind, epi_extra_src(e, kind), m * ldc + n0, x) fetched, kind = epi_extra_kind(e).
__device__ __forceinline__ void epilogue8(const EpiParams& e, int64_t m, int64_t n0, float* v, int kind, const EpiExtra& x) {
  const int64_t off = m * e.ldc + n0;
  if (epi_has_bias(e.mode) && e.bias) {
    const float4 b0 = *reinterpret_cast<const float4*>(e.bias + n0), b1 = *reinterpret_cast<const float4*>(e.bias + n0 + 4);
    v[0] += b0.x; v[1] += b0.y; v[2] += b0.z; v[3] += b0.w; v[4] += b1.x; v[5] += b1.y; v[6] += b1.z; v[7] += b1.w;
  }
  if (kind == kExtraAuxF32) {
    add8(v, x.lo, x.hi);
  } else if (kind == kExtraAuxBf16) {
    const bf16x8 u = __builtin_bit_cast(bf16x8, x.lo);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] *= gelu_grad_f((float)u[i]);
  }
  const bool two = e.mode == kEpiBiasGelu;
  float hh[8];
  if (two) {
#pragma unroll
    for (int i = 0; i < 8; ++i) hh[i] = gelu_f(v[i]);
  }
  if (e.out_bf16) {
    bf16x8 o;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (bf16)v[i];
    *reinterpret_cast<bf16x8*>(reinterpret_cast<bf16*>(e.C) + off) = o;
    if (two) {
      bf16x8 h;
#pragma unroll
      for (int i = 0; i < 8; ++i) h[i] = (bf16)hh[i];
      *reinterpret_cast<bf16x8*>(reinterpret_cast<bf16*>(e.C2) + off) = h;
    }
  } else {
    float* c = reinterpret_cast<float*>(e.C) + off;
    if (kind == kExtraOldC) {
      add8(v, x.lo, x.hi);
    } else if (e.accumulate) {   // accumulating into the output of a residual epilogue: no slot left to fetch ahead
      const uint4 o0 = *reinterpret_cast<const uint4*>(c), o1 = *reinterpret_cast<const uint4*>(c + 4);
      add8(v, o0, o1);
    }
    *reinterpret_cast<float4*>(c) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4*>(c + 4) = make_float4(v[4], v[5], v[6], v[7]);
    if (two) {
      float* c2 = reinterpret_cast<float*>(e.C2) + off;
      *reinterpret_cast<float4*>(c2) = make_float4(hh[0], hh[1], hh[2], hh[3]);
      *reinterpret_cast<float4*>(c2 + 4) = make_float4(hh[4], hh[5], hh[6], hh[7]);
    }
  }
}

// ---- epilogues of the dedicated kernel instantiations ---------------------------------------------------------
// Adam on 8 consecutive elements at offset off of w, m, v (and the bf16 copy): g[8] is the gradient the GEMM just
// produced, xw / xm / xv what was fetched from w, m, v (32 bytes each).  26 bytes of traffic per parameter - the
// gradient itself never reaches memory unless e.C asks for it.
__device__ __forceinline__ void unpack8(const EpiExtra& x, float* o) {
  o[0] = __uint_as_float(x.lo.x); o[1] = __uint_as_float(x.lo.y); o[2] = __uint_as_float(x.lo.z); o[3] = __uint_as_float(x.lo.w);
  o[4] = __uint_as_float(x.hi.x); o[5] = __uint_as_float(x.hi.y); o[6] = __uint_as_float(x.hi.z); o[7] = __uint_as_float(x.hi.w);
}
__device__ __forceinline__ void store8(float* p, const float* o) {
  *reinterpret_cast<float4*>(p) = make_float4(o[0], o[1], o[2], o[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(o[4], o[5], o[6], o[7]);
}
__device__ __forceinline__ void epilogue8_adam(const EpiParams& e, int64_t off, const float* g, const EpiExtra& xw,
                                               const EpiExtra& xm, const EpiExtra& xv, float ic1, float ic2) {
  float w[8], m[8], v[8];
  unpack8(xw, w);
  unpack8(xm, m);
  unpack8(xv, v);
#pragma unroll
  for (int i = 0; i < 8; ++i) adam_one(w[i], m[i], v[i], g[i], e.ad_lr, e.ad_b1, e.ad_b2, e.ad_eps, ic1, ic2);
  store8(e.ad_w + off, w);
  store8(e.ad_m + off, m);
  store8(e.ad_v + off, v);
  if (e.ad_wlp) {
    bf16x8 o;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (bf16)w[i];
    *reinterpret_cast<bf16x8*>(e.ad_wlp + off) = o;
  }
  if (e.C) store8(reinterpret_cast<float*>(e.C) + off, g);
}

// Target token of row r = b*T + t of the logits: tokens[b*(T+1) + t + 1], clamped into [0, V) as everywhere.
__device__ __forceinline__ int xent_target(const EpiParams& e, int64_t r) {
  const int b = (int)(r / e.xe_T), t = (int)(r - (int64_t)b * e.xe_T);
  const int id = e.xe_tokens[(size_t)b * (e.xe_T + 1) + t + 1];
  return id < 0 ? 0 : (id >= e.xe_V ? e.xe_V - 1 : id);
}
// Softmax statistics of 8 consecutive logits z[8] of row m, columns n..n+7; the 8 lanes that hold the 64 columns of
// one row segment (lane & 7 = 0..7) combine theirs, lane 0 of them writes (max, sum exp(z - max)) of the group.
__device__ __forceinline__ void epilogue8_xent_stats(const EpiParams& e, int64_t m, int64_t n, const float* z, int c8) {
  float mx = z[0];
#pragma unroll
  for (int i = 1; i < 8; ++i) mx = fmaxf(mx, z[i]);
#pragma unroll
  for (int o = 1; o < 8; o <<= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) sum += __expf(z[i] - mx);
#pragma unroll
  for (int o = 1; o < 8; o <<= 1) sum += __shfl_xor(sum, o, 64);
  if (c8 == 0) *reinterpret_cast<float2*>(e.xe_part + 2 * (m * e.xe_groups + (n >> 6))) = make_float2(mx, sum);
  const int tgt = xent_target(e, m);
  if (tgt >= n && tgt < n + 8) {
    float zt = z[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) zt = (tgt - (int)n == i) ? z[i] : zt;
    e.xe_zt[m] = zt;
  }
}
// (softmax - onehot) / N of 8 consecutive logits; x.lo.x holds lse[m], x.lo.y the target id (fetched ahead).
__device__ __forceinline__ void epilogue8_xent_grad(const EpiParams& e, int64_t m, int64_t n, const float* z, const EpiExtra& x) {
  const float lse = __uint_as_float(x.lo.x);
  const int tgt = (int)x.lo.y;
  bf16x8 o;
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = (bf16)((__expf(z[i] - lse) - ((int)n + i == tgt ? 1.f : 0.f)) * e.xe_inv_n);
  *reinterpret_cast<bf16x8*>(reinterpret_cast<bf16*>(e.C) + m * e.ldc + n) = o;
}

// Workgroup id -> output tile, XCD-aware (see file header).
__device__ __forceinline__ void tile_of_block(int pid, int nblk, int tiles_m, int tiles_n, int& tm, int& tn) {
  constexpr int kXcd = 8, kGroup = 8;
  const int q = nblk / kXcd, r = nblk % kXcd;
  const int xcd = pid % kXcd, j = pid / kXcd;
  const int logical = xcd * q + (xcd < r ? xcd : r) + j;
  const int per_group = kGroup * tiles_n;
  const int group = logical / per_group;
  const int first_m = group * kGroup;
  const int gsize = tiles_m - first_m < kGroup ? tiles_m - first_m : kGroup;
  const int in_group = logical - group * per_group;
  tm = first_m + in_group % gsize;
  tn = in_group / gsize;
}

struct GemmBf16Params {
  const bf16* A;
  const bf16* B;
  int64_t M, N, K, lda, ldb;
  int tiles_m, tiles_n;
  float* b_colsum;          // ring kernel, k-major B only: out[n] (=|+=) sum_k B[k][n]; null: not wanted
  int colsum_accumulate;
  EpiParams epi;
};

// Epilogue of the MFMA kernels.  acc[i][j][r] is element m = 32 i + lane%32, n = 32 j + 8 (r/4) + 4 (lane/32) + r%4
// of the wave tile (rows mw0.., columns nw0..): a lane owns one row fragment of 4 columns, so storing straight
// from the accumulators would scatter 8-byte pieces over 32 rows per instruction.  Instead each wave parks one
// 32 x 64 block at a time in its own slice of LDS (the operand tiles are dead by now) and reads it back
// row-wise: 8 lanes cover the 64 columns of a row with 8 consecutive values each, so every global access of
// the epilogue (output, residual, saved pre-activation) is a 16-byte vector and every row segment a full
// 128-byte line or more.  What a segment needs from memory besides the accumulators is fetched one 32-row block
// ahead.  All waves of the block must call (it synchronises the block).
// Parks 32-row block i, 64-column half h of a wave tile in `stage` (rows of ld floats), from either accumulator
// layout: 32 x 32 MFMA blocks (layout above) or 16 x 16 blocks, where acc[a][b][r] is element m = 16 a + lane%16,
// n = 16 b + 4 (lane/16) + r.  Both write 16-byte pieces that tile the banks without conflicts at ld = 68.
template <int FM, int FN>
__device__ __forceinline__ void stage_block(float* stage, int ld, const f32x16 (&acc)[FM][FN], int i, int h, int lane) {
  const int lrow = lane & 31, lhalf = lane >> 5;
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int qq = 0; qq < 4; ++qq)
      *reinterpret_cast<float4*>(stage + lrow * ld + j * 32 + qq * 8 + lhalf * 4) =
          make_float4(acc[i][2 * h + j][qq * 4], acc[i][2 * h + j][qq * 4 + 1], acc[i][2 * h + j][qq * 4 + 2],
                      acc[i][2 * h + j][qq * 4 + 3]);
}
template <int FM16, int FN16>
__device__ __forceinline__ void stage_block(float* stage, int ld, const f32x4 (&acc)[FM16][FN16], int i, int h, int lane) {
  const int lrow = lane & 15, lq = lane >> 4;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
      *reinterpret_cast<float4*>(stage + (a * 16 + lrow) * ld + b * 16 + lq * 4) =
          make_float4(acc[2 * i + a][4 * h + b][0], acc[2 * i + a][4 * h + b][1], acc[2 * i + a][4 * h + b][2],
                      acc[2 * i + a][4 * h + b][3]);
}

// FM, FN: the wave tile in units of 32 rows / 32 columns, whatever the accumulator layout.
template <int FM, int FN, bool EDGE, int KIND, typename Acc>
__device__ __forceinline__ void gemm_epilogue_staged_kind(bf16* smem, Acc& acc, const GemmBf16Params& p,
                                                          int64_t mw0, int64_t nw0, int wave, int lane) {
  static_assert(FN % 2 == 0, "epilogue staging works on 64-column halves of the wave tile");
  constexpr int kLdS = 64 + 4;   // floats; 272-byte rows keep the 16-byte LDS accesses conflict-free
  static_assert(!EDGE || KIND <= kExtraOldC, "the dedicated epilogues exist for full tiles only");
  constexpr bool kAhead = KIND != kExtraNone && KIND != kExtraXentStats;
  const int r8 = lane >> 3, c8 = lane & 7;
  const void* const extra_src = epi_extra_src(p.epi, KIND);
  const int64_t M = p.M, N = p.N, ldc = p.epi.ldc;
  float ic1 = 0.f, ic2 = 0.f;   // Adam's bias corrections
  if (KIND == kExtraAdam) {
    ic1 = p.epi.ad_c ? p.epi.ad_c[0] : p.epi.ad_ic1;
    ic2 = p.epi.ad_c ? p.epi.ad_c[1] : p.epi.ad_ic2;
  }
  // Row segment `it` of 32-row block i, column half h: the fetch of what this lane needs there (x2, x3: the second
  // and third array of the Adam epilogue).
  auto fetch = [&](int h, int i, int it, EpiExtra& x, EpiExtra& x2, EpiExtra& x3) {
    const int64_t m = mw0 + i * 32 + it * 8 + r8, n = nw0 + h * 64 + c8 * 8;
    if (KIND == kExtraAdam) {
      epi_extra_load(kExtraAuxF32, p.epi.ad_w, m * ldc + n, x);
      epi_extra_load(kExtraAuxF32, p.epi.ad_m, m * ldc + n, x2);
      epi_extra_load(kExtraAuxF32, p.epi.ad_v, m * ldc + n, x3);
    } else if (KIND == kExtraXentGrad) {
      x.lo.x = __float_as_uint(p.epi.xe_lse[m]);
      x.lo.y = (uint32_t)xent_target(p.epi, m);
    } else if (!EDGE || (m < M && n + 7 < N)) {
      epi_extra_load(KIND, extra_src, m * ldc + n, x);
    }
  };
  // Between the staging writes and the row-wise reads of a wave's private slice.  With extras in flight a block
  // barrier would wait for them (and for the stores); a wave's LDS accesses execute in issue order, so keeping
  // the compiler from reordering them is enough.  Without extras the plain barrier measured faster.
  auto sync = [] {
    if (kAhead) {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    } else {
      __syncthreads();
    }
  };
  __syncthreads();   // every wave is done with the operand tiles
  float* stage = reinterpret_cast<float*>(smem) + wave * (32 * kLdS);
  // Extras are fetched kSlots row segments ahead of their use: a whole 32-row block (four segments) where a segment
  // needs 16 or 32 bytes per lane, two segments for Adam's 96 bytes (a block's worth would not fit the registers
  // next to the accumulators still waiting to be parked).
  constexpr int kSlots = KIND == kExtraAdam ? 2 : 4;
  EpiExtra q[kSlots] = {};
  EpiExtra q2[kSlots] = {}, q3[kSlots] = {};   // Adam only (dead otherwise)
  if (kAhead) {
#pragma unroll
    for (int it = 0; it < kSlots; ++it) fetch(0, 0, it, q[it], q2[it], q3[it]);
  }
#pragma unroll
  for (int h = 0; h < FN / 2; ++h) {
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      stage_block(stage, kLdS, acc, i, h, lane);
      sync();
      const bool wrap = i + 1 == FM;
      const int ni = wrap ? 0 : i + 1, nh = wrap ? h + 1 : h;
      auto segment = [&](int it, EpiExtra& slot, EpiExtra& slot2, EpiExtra& slot3) {
        const int row = it * 8 + r8;
        const float4 v0 = *reinterpret_cast<const float4*>(stage + row * kLdS + c8 * 8);
        const float4 v1 = *reinterpret_cast<const float4*>(stage + row * kLdS + c8 * 8 + 4);
        float v[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
        const EpiExtra x = slot, x2 = slot2, x3 = slot3;
        if (kAhead) {   // the segment kSlots further on takes over the slot
          if (it + kSlots < 4) fetch(h, i, it + kSlots, slot, slot2, slot3);
          else if (nh < FN / 2) fetch(nh, ni, it + kSlots - 4, slot, slot2, slot3);
        }
        const int64_t m = mw0 + i * 32 + row;
        const int64_t n = nw0 + h * 64 + c8 * 8;
        if (KIND == kExtraAdam) {
          epilogue8_adam(p.epi, m * ldc + n, v, x, x2, x3, ic1, ic2);
        } else if (KIND == kExtraXentStats) {
          epilogue8_xent_stats(p.epi, m, n, v, c8);
        } else if (KIND == kExtraXentGrad) {
          epilogue8_xent_grad(p.epi, m, n, v, x);
        } else if (!EDGE || (m < M && n + 7 < N)) {
          epilogue8(p.epi, m, n, v, KIND, x);
        } else if (m < M) {
          for (int e = 0; e < 8; ++e)
            if (n + e < N) epilogue1<true>(p.epi, m, n + e, v[e]);
        }
      };
      if (kAhead) {   // unrolled: each segment has its own registers for what was fetched ahead
#pragma unroll
        for (int it = 0; it < 4; ++it) segment(it, q[it % kSlots], q2[it % kSlots], q3[it % kSlots]);
      } else {
#pragma unroll 1
        for (int it = 0; it < 4; ++it) segment(it, q[0], q2[0], q3[0]);
      }
      sync();
    }
  }
}

// EPISET: which epilogues the instantiation carries: 0 the general ones (store, bias, residual, GELU, GELU', add-to);
// 1 the two of the LM head fused with the loss (statistics; gradient of the logits); 2 Adam on the product.  The
// dedicated sets have kernel instantiations of their own so that the general kernels do not grow.
constexpr int kEpiSetGeneral = 0, kEpiSetXent = 1, kEpiSetAdam = 2;
template <int FM, int FN, bool EDGE, int EPISET = kEpiSetGeneral, typename Acc>
__device__ __forceinline__ void gemm_epilogue_staged(bf16* smem, Acc& acc, const GemmBf16Params& p,
                                                     int64_t mw0, int64_t nw0, int wave, int lane) {
  if constexpr (EPISET == kEpiSetAdam) {
    gemm_epilogue_staged_kind<FM, FN, EDGE, kExtraAdam>(smem, acc, p, mw0, nw0, wave, lane);
    return;
  } else if constexpr (EPISET == kEpiSetXent) {
    if (p.epi.mode == kEpiXentStats) gemm_epilogue_staged_kind<FM, FN, EDGE, kExtraXentStats>(smem, acc, p, mw0, nw0, wave, lane);
    else gemm_epilogue_staged_kind<FM, FN, EDGE, kExtraXentGrad>(smem, acc, p, mw0, nw0, wave, lane);
    return;
  }
  switch (epi_extra_kind(p.epi)) {   // uniform over the launch
    case kExtraAuxBf16: gemm_epilogue_staged_kind<FM, FN, EDGE, kExtraAuxBf16>(smem, acc, p, mw0, nw0, wave, lane); break;
    case kExtraAuxF32: gemm_epilogue_staged_kind<FM, FN, EDGE, kExtraAuxF32>(smem, acc, p, mw0, nw0, wave, lane); break;
    case kExtraOldC: gemm_epilogue_staged_kind<FM, FN, EDGE, kExtraOldC>(smem, acc, p, mw0, nw0, wave, lane); break;
    default: gemm_epilogue_staged_kind<FM, FN, EDGE, kExtraNone>(smem, acc, p, mw0, nw0, wave, lane); break;
  }
}

// Ring-buffered variant for full tiles (gemm_ring.hip).
bool gemm_ring_supported(int64_t M, int64_t N, int64_t K);
hipError_t launch_gemm_ring(hipStream_t s, const GemmBf16Params& p, bool a_kmajor, bool b_kmajor);
// The same kernel on 128 x 256 tiles (row-major A only; p.tiles_m counts 128-row tiles): for problems with at most
// 128 full tiles, which would otherwise occupy half the chip.
hipError_t launch_gemm_ring_half(hipStream_t s, const GemmBf16Params& p, bool b_kmajor);
// n <= kRingGroupMax problems of one operand layout in a single launch, problem i's workgroups before problem i+1's.
constexpr int kRingGroupMax = 3;
struct GemmRingGroup {
  GemmBf16Params p[kRingGroupMax];
  int first[kRingGroupMax + 1];   // workgroup ranges; unused problems have empty ranges
};
hipError_t launch_gemm_ring_group(hipStream_t s, const GemmBf16Params* p, int n, bool a_kmajor, bool b_kmajor);
hipError_t gemm_ring_init();

}  // namespace pw
