// bf16 MFMA GEMM, ring-buffered variant for full tiles: global memory -> LDS directly
// (global_load_lds_dwordx4, no staging registers, no LDS store instructions) into a two-stage ring of
// 64-deep k tiles - the next tile is in flight while one is multiplied - and transposing LDS reads
// (ds_read_b64_tr_b16) for operands stored k-major, so no data is ever regrouped in registers.
//
// Facts about the two gfx950 instructions, checked on the device with in-bounds probes:
//  * global_load_lds_dwordx4: the wave's 64 lanes deposit their 16 bytes at LDS base + 16*lane, in lane
//    order, whatever global address each lane supplied.  A swizzled LDS layout is therefore obtained by
//    choosing which global chunk each lane fetches.
//  * ds_read_b64_tr_b16: within each group of 16 lanes, lane i receives element i%4 of the four 8-byte
//    pieces addressed by lanes i/4, i/4 + 4, i/4 + 8, i/4 + 12 of the group.  If lane L of the group
//    points at [k0 + L/4][r0 + 4*(L%4)] of a k-major tile, lane i ends up with k0..k0+3 of row r0 + i:
//    half of an MFMA operand fragment.
//
// LDS layouts (one stage = A tile then B tile, 32 KiB each, no padding):
//  * operand stored [row][k] in memory: LDS [256 rows][8 chunks of 8 k]; chunk c of row r sits at
//    position c ^ ((r >> 1) & 7): the 16-byte fragment reads of 16 consecutive rows hit 16 distinct
//    bank groups.
//  * operand stored [k][row] in memory: LDS [64 k][32 chunks of 8 rows]; chunk c of k-row k sits at
//    position c ^ (4 * (k & 3)) ^ (2 * ((k >> 3) & 1)): the eight k-rows (k0..k0+3 and k0+8..k0+11, 16 rows
//    each) that the first 32 lanes of one transposing read touch fall into eight different 32-byte bank windows.
#include "common.hpp"
#include "gemm_common.hpp"
#include "kernels.hpp"
#include <type_traits>

namespace pw {

namespace {

constexpr int kRT = 256;            // tile is kRT x kRT
constexpr int kRBK = 64;            // k per stage
constexpr int kRStages = 2;
constexpr int kRingHM = 2;          // 16-row blocks of A per unit of the main loop (see ring_tile); 4 spills registers
constexpr int kROperand = kRT * kRBK;            // elements per full operand tile (32 KiB)
// Elements per stage: an A tile of TM rows (256, or 128 for problems that would otherwise leave half the chip
// idle) and a B tile of 256 rows.
template <int TM> constexpr int ring_stage() { return (TM + kRT) * kRBK; }

typedef __attribute__((address_space(3))) void* lds_ptr;
typedef const __attribute__((address_space(1))) void* gbl_ptr;
typedef short short4v __attribute__((ext_vector_type(4)));

// 16 bytes per lane from global memory straight into LDS at lds_off + 16*lane (lds_off: wave-uniform byte
// offset).  Issued through inline assembly on purpose: the compiler then keeps no record of an LDS write in
// flight, and so neither drains the vector-memory counter before unrelated LDS reads nor at barriers.  The
// kernel waits for the tile it needs with an explicit s_waitcnt (see the main loop).
__device__ __forceinline__ void dma16(const bf16* g, uint32_t lds_off) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(g), "s"(lds_off) : "memory", "m0");
}

// One of this wave's PER direct-load instructions (1 KiB each; 32 per operand tile, shared evenly by the waves)
// of an operand tile.  base: operand; ld: leading dimension; row0: first tile row (m or n); k0: first k of the
// stage; j: 0..PER-1.
template <bool KMAJOR, int PER>
__device__ __forceinline__ void issue_one(const bf16* __restrict__ base, int64_t ld, int64_t row0, int64_t k0,
                                          uint32_t lds_tile_off, int wave, int lane, int j) {
  const int instr = wave * PER + j;
  const bf16* g;
  if (!KMAJOR) {
    const int r = instr * 8 + (lane >> 3);        // 8 rows x 128 bytes per instruction
    const int c = (lane & 7) ^ ((r >> 1) & 7);
    g = base + (row0 + r) * ld + k0 + c * 8;
  } else {
    const int k = instr * 2 + (lane >> 5);        // 2 k-rows x 512 bytes per instruction
    const int c = (lane & 31) ^ (4 * (k & 3)) ^ (2 * ((k >> 3) & 1));
    g = base + (k0 + k) * ld + row0 + c * 8;
  }
  dma16(g, lds_tile_off + instr * 1024);
}

// One operand fragment of v_mfma_f32_16x16x32_bf16 for this lane: row frag_row0 + lane % 16 of the tile, the 8
// k-values 32 kk + 8 (lane / 16) .. + 7.  (Both operands of that instruction have this lane layout.)
template <bool KMAJOR>
__device__ __forceinline__ bf16x8 read_fragment(const bf16* lds_tile, int frag_row0, int kk, int lane) {
  if (!KMAJOR) {
    const int r = frag_row0 + (lane & 15);
    const int c = (4 * kk + (lane >> 4)) ^ ((r >> 1) & 7);
    return *reinterpret_cast<const bf16x8*>(lds_tile + r * kRBK + c * 8);
  } else {
    const int grp = lane >> 4, L = lane & 15;
    const int row = frag_row0 + 4 * (L & 3);                      // first of the 4 rows this lane points at
    const int kbase = kk * 32 + 8 * grp + (L >> 2);
    union { bf16x8 v; short4v h[2]; } u;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int k = kbase + 4 * t;
      const int c = (row >> 3) ^ (4 * (k & 3)) ^ (2 * ((k >> 3) & 1));
      const bf16* p = lds_tile + k * kRT + c * 8 + (row & 7);
      u.h[t] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)p);
    }
    return u.v;
  }
}

// One TM x 256 output tile of problem p (TM = 256, or 128 for problems of few tiles); pid: index of the tile's
// workgroup among the problem's own.  Waves form a 2 x NW grid: NW = 4 -> 8 waves with (TM / 2) x 64 wave tiles.  The products are 16 x 16 x 32 MFMAs: on
// operands with random mantissas the chip runs into its board power limit, and per flop that shape draws less
// than the 32 x 32 x 16 one (same loop, same LDS bytes: 2.06 against 1.82 PFLOP/s sustained).
template <bool A_KMAJOR, bool B_KMAJOR, int NW, int TM, int EPISET = kEpiSetGeneral>
__device__ __forceinline__ void ring_tile(const GemmBf16Params& p, int pid, bf16* smem) {
  static_assert(TM == kRT || (TM == 128 && !A_KMAJOR), "the half-height tile exists for row-major A only");
  constexpr int kRStage = ring_stage<TM>();
  constexpr int kAOperand = TM * kRBK;                // elements of the A tile
  int tm, tn;
  tile_of_block(pid, p.tiles_m * p.tiles_n, p.tiles_m, p.tiles_n, tm, tn);
  const int64_t m0 = (int64_t)tm * TM, n0 = (int64_t)tn * kRT;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = wave / NW, wn = wave % NW;
  constexpr int kWaveN = kRT / NW;                    // columns of a wave tile
  constexpr int kWaveM = TM / 2;                      // rows of a wave tile
  constexpr int FM = kWaveM / 16, FN = kWaveN / 16;   // 16 x 16 accumulator blocks of the wave tile
  constexpr int HM = kRingHM;                         // a unit of work: HM row blocks x FN column blocks, one 32-deep k-step
  constexpr int UPS = FM / HM;                        // units per k-step
  constexpr int PER_A = TM / 8 / (2 * NW);            // direct-load instructions (1 KiB each) per A tile and wave
  constexpr int PER_B = kRT / 8 / (2 * NW);           // ... per B tile and wave
  constexpr int PER = PER_A + PER_B;
  static_assert(HM * FN >= PER, "one direct load at most goes out behind each MFMA of the last unit");
  constexpr int kIssueEvery = HM * FN / PER;          // ... behind every kIssueEvery-th MFMA, until all PER are out

  f32x4 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;

  // Column sums of a k-major B (the bias gradient that goes with a weight gradient): the waves of the first tile
  // row that own the B columns (wm == 0) add up the fragments they read anyway.
  const bool do_colsum = B_KMAJOR && p.b_colsum != nullptr && tm == 0 && wm == 0;
  float cs[FN];
#pragma unroll
  for (int j = 0; j < FN; ++j) cs[j] = 0.f;
  auto add_colsum = [&](const bf16x8* bfr) {
    if (do_colsum) {
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        float t = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) t += (float)bfr[j][e];
        cs[j] += t;
      }
    }
  };

  const int kt_total = (int)(p.K / kRBK);
  const uint32_t smem_off = (uint32_t)(uintptr_t)(lds_ptr)smem;   // byte offset of the ring inside LDS
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  // idx 0..PER_A-1: A tile instructions, PER_A..PER-1: B tile instructions of k-tile kt
  auto issue_idx = [&](int kt, int idx) {
    const uint32_t stage = smem_off + (uint32_t)(kt % kRStages) * (kRStage * 2);
    if (idx < PER_A) issue_one<A_KMAJOR, PER_A>(p.A, p.lda, m0, (int64_t)kt * kRBK, stage, wave_s, lane, idx);
    else issue_one<B_KMAJOR, PER_B>(p.B, p.ldb, n0, (int64_t)kt * kRBK, stage + kAOperand * 2, wave_s, lane, idx - PER_A);
  };
  // A unit u of a k-tile: k-step u / UPS (32 deep), row blocks HM (u % UPS) .. + HM - 1 of the wave tile.
  auto load_a = [&](int stage, int u, bf16x8* af) {
    const bf16* a_tile = smem + stage * kRStage;
#pragma unroll
    for (int i = 0; i < HM; ++i) af[i] = read_fragment<A_KMAJOR>(a_tile, wm * kWaveM + ((u % UPS) * HM + i) * 16, u / UPS, lane);
  };
  auto load_b = [&](int stage, int ks, bf16x8* bfr) {
    const bf16* b_tile = smem + stage * kRStage + kAOperand;
#pragma unroll
    for (int j = 0; j < FN; ++j) bfr[j] = read_fragment<B_KMAJOR>(b_tile, wn * kWaveN + j * 16, ks, lane);
  };
  auto wait_and_sync = [&]() {
    // all of this wave's LDS reads and its share of the tile in flight are complete ...
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    // ... and after the (bare, fence-less) barrier so are everyone else's: the tile in flight is visible and
    // the stage just consumed may be overwritten.
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };

  // The MFMA stream runs across k-tiles without a gap.  A k-tile is four units of HM x FN MFMAs (two 32-deep
  // k-steps, two halves of the wave tile's rows each).  Fragments are double-buffered in registers: the A fragments
  // of unit u+1 (and the B fragments of the next k-step with them) are read before the MFMAs of unit u.  The one
  // barrier per k-tile sits in front of the MFMAs of the LAST unit: by then every wave has finished reading the
  // current stage, so behind the barrier the first fragments of the next tile are fetched and the direct loads of
  // the tile after next are issued between those last MFMAs.
  // Prologue: both stages are free, so the first two k-tiles go out back to back; only the first is waited for.
#pragma unroll
  for (int idx = 0; idx < PER; ++idx) issue_idx(0, idx);
  if (kt_total > 1) {
#pragma unroll
    for (int idx = 0; idx < PER; ++idx) issue_idx(1, idx);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PER) : "memory");   // all but the second tile's loads have landed
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  } else {
    wait_and_sync();
  }
  bf16x8 af[2][HM], bfr[2][FN];
  load_a(0, 0, af[0]);
  load_b(0, 0, bfr[0]);
  constexpr int KU = UPS * (kRBK / 32);   // units per tile
  static_assert(KU % 2 == 0 && (kRBK / 32) % 2 == 0, "fragment buffers alternate and must be in phase at every tile start");
  auto mfma = [&](int u, int i, int j) {
    const int row = (u % UPS) * HM + i;
    acc[row][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr[(u / UPS) & 1][j], af[u & 1][i], acc[row][j], 0, 0, 0);
  };
  // Column order within a unit: back and forth, so that every MFMA shares an operand with the one before it
  // (fewer operand bits change between issues: +2 % sustained rate under the power limit).
  static_assert(HM % 2 == 0, "a unit ends on the column it started with");
  auto snake = [](int i, int jj) { return (i & 1) ? FN - 1 - jj : jj; };
  // One k-tile.  MORE: another tile follows (already in flight); MORE2: the one after that exists and is issued here.
  auto k_tile = [&](int kt, auto more, auto more2) {
    const int stage = kt & 1;
#pragma unroll
    for (int u = 0; u < KU - 1; ++u) {
      // unit 0 starts with one MFMA on fragments fetched during the previous tile, so that the wait for
      // those does not also cover the reads issued here.
      if (u == 0) {
        mfma(0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
      load_a(stage, u + 1, af[(u + 1) & 1]);
      if (u % UPS == 0 && u + UPS < KU) load_b(stage, u / UPS + 1, bfr[(u / UPS + 1) & 1]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < HM; ++i)
#pragma unroll
        for (int jj = 0; jj < FN; ++jj) {
          const int j = snake(i, jj);
          if (u != 0 || i != 0 || j != 0) mfma(u, i, j);
        }
      if (u % UPS == 0) add_colsum(bfr[(u / UPS) & 1]);
      __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (decltype(more)::value) {
      wait_and_sync();
      load_a(stage ^ 1, 0, af[0]);
      load_b(stage ^ 1, 0, bfr[0]);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int i = 0; i < HM; ++i)
#pragma unroll
      for (int jj = 0; jj < FN; ++jj) {
        mfma(KU - 1, i, snake(i, jj));
        if constexpr (decltype(more2)::value) {
          if ((i * FN + jj) % kIssueEvery == 0 && (i * FN + jj) / kIssueEvery < PER) issue_idx(kt + 2, (i * FN + jj) / kIssueEvery);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    __builtin_amdgcn_sched_barrier(0);
  };
  using yes = std::integral_constant<bool, true>;
  using no = std::integral_constant<bool, false>;
  int kt = 0;
  for (; kt + 2 < kt_total; ++kt) k_tile(kt, yes{}, yes{});
  if (kt + 1 < kt_total) { k_tile(kt, yes{}, no{}); ++kt; }
  k_tile(kt, no{}, no{});
  if (do_colsum) {
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      float t = cs[j] + __shfl_xor(cs[j], 16, 64);   // the four k-groups of the fragment
      t += __shfl_xor(t, 32, 64);
      if (lane < 16) {
        float* o = p.b_colsum + n0 + wn * kWaveN + j * 16 + lane;
        *o = p.colsum_accumulate ? *o + t : t;
      }
    }
  }
  gemm_epilogue_staged<kWaveM / 32, kWaveN / 32, false, EPISET>(smem, acc, p, m0 + wm * kWaveM, n0 + wn * kWaveN, wave, lane);
}

template <bool A_KMAJOR, bool B_KMAJOR, int NW, int TM, int EPISET = kEpiSetGeneral>
__global__ __launch_bounds__(2 * NW * 64) void gemm_ring_kernel(GemmBf16Params p) {
  extern __shared__ __attribute__((aligned(16))) bf16 smem[];
  ring_tile<A_KMAJOR, B_KMAJOR, NW, TM, EPISET>(p, blockIdx.x, smem);
}

// Up to three independent problems of the same operand layout in one launch: workgroups [first[i], first[i+1])
// work on problem i.  Lets GEMMs that each fill only part of the chip share one round of workgroups.
template <bool A_KMAJOR, bool B_KMAJOR, int NW, int EPISET = kEpiSetGeneral>
__global__ __launch_bounds__(2 * NW * 64) void gemm_ring_group_kernel(GemmRingGroup g) {
  extern __shared__ __attribute__((aligned(16))) bf16 smem[];
  const int bid = (int)blockIdx.x;
  const int which = bid < g.first[1] ? 0 : (bid < g.first[2] ? 1 : 2);
  const GemmBf16Params p = which == 0 ? g.p[0] : (which == 1 ? g.p[1] : g.p[2]);
  ring_tile<A_KMAJOR, B_KMAJOR, NW, kRT, EPISET>(p, bid - g.first[which], smem);
}

template <int TM> constexpr size_t ring_smem_bytes() { return (size_t)kRStages * ring_stage<TM>() * sizeof(bf16); }
constexpr size_t kRSmemBytes = ring_smem_bytes<kRT>();   // 128 KiB (96 KiB with the half-height A tile)
static_assert(ring_smem_bytes<128>() >= 8 * 32 * 68 * 4, "epilogue staging must fit");

// Waves along n.  4 (8 waves, 128 x 64 wave tiles) is what runs; 2 (4 waves, 128 x 128 wave tiles, accumulators in
// AGPRs, a third fewer LDS fragment reads per MFMA) measured the same within noise with 32 x 32 MFMA blocks on every
// shape of the step, so it is not instantiated.
constexpr int kRingNW = 4;

template <bool AK, bool BK_, int NW>
hipError_t prepare_ring_variant() {
  static bool attr_done = false;
  if (attr_done) return hipSuccess;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_ring_kernel<AK, BK_, NW, kRT>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)kRSmemBytes);
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_ring_group_kernel<AK, BK_, NW>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kRSmemBytes);
  if constexpr (!AK) {
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_ring_kernel<AK, BK_, NW, 128>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)ring_smem_bytes<128>());
  }
  if constexpr (!AK && BK_) {   // the forward layout also carries the LM head's loss epilogues
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_ring_kernel<AK, BK_, NW, kRT, kEpiSetXent>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)kRSmemBytes);
  }
  if constexpr (AK && BK_) {    // the weight-gradient layout also carries the Adam epilogue
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_ring_kernel<AK, BK_, NW, kRT, kEpiSetAdam>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)kRSmemBytes);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_ring_group_kernel<AK, BK_, NW, kEpiSetAdam>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)kRSmemBytes);
  }
  if (e == hipSuccess) attr_done = true;
  return e;
}

// Which set of epilogues the problems of one launch need (all of one set), or -1.
static int epi_set_of(const GemmBf16Params* p, int n) {
  auto set_of = [](int mode) { return mode == kEpiAdam ? kEpiSetAdam : (mode == kEpiXentStats || mode == kEpiXentGrad) ? kEpiSetXent : kEpiSetGeneral; };
  const int set = set_of(p[0].epi.mode);
  for (int i = 1; i < n; ++i)
    if (set_of(p[i].epi.mode) != set) return -1;
  return set;
}

template <bool AK, bool BK_, int NW>
hipError_t launch_ring_variant(hipStream_t s, const GemmBf16Params* p, int n) {
  hipError_t e = prepare_ring_variant<AK, BK_, NW>();
  if (e != hipSuccess) return e;
  const int set = epi_set_of(p, n);
  if (set < 0) return hipErrorInvalidValue;
  if (set == kEpiSetXent) {
    if constexpr (!AK && BK_) {
      if (n != 1) return hipErrorInvalidValue;
      gemm_ring_kernel<AK, BK_, NW, kRT, kEpiSetXent><<<p[0].tiles_m * p[0].tiles_n, 2 * NW * 64, kRSmemBytes, s>>>(p[0]);
      return hipGetLastError();
    } else {
      return hipErrorInvalidValue;
    }
  }
  if (set == kEpiSetAdam) {
    if constexpr (!(AK && BK_)) return hipErrorInvalidValue;
  }
  if (n == 1) {
    if constexpr (AK && BK_) {
      if (set == kEpiSetAdam) {
        gemm_ring_kernel<AK, BK_, NW, kRT, kEpiSetAdam><<<p[0].tiles_m * p[0].tiles_n, 2 * NW * 64, kRSmemBytes, s>>>(p[0]);
        return hipGetLastError();
      }
    }
    gemm_ring_kernel<AK, BK_, NW, kRT><<<p[0].tiles_m * p[0].tiles_n, 2 * NW * 64, kRSmemBytes, s>>>(p[0]);
  } else {
    GemmRingGroup g{};
    int total = 0;
    for (int i = 0; i < kRingGroupMax; ++i) {
      g.first[i] = total;
      if (i < n) {
        g.p[i] = p[i];
        total += p[i].tiles_m * p[i].tiles_n;
      }
    }
    g.first[kRingGroupMax] = total;
    if constexpr (AK && BK_) {
      if (set == kEpiSetAdam) {
        gemm_ring_group_kernel<AK, BK_, NW, kEpiSetAdam><<<total, 2 * NW * 64, kRSmemBytes, s>>>(g);
        return hipGetLastError();
      }
    }
    gemm_ring_group_kernel<AK, BK_, NW><<<total, 2 * NW * 64, kRSmemBytes, s>>>(g);
  }
  return hipGetLastError();
}

template <bool BK_, int NW>
hipError_t launch_ring_half(hipStream_t s, const GemmBf16Params& p) {
  hipError_t e = prepare_ring_variant<false, BK_, NW>();
  if (e != hipSuccess) return e;
  gemm_ring_kernel<false, BK_, NW, 128><<<p.tiles_m * p.tiles_n, 2 * NW * 64, ring_smem_bytes<128>(), s>>>(p);
  return hipGetLastError();
}

template <int NW>
hipError_t launch_ring_nw(hipStream_t s, const GemmBf16Params* p, int n, bool ak, bool bk) {
  if (!ak && !bk) return launch_ring_variant<false, false, NW>(s, p, n);
  if (!ak && bk) return launch_ring_variant<false, true, NW>(s, p, n);
  if (ak && bk) return launch_ring_variant<true, true, NW>(s, p, n);
  return launch_ring_variant<true, false, NW>(s, p, n);
}

}  // namespace

hipError_t launch_gemm_ring(hipStream_t s, const GemmBf16Params& p, bool ak, bool bk) {
  return launch_ring_nw<kRingNW>(s, &p, 1, ak, bk);
}
hipError_t launch_gemm_ring_group(hipStream_t s, const GemmBf16Params* p, int n, bool ak, bool bk) {
  if (n < 1 || n > kRingGroupMax) return hipErrorInvalidValue;
  return launch_ring_nw<kRingNW>(s, p, n, ak, bk);
}

// 128 x 256 tiles (p.tiles_m counts 128-row tiles), A row-major.
hipError_t launch_gemm_ring_half(hipStream_t s, const GemmBf16Params& p, bool bk) {
  return bk ? launch_ring_half<true, kRingNW>(s, p) : launch_ring_half<false, kRingNW>(s, p);
}

bool gemm_ring_supported(int64_t M, int64_t N, int64_t K) { return M % kRT == 0 && N % kRT == 0 && K % kRBK == 0 && K >= kRBK; }

// Sets the dynamic-LDS attribute of every variant up front (never inside a stream capture).
hipError_t gemm_ring_init() {
  hipError_t e = prepare_ring_variant<false, false, kRingNW>();
  if (e == hipSuccess) e = prepare_ring_variant<false, true, kRingNW>();
  if (e == hipSuccess) e = prepare_ring_variant<true, true, kRingNW>();
  if (e == hipSuccess) e = prepare_ring_variant<true, false, kRingNW>();
  return e;
}

}  // namespace pw
