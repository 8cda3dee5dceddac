// GEMM engine: C[M,N] = op(A)[M,K] . op(B)[K,N], fp32 accumulation, fused epilogues; argument checks and the
// choice of kernel for every problem (launch_gemm, launch_gemm_pair).
//
// bf16 problems made of full 256 x 256 tiles that fill the chip go to the ring-buffered kernel of gemm_ring.hip
// (direct global->LDS loads): that is every GEMM of the large workloads.  The kernel in this file takes the rest
// - any shape, ragged edges, few tiles: v_mfma_f32_32x32x16_bf16 tiles, 64-wide wavefronts, block tile
// BM x BN x 64 staged through registers into double-buffered LDS.  In LDS both operand
// tiles are always [row][k] with k contiguous (row = m for A, n for B), padded to 72 elements per row so
// that the 16-byte fragment reads of 32 consecutive rows fall in distinct bank groups.  Operands stored
// k-major in memory (B of a forward GEMM, both operands of a weight-gradient GEMM) are transposed on the
// way in: a thread fetches a 4(k) x 8(row) block with four 16-byte loads, regroups it with v_perm_b32
// into eight 4(k)-element pieces and stores those with 8-byte LDS writes.  The main loop is therefore the
// same for every layout.  The MFMA is issued with the B fragment as its first operand, so a lane ends up
// with 4 consecutive n for one m: epilogue loads/stores are 8- or 16-byte vectors.
//
// Launch mapping: one workgroup per output tile, 1-D grid.  Hardware deals consecutive workgroup ids
// round-robin to the 8 XCDs (each with its own L2), so ids are first regrouped so that every XCD owns a
// contiguous range of tiles, and within the range tiles are walked in groups of 8 tile-rows so that
// concurrently resident workgroups share A and B panels through that XCD's L2.
//
// fp32 path: a plain LDS-tiled ALU kernel; it serves the small fp32 configuration only.
#include "common.hpp"
#include <algorithm>
#include <cmath>

#include "gemm_common.hpp"
#include "kernels.hpp"

#include <cstdlib>
#include <map>
#include <tuple>
#include <vector>

#ifndef PW_WM
#define PW_WM 2
#define PW_WN 4
#endif

namespace pw {

// ======================================================================================================
// bf16 MFMA kernel
// ======================================================================================================
constexpr int kBK = 64;          // k extent of one LDS stage
constexpr int kLdk = kBK + 8;    // padded row length in LDS (elements)


// Global -> registers for one operand tile of ROWS rows x 64 k.  Each thread owns CNT pieces.
//   row-major-k operand (KMAJOR = false): piece = 16 bytes = 8 consecutive k of one row.
//   k-major operand     (KMAJOR = true):  piece = 4 k x 8 rows, held as four 16-byte loads.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <int ROWS, int NT, bool KMAJOR, bool EDGE>
struct TileLoader {
  static constexpr int kPieces = KMAJOR ? (kBK / 4) * (ROWS / 8) : ROWS * (kBK / 8);
  static constexpr int CNT = (kPieces + NT - 1) / NT;
  static constexpr bool kPartial = kPieces % NT != 0;   // some threads own no piece in the last round
  u32x4 reg[KMAJOR ? CNT * 4 : CNT];

  // k-major pieces: which 8-row chunk (rc) and which 4-k group (kq) piece `id` covers.  The 8-byte LDS
  // stores of one 32-lane half-wave land on bank (32*(rc&1) + 2*kq + const) mod 64, so a half-wave is given
  // 2 adjacent row chunks x all 16 k-groups: 32 distinct 8-byte slots, no bank conflict.  (The price is
  // that a half-wave's global loads cover 32 bytes x 16 rows instead of whole 128-byte lines.)
  static __device__ __forceinline__ int piece_rc(int id) { return (id & 1) | ((id >> 5) << 1); }
  static __device__ __forceinline__ int piece_kq(int id) { return (id >> 1) & 15; }

  // p: operand base; ld: leading dimension; row0: first row (m or n) of the tile; k0: first k;
  // rows_total / k_total: operand extents (used only when EDGE).
  __device__ __forceinline__ void load(const bf16* __restrict__ p, int64_t ld, int64_t row0, int64_t k0,
                                       int64_t rows_total, int64_t k_total) {
#pragma unroll
    for (int i = 0; i < CNT; ++i) {
      const int id = threadIdx.x + i * NT;
      if (kPartial && id >= kPieces) continue;
      if (!KMAJOR) {
        const int r = id >> 3, kc = id & 7;
        const int64_t row = row0 + r, k = k0 + kc * 8;
        if (!EDGE || (row < rows_total && k < k_total))
          reg[i] = *reinterpret_cast<const u32x4*>(p + row * ld + k);
        else
          reg[i] = u32x4{0, 0, 0, 0};
      } else {
        const int rc = piece_rc(id), kq = piece_kq(id);
        const int64_t row = row0 + rc * 8;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int64_t k = k0 + kq * 4 + j;
          if (!EDGE || (row < rows_total && k < k_total))
            reg[i * 4 + j] = *reinterpret_cast<const u32x4*>(p + k * ld + row);
          else
            reg[i * 4 + j] = u32x4{0, 0, 0, 0};
        }
      }
    }
  }

  // registers -> LDS tile [ROWS][kLdk]
  __device__ __forceinline__ void store(bf16* __restrict__ tile) const {
#pragma unroll
    for (int i = 0; i < CNT; ++i) {
      const int id = threadIdx.x + i * NT;
      if (kPartial && id >= kPieces) continue;
      if (!KMAJOR) {
        const int r = id >> 3, kc = id & 7;
        *reinterpret_cast<u32x4*>(tile + r * kLdk + kc * 8) = reg[i];
      } else {
        const int rc = piece_rc(id), kq = piece_kq(id);
        const u32x4 w0 = reg[i * 4 + 0], w1 = reg[i * 4 + 1], w2 = reg[i * 4 + 2], w3 = reg[i * 4 + 3];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
          // rows 2*e2 (low halves) and 2*e2+1 (high halves) of the 8-row group; 4 consecutive k each
          u32x2 lo, hi;
          lo.x = __builtin_amdgcn_perm(w1[e2], w0[e2], 0x05040100u);
          lo.y = __builtin_amdgcn_perm(w3[e2], w2[e2], 0x05040100u);
          hi.x = __builtin_amdgcn_perm(w1[e2], w0[e2], 0x07060302u);
          hi.y = __builtin_amdgcn_perm(w3[e2], w2[e2], 0x07060302u);
          *reinterpret_cast<u32x2*>(tile + (rc * 8 + 2 * e2) * kLdk + kq * 4) = lo;
          *reinterpret_cast<u32x2*>(tile + (rc * 8 + 2 * e2 + 1) * kLdk + kq * 4) = hi;
        }
      }
    }
  }
};

template <int BM, int BN, int WM, int WN, bool A_KMAJOR, bool B_KMAJOR, bool EDGE>
__global__ __launch_bounds__(64 * WM * WN) void gemm_bf16_kernel(GemmBf16Params p) {
  constexpr int NT = 64 * WM * WN;
  constexpr int TM = BM / WM, TN = BN / WN;   // wave tile
  constexpr int FM = TM / 32, FN = TN / 32;   // 32x32 MFMA tiles per wave
  static_assert(TM % 32 == 0 && TN % 32 == 0, "wave tile must be a multiple of the MFMA tile");
  // One LDS allocation: [stage 0: A tile, B tile][stage 1: A tile, B tile].  Addresses are formed from the
  // __shared__ symbol directly so that every access stays an LDS (ds_*) instruction.
  extern __shared__ __attribute__((aligned(16))) bf16 smem[];
  constexpr int kStage = (BM + BN) * kLdk;   // elements per stage
  constexpr int kBoff = BM * kLdk;           // B tile offset inside a stage

  int tm, tn;
  tile_of_block(blockIdx.x, p.tiles_m * p.tiles_n, p.tiles_m, p.tiles_n, tm, tn);
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = wave / WN, wn = wave % WN;
  const int lrow = lane & 31, lhalf = lane >> 5;

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  TileLoader<BM, NT, A_KMAJOR, EDGE> la;
  TileLoader<BN, NT, B_KMAJOR, EDGE> lb;
  const int64_t kt_total = (p.K + kBK - 1) / kBK;

  la.load(p.A, p.lda, m0, 0, p.M, p.K);
  lb.load(p.B, p.ldb, n0, 0, p.N, p.K);
  la.store(smem);
  lb.store(smem + kBoff);
  __syncthreads();

  auto compute = [&](int cur) {
    const bf16* a_tile = smem + cur * kStage + (wm * TM + lrow) * kLdk + lhalf * 8;
    const bf16* b_tile = smem + cur * kStage + kBoff + (wn * TN + lrow) * kLdk + lhalf * 8;
#pragma unroll
    for (int kk = 0; kk < kBK / 16; ++kk) {
      bf16x8 af[FM], bfr[FN];
#pragma unroll
      for (int i = 0; i < FM; ++i) af[i] = *reinterpret_cast<const bf16x8*>(a_tile + i * 32 * kLdk + kk * 16);
#pragma unroll
      for (int j = 0; j < FN; ++j) bfr[j] = *reinterpret_cast<const bf16x8*>(b_tile + j * 32 * kLdk + kk * 16);
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
    }
  };
  // Steady state: fetch tile kt+1 into registers, multiply tile kt out of LDS, park tile kt+1 in the other
  // LDS stage, one barrier.  The last tile has nothing to fetch and is peeled off.
  for (int64_t kt = 0; kt + 1 < kt_total; ++kt) {
    const int cur = (int)(kt & 1);
    la.load(p.A, p.lda, m0, (kt + 1) * kBK, p.M, p.K);
    lb.load(p.B, p.ldb, n0, (kt + 1) * kBK, p.N, p.K);
    compute(cur);
    la.store(smem + (cur ^ 1) * kStage);
    lb.store(smem + (cur ^ 1) * kStage + kBoff);
    __syncthreads();
  }
  compute((int)((kt_total - 1) & 1));

  gemm_epilogue_staged<FM, FN, EDGE>(smem, acc, p, m0 + wm * TM, n0 + wn * TN, wave, lane);
}

// The kernels use more than the default 64 KiB of dynamic LDS: raise the limit once per variant (done for all
// variants by gemm_init() so that it never happens inside a stream capture).
template <int BM, int BN, int WM, int WN, bool AK, bool BK_, bool EDGE>
static hipError_t prepare_bf16_variant() {
  constexpr size_t smem = (size_t)2 * (BM + BN) * kLdk * sizeof(bf16);
  static bool attr_done = false;   // per instantiation
  if (attr_done) return hipSuccess;
  auto kern = gemm_bf16_kernel<BM, BN, WM, WN, AK, BK_, EDGE>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e == hipSuccess) attr_done = true;
  return e;
}

template <int BM, int BN, int WM, int WN, bool AK, bool BK_, bool EDGE>
static hipError_t launch_bf16_variant(hipStream_t s, const GemmBf16Params& p) {
  constexpr int NT = 64 * WM * WN;
  constexpr size_t smem = (size_t)2 * (BM + BN) * kLdk * sizeof(bf16);
  hipError_t e = prepare_bf16_variant<BM, BN, WM, WN, AK, BK_, EDGE>();
  if (e != hipSuccess) return e;
  gemm_bf16_kernel<BM, BN, WM, WN, AK, BK_, EDGE><<<p.tiles_m * p.tiles_n, NT, smem, s>>>(p);
  return hipGetLastError();
}

template <int BM, int BN, int WM, int WN>
static hipError_t prepare_bf16_tile() {
  hipError_t e = hipSuccess;
#define PW_PREP(AK, BKM)                                                               \
  if (e == hipSuccess) e = prepare_bf16_variant<BM, BN, WM, WN, AK, BKM, true>();      \
  if (e == hipSuccess) e = prepare_bf16_variant<BM, BN, WM, WN, AK, BKM, false>()
  PW_PREP(false, false);
  PW_PREP(false, true);
  PW_PREP(true, true);
  PW_PREP(true, false);
#undef PW_PREP
  return e;
}

static bool g_use_ring = true;

hipError_t gemm_init() {
  const char* env = getenv("PW_GEMM_RING");      // PW_GEMM_RING=0 selects the register-staged kernel everywhere
  g_use_ring = !(env && env[0] == '0');
  hipError_t e = gemm_ring_init();
  if (e == hipSuccess) e = prepare_bf16_tile<256, 256, PW_WM, PW_WN>();
  if (e == hipSuccess) e = prepare_bf16_tile<128, 128, 2, 2>();
  return e;
}

template <int BM, int BN, int WM, int WN>
static hipError_t launch_bf16_tile(hipStream_t s, const GemmBf16Params& p, bool ak, bool bk, bool edge) {
#define PW_DISPATCH(AK, BKM)                                                                  \
  return edge ? launch_bf16_variant<BM, BN, WM, WN, AK, BKM, true>(s, p)                      \
              : launch_bf16_variant<BM, BN, WM, WN, AK, BKM, false>(s, p)
  if (!ak && !bk) { PW_DISPATCH(false, false); }
  if (!ak && bk) { PW_DISPATCH(false, true); }
  if (ak && bk) { PW_DISPATCH(true, true); }
  PW_DISPATCH(true, false);
#undef PW_DISPATCH
}

// ======================================================================================================
// fp32 ALU kernel: 64x64 tile, 256 threads, 4x4 outputs per thread, BK = 16.  Any M, N, K.
// ======================================================================================================
struct GemmF32Params {
  const float* A;
  const float* B;
  int64_t M, N, K;
  int64_t sam, sak, sbn, sbk;   // element strides: A(m,k) = A[m*sam + k*sak], B(k,n) = B[n*sbn + k*sbk]
  EpiParams epi;
};

__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmF32Params p) {
  __shared__ float As[16][64 + 4];
  __shared__ float Bs[16][64 + 4];
  const int64_t m0 = (int64_t)blockIdx.y * 64, n0 = (int64_t)blockIdx.x * 64;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4] = {};
  for (int64_t k0 = 0; k0 < p.K; k0 += 16) {
    for (int idx = threadIdx.x; idx < 16 * 64; idx += 256) {
      // consecutive threads walk the dimension that is contiguous in memory
      int r, k;
      if (p.sak == 1) { k = idx & 15; r = idx >> 4; } else { r = idx & 63; k = idx >> 6; }
      const int64_t m = m0 + r, kk = k0 + k;
      As[k][r] = (m < p.M && kk < p.K) ? p.A[m * p.sam + kk * p.sak] : 0.f;
    }
    for (int idx = threadIdx.x; idx < 16 * 64; idx += 256) {
      int r, k;
      if (p.sbk == 1) { k = idx & 15; r = idx >> 4; } else { r = idx & 63; k = idx >> 6; }
      const int64_t n = n0 + r, kk = k0 + k;
      Bs[k][r] = (n < p.N && kk < p.K) ? p.B[n * p.sbn + kk * p.sbk] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const float4 a = *reinterpret_cast<const float4*>(&As[k][ty * 4]);
      const float4 b = *reinterpret_cast<const float4*>(&Bs[k][tx * 4]);
      const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += av[i] * bv[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t m = m0 + ty * 4 + i;
    if (m >= p.M) continue;
    const int64_t n = n0 + tx * 4;
    const bool vec_ok = n + 3 < p.N && (p.epi.ldc & 3) == 0;
    if (vec_ok) {
      epilogue4<false>(p.epi, m, n, acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (n + j < p.N) epilogue1<false>(p.epi, m, n + j, acc[i][j]);
    }
  }
}

// ======================================================================================================
// host side
// ======================================================================================================
namespace {
struct ProfiledLaunch {
  hipEvent_t start, stop;
  double flops;
  bool optimizer = false;   // the launch carried the Adam epilogue: MFMA work plus 26 bytes per output element
  GemmShapeKey key{};       // shape, layouts and epilogue (of the first member of a shared launch)
};
struct ShapeLess {
  bool operator()(const GemmShapeKey& x, const GemmShapeKey& y) const {
    return std::tie(x.M, x.N, x.K, x.a_kmajor, x.b_kmajor, x.epilogue, x.members) <
           std::tie(y.M, y.N, y.K, y.a_kmajor, y.b_kmajor, y.epilogue, y.members);
  }
};
std::vector<GemmShapeRow> g_shape_rows;   // per-shape totals as of the last gemm_profile_end
GemmShapeKey shape_key(const GemmArgs& a, int members) {
  return GemmShapeKey{a.M, a.N, a.K, a.a_kmajor, a.b_kmajor, a.epilogue, members};
}
int64_t g_fused_launches = 0;   // what the last gemm_profile_end saw of such launches
double g_fused_ms = 0.0, g_fused_flops = 0.0;
bool g_profile_on = false;
std::vector<ProfiledLaunch> g_profile;
std::vector<hipEvent_t> g_profile_free;

hipEvent_t profile_event() {
  if (!g_profile_free.empty()) {
    hipEvent_t e = g_profile_free.back();
    g_profile_free.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  (void)hipEventCreate(&e);
  return e;
}
}  // namespace

void gemm_profile_begin() {
  for (auto& p : g_profile) {
    g_profile_free.push_back(p.start);
    g_profile_free.push_back(p.stop);
  }
  g_profile.clear();
  g_profile_on = true;
}

void gemm_profile_pause() { g_profile_on = false; }

hipError_t gemm_profile_end(int64_t* launches, double* total_ms, double* total_flops) {
  g_profile_on = false;
  double ms = 0.0, fl = 0.0;
  int64_t n = 0;
  g_fused_launches = 0;
  g_fused_ms = g_fused_flops = 0.0;
  hipError_t err = hipSuccess;
  std::map<GemmShapeKey, GemmShapeRow, ShapeLess> by_shape;
  for (auto& p : g_profile) {
    hipError_t e = hipEventSynchronize(p.stop);
    float t = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&t, p.start, p.stop);
    if (e != hipSuccess) err = e;
    GemmShapeRow& row = by_shape[p.key];
    row.key = p.key;
    row.launches++;
    row.total_ms += t;
    row.total_flops += p.flops;
    if (p.optimizer) {
      g_fused_launches++;
      g_fused_ms += t;
      g_fused_flops += p.flops;
    } else {
      n++;
      ms += t;
      fl += p.flops;
    }
    g_profile_free.push_back(p.start);
    g_profile_free.push_back(p.stop);
  }
  if (launches) *launches = n;
  if (total_ms) *total_ms = ms;
  if (total_flops) *total_flops = fl;
  g_profile.clear();
  g_shape_rows.clear();
  for (auto& kv : by_shape) g_shape_rows.push_back(kv.second);
  std::stable_sort(g_shape_rows.begin(), g_shape_rows.end(),
                   [](const GemmShapeRow& x, const GemmShapeRow& y) { return x.total_ms > y.total_ms; });
  return err;
}

int gemm_profile_shapes(GemmShapeRow* rows, int cap) {
  const int n = (int)g_shape_rows.size();
  for (int i = 0; rows && i < n && i < cap; ++i) rows[i] = g_shape_rows[i];
  return n;
}

void gemm_profile_fused(int64_t* launches, double* total_ms, double* total_flops) {
  if (launches) *launches = g_fused_launches;
  if (total_ms) *total_ms = g_fused_ms;
  if (total_flops) *total_flops = g_fused_flops;
}

static hipError_t launch_gemm_impl(hipStream_t s, const GemmArgs& a);

hipError_t launch_gemm(hipStream_t s, const GemmArgs& a) {
  const bool timed = g_profile_on && a.dtype == kBF16 && a.M > 0 && a.N > 0;
  if (!timed) return launch_gemm_impl(s, a);
  ProfiledLaunch p{profile_event(), profile_event(), 2.0 * (double)a.M * (double)a.N * (double)a.K, a.epilogue == kEpiAdam,
                   shape_key(a, 1)};
  if (!p.start || !p.stop) return hipErrorOutOfMemory;
  hipError_t e = hipEventRecord(p.start, s);
  if (e == hipSuccess) e = launch_gemm_impl(s, a);
  if (e == hipSuccess) e = hipEventRecord(p.stop, s);
  if (e == hipSuccess) g_profile.push_back(p);
  return e;
}

// Argument checks shared by every path; *empty is set when there is nothing to compute.
static hipError_t check_gemm_args(const GemmArgs& a, bool* empty) {
  *empty = false;
  const bool no_c = a.epilogue == kEpiAdam || a.epilogue == kEpiXentStats;   // C optional / unused there
  if (!a.A || !a.B || (!a.C && !no_c) || a.M < 0 || a.N < 0 || a.K < 0) return hipErrorInvalidValue;
  if (a.epilogue < kEpiStore || a.epilogue > kEpiXentGrad) return hipErrorInvalidValue;
  if (a.epilogue == kEpiAdam) {
    const AdamEpi& d = a.adam;
    if (!d.w || !d.m || !d.v || (!d.c_dev && d.t < 1) || a.out_dtype != kF32 || a.accumulate) return hipErrorInvalidValue;
    if (((uintptr_t)d.w | (uintptr_t)d.m | (uintptr_t)d.v | (uintptr_t)d.w_bf16 | (uintptr_t)d.c_dev) & 15) return hipErrorInvalidValue;
  }
  if (a.epilogue == kEpiXentStats || a.epilogue == kEpiXentGrad) {
    const XentEpi& x = a.xent;
    if (!x.tokens || x.T < 1 || a.M % x.T || a.accumulate) return hipErrorInvalidValue;
    if (a.epilogue == kEpiXentStats && (!x.part || !x.zt || ((uintptr_t)x.part & 7))) return hipErrorInvalidValue;
    if (a.epilogue == kEpiXentGrad && (!x.lse || a.out_dtype != kBF16)) return hipErrorInvalidValue;
  }
  if (a.lda < (a.a_kmajor ? a.M : a.K) || a.ldb < (a.b_kmajor ? a.N : a.K) || a.ldc < a.N) return hipErrorInvalidValue;
  if ((a.epilogue == kEpiBiasResidual || a.epilogue == kEpiGeluBwd) && !a.aux) return hipErrorInvalidValue;
  if (a.epilogue == kEpiBiasGelu && !a.C2) return hipErrorInvalidValue;
  if (a.accumulate && (a.out_dtype != kF32 || a.epilogue != kEpiStore)) return hipErrorInvalidValue;
  if (a.epilogue == kEpiBiasResidual && a.out_dtype != kF32) return hipErrorInvalidValue;
  if (a.out_dtype == kBF16 && a.dtype != kBF16) return hipErrorInvalidValue;
  if (a.M == 0 || a.N == 0) { *empty = true; return hipSuccess; }
  if (a.M > (1LL << 30) || a.N > (1LL << 30) || a.K > (1LL << 30)) return hipErrorInvalidValue;
  if (a.dtype == kF32) {
    if (a.out_dtype != kF32) return hipErrorInvalidValue;
    // vector epilogue accesses need 16-byte alignment; the kernel falls back to scalars when ldc % 4 != 0
    if (((uintptr_t)a.C | (uintptr_t)a.C2 | (uintptr_t)a.aux | (uintptr_t)a.bias) & 15) return hipErrorInvalidValue;
    return hipSuccess;
  }
  if (a.dtype != kBF16) return hipErrorInvalidValue;
  // 16-byte vector loads: every row start and every k offset of a piece must be 16-byte aligned
  if ((a.K % 8) || (a.lda % 8) || (a.ldb % 8)) return hipErrorInvalidValue;
  if ((a.a_kmajor && a.M % 8) || (a.b_kmajor && a.N % 8)) return hipErrorInvalidValue;
  if (((uintptr_t)a.A | (uintptr_t)a.B) & 15) return hipErrorInvalidValue;
  if (((uintptr_t)a.C | (uintptr_t)a.C2 | (uintptr_t)a.aux | (uintptr_t)a.bias) & 15) return hipErrorInvalidValue;
  if (a.ldc % 8) return hipErrorInvalidValue;
  return hipSuccess;
}

static EpiParams epi_of(const GemmArgs& a) {
  EpiParams e;
  e.mode = a.epilogue;
  e.out_bf16 = a.out_dtype == kBF16;
  e.accumulate = a.accumulate;
  e.bias = a.bias;
  e.aux = a.aux;
  e.C = a.C;
  e.C2 = a.C2;
  e.ldc = a.ldc;
  e.ad_w = a.adam.w; e.ad_m = a.adam.m; e.ad_v = a.adam.v; e.ad_wlp = (bf16*)a.adam.w_bf16; e.ad_c = a.adam.c_dev;
  e.ad_lr = a.adam.lr; e.ad_b1 = a.adam.b1; e.ad_b2 = a.adam.b2; e.ad_eps = a.adam.eps;
  e.ad_ic1 = e.ad_ic2 = 0.f;
  if (a.epilogue == kEpiAdam && !a.adam.c_dev) {   // the expressions of the Adam kernel
    e.ad_ic1 = 1.f / (1.f - powf(a.adam.b1, (float)a.adam.t));
    e.ad_ic2 = 1.f / (1.f - powf(a.adam.b2, (float)a.adam.t));
  }
  e.xe_tokens = a.xent.tokens; e.xe_part = a.xent.part; e.xe_zt = a.xent.zt; e.xe_lse = a.xent.lse;
  e.xe_inv_n = a.xent.inv_n; e.xe_T = a.xent.T; e.xe_V = (int)a.N; e.xe_groups = (int)(a.N / 64);
  return e;
}

static GemmBf16Params bf16_params_of(const GemmArgs& a, int tile) {
  GemmBf16Params p;
  p.A = (const bf16*)a.A;
  p.B = (const bf16*)a.B;
  p.M = a.M; p.N = a.N; p.K = a.K; p.lda = a.lda; p.ldb = a.ldb;
  p.tiles_m = (int)((a.M + tile - 1) / tile);
  p.tiles_n = (int)((a.N + tile - 1) / tile);
  p.b_colsum = a.b_colsum;
  p.colsum_accumulate = a.accumulate;
  p.epi = epi_of(a);
  return p;
}

// The ring-buffered kernel takes full 256 x 256 tiles only.
static bool ring_eligible(const GemmArgs& a) {
  return g_use_ring && a.dtype == kBF16 && gemm_ring_supported(a.M, a.N, a.K);
}

// The Adam epilogue lives in the ring kernel's weight-gradient instantiation (full 256 x 256 tiles, both operands
// k-major, fp32 product), alone when the problem fills most of the chip or as a member of a shared launch.
bool gemm_adam_fusable(const GemmArgs& a, bool grouped) {
  return ring_eligible(a) && a.a_kmajor && a.b_kmajor && a.out_dtype == kF32 && !a.accumulate &&
         (grouped || (a.M / 256) * (a.N / 256) >= 150);
}
// The loss epilogues live in the ring kernel's forward-layout instantiation.
bool gemm_xent_fusable(const GemmArgs& a) {
  return ring_eligible(a) && !a.a_kmajor && a.b_kmajor && (a.M / 256) * (a.N / 256) >= 150 && a.N <= (1 << 24);
}

bool gemm_colsum_fusable(const GemmArgs& a, bool paired) {
  return ring_eligible(a) && a.a_kmajor && a.b_kmajor && a.out_dtype == kF32 &&
         (a.epilogue == kEpiStore || a.epilogue == kEpiAdam) && (paired || (a.M / 256) * (a.N / 256) >= 150);
}

static hipError_t launch_gemm_impl(hipStream_t s, const GemmArgs& a) {
  bool empty;
  hipError_t err = check_gemm_args(a, &empty);
  if (err != hipSuccess || empty) return err;
  if (a.b_colsum && (!gemm_colsum_fusable(a, false) || ((uintptr_t)a.b_colsum & 3))) return hipErrorInvalidValue;
  if (a.epilogue == kEpiAdam)
    return gemm_adam_fusable(a, false) ? launch_gemm_ring(s, bf16_params_of(a, 256), true, true) : hipErrorInvalidValue;
  if (a.epilogue == kEpiXentStats || a.epilogue == kEpiXentGrad)
    return gemm_xent_fusable(a) ? launch_gemm_ring(s, bf16_params_of(a, 256), false, true) : hipErrorInvalidValue;

  if (a.dtype == kF32) {
    GemmF32Params p;
    p.A = (const float*)a.A;
    p.B = (const float*)a.B;
    p.M = a.M; p.N = a.N; p.K = a.K;
    p.sam = a.a_kmajor ? 1 : a.lda; p.sak = a.a_kmajor ? a.lda : 1;
    p.sbn = a.b_kmajor ? 1 : a.ldb; p.sbk = a.b_kmajor ? a.ldb : 1;
    p.epi = epi_of(a);
    dim3 grid((unsigned)((a.N + 63) / 64), (unsigned)((a.M + 63) / 64));
    if (grid.y > 65535) return hipErrorInvalidValue;
    gemm_f32_kernel<<<grid, 256, 0, s>>>(p);
    return hipGetLastError();
  }
  // Full tiles whose last round would occupy at most half the chip (384 tiles: a round of 256, then 128), A
  // row-major: the columns of that last round become a problem of their own, which takes the 128 x 256 tiles below.
  if (ring_eligible(a) && !a.a_kmajor && !a.b_colsum) {
    const int64_t tm = a.M / 256, tiles = tm * (a.N / 256), rest = tiles % 256;
    if (tiles > 256 && rest > 0 && rest <= 128 && rest % tm == 0) {
      const int64_t n2 = rest / tm * 256, n1 = a.N - n2;
      const int64_t out_size = a.out_dtype == kBF16 ? 2 : 4;
      const int64_t aux_size = a.epilogue == kEpiBiasResidual ? 4 : 2;
      GemmArgs head = a, tail = a;
      head.N = n1;
      tail.N = n2;
      tail.B = (const char*)a.B + (a.b_kmajor ? n1 : n1 * a.ldb) * 2;
      if (a.bias) tail.bias = a.bias + n1;
      if (a.aux) tail.aux = (const char*)a.aux + n1 * aux_size;
      tail.C = (char*)a.C + n1 * out_size;
      if (a.C2) tail.C2 = (char*)a.C2 + n1 * out_size;
      err = launch_gemm_impl(s, head);
      return err != hipSuccess ? err : launch_gemm_impl(s, tail);
    }
  }
  // Full 256x256 tiles with enough of them to fill the chip: the ring-buffered kernel.
  if (ring_eligible(a) && (a.M / 256) * (a.N / 256) >= 150)
    return launch_gemm_ring(s, bf16_params_of(a, 256), a.a_kmajor, a.b_kmajor);
  // At most half the chip in full tiles, A row-major: the ring kernel on 128 x 256 tiles.
  if (ring_eligible(a) && !a.a_kmajor && (a.M / 256) * (a.N / 256) <= 128 && (a.M / 128) * (a.N / 256) >= 64) {
    GemmBf16Params p = bf16_params_of(a, 256);
    p.tiles_m = (int)(a.M / 128);
    return launch_gemm_ring_half(s, p, a.b_kmajor);
  }
  // Tile choice: 256x256 when that still yields at least one workgroup per CU; otherwise 128x128.
  const int64_t big_tiles = ((a.M + 255) / 256) * ((a.N + 255) / 256);
  if (big_tiles >= 150) {
    const bool edge = (a.M % 256) || (a.N % 256) || (a.K % kBK);
    return launch_bf16_tile<256, 256, PW_WM, PW_WN>(s, bf16_params_of(a, 256), a.a_kmajor, a.b_kmajor, edge);
  }
  const GemmBf16Params p = bf16_params_of(a, 128);
  if ((int64_t)p.tiles_m * p.tiles_n > (1 << 24)) return hipErrorInvalidValue;
  const bool edge = (a.M % 128) || (a.N % 128) || (a.K % kBK);
  return launch_bf16_tile<128, 128, 2, 2>(s, p, a.a_kmajor, a.b_kmajor, edge);
}

// Up to three independent GEMMs.  When all are ring-kernel problems of one operand layout, together fill at least
// most of the chip, and at least one of them would leave part of it idle (or miss the ring kernel) alone, they
// share a single launch (their tiles run side by side); otherwise one launch each.
bool gemm_group_shares_launch(const GemmArgs* a, int n) {
  if (n < 2 || n > kRingGroupMax) return false;
  int64_t total = 0;
  bool all_full_rounds = true;
  for (int i = 0; i < n; ++i) {
    if (a[i].M <= 0 || a[i].N <= 0 || !ring_eligible(a[i])) return false;
    if (a[i].a_kmajor != a[0].a_kmajor || a[i].b_kmajor != a[0].b_kmajor) return false;
    const int64_t t = (a[i].M / 256) * (a[i].N / 256);
    total += t;
    all_full_rounds = all_full_rounds && t % 256 == 0;
  }
  return total >= 150 && total <= (1 << 20) && !all_full_rounds;
}
bool gemm_pair_shares_launch(const GemmArgs& a0, const GemmArgs& a1) {
  const GemmArgs a[2] = {a0, a1};
  return gemm_group_shares_launch(a, 2);
}

hipError_t launch_gemm_group(hipStream_t s, const GemmArgs* a, int n) {
  if (n < 1 || n > kRingGroupMax || !a) return hipErrorInvalidValue;
  bool empty[kRingGroupMax], any_empty = false;
  for (int i = 0; i < n; ++i) {
    const hipError_t err = check_gemm_args(a[i], &empty[i]);
    if (err != hipSuccess) return err;
    any_empty = any_empty || empty[i];
  }
  const bool shared = !any_empty && gemm_group_shares_launch(a, n);
  for (int i = 0; i < n; ++i) {   // checked before anything is launched
    if (a[i].b_colsum && !gemm_colsum_fusable(a[i], shared)) return hipErrorInvalidValue;
    if (a[i].epilogue == kEpiAdam && !gemm_adam_fusable(a[i], shared)) return hipErrorInvalidValue;
    if (shared && (a[i].epilogue == kEpiAdam) != (a[0].epilogue == kEpiAdam)) return hipErrorInvalidValue;
    if (a[i].epilogue == kEpiXentStats || a[i].epilogue == kEpiXentGrad) return hipErrorInvalidValue;
  }
  if (!shared) {
    for (int i = 0; i < n; ++i) {
      const hipError_t err = launch_gemm(s, a[i]);
      if (err != hipSuccess) return err;
    }
    return hipSuccess;
  }
  // the larger problems' workgroups first
  int order[kRingGroupMax];
  double flops = 0.0;
  for (int i = 0; i < n; ++i) {
    order[i] = i;
    flops += 2.0 * (double)a[i].M * (double)a[i].N * (double)a[i].K;
  }
  std::stable_sort(order, order + n, [&](int x, int y) { return a[x].M * a[x].N > a[y].M * a[y].N; });
  GemmBf16Params p[kRingGroupMax];
  for (int i = 0; i < n; ++i) p[i] = bf16_params_of(a[order[i]], 256);
  const bool timed = g_profile_on;
  ProfiledLaunch pl{nullptr, nullptr, flops, a[0].epilogue == kEpiAdam, shape_key(a[order[0]], n)};
  hipError_t err = hipSuccess;
  if (timed) {
    pl.start = profile_event();
    pl.stop = profile_event();
    if (!pl.start || !pl.stop) return hipErrorOutOfMemory;
    err = hipEventRecord(pl.start, s);
    if (err != hipSuccess) return err;
  }
  err = launch_gemm_ring_group(s, p, n, a[0].a_kmajor, a[0].b_kmajor);
  if (timed && err == hipSuccess) {
    err = hipEventRecord(pl.stop, s);
    if (err == hipSuccess) g_profile.push_back(pl);
  }
  return err;
}

hipError_t launch_gemm_pair(hipStream_t s, const GemmArgs& a0, const GemmArgs& a1) {
  const GemmArgs a[2] = {a0, a1};
  return launch_gemm_group(s, a, 2);
}

}  // namespace pw
