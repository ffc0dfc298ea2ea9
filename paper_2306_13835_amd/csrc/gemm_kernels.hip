// fp16 x fp16 -> fp32 dense products of the shard forward pass on the CDNA4
// matrix cores:  C[M,N] = A[M,K] * W[N,K]^T  (+ epilogue).
//
// These are the column-parallel (q|k|v, fc1) and row-parallel (out-proj, fc2)
// projections a tensor-parallel worker evaluates on a batch entry (paper,
// Section 3.1) and the tied vocabulary-slice head.  Both operands are
// contiguous along K, which is exactly the operand order of the
// v_mfma_f32_32x32x16_f16 instruction: every lane feeds 8 consecutive K
// values of one row (A) or one column (W^T) per step.
//
// Tiling: a workgroup of 4 wavefronts owns a BM x BN tile of C and walks K in
// steps of 64 through two LDS stages (global -> registers -> LDS, one barrier
// per step).  LDS rows are padded by 16 bytes so the 16-byte fragment reads of
// 32 consecutive rows fall on distinct banks.  Workgroup ids are remapped so
// that each of the 8 XCDs (round-robin dispatch) works on a contiguous range
// of W tiles and re-reads them from its own L2.
//
// Roofline: MFMA fp16 when M is a few hundred or more; HBM (W streamed once)
// for M <= 64.  Algorithmic work 2*M*N*K flop, bytes 2*(M*K + N*K) + output.
#include <type_traits>

#include "computron.h"
#include "kernels.h"

namespace ctn {

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// The switches a launch runs under: the caller's (a context's, or a test's) or the defaults.  They are
// scoped to the host thread for the duration of one launch_gemm call, never process wide.
thread_local const GemmTuning* t_tuning = nullptr;
const GemmTuning kDefaultTuning{};
inline const GemmTuning& tuning() { return t_tuning ? *t_tuning : kDefaultTuning; }
struct TuningScope {
  const GemmTuning* prev;
  explicit TuningScope(const GemmTuning* t) : prev(t_tuning) { t_tuning = t; }
  ~TuningScope() { t_tuning = prev; }
};

constexpr int LDS_PAD = 8;      // halves of padding per LDS row (16 bytes)
constexpr int kXcds = 8;

// Workgroup id -> tile id such that XCD x (ids congruent to x mod 8) owns a
// contiguous slice of the tile sequence.
__device__ inline int xcd_remap(int id, int total) {
  const int chunk = total / kXcds, rem = total % kXcds;
  const int x = id % kXcds, slot = id / kXcds;
  return x * chunk + (x < rem ? x : rem) + slot;
}

// Up to three products that share A run as one launch ("parts"): part p
// multiplies by W[p] (N rows), adds bias[p] and writes columns [p*N, (p+1)*N)
// of an output with row stride ldc.  This is how q, k and v are projected
// together although their weights are separate tensors.
struct GemmArgs {
  const _Float16* A;
  const _Float16* W[3];
  const _Float16* bias[3];
  void* out;
  int M, N, K, ldc, parts;
  // Split-K (small M): the K range is cut into `splits` slices, one workgroup per (tile, slice);
  // every slice stores its fp32 partial tile into partial[slice][M][parts*N] and a second kernel
  // adds the slices in a fixed order and applies the epilogue.  splits == 1: no partials.
  int splits;
  float* partial;
};
constexpr int EPI_PARTIAL = 100;   // internal epilogue: store the raw accumulator into the slice's partial buffer

// Epilogue of one wavefront's TM x TN grid of 32x32 accumulator tiles whose first element is (m_w, n_w).
// Accumulator layout of the 32x32 tile: lane holds column (lane % 32) and
// rows 8*(e/4) + 4*(lane/32) + e%4 for e = 0..15.
template <int TM, int TN, int EPI>
__device__ __forceinline__ void store_tile(const GemmArgs& g, const float16v (&acc)[TM][TN], const _Float16* __restrict__ bias,
                                           void* __restrict__ out, int m_w, int n_w, int col0, int ldc, int split, int lane) {
  const int M = g.M, N = g.N;
  const int col_in = lane & 31, row_in = (lane >> 5) * 4;
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int n = n_w + j * 32 + col_in;
    if (n >= N) continue;
    float bv = 0.f;
    if (EPI != CTN_EPI_F32 && EPI != EPI_PARTIAL) bv = static_cast<float>(bias[n]);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = m_w + i * 32 + 8 * (e >> 2) + row_in + (e & 3);
        if (m >= M) continue;
        const int64_t o = static_cast<int64_t>(m) * ldc + col0 + n;
        const float v = acc[i][j][e] + bv;
        if (EPI == EPI_PARTIAL) {
          g.partial[(static_cast<int64_t>(split) * M + m) * (static_cast<int64_t>(N) * g.parts) + col0 + n] = v;
        } else if (EPI == CTN_EPI_BIAS_F16) {
          static_cast<_Float16*>(out)[o] = static_cast<_Float16>(v);
        } else if (EPI == CTN_EPI_BIAS_RELU_F16) {
          static_cast<_Float16*>(out)[o] = static_cast<_Float16>(v > 0.f ? v : 0.f);
        } else if (EPI == CTN_EPI_BIAS_RESID_F32) {
          static_cast<float*>(out)[o] += v;
        } else {
          static_cast<float*>(out)[o] = v;
        }
      }
    }
  }
}

template <int BM, int BN, int BK, int WM, int WN, int EPI>
__device__ __forceinline__ void gemm_nt_body(const GemmArgs& g) {
  constexpr int THREADS = (BM / WM) * (BN / WN) * 64;
  constexpr int LDS_ROW = BK + LDS_PAD;
  constexpr int LPR = BK / 8;          // 16-byte lanes per tile row in the cooperative load
  constexpr int RPP = THREADS / LPR;   // tile rows covered by one pass of the workgroup
  static_assert(BK == 32 || BK == 64, "K extent of one LDS stage");
  static_assert(BM % RPP == 0 && BN % RPP == 0, "cooperative load covers whole passes");
  static_assert(THREADS >= 256 && THREADS <= 1024, "4 to 16 wavefronts per workgroup");
  static_assert(WM % 32 == 0 && WN % 32 == 0 && BM % 32 == 0 && BN % 32 == 0, "32x32 MFMA tiles");
  constexpr int TM = WM / 32, TN = WN / 32;     // MFMA tiles per wavefront
  constexpr int PA = BM / RPP, PB = BN / RPP;   // passes of the cooperative loads

  __shared__ __attribute__((aligned(16))) _Float16 As[2][BM][LDS_ROW];
  __shared__ __attribute__((aligned(16))) _Float16 Bs[2][BN][LDS_ROW];

  const int M = g.M, N = g.N, K = g.K;
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  int tile = xcd_remap(blockIdx.x, tiles_m * tiles_n * g.parts * g.splits);
  const int split = tile / (tiles_m * tiles_n * g.parts);
  tile -= split * tiles_m * tiles_n * g.parts;
  const int part = tile / (tiles_m * tiles_n);
  tile -= part * tiles_m * tiles_n;
  const int m0 = (tile % tiles_m) * BM, n0 = (tile / tiles_m) * BN;   // m fastest: W tile shared by neighbours
  const _Float16* __restrict__ A = g.A;
  const _Float16* __restrict__ W = part == 0 ? g.W[0] : (part == 1 ? g.W[1] : g.W[2]);
  const _Float16* __restrict__ bias = part == 0 ? g.bias[0] : (part == 1 ? g.bias[1] : g.bias[2]);
  void* __restrict__ out = g.out;
  const int ldc = g.ldc, col0 = part * N;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave % (BM / WM)) * WM, wn0 = (wave / (BM / WM)) * WN;
  const int lrow = tid / LPR, lcol = (tid % LPR) * 8;   // cooperative load: RPP rows x LPR lanes x 16 B

  float16v acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  u32x4 ra[PA], rb[PB];
  auto load_global = [&](int k0) {
    const int kc = k0 + lcol;
#pragma unroll
    for (int p = 0; p < PA; ++p) {
      const int r = m0 + p * RPP + lrow;
      ra[p] = u32x4{0u, 0u, 0u, 0u};
      if (r < M && kc < K) ra[p] = *reinterpret_cast<const u32x4*>(A + static_cast<int64_t>(r) * K + kc);
    }
#pragma unroll
    for (int p = 0; p < PB; ++p) {
      const int r = n0 + p * RPP + lrow;
      rb[p] = u32x4{0u, 0u, 0u, 0u};
      if (r < N && kc < K) rb[p] = *reinterpret_cast<const u32x4*>(W + static_cast<int64_t>(r) * K + kc);
    }
  };
  auto store_lds = [&](int buf) {
#pragma unroll
    for (int p = 0; p < PA; ++p) *reinterpret_cast<u32x4*>(&As[buf][p * RPP + lrow][lcol]) = ra[p];
#pragma unroll
    for (int p = 0; p < PB; ++p) *reinterpret_cast<u32x4*>(&Bs[buf][p * RPP + lrow][lcol]) = rb[p];
  };

  // this workgroup's slice of the K steps (all of them when splits == 1)
  const int ksteps_all = (K + BK - 1) / BK;
  const int kt_begin = static_cast<int>(static_cast<int64_t>(ksteps_all) * split / g.splits);
  const int kt_end = static_cast<int>(static_cast<int64_t>(ksteps_all) * (split + 1) / g.splits);
  const int ksteps = kt_end - kt_begin;
  const int kbase = kt_begin * BK;
  if (ksteps > 0) {
    load_global(kbase);
    store_lds(0);
  }
  __syncthreads();

  const int frow = lane & 31, fcol = (lane >> 5) * 8;
  for (int kt = 0; kt < ksteps; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < ksteps) load_global(kbase + (kt + 1) * BK);   // in flight while this stage is multiplied
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      half8 af[TM], bf[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        af[i] = *reinterpret_cast<const half8*>(&As[buf][wm0 + i * 32 + frow][ks * 16 + fcol]);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        bf[j] = *reinterpret_cast<const half8*>(&Bs[buf][wn0 + j * 32 + frow][ks * 16 + fcol]);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < ksteps) {
      store_lds(buf ^ 1);    // the other stage was last read before the previous barrier
      __syncthreads();
    }
  }

  store_tile<TM, TN, EPI>(g, acc, bias, out, m0 + wm0, n0 + wn0, col0, ldc, split, lane);
}

// Two entry points over the same body: with and without an explicit target of two wavefronts
// per SIMD (at most 256 VGPRs).
template <int BM, int BN, int BK, int WM, int WN, int EPI>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void gemm_nt_kernel(const GemmArgs g) {
  gemm_nt_body<BM, BN, BK, WM, WN, EPI>(g);
}
template <int BM, int BN, int BK, int WM, int WN, int EPI>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64, 2) void gemm_nt_kernel_occ2(const GemmArgs g) {
  gemm_nt_body<BM, BN, BK, WM, WN, EPI>(g);
}

// ---- the same tiles with the global loads running two K steps ahead -----------------------------------------
//
// gemm_nt_body keeps one stage of global loads in flight and ends every step with a fenced barrier, which
// (on this target) also waits for every outstanding vector memory operation.  Here the loads of step k + 2
// are issued at the top of step k into a second register set and a raw s_barrier (after s_waitcnt lgkmcnt(0):
// the stage stores are complete) ends the step, so two stages of operands are on their way while one is
// multiplied.  Weights that come from HBM every time, as inside a forward pass, have about twice the latency of
// the warm operands of a tuning loop; this is where the second stage pays (2048 x 5120 x 5376, weights rotating
// through 8 copies: 156 against 183 us).  The step is branch free (loads past the end re-read the last step and
// land in a stage nobody reads) so that the waits for the staged loads stay partial (vmcnt(n), n > 0), and
// scheduling barriers keep the loads at the top of the step.  Same K order and epilogue: bit-equal results.
// Needs K % BK == 0; rows past M or N re-read the last valid row and are not stored.
__device__ __forceinline__ void stage_stores_done_barrier() {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
#endif
}

template <int BM, int BN, int BK, int WM, int WN, int EPI>
__device__ __forceinline__ void gemm_nt_deep_body(const GemmArgs& g) {
  constexpr int THREADS = (BM / WM) * (BN / WN) * 64;
  constexpr int LDS_ROW = BK + LDS_PAD;
  constexpr int LPR = BK / 8, RPP = THREADS / LPR;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int PA = BM / RPP, PB = BN / RPP;
  static_assert(BM % RPP == 0 && BN % RPP == 0, "cooperative load covers whole passes");

  __shared__ __attribute__((aligned(16))) _Float16 As[2][BM][LDS_ROW];
  __shared__ __attribute__((aligned(16))) _Float16 Bs[2][BN][LDS_ROW];

  const int M = g.M, N = g.N, K = g.K;
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  int tile = xcd_remap(blockIdx.x, tiles_m * tiles_n * g.parts * g.splits);
  const int split = tile / (tiles_m * tiles_n * g.parts);
  tile -= split * tiles_m * tiles_n * g.parts;
  const int part = tile / (tiles_m * tiles_n);
  tile -= part * tiles_m * tiles_n;
  const int m0 = (tile % tiles_m) * BM, n0 = (tile / tiles_m) * BN;
  const _Float16* __restrict__ A = g.A;
  const _Float16* __restrict__ W = part == 0 ? g.W[0] : (part == 1 ? g.W[1] : g.W[2]);
  const _Float16* __restrict__ bias = part == 0 ? g.bias[0] : (part == 1 ? g.bias[1] : g.bias[2]);
  const int ldc = g.ldc, col0 = part * N;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave % (BM / WM)) * WM, wn0 = (wave / (BM / WM)) * WN;
  const int lrow = tid / LPR, lcol = (tid % LPR) * 8;

  float16v acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const _Float16* pa[PA];
  const _Float16* pb[PB];
#pragma unroll
  for (int p = 0; p < PA; ++p) {
    const int r = m0 + p * RPP + lrow;
    pa[p] = A + static_cast<int64_t>(r < M ? r : M - 1) * K + lcol;
  }
#pragma unroll
  for (int p = 0; p < PB; ++p) {
    const int r = n0 + p * RPP + lrow;
    pb[p] = W + static_cast<int64_t>(r < N ? r : N - 1) * K + lcol;
  }
  u32x4 ra[2][PA], rb[2][PB];
  auto load_global = [&](int set, int k0) {
#pragma unroll
    for (int p = 0; p < PA; ++p) ra[set][p] = *reinterpret_cast<const u32x4*>(pa[p] + k0);
#pragma unroll
    for (int p = 0; p < PB; ++p) rb[set][p] = *reinterpret_cast<const u32x4*>(pb[p] + k0);
  };
  auto store_lds = [&](int set, int buf) {
#pragma unroll
    for (int p = 0; p < PA; ++p) *reinterpret_cast<u32x4*>(&As[buf][p * RPP + lrow][lcol]) = ra[set][p];
#pragma unroll
    for (int p = 0; p < PB; ++p) *reinterpret_cast<u32x4*>(&Bs[buf][p * RPP + lrow][lcol]) = rb[set][p];
  };

  const int ksteps_all = K / BK;
  const int kt_begin = static_cast<int>(static_cast<int64_t>(ksteps_all) * split / g.splits);
  const int kt_end = static_cast<int>(static_cast<int64_t>(ksteps_all) * (split + 1) / g.splits);
  const int ksteps = kt_end - kt_begin;
  const int kbase = kt_begin * BK;
  const int frow = lane & 31, fcol = (lane >> 5) * 8;

  // One K step; `par` (its parity, compile time) names the stage multiplied and the register set refilled.
  auto step = [&](int kt, auto par_c) {
    constexpr int par = decltype(par_c)::value;
    const int ahead = kt + 2 < ksteps ? kt + 2 : ksteps - 1;
    load_global(par, kbase + ahead * BK);             // this set's previous content went to LDS one step ago
    __builtin_amdgcn_sched_barrier(0);                // keep the loads up here, two steps ahead of their use
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      half8 af[TM], bf[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        af[i] = *reinterpret_cast<const half8*>(&As[par][wm0 + i * 32 + frow][ks * 16 + fcol]);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        bf[j] = *reinterpret_cast<const half8*>(&Bs[par][wn0 + j * 32 + frow][ks * 16 + fcol]);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    store_lds(par ^ 1, par ^ 1);                      // step kt + 1, loaded one step ago (past the end: unused)
    stage_stores_done_barrier();
  };

  if (ksteps > 0) {
    load_global(0, kbase);
    store_lds(0, 0);
    load_global(1, kbase + (ksteps > 1 ? BK : 0));
    stage_stores_done_barrier();
    int kt = 0;
    for (; kt + 2 <= ksteps; kt += 2) {
      step(kt, std::integral_constant<int, 0>{});
      step(kt + 1, std::integral_constant<int, 1>{});
    }
    if (kt < ksteps) step(kt, std::integral_constant<int, 0>{});
  }
  store_tile<TM, TN, EPI>(g, acc, bias, g.out, m0 + wm0, n0 + wn0, col0, ldc, split, lane);
}

template <int BM, int BN, int BK, int WM, int WN, int EPI>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void gemm_nt_deep_kernel(const GemmArgs g) {
  gemm_nt_deep_body<BM, BN, BK, WM, WN, EPI>(g);
}
template <int BM, int BN, int BK, int WM, int WN, int EPI>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64, 2) void gemm_nt_deep_kernel_occ2(const GemmArgs g) {
  gemm_nt_deep_body<BM, BN, BK, WM, WN, EPI>(g);
}


template <int BM, int BN, int BK, int WM, int WN>
hipError_t launch_tiles(const GemmArgs& g, int epi, hipStream_t s) {
  const int tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN) * g.parts * g.splits;
  const dim3 grid(tiles), block((BM / WM) * (BN / WN) * 64);
  // two wavefronts per SIMD is what LDS allows anyway for these shapes (two 4-wave workgroups of up to
  // 80 KiB, or one 8-wave workgroup); stating it keeps the register allocation at or below 256
  constexpr int kWaves = (BM / WM) * (BN / WN);
  constexpr bool kOcc2 = WM * WN >= 64 * 64 && WM * WN <= 128 * 64 &&
                         ((kWaves == 4 && 4 * (BM + BN) * (BK + 8) <= 80 * 1024) || kWaves == 8);
  // (128x128 per wavefront already fills the register file with accumulators: no room for a second set;
  // the 8-wave tiles sit at their 128-register limit and measured 7 % slower with it)
  const bool deep = tuning().deep_loads && g.K % BK == 0 && WM * WN < 128 * 128 && kWaves <= 4;
#define CTN_GEMM(E)                                                                                  \
  do {                                                                                               \
    if constexpr (kOcc2) {                                                                           \
      if (deep) hipLaunchKernelGGL((gemm_nt_deep_kernel_occ2<BM, BN, BK, WM, WN, E>), grid, block, 0, s, g); \
      else hipLaunchKernelGGL((gemm_nt_kernel_occ2<BM, BN, BK, WM, WN, E>), grid, block, 0, s, g);   \
    } else {                                                                                         \
      if (deep) hipLaunchKernelGGL((gemm_nt_deep_kernel<BM, BN, BK, WM, WN, E>), grid, block, 0, s, g); \
      else hipLaunchKernelGGL((gemm_nt_kernel<BM, BN, BK, WM, WN, E>), grid, block, 0, s, g);        \
    }                                                                                                \
  } while (0)
  switch (epi) {
    case EPI_PARTIAL: CTN_GEMM(EPI_PARTIAL); break;
    case CTN_EPI_BIAS_F16: CTN_GEMM(CTN_EPI_BIAS_F16); break;
    case CTN_EPI_BIAS_RELU_F16: CTN_GEMM(CTN_EPI_BIAS_RELU_F16); break;
    case CTN_EPI_BIAS_RESID_F32: CTN_GEMM(CTN_EPI_BIAS_RESID_F32); break;
    case CTN_EPI_F32: CTN_GEMM(CTN_EPI_F32); break;
    default: return hipErrorInvalidValue;
  }
#undef CTN_GEMM
  return hipGetLastError();
}


// ---- 128x128x64 tiles with direct global -> LDS stage fills -------------------------------------------------
//
// The same tile, wavefront layout, K order and epilogue as gemm_nt_body<128,128,64,64,64>, hence the same
// results bit for bit; what differs is how a stage gets into LDS.  global_load_lds_dwordx4 writes 1 KiB per
// wave instruction (8 rows of 128 bytes) straight into LDS: no registers hold the stage, no ds_write is
// issued, and the fill of the next stage overlaps with the fragment reads of the current one.  Rows are not
// padded (the instruction writes wave-contiguously); instead the 16-byte chunk c of row r is stored at
// position c ^ ((r >> 1) & 7), which spreads the 16 rows a fragment read touches per cycle over all banks.
// The compiler orders an LDS read behind every direct-to-LDS load that may alias it by waiting for vmcnt(0),
// which would serialise the fill of the next stage with the products of this one; fragment reads and their
// waits are therefore written in inline assembly, and the two places where the fill must have landed (before
// the first step, at the end of every step) wait and synchronise explicitly with s_waitcnt + s_barrier.
// Needs K % 64 == 0 (a ragged K cannot be zero-filled this way); rows past M or N re-read the last valid row
// and their results are not stored.  Measured against the register-staged loop on operands that sit in the
// last-level cache: 12-22 % faster on products of 600 tiles and more (M = 2048 shapes), 1-12 % on the M = 1024
// ones; with weights streamed from HBM, as inside a forward pass, 5-12 % on the M = 1024 shapes.
__device__ __forceinline__ void fill16(const _Float16* g, _Float16* l) {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_global_load_lds(g, l, 16, 0, 0);
#endif
}
__device__ __forceinline__ half8 frag16(unsigned lds_addr) {
  half8 v = {0, 0, 0, 0, 0, 0, 0, 0};   // (overwritten by the read; the host pass sees no assembly)
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(lds_addr));
#endif
  return v;
}
__device__ __forceinline__ void fills_landed_barrier() {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
#endif
}

template <int EPI>
__global__ __launch_bounds__(256, 2) void gemm_dma_kernel(const GemmArgs g) {
  constexpr int BM = 128, BN = 128, BK = 64, TM = 2, TN = 2;
  constexpr unsigned STAGE = BM * BK * 2;            // bytes of one operand's stage
  __shared__ __attribute__((aligned(1024))) _Float16 As[2][BM][BK];
  __shared__ __attribute__((aligned(1024))) _Float16 Bs[2][BN][BK];

  const int M = g.M, N = g.N, K = g.K;
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  int tile = xcd_remap(blockIdx.x, tiles_m * tiles_n * g.parts * g.splits);
  const int split = tile / (tiles_m * tiles_n * g.parts);
  tile -= split * tiles_m * tiles_n * g.parts;
  const int part = tile / (tiles_m * tiles_n);
  tile -= part * tiles_m * tiles_n;
  const int m0 = (tile % tiles_m) * BM, n0 = (tile / tiles_m) * BN;
  const _Float16* __restrict__ A = g.A;
  const _Float16* __restrict__ W = part == 0 ? g.W[0] : (part == 1 ? g.W[1] : g.W[2]);
  const _Float16* __restrict__ bias = part == 0 ? g.bias[0] : (part == 1 ? g.bias[1] : g.bias[2]);
  const int ldc = g.ldc, col0 = part * N;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave % 2) * 64, wn0 = (wave / 2) * 64;

  float16v acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // Stage fill: wave w issues, per operand, four instructions of 8 rows each (rows 32w + 8i + lane / 8);
  // lane % 8 is the LDS position inside the row, so the lane fetches the chunk that belongs there.
  const int lr = lane >> 3, lp = lane & 7;
  const _Float16* ga[4];
  const _Float16* gb[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = (wave * 4 + i) * 8 + lr, c = lp ^ ((r >> 1) & 7);
    const int ra = m0 + r < M ? m0 + r : M - 1, rb = n0 + r < N ? n0 + r : N - 1;
    ga[i] = A + static_cast<int64_t>(ra) * K + c * 8;
    gb[i] = W + static_cast<int64_t>(rb) * K + c * 8;
  }
  auto fill_stage = [&](int buf, int k0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      fill16(ga[i] + k0, &As[buf][(wave * 4 + i) * 8][0]);
      fill16(gb[i] + k0, &Bs[buf][(wave * 4 + i) * 8][0]);
    }
  };
  // Fragment addresses (bytes from the start of a stage), one per k16 sub-step.
  const int frow = lane & 31, fg = lane >> 5;
  unsigned fa[TM][4], fb[TN][4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int r = wm0 + i * 32 + frow;
      fa[i][ks] = r * (BK * 2) + (((2 * ks + fg) ^ ((r >> 1) & 7)) * 16);
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int r = wn0 + j * 32 + frow;
      fb[j][ks] = r * (BK * 2) + (((2 * ks + fg) ^ ((r >> 1) & 7)) * 16);
    }
  }
  // (the low 32 bits of a pointer into LDS are the LDS byte address)
  const unsigned as_base = static_cast<unsigned>(reinterpret_cast<uintptr_t>(&As[0][0][0]));
  const unsigned bs_base = static_cast<unsigned>(reinterpret_cast<uintptr_t>(&Bs[0][0][0]));

  const int ksteps_all = K / BK;
  const int kt_begin = static_cast<int>(static_cast<int64_t>(ksteps_all) * split / g.splits);
  const int kt_end = static_cast<int>(static_cast<int64_t>(ksteps_all) * (split + 1) / g.splits);
  const int ksteps = kt_end - kt_begin;
  const int kbase = kt_begin * BK;
  // Two register sets for the fragments: the reads of sub-step ks + 1 are in flight while the products of
  // sub-step ks run, and the barrier that ends a stage sits in front of the last sub-step's products, with the
  // first fragment reads of the next stage issued right behind it, so that no product waits for an LDS read
  // that has not had a block of products to arrive in (4 x 256 forward of the 6.7B/TP2 shard 10.35 -> 10.18 ms).
  half8 af0[TM], bf0[TN], af1[TM], bf1[TN];
  auto read_frags = [&](half8 (&af)[TM], half8 (&bf)[TN], int buf, int ks) {
    const unsigned a0 = as_base + buf * STAGE, b0 = bs_base + buf * STAGE;
#pragma unroll
    for (int i = 0; i < TM; ++i) af[i] = frag16(a0 + fa[i][ks]);
#pragma unroll
    for (int j = 0; j < TN; ++j) bf[j] = frag16(b0 + fb[j][ks]);
  };
  auto products = [&](const half8 (&af)[TM], const half8 (&bf)[TN]) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[j], acc[i][j], 0, 0, 0);
  };
#if defined(__HIP_DEVICE_COMPILE__)
#define CTN_FRAGS_READY(AF, BF) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(AF[0]), "+v"(AF[1]), "+v"(BF[0]), "+v"(BF[1]))
#else
#define CTN_FRAGS_READY(AF, BF)
#endif

  if (ksteps > 0) {
    fill_stage(0, kbase);
    fills_landed_barrier();
    if (ksteps > 1) fill_stage(1, kbase + BK);
    read_frags(af0, bf0, 0, 0);
    for (int kt = 0; kt < ksteps; ++kt) {
      const int buf = kt & 1;
      CTN_FRAGS_READY(af0, bf0);
      read_frags(af1, bf1, buf, 1);
      products(af0, bf0);
      CTN_FRAGS_READY(af1, bf1);
      read_frags(af0, bf0, buf, 2);
      products(af1, bf1);
      CTN_FRAGS_READY(af0, bf0);
      read_frags(af1, bf1, buf, 3);
      products(af0, bf0);
      CTN_FRAGS_READY(af1, bf1);
      // this wavefront has read stage kt for the last time; the fill of stage kt + 1 was issued a step ago
      if (kt + 1 < ksteps) {
        fills_landed_barrier();                        // stage kt + 1 complete everywhere, stage kt free everywhere
        if (kt + 2 < ksteps) fill_stage(buf, kbase + (kt + 2) * BK);
        read_frags(af0, bf0, buf ^ 1, 0);
      }
      products(af1, bf1);
    }
  }
#undef CTN_FRAGS_READY
  store_tile<TM, TN, EPI>(g, acc, bias, g.out, m0 + wm0, n0 + wn0, col0, ldc, split, lane);
}


hipError_t launch_dma_tiles(const GemmArgs& g, int epi, hipStream_t s) {
  const int tiles = ((g.M + 127) / 128) * ((g.N + 127) / 128) * g.parts * g.splits;
  const dim3 grid(tiles), block(256);
#define CTN_GEMM(E) hipLaunchKernelGGL((gemm_dma_kernel<E>), grid, block, 0, s, g)
  switch (epi) {
    case EPI_PARTIAL: CTN_GEMM(EPI_PARTIAL); break;
    case CTN_EPI_BIAS_F16: CTN_GEMM(CTN_EPI_BIAS_F16); break;
    case CTN_EPI_BIAS_RELU_F16: CTN_GEMM(CTN_EPI_BIAS_RELU_F16); break;
    case CTN_EPI_BIAS_RESID_F32: CTN_GEMM(CTN_EPI_BIAS_RESID_F32); break;
    case CTN_EPI_F32: CTN_GEMM(CTN_EPI_F32); break;
    default: return hipErrorInvalidValue;
  }
#undef CTN_GEMM
  return hipGetLastError();
}


// ---- M <= 64: weights streamed once from HBM ---------------------------------
//
// With a few dozen tokens the product is bound by reading W once (M flop per
// weight byte is far below the machine balance).  What matters is the number
// of bytes in flight, not the matrix cores: a workgroup of 16 wavefronts owns
// 16 output features and ALL tokens; wavefront w takes the 32-wide K chunks
// w, w+16, w+32, ... so that at any moment the 16 wavefronts read 1 KiB of
// each of the 16 weight rows, four chunks ahead.  Fragments go from global
// memory straight into v_mfma_f32_16x16x32_f16 operands (no LDS staging: no
// operand is reused inside the workgroup).  The 16 partial tiles are summed
// through LDS in a fixed order, so results do not depend on timing.
typedef float float4v __attribute__((ext_vector_type(4)));
constexpr int SK_WAVES = 16;

// MT = 16-token tiles (M <= 16*MT), NT = 16-feature tiles per workgroup, UNROLL = K chunks in flight.
// Every A fragment is used for NT products, so the L2 traffic for A is M/(16*NT) times that of W.
template <int MT, int NT, int UNROLL, int EPI>
__global__ __launch_bounds__(SK_WAVES * 64) void gemm_skinny_kernel(const GemmArgs g) {
  constexpr int BN = 16 * NT;
  __shared__ float part[SK_WAVES][MT * 16][BN + 1];
  const int M = g.M, N = g.N, K = g.K;
  const int tiles_n = (N + BN - 1) / BN;
  const int part_id = blockIdx.x / tiles_n;
  const int n0 = (blockIdx.x % tiles_n) * BN;
  const _Float16* __restrict__ A = g.A;
  const _Float16* __restrict__ W = part_id == 0 ? g.W[0] : (part_id == 1 ? g.W[1] : g.W[2]);
  const _Float16* __restrict__ bias = part_id == 0 ? g.bias[0] : (part_id == 1 ? g.bias[1] : g.bias[2]);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, kg = lane >> 4;          // operand row / column and 8-wide K group of this lane

  float4v acc[MT][NT];
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[t][j] = float4v{0.f, 0.f, 0.f, 0.f};

  const _Float16* wrow[NT];
  bool n_ok[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int n_row = n0 + j * 16 + r16;
    n_ok[j] = n_row < N;
    wrow[j] = W + static_cast<int64_t>(n_ok[j] ? n_row : 0) * K;
  }
  const int chunks = (K + 31) / 32;
  for (int c0 = wave; c0 < chunks; c0 += SK_WAVES * UNROLL) {
    half8 wf[UNROLL][NT], af[UNROLL][MT];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int k = (c0 + u * SK_WAVES) * 32 + kg * 8;
      const bool k_ok = k < K;                         // also false for chunks past the end
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        wf[u][j] = half8{0, 0, 0, 0, 0, 0, 0, 0};
        if (k_ok && n_ok[j]) wf[u][j] = *reinterpret_cast<const half8*>(wrow[j] + k);
      }
#pragma unroll
      for (int t = 0; t < MT; ++t) {
        const int m = t * 16 + r16;
        af[u][t] = half8{0, 0, 0, 0, 0, 0, 0, 0};
        if (k_ok && m < M) af[u][t] = *reinterpret_cast<const half8*>(A + static_cast<int64_t>(m) * K + k);
      }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
#pragma unroll
      for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int j = 0; j < NT; ++j)
          acc[t][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(af[u][t], wf[u][j], acc[t][j], 0, 0, 0);
  }
  // accumulator layout of a 16x16 tile: lane holds column (lane % 16), rows 4*(lane/16) + e
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) part[wave][t * 16 + 4 * kg + e][j * 16 + r16] = acc[t][j][e];
  __syncthreads();
  for (int idx = tid; idx < MT * 16 * BN; idx += SK_WAVES * 64) {
    const int m = idx / BN, j = idx % BN, n = n0 + j;
    if (m >= M || n >= N) continue;
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < SK_WAVES; ++w) v += part[w][m][j];      // fixed order: deterministic
    if (EPI != CTN_EPI_F32) v += static_cast<float>(bias[n]);
    const int64_t o = static_cast<int64_t>(m) * g.ldc + part_id * N + n;
    if (EPI == CTN_EPI_BIAS_F16) {
      static_cast<_Float16*>(g.out)[o] = static_cast<_Float16>(v);
    } else if (EPI == CTN_EPI_BIAS_RELU_F16) {
      static_cast<_Float16*>(g.out)[o] = static_cast<_Float16>(v > 0.f ? v : 0.f);
    } else if (EPI == CTN_EPI_BIAS_RESID_F32) {
      static_cast<float*>(g.out)[o] += v;
    } else {
      static_cast<float*>(g.out)[o] = v;
    }
  }
}

// M <= 16, long rows: the same product with W read row-contiguously.  In the kernel above a wave
// instruction touches 16 rows x 64 bytes; here wavefront w reads 1 KiB of row n0 + w per
// instruction (a 512-wide K window, two windows ahead), the 16 x 512 window is transposed through
// LDS (rows padded by 16 bytes: fragment reads are free of bank conflicts) and wavefront w then
// multiplies the window's K chunk w.  Measured with cold weights at M = 8: 15.1 us against 18.9 us
// for a 67 MB matrix.  The 16 partial tiles are summed through LDS in wavefront order.
constexpr int RS_WIN = 512, RS_ROW = RS_WIN + 8, RS_AHEAD = 2;
static_assert(RS_AHEAD % 2 == 0, "the LDS stage alternates with the position inside a trip");
template <int EPI>
__global__ __launch_bounds__(SK_WAVES * 64) void gemm_rowstream_kernel(const GemmArgs g) {
  // Two stages each of the weight window and of the activation window, [16 rows][RS_ROW]; the 16 partial tiles
  // of the end reuse the weight stages (two workgroups of 66.6 KB fit a CU's LDS, three arrays side by side would not).
  constexpr int kStage = 16 * RS_ROW;                  // halves per stage
  __shared__ __attribute__((aligned(16))) _Float16 smem[4 * kStage];
  _Float16 (*wt)[16][RS_ROW] = reinterpret_cast<_Float16 (*)[16][RS_ROW]>(smem);
  _Float16 (*at)[16][RS_ROW] = reinterpret_cast<_Float16 (*)[16][RS_ROW]>(smem + 2 * kStage);
  float (*part)[16][17] = reinterpret_cast<float (*)[16][17]>(smem);
  static_assert(sizeof(float) * SK_WAVES * 16 * 17 <= sizeof(_Float16) * 2 * kStage, "partial tiles fit the weight stages");
  const int M = g.M, N = g.N, K = g.K;
  const int tiles_n = (N + 15) / 16;
  const int part_id = blockIdx.x / tiles_n;
  const int n0 = (blockIdx.x % tiles_n) * 16;
  const _Float16* __restrict__ A = g.A;
  const _Float16* __restrict__ W = part_id == 0 ? g.W[0] : (part_id == 1 ? g.W[1] : g.W[2]);
  const _Float16* __restrict__ bias = part_id == 0 ? g.bias[0] : (part_id == 1 ? g.bias[1] : g.bias[2]);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, kg = lane >> 4;
  const bool row_ok = n0 + wave < N;
  const bool tok_ok = wave < M;                        // wavefront w also fetches token w's activations
  const _Float16* wrow = W + static_cast<int64_t>(row_ok ? n0 + wave : 0) * K;
  const _Float16* arow = A + static_cast<int64_t>(tok_ok ? wave : 0) * K;
  const int steps = (K + RS_WIN - 1) / RS_WIN;
  // Loads are branch free (an address that is always valid, zeros selected afterwards where the window or the
  // row does not exist) and the barrier is a raw one: a fenced barrier, or a branch around a load, makes the
  // compiler wait for every outstanding load, and the windows that are meant to be in flight would not be.
  // (the zeros are selected where a value is consumed, not where it is loaded: a select right behind the load
  // would wait for it)
  const half8 zero8 = half8{0, 0, 0, 0, 0, 0, 0, 0};
  auto in_k = [&](int p) { return p * RS_WIN + lane * 8 < K; };             // (p >= steps implies false)
  auto load_w = [&](int p) {                            // this lane's 16 bytes of window p of its wave's weight row
    return *reinterpret_cast<const half8*>(wrow + (row_ok && in_k(p) ? p * RS_WIN + lane * 8 : 0));
  };
  // The activations take the same road as the weights: wavefront w reads 1 KiB of token w's row per window
  // (M of the 16 wavefronts; the others store zeros) and the 16 x 512 window is transposed through LDS.  Loading
  // the operand fragments straight from global memory instead (16 rows x 64 bytes per wave instruction, by all
  // 16 wavefronts, half of each cache line unused) cost the load path of a CU twice what the weights cost it.
  auto load_a = [&](int p) {
    return *reinterpret_cast<const half8*>(arow + (tok_ok && in_k(p) ? p * RS_WIN + lane * 8 : 0));
  };
  // Issue order matters: vector memory returns in order, so a load waited for takes everything older with it.
  // Window p + RS_AHEAD of both operands is asked for while window p is being stored and multiplied.
  half8 wr[RS_AHEAD], ar[RS_AHEAD];
#pragma unroll
  for (int u = 0; u < RS_AHEAD; ++u) {
    ar[u] = load_a(u);
    __builtin_amdgcn_sched_barrier(0);
    wr[u] = load_w(u);
    __builtin_amdgcn_sched_barrier(0);
  }
  float4v acc = float4v{0.f, 0.f, 0.f, 0.f};
  for (int p0 = 0; p0 < steps; p0 += RS_AHEAD) {
#pragma unroll
    for (int u = 0; u < RS_AHEAD; ++u) {
      const int p = p0 + u, buf = u & 1;               // (RS_AHEAD is even: the stage alternates with u)
      // past the last window the same code runs on zeros: no branch, and zeros add nothing
      *reinterpret_cast<half8*>(&at[buf][wave][lane * 8]) = (tok_ok && in_k(p)) ? ar[u] : zero8;
      *reinterpret_cast<half8*>(&wt[buf][wave][lane * 8]) = (row_ok && in_k(p)) ? wr[u] : zero8;
      __builtin_amdgcn_sched_barrier(0);
      ar[u] = load_a(p + RS_AHEAD);
      __builtin_amdgcn_sched_barrier(0);
      wr[u] = load_w(p + RS_AHEAD);
      __builtin_amdgcn_sched_barrier(0);
      stage_stores_done_barrier();                      // one per window: the other stage was last read before the previous one
      const half8 bf = *reinterpret_cast<const half8*>(&wt[buf][r16][wave * 32 + kg * 8]);
      const half8 af = *reinterpret_cast<const half8*>(&at[buf][r16][wave * 32 + kg * 8]);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(af, bf, acc, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  __syncthreads();                                      // the stages have been read for the last time: they become `part`
  // accumulator layout of a 16x16 tile: lane holds column (lane % 16), rows 4*(lane/16) + e
#pragma unroll
  for (int e = 0; e < 4; ++e) part[wave][4 * kg + e][r16] = acc[e];
  __syncthreads();
  if (tid < 256) {
    const int m = tid / 16, j = tid % 16, n = n0 + j;
    if (m < M && n < N) {
      float v = 0.f;
#pragma unroll
      for (int w = 0; w < SK_WAVES; ++w) v += part[w][m][j];      // fixed order: deterministic
      if (EPI != CTN_EPI_F32) v += static_cast<float>(bias[n]);
      const int64_t o = static_cast<int64_t>(m) * g.ldc + part_id * N + n;
      if (EPI == CTN_EPI_BIAS_F16) {
        static_cast<_Float16*>(g.out)[o] = static_cast<_Float16>(v);
      } else if (EPI == CTN_EPI_BIAS_RELU_F16) {
        static_cast<_Float16*>(g.out)[o] = static_cast<_Float16>(v > 0.f ? v : 0.f);
      } else if (EPI == CTN_EPI_BIAS_RESID_F32) {
        static_cast<float*>(g.out)[o] += v;
      } else {
        static_cast<float*>(g.out)[o] = v;
      }
    }
  }
}

hipError_t launch_rowstream(const GemmArgs& g, int epi, hipStream_t s) {
  const dim3 grid(((g.N + 15) / 16) * g.parts), block(SK_WAVES * 64);
#define CTN_RS(E) hipLaunchKernelGGL((gemm_rowstream_kernel<E>), grid, block, 0, s, g)
  switch (epi) {
    case CTN_EPI_BIAS_F16: CTN_RS(CTN_EPI_BIAS_F16); break;
    case CTN_EPI_BIAS_RELU_F16: CTN_RS(CTN_EPI_BIAS_RELU_F16); break;
    case CTN_EPI_BIAS_RESID_F32: CTN_RS(CTN_EPI_BIAS_RESID_F32); break;
    case CTN_EPI_F32: CTN_RS(CTN_EPI_F32); break;
    default: return hipErrorInvalidValue;
  }
#undef CTN_RS
  return hipGetLastError();
}

template <int MT, int NT, int UNROLL>
hipError_t launch_skinny(const GemmArgs& g, int epi, hipStream_t s) {
  const dim3 grid(((g.N + 16 * NT - 1) / (16 * NT)) * g.parts), block(SK_WAVES * 64);
#define CTN_SK(E) hipLaunchKernelGGL((gemm_skinny_kernel<MT, NT, UNROLL, E>), grid, block, 0, s, g)
  switch (epi) {
    case CTN_EPI_BIAS_F16: CTN_SK(CTN_EPI_BIAS_F16); break;
    case CTN_EPI_BIAS_RELU_F16: CTN_SK(CTN_EPI_BIAS_RELU_F16); break;
    case CTN_EPI_BIAS_RESID_F32: CTN_SK(CTN_EPI_BIAS_RESID_F32); break;
    case CTN_EPI_F32: CTN_SK(CTN_EPI_F32); break;
    default: return hipErrorInvalidValue;
  }
#undef CTN_SK
  return hipGetLastError();
}

// variant 0: 16 features per workgroup (most workgroups); variant 1: 32 (half the A traffic)
hipError_t launch_skinny_any(const GemmArgs& g, int epi, hipStream_t s, int variant) {
  if (g.M <= 16) return variant ? launch_skinny<1, 2, 4>(g, epi, s) : launch_skinny<1, 1, 4>(g, epi, s);
  if (g.M <= 32) return variant ? launch_skinny<2, 2, 2>(g, epi, s) : launch_skinny<2, 1, 4>(g, epi, s);
  if (g.M <= 48) return variant ? launch_skinny<3, 2, 2>(g, epi, s) : launch_skinny<3, 1, 4>(g, epi, s);
  return variant ? launch_skinny<4, 2, 2>(g, epi, s) : launch_skinny<4, 1, 4>(g, epi, s);
}

// Second pass of a split-K product: out = epilogue(sum over slices, in slice order).
template <int EPI>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const GemmArgs g) {
  const int64_t ncols = static_cast<int64_t>(g.N) * g.parts;
  const int64_t total = static_cast<int64_t>(g.M) * ncols;
  for (int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; idx < total;
       idx += static_cast<int64_t>(gridDim.x) * 256) {
    const int64_t m = idx / ncols, c = idx % ncols;
    const int part = static_cast<int>(c / g.N), n = static_cast<int>(c % g.N);
    float v = 0.f;
    for (int sidx = 0; sidx < g.splits; ++sidx) v += g.partial[(static_cast<int64_t>(sidx) * g.M + m) * ncols + c];
    const _Float16* bias = part == 0 ? g.bias[0] : (part == 1 ? g.bias[1] : g.bias[2]);
    if (EPI != CTN_EPI_F32) v += static_cast<float>(bias[n]);
    const int64_t o = m * g.ldc + c;
    if (EPI == CTN_EPI_BIAS_F16) {
      static_cast<_Float16*>(g.out)[o] = static_cast<_Float16>(v);
    } else if (EPI == CTN_EPI_BIAS_RELU_F16) {
      static_cast<_Float16*>(g.out)[o] = static_cast<_Float16>(v > 0.f ? v : 0.f);
    } else if (EPI == CTN_EPI_BIAS_RESID_F32) {
      static_cast<float*>(g.out)[o] += v;
    } else {
      static_cast<float*>(g.out)[o] = v;
    }
  }
}

// The same pass four columns per thread with every slice's load issued before the first is used
// (MAXS loads in flight; slices past the last re-read slice 0 and are dropped by a select): one
// memory round trip per element instead of one per slice.  Same order of additions, same bits.
// Needs N and ldc to be multiples of 4.
typedef _Float16 half4r __attribute__((ext_vector_type(4)));
template <int EPI, int MAXS>
__global__ __launch_bounds__(256) void splitk_reduce4_kernel(const GemmArgs g) {
  const int64_t ncols4 = static_cast<int64_t>(g.N) * g.parts / 4;
  const int64_t total4 = static_cast<int64_t>(g.M) * ncols4;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= total4) return;
  const int64_t m = idx / ncols4, c = (idx % ncols4) * 4;
  const int part = static_cast<int>(c / g.N), n = static_cast<int>(c % g.N);
  const float4v* src = reinterpret_cast<const float4v*>(g.partial) + idx;
  float4v p[MAXS];
#pragma unroll
  for (int sl = 0; sl < MAXS; ++sl) p[sl] = src[(sl < g.splits ? sl : 0) * total4];
  const int64_t o = m * g.ldc + c;
  float4v r = {0.f, 0.f, 0.f, 0.f};
  if (EPI == CTN_EPI_BIAS_RESID_F32) r = *reinterpret_cast<const float4v*>(static_cast<float*>(g.out) + o);
  half4r bias = {0, 0, 0, 0};
  if (EPI != CTN_EPI_F32) {
    const _Float16* bp = part == 0 ? g.bias[0] : (part == 1 ? g.bias[1] : g.bias[2]);
    bias = *reinterpret_cast<const half4r*>(bp + n);
  }
  float4v v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int sl = 0; sl < MAXS; ++sl) v += sl < g.splits ? p[sl] : float4v{0.f, 0.f, 0.f, 0.f};
  if (EPI != CTN_EPI_F32) {
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] += static_cast<float>(bias[e]);
  }
  if (EPI == CTN_EPI_BIAS_F16 || EPI == CTN_EPI_BIAS_RELU_F16) {
    half4r h;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      h[e] = static_cast<_Float16>(EPI == CTN_EPI_BIAS_RELU_F16 ? (v[e] > 0.f ? v[e] : 0.f) : v[e]);
    *reinterpret_cast<half4r*>(static_cast<_Float16*>(g.out) + o) = h;
  } else if (EPI == CTN_EPI_BIAS_RESID_F32) {
    *reinterpret_cast<float4v*>(static_cast<float*>(g.out) + o) = r + v;
  } else {
    *reinterpret_cast<float4v*>(static_cast<float*>(g.out) + o) = v;
  }
}

template <int EPI>
void launch_reduce4(const GemmArgs& g, hipStream_t s) {
  const int64_t total4 = static_cast<int64_t>(g.M) * g.N * g.parts / 4;
  const dim3 grid(static_cast<unsigned>((total4 + 255) / 256)), block(256);
  if (g.splits <= 4) hipLaunchKernelGGL((splitk_reduce4_kernel<EPI, 4>), grid, block, 0, s, g);
  else if (g.splits <= 8) hipLaunchKernelGGL((splitk_reduce4_kernel<EPI, 8>), grid, block, 0, s, g);
  else hipLaunchKernelGGL((splitk_reduce4_kernel<EPI, 16>), grid, block, 0, s, g);
}


hipError_t launch_splitk_reduce(const GemmArgs& g, int epi, hipStream_t s) {
  if (tuning().reduce4 && g.N % 4 == 0 && g.ldc % 4 == 0 && g.splits <= 16 &&
      reinterpret_cast<uintptr_t>(g.out) % 16 == 0 && reinterpret_cast<uintptr_t>(g.partial) % 16 == 0 &&
      (epi == CTN_EPI_F32 || (reinterpret_cast<uintptr_t>(g.bias[0]) % 8 == 0 &&
                              (g.parts < 2 || reinterpret_cast<uintptr_t>(g.bias[1]) % 8 == 0) &&
                              (g.parts < 3 || reinterpret_cast<uintptr_t>(g.bias[2]) % 8 == 0)))) {
    switch (epi) {
      case CTN_EPI_BIAS_F16: launch_reduce4<CTN_EPI_BIAS_F16>(g, s); break;
      case CTN_EPI_BIAS_RELU_F16: launch_reduce4<CTN_EPI_BIAS_RELU_F16>(g, s); break;
      case CTN_EPI_BIAS_RESID_F32: launch_reduce4<CTN_EPI_BIAS_RESID_F32>(g, s); break;
      case CTN_EPI_F32: launch_reduce4<CTN_EPI_F32>(g, s); break;
      default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
  const int64_t total = static_cast<int64_t>(g.M) * g.N * g.parts;
  const dim3 grid(static_cast<unsigned>((total + 255) / 256)), block(256);
#define CTN_RED(E) hipLaunchKernelGGL((splitk_reduce_kernel<E>), grid, block, 0, s, g)
  switch (epi) {
    case CTN_EPI_BIAS_F16: CTN_RED(CTN_EPI_BIAS_F16); break;
    case CTN_EPI_BIAS_RELU_F16: CTN_RED(CTN_EPI_BIAS_RELU_F16); break;
    case CTN_EPI_BIAS_RESID_F32: CTN_RED(CTN_EPI_BIAS_RESID_F32); break;
    case CTN_EPI_F32: CTN_RED(CTN_EPI_F32); break;
    default: return hipErrorInvalidValue;
  }
#undef CTN_RED
  return hipGetLastError();
}


hipError_t launch_config(int cfg, const GemmArgs& g, int epi, hipStream_t s) {
  switch (cfg) {
    case 0:
      if (tuning().direct_fill && g.K % 64 == 0) return launch_dma_tiles(g, epi, s);
      return launch_tiles<128, 128, 64, 64, 64>(g, epi, s);
    case 17: return launch_tiles<128, 128, 64, 64, 64>(g, epi, s);   // the register-staged loop, whatever K
    case 1: return launch_tiles<128, 64, 64, 64, 32>(g, epi, s);
    case 2: return launch_tiles<256, 128, 32, 128, 64>(g, epi, s);
    case 3: return launch_tiles<128, 256, 32, 64, 128>(g, epi, s);
    case 4: return launch_tiles<256, 128, 64, 128, 64>(g, epi, s);
    case 5: return launch_tiles<128, 128, 32, 64, 64>(g, epi, s);
    case 6: return launch_tiles<64, 64, 64, 32, 32>(g, epi, s);
    case 7: return launch_tiles<32, 128, 64, 32, 32>(g, epi, s);
    case 8: return launch_tiles<256, 256, 32, 128, 128>(g, epi, s);
    case 11: return launch_tiles<256, 128, 64, 64, 64>(g, epi, s);    // 8 wavefronts
    case 12: return launch_tiles<256, 256, 32, 64, 64>(g, epi, s);    // 16 wavefronts
    case 13: return launch_tiles<256, 128, 32, 64, 64>(g, epi, s);    // 8 wavefronts, smaller stages
    case 16: return g.M <= 16 ? launch_rowstream(g, epi, s) : hipErrorInvalidValue;
    case 9: return g.M <= 64 ? launch_skinny_any(g, epi, s, 0) : hipErrorInvalidValue;
    case 10: return g.M <= 64 ? launch_skinny_any(g, epi, s, 1) : hipErrorInvalidValue;
    default: return hipErrorInvalidValue;
  }
}

// Split-K for small M: enough (tile, slice) workgroups to fill the chip once (32-row tiles) or twice, each slice at
// least two K steps long, the partial buffer permitting.  Returns 1 when splitting does not pay.
int choose_splits(const GemmArgs& g, int bm, int bn, size_t partial_floats) {
  const int tiles = ((g.M + bm - 1) / bm) * ((g.N + bn - 1) / bn) * g.parts;
  const int ksteps = (g.K + 63) / 64;
  // (measured on whole forward passes, workgroup targets from 128 to 2048: the 32x128 tiles of up to 32 rows do
  // best with one workgroup per CU, 3 x 8 tokens 2.77 -> 2.54 ms on the 6.7B/TP2 shard, 3.27 -> 2.91 ms on the
  // 13B/TP4 shard; the 64x64 tiles with two, every other target 5-25 % slower)
  const int target = bm <= 32 ? 256 : 512;
  int splits = target / (tiles > 0 ? tiles : 1);
  if (splits > ksteps / 2) splits = ksteps / 2;
  if (splits > 16) splits = 16;
  const size_t per_slice = static_cast<size_t>(g.M) * g.N * g.parts;
  if (per_slice && splits > static_cast<int>(partial_floats / per_slice)) splits = static_cast<int>(partial_floats / per_slice);
  return splits < 2 ? 1 : splits;
}

hipError_t launch_splitk(GemmArgs g, int cfg, int splits, int epi, hipStream_t s, PendingSum* defer) {
  g.splits = splits;
  hipError_t e = launch_config(cfg, g, EPI_PARTIAL, s);
  if (e != hipSuccess) return e;
  if (tuning().defer_sums && defer && epi == CTN_EPI_BIAS_RESID_F32 && g.parts == 1 && g.ldc == g.N) {
    // the caller's next kernel, a LayerNorm, reads x anyway and finishes the update there (with
    // few rows its variant that keeps every slice's load in flight at once: one kernel and one
    // memory round trip in place of two kernels)
    defer->partial = g.partial;
    defer->splits = splits;
    defer->bias = g.bias[0];
    return hipSuccess;
  }
  return launch_splitk_reduce(g, epi, s);
}


hipError_t dispatch(const GemmArgs& g, int epi, hipStream_t s, size_t partial_floats, PendingSum* defer = nullptr,
                    bool allow_tail = true) {
  if (defer) *defer = PendingSum{};
  if (g.M <= 0 || g.N <= 0) return hipSuccess;
  if (g.K <= 0 || g.K % 8 || g.parts < 1 || g.parts > 3) return hipErrorInvalidValue;
  for (int p = 0; p < g.parts; ++p)
    if (!g.W[p] || (epi != CTN_EPI_F32 && !g.bias[p])) return hipErrorInvalidValue;
  // operands are read in 16-byte pieces (K is a multiple of 8, so every row then starts on such a boundary)
  if (reinterpret_cast<uintptr_t>(g.A) % 16 || reinterpret_cast<uintptr_t>(g.out) % 4) return hipErrorInvalidValue;
  for (int p = 0; p < g.parts; ++p)
    if (reinterpret_cast<uintptr_t>(g.W[p]) % 16 || reinterpret_cast<uintptr_t>(g.bias[p]) % 2) return hipErrorInvalidValue;
  if (tuning().force_tile == 14 || tuning().force_tile == 15) {       // tuning hook: split-K over 64x64 / 32x128 tiles
    const int cfg = tuning().force_tile == 14 ? 6 : 7;
    const int splits = g.partial ? choose_splits(g, cfg == 6 ? 64 : 32, cfg == 6 ? 64 : 128, partial_floats) : 1;
    return splits > 1 ? launch_splitk(g, cfg, splits, epi, s, defer) : launch_config(cfg, g, epi, s);
  }
  if (tuning().force_tile >= 0 && !(tuning().force_tile >= 9 && tuning().force_tile <= 10 && g.M > 64) && !(tuning().force_tile == 16 && g.M > 16))
    return launch_config(tuning().force_tile, g, epi, s);
  if (g.M <= 64) {
    // measured on MI355X: very wide outputs (the vocabulary head) re-read A too often in the
    // streaming kernel; mid-size outputs take 32 features per workgroup to halve A's L2 traffic
    const int64_t n_total = static_cast<int64_t>(g.N) * g.parts;
    // The row-stream kernel launches one workgroup per 16 features.  A count a little over one per CU (320 for
    // the 5120 features of a 13B/TP4 layer) leaves most CUs waiting for the few that got two, and its cost
    // grows with the tokens (every workgroup reads all of A); from 9 tokens on the K-sliced tiles do better
    // there: 13B/TP4 forward of 12 tokens 2.88 -> 2.72 ms, of 16 tokens 3.16 -> 2.78 ms (8 tokens: 2.69 either way).
    const int rs_wgs = ((g.N + 15) / 16) * g.parts;
    const bool rs_poor = g.M > 8 && g.partial && rs_wgs > 256 && rs_wgs * 10 < 512 * 7;
    if (g.M <= 16 && g.K >= 4096 && !rs_poor) return launch_rowstream(g, epi, s);   // long rows: row-contiguous reads pay
    if (n_total > 16384) return launch_config(g.M <= 32 ? 7 : 6, g, epi, s);
    if ((g.M > 16 || rs_poor) && g.partial) {                        // LDS-staged tiles, K split across workgroups
      const int cfg = g.M <= 32 ? 7 : 6;
      const int splits = choose_splits(g, cfg == 6 ? 64 : 32, cfg == 6 ? 64 : 128, partial_floats);
      if (splits > 1) return launch_splitk(g, cfg, splits, epi, s, defer);
    }
    return launch_skinny_any(g, epi, s, n_total >= 6144 ? 1 : 0);
  }
  if (g.M <= 256 && g.partial && static_cast<int64_t>(g.N) * g.parts <= 16384) {
    // A few requests batched (the paper's workloads: up to 32 requests of 8 tokens): still bound by streaming
    // the weights once, so the same K-sliced 64x64 tiles as for 64 tokens, as long as slicing adds workgroups.
    const int splits = choose_splits(g, 64, 64, partial_floats);
    if (splits > 1) return launch_splitk(g, 6, splits, epi, s, defer);
  }
  // Tile choice by how the tile count fills 256 CUs (two workgroups per CU for the big tiles):
  const int t0 = ((g.M + 127) / 128) * ((g.N + 127) / 128) * g.parts;
  if (g.partial && t0 <= 256 && g.K >= 2048) {
    // at most one 128x128 tile per CU and a long K: two to four K slices fill the second workgroup
    // slot of every CU; the ordered reduction costs one more small kernel (or is left to the LayerNorm
    // that follows).  K = 2048 still pays: the out-projection of the 6.7B/TP2 shard at 1024 tokens,
    // 10.24 -> 10.08 ms per forward pass against 128x64 tiles in one pass.
    int splits = 512 / t0;
    if (splits > 4) splits = 4;
    const size_t per_slice = static_cast<size_t>(g.M) * g.N * g.parts;
    if (splits > static_cast<int>(partial_floats / per_slice)) splits = static_cast<int>(partial_floats / per_slice);
    if (splits >= 2) return launch_splitk(g, 0, splits, epi, s, defer);
  }
  if (t0 <= 128) return launch_config(6, g, epi, s);               // few tiles: 64x64
  if (t0 <= 320) return launch_config(1, g, epi, s);               // under one round: 128x64 doubles the count
  // A last round that fills at most half of the 512 slots (640 tiles of a 13B/TP4 layer, 1576 of the
  // vocabulary head) costs nearly a whole round.  The columns of the full rounds go out as one product and
  // the remaining columns as a second one whose tiles are cut along K, so that its workgroups fill the
  // chip too and each takes a fraction of a tile's time; a third, small kernel adds the slices in order.
  if (tuning().tail_split && allow_tail && g.partial && g.parts == 1 && t0 > 512 && t0 % 512 && t0 % 512 <= 256 &&
      g.K >= 2048 && g.K % 64 == 0) {
    const int tiles_m = (g.M + 127) / 128, tiles_n = (g.N + 127) / 128;
    const int n_main = (t0 / 512) * 512 / tiles_m;                  // column tiles of the full rounds
    const int tail_tiles = (tiles_n - n_main) * tiles_m;
    GemmArgs tail = g;
    tail.N = g.N - n_main * 128;
    int splits = 512 / tail_tiles;
    if (splits > 4) splits = 4;
    if (splits > g.K / 64 / 4) splits = g.K / 64 / 4;               // a slice keeps at least four K steps
    const size_t per_slice = static_cast<size_t>(g.M) * tail.N;
    if (splits > static_cast<int>(partial_floats / per_slice)) splits = static_cast<int>(partial_floats / per_slice);
    if (n_main > 0 && tail.N > 0 && splits >= 2) {
      GemmArgs main_part = g;
      main_part.N = n_main * 128;
      hipError_t e = dispatch(main_part, epi, s, partial_floats, nullptr, false);
      if (e != hipSuccess) return e;
      const size_t skip = static_cast<size_t>(n_main) * 128;
      tail.W[0] = g.W[0] + skip * g.K;
      if (tail.bias[0]) tail.bias[0] = g.bias[0] + skip;
      const size_t elem = (epi == CTN_EPI_BIAS_F16 || epi == CTN_EPI_BIAS_RELU_F16) ? 2 : 4;
      tail.out = static_cast<char*>(g.out) + skip * elem;
      return launch_splitk(tail, 0, splits, epi, s, nullptr);
    }
  }
  // Plenty of tiles: 128x128x64 (4 wavefronts) or 256x128x32 (8 wavefronts of 64x64), both two
  // workgroups per CU, i.e. 512 per round.  The wide tile moves 1.15 times the flops per unit time
  // when its rounds are full (measured at 1500-3000 tiles); what decides is the last, partly
  // filled round, so compare rounds x work per tile: (M=2048, N=10240) 3 rounds of 128x128 beat 2
  // rounds of 256x128, (M=4096, N=8192) 2 wide rounds beat 4 narrow ones.
  const int t_wide = ((g.M + 255) / 256) * ((g.N + 127) / 128) * g.parts;
  const int rounds_narrow = (t0 + 511) / 512, rounds_wide = (t_wide + 511) / 512;
  // (measured inside the forward pass, weights coming from HBM: this rule still holds with direct-to-LDS
  // fills in the 128x128x64 tile, whose advantage over the wide tile is confined to operands that are already
  // in the last-level cache)
  // Where that comparison favoured the wide tile, the 128x128x64 tile with its loads two steps ahead now does
  // a little better still inside the forward pass (13B shards: 22.5 -> 22.2 and 19.6 -> 19.4 ms).
  if (173 * rounds_wide < 100 * rounds_narrow) {
    // a short K (the out-projection of a finely split shard: K = hidden / TP) has few steps per tile to hide
    // a stage's latency behind; half-size steps do better (13B / TP4 forward 22.4 -> 21.9 ms)
    if (g.K <= 2560) return launch_config(5, g, epi, s);
    return launch_config(tuning().deep_loads && g.K % 64 == 0 ? 17 : 13, g, epi, s);
  }
  return launch_config(0, g, epi, s);
}

}  // namespace

int gemm_tuning_set(GemmTuning& t, int cfg) {
  if (cfg == 100 || cfg == 101) {      // direct-to-LDS stage fills off / on
    t.direct_fill = cfg == 101;
    return 0;
  }
  if (cfg == 102 || cfg == 103) {      // global loads two steps ahead off / on
    t.deep_loads = cfg == 103;
    return 0;
  }
  if (cfg == 108 || cfg == 109) {      // K-sliced tail columns off / on
    t.tail_split = cfg == 109;
    return 0;
  }
  if (cfg == 106 || cfg == 107) {      // four-column split-K reduction off / on
    t.reduce4 = cfg == 107;
    return 0;
  }
  if (cfg == 104 || cfg == 105) {      // summation of split residual products left to LayerNorm off / on
    t.defer_sums = cfg == 105;
    return 0;
  }
  if (cfg < -1 || cfg > 17) return -1;
  t.force_tile = cfg;
  return 0;
}

hipError_t launch_gemm(const _Float16* A, const _Float16* W, const _Float16* bias, void* out, int M, int N,
                       int K, int epi, hipStream_t s, float* partial, size_t partial_floats, PendingSum* defer,
                       const GemmTuning* tune) {
  const TuningScope scope(tune);
  GemmArgs g{};
  g.A = A; g.W[0] = W; g.bias[0] = bias; g.out = out;
  g.M = M; g.N = N; g.K = K; g.ldc = N; g.parts = 1; g.splits = 1; g.partial = partial;
  return dispatch(g, epi, s, partial_floats, defer);
}

hipError_t launch_gemm3(const _Float16* A, const _Float16* const W[3], const _Float16* const bias[3], void* out,
                        int M, int N, int K, int epi, hipStream_t s, float* partial, size_t partial_floats,
                        const GemmTuning* tune) {
  const TuningScope scope(tune);
  GemmArgs g{};
  g.A = A; g.out = out;
  for (int p = 0; p < 3; ++p) { g.W[p] = W[p]; g.bias[p] = bias[p]; }
  g.M = M; g.N = N; g.K = K; g.ldc = 3 * N; g.parts = 3; g.splits = 1; g.partial = partial;
  return dispatch(g, epi, s, partial_floats);
}

}  // namespace ctn
