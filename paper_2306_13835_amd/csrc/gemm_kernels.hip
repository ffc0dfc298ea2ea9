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
#include "computron.h"
#include "kernels.h"

namespace ctn {

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int BK = 64;          // K extent of one LDS stage
constexpr int LDS_PAD = 8;      // halves of padding per LDS row (16 bytes)
constexpr int LDS_ROW = BK + LDS_PAD;
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
};

template <int BM, int BN, int WM, int WN, int EPI>
__global__ __launch_bounds__(256) void gemm_nt_kernel(const GemmArgs g) {
  static_assert((BM / WM) * (BN / WN) == 4, "four wavefronts per workgroup");
  static_assert(WM % 32 == 0 && WN % 32 == 0 && BM % 32 == 0 && BN % 32 == 0, "32x32 MFMA tiles");
  constexpr int TM = WM / 32, TN = WN / 32;     // MFMA tiles per wavefront
  constexpr int PA = BM / 32, PB = BN / 32;     // 32-row passes of the cooperative loads

  __shared__ __attribute__((aligned(16))) _Float16 As[2][BM][LDS_ROW];
  __shared__ __attribute__((aligned(16))) _Float16 Bs[2][BN][LDS_ROW];

  const int M = g.M, N = g.N, K = g.K;
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  int tile = xcd_remap(blockIdx.x, tiles_m * tiles_n * g.parts);
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
  const int lrow = tid >> 3, lcol = (tid & 7) * 8;   // cooperative load: 32 rows x 8 lanes x 16 B

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
      const int r = m0 + p * 32 + lrow;
      ra[p] = u32x4{0u, 0u, 0u, 0u};
      if (r < M && kc < K) ra[p] = *reinterpret_cast<const u32x4*>(A + static_cast<int64_t>(r) * K + kc);
    }
#pragma unroll
    for (int p = 0; p < PB; ++p) {
      const int r = n0 + p * 32 + lrow;
      rb[p] = u32x4{0u, 0u, 0u, 0u};
      if (r < N && kc < K) rb[p] = *reinterpret_cast<const u32x4*>(W + static_cast<int64_t>(r) * K + kc);
    }
  };
  auto store_lds = [&](int buf) {
#pragma unroll
    for (int p = 0; p < PA; ++p) *reinterpret_cast<u32x4*>(&As[buf][p * 32 + lrow][lcol]) = ra[p];
#pragma unroll
    for (int p = 0; p < PB; ++p) *reinterpret_cast<u32x4*>(&Bs[buf][p * 32 + lrow][lcol]) = rb[p];
  };

  const int ksteps = (K + BK - 1) / BK;
  load_global(0);
  store_lds(0);
  __syncthreads();

  const int frow = lane & 31, fcol = (lane >> 5) * 8;
  for (int kt = 0; kt < ksteps; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < ksteps) load_global((kt + 1) * BK);   // in flight while this stage is multiplied
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

  // Accumulator layout of the 32x32 tile: lane holds column (lane % 32) and
  // rows 8*(e/4) + 4*(lane/32) + e%4 for e = 0..15.
  const int col_in = lane & 31, row_in = (lane >> 5) * 4;
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int n = n0 + wn0 + j * 32 + col_in;
    if (n >= N) continue;
    float bv = 0.f;
    if (EPI != CTN_EPI_F32) bv = static_cast<float>(bias[n]);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = m0 + wm0 + i * 32 + 8 * (e >> 2) + row_in + (e & 3);
        if (m >= M) continue;
        const int64_t o = static_cast<int64_t>(m) * ldc + col0 + n;
        const float v = acc[i][j][e] + bv;
        if (EPI == CTN_EPI_BIAS_F16) {
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

template <int BM, int BN, int WM, int WN>
hipError_t launch_tiles(const GemmArgs& g, int epi, hipStream_t s) {
  const int tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN) * g.parts;
  const dim3 grid(tiles), block(256);
#define CTN_GEMM(E) hipLaunchKernelGGL((gemm_nt_kernel<BM, BN, WM, WN, E>), grid, block, 0, s, g)
  switch (epi) {
    case CTN_EPI_BIAS_F16: CTN_GEMM(CTN_EPI_BIAS_F16); break;
    case CTN_EPI_BIAS_RELU_F16: CTN_GEMM(CTN_EPI_BIAS_RELU_F16); break;
    case CTN_EPI_BIAS_RESID_F32: CTN_GEMM(CTN_EPI_BIAS_RESID_F32); break;
    case CTN_EPI_F32: CTN_GEMM(CTN_EPI_F32); break;
    default: return hipErrorInvalidValue;
  }
#undef CTN_GEMM
  return hipGetLastError();
}

}  // namespace

static hipError_t dispatch(const GemmArgs& g, int epi, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0) return hipSuccess;
  if (g.K <= 0 || g.K % 8 || g.parts < 1 || g.parts > 3) return hipErrorInvalidValue;
  for (int p = 0; p < g.parts; ++p)
    if (!g.W[p] || (epi != CTN_EPI_F32 && !g.bias[p])) return hipErrorInvalidValue;
  if (g.M <= 32) return launch_tiles<32, 128, 32, 32>(g, epi, s);
  if (g.M <= 64) return launch_tiles<64, 64, 32, 32>(g, epi, s);
  return launch_tiles<128, 128, 64, 64>(g, epi, s);
}

hipError_t launch_gemm(const _Float16* A, const _Float16* W, const _Float16* bias, void* out, int M, int N,
                       int K, int epi, hipStream_t s) {
  GemmArgs g{};
  g.A = A; g.W[0] = W; g.bias[0] = bias; g.out = out;
  g.M = M; g.N = N; g.K = K; g.ldc = N; g.parts = 1;
  return dispatch(g, epi, s);
}

hipError_t launch_gemm3(const _Float16* A, const _Float16* const W[3], const _Float16* const bias[3], void* out,
                        int M, int N, int K, int epi, hipStream_t s) {
  GemmArgs g{};
  g.A = A; g.out = out;
  for (int p = 0; p < 3; ++p) { g.W[p] = W[p]; g.bias[p] = bias[p]; }
  g.M = M; g.N = N; g.K = K; g.ldc = 3 * N; g.parts = 3;
  return dispatch(g, epi, s);
}

}  // namespace ctn
