// Internal launch interface of the HIP kernels (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <cstddef>
#include <cstdint>

namespace ctn {

// ---- copy (swap-in / swap-out) ---------------------------------------------
constexpr int kCopyMaxSegs = 16;
struct CopySeg {
  const void* src;
  void* dst;
  uint64_t n16;  // number of 16-byte units
};
struct CopyTable {
  int32_t n;
  int32_t threads;                          // workgroup size the chunk counts were made for
  uint32_t chunk_prefix[kCopyMaxSegs + 1];  // chunks before segment i
  CopySeg seg[kCopyMaxSegs];
};
// Width of a copy launch is given in wavefronts: a multiple of 4 runs as workgroups of 256 threads, another
// even count as workgroups of 128, an odd count as single-wavefront workgroups.
int copy_workgroup_threads(int waves);
// Fills chunk_prefix from seg[].n16 for workgroups of `threads`; returns false if the table is too large.
bool copy_table_finish(CopyTable& t, int threads);
enum { kCopyH2D = 0, kCopyD2H = 1, kCopyOther = 2 };
// waves <= 0: the library default.  The table must have been finished for copy_workgroup_threads(waves).
hipError_t launch_copy_table(const CopyTable& t, int waves, hipStream_t s, int dir);
int default_copy_waves();

// A residual update that a split-K product has left undone: x[row][col] += sum over slices (in
// slice order) of partial[slice][row][col] + bias[col].  splits == 0: nothing pending.
struct PendingSum {
  const float* partial = nullptr;
  int splits = 0;
  const _Float16* bias = nullptr;
};

// ---- elementwise -------------------------------------------------------------
hipError_t launch_embed(const int32_t* ids, const _Float16* tok, const _Float16* pos, float* x, int M,
                        int seq, int hidden, int vocab_local, int rank, hipStream_t s);
// pending (optional): apply that residual update to x (x is written back) before normalising.
hipError_t launch_layernorm(float* x, const _Float16* g, const _Float16* b, _Float16* out, int rows, int hidden,
                            hipStream_t s, const PendingSum* pending = nullptr);

// ---- dense products ------------------------------------------------------------
// Switches for tests and tuning runs; the defaults are what the library uses.  The values of
// gemm_tuning_set are listed at ctn_debug_gemm_tile in the test header.
struct GemmTuning {
  int force_tile = -1;        // >= 0: one tile configuration for every product
  bool deep_loads = true;     // register-staged tiles keep a second stage of loads in flight
  bool direct_fill = true;    // 128x128x64 tiles filled straight from global memory into LDS
  bool reduce4 = true;        // the second pass of a K-sliced product reads four columns per thread
  bool defer_sums = true;     // a K-sliced row-parallel product may leave its sum to the next LayerNorm
  bool tail_split = true;     // columns of a thinly filled last round of tiles computed in K slices
};
int gemm_tuning_set(GemmTuning& t, int cfg);   // 0, or -1 for a value that means nothing
// partial / partial_floats: optional fp32 scratch (device) that allows small-M products to split K
// across workgroups; nullptr keeps every product in one pass.
// defer (optional, residual epilogue only): when the product is split, leave the summation of the
// slices and the residual update to the caller (*defer describes it) instead of running the reduce kernel.
// tune (optional): switches for this call; nullptr = defaults.
hipError_t launch_gemm(const _Float16* A, const _Float16* W, const _Float16* bias, void* out, int M, int N,
                       int K, int epilogue, hipStream_t s, float* partial = nullptr, size_t partial_floats = 0,
                       PendingSum* defer = nullptr, const GemmTuning* tune = nullptr);
// Three products sharing A in one launch: out[M, 3N] = [A W0^T + b0 | A W1^T + b1 | A W2^T + b2].
hipError_t launch_gemm3(const _Float16* A, const _Float16* const W[3], const _Float16* const bias[3], void* out,
                        int M, int N, int K, int epilogue, hipStream_t s, float* partial = nullptr,
                        size_t partial_floats = 0, const GemmTuning* tune = nullptr);
hipError_t launch_attention(const _Float16* qkv, _Float16* out, int batch, int seq, int heads, int head_dim,
                            hipStream_t s);

}  // namespace ctn
