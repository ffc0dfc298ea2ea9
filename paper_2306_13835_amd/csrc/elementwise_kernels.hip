// Token/position embedding and LayerNorm of the shard forward pass.
//
// The paper only names the model (OPT, Section 5.1); these are the public OPT
// decoder's steps at the rank's shapes.  Both kernels are bound by HBM
// bandwidth: embed reads 2*hidden*2 B and writes 4*hidden B per token,
// LayerNorm reads 4*hidden B and writes 2*hidden B per row.
#include "kernels.h"
#include "layout.hpp"

namespace ctn {

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));

// One workgroup per token row.  Vocabulary-parallel lookup: ids outside this
// rank's slice contribute a zero row; positions are shifted by two rows.
__global__ __launch_bounds__(256) void embed_kernel(const int32_t* __restrict__ ids,
                                                    const _Float16* __restrict__ tok,
                                                    const _Float16* __restrict__ pos, float* __restrict__ x,
                                                    int seq, int hidden, int vocab_local, int rank) {
  const int m = blockIdx.x;
  const int64_t local = static_cast<int64_t>(ids[m]) - static_cast<int64_t>(rank) * vocab_local;
  const bool inside = local >= 0 && local < vocab_local;
  const half8* trow = reinterpret_cast<const half8*>(tok + (inside ? local : 0) * hidden);
  const half8* prow = reinterpret_cast<const half8*>(pos + static_cast<int64_t>(m % seq + 2) * hidden);
  float* xr = x + static_cast<int64_t>(m) * hidden;
  for (int c = threadIdx.x; c < hidden / 8; c += blockDim.x) {
    half8 p = prow[c];
    half8 t = {0, 0, 0, 0, 0, 0, 0, 0};
    if (inside) t = trow[c];
    float4v lo, hi;
    for (int e = 0; e < 4; ++e) {
      lo[e] = static_cast<float>(t[e]) + static_cast<float>(p[e]);
      hi[e] = static_cast<float>(t[e + 4]) + static_cast<float>(p[e + 4]);
    }
    reinterpret_cast<float4v*>(xr)[2 * c] = lo;
    reinterpret_cast<float4v*>(xr)[2 * c + 1] = hi;
  }
}

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// One workgroup of WAVES wavefronts per row, the row held in registers (NV
// float4 per lane): mean, then the mean of squared deviations (biased), each
// reduced across the wavefront by shuffles and across wavefronts through LDS,
// then normalise, scale, shift, round to fp16.  Several wavefronts per row
// keep enough loads in flight per CU when there are only a few thousand rows.
// FUSE: first finish a split-K product's residual update of this row (x +=
// slices + bias, written back to x), in the same order of additions as the
// stand-alone reduction.
constexpr int kFewRows = 256;   // up to here rows go to the wide one-round-trip kernel

template <int WAVES>
__device__ inline float block_sum(float v, float* scratch) {
  v = wave_sum(v);
  if (WAVES == 1) return v;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();                       // scratch may still be read from the previous reduction
  if (lane == 0) scratch[wave] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int w = 0; w < WAVES; ++w) t += scratch[w];    // same order in every thread
  return t;
}

template <int NV, int WAVES, bool FUSE>
__global__ __launch_bounds__(WAVES * 64) void layernorm_kernel(float* __restrict__ x, const _Float16* __restrict__ g,
                                                               const _Float16* __restrict__ b,
                                                               _Float16* __restrict__ out, int rows, int hidden,
                                                               const PendingSum pend) {
  __shared__ float scratch[WAVES];
  const int row = blockIdx.x;
  float4v* xr = reinterpret_cast<float4v*>(x + static_cast<int64_t>(row) * hidden);
  const int nvec = hidden / 4;
  float4v v[NV];
  half4 gg[NV], bb[NV];      // gain and bias travel together with the row: one memory round trip, not two
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = threadIdx.x + i * WAVES * 64;
    if (c < nvec) {
      v[i] = xr[c];
      gg[i] = reinterpret_cast<const half4*>(g)[c];
      bb[i] = reinterpret_cast<const half4*>(b)[c];
      if (FUSE) {
        float4v t = {0.f, 0.f, 0.f, 0.f};
        for (int sl = 0; sl < pend.splits; ++sl)
          t += reinterpret_cast<const float4v*>(pend.partial + (static_cast<int64_t>(sl) * rows + row) * hidden)[c];
        const half4 pb = reinterpret_cast<const half4*>(pend.bias)[c];
#pragma unroll
        for (int e = 0; e < 4; ++e) t[e] += static_cast<float>(pb[e]);
        v[i] += t;
        xr[c] = v[i];
      }
      sum += (v[i][0] + v[i][1]) + (v[i][2] + v[i][3]);
    } else {
      v[i] = float4v{0.f, 0.f, 0.f, 0.f};
    }
  }
  const float mean = block_sum<WAVES>(sum, scratch) / static_cast<float>(hidden);
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = threadIdx.x + i * WAVES * 64;
    if (c < nvec) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[i][e] -= mean;
        sq += v[i][e] * v[i][e];
      }
    }
  }
  const float var = block_sum<WAVES>(sq, scratch) / static_cast<float>(hidden);
  const float inv = 1.0f / sqrtf(var + 1e-5f);
  _Float16* orow = out + static_cast<int64_t>(row) * hidden;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = threadIdx.x + i * WAVES * 64;
    if (c < nvec) {
      half4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        o[e] = static_cast<_Float16>(v[i][e] * inv * static_cast<float>(gg[i][e]) + static_cast<float>(bb[i][e]));
      reinterpret_cast<half4*>(orow)[c] = o;
    }
  }
}

// Few rows (a small batch), with or without a pending split-K residual update (MAXS = 0: none):
// one workgroup per row, wide enough that a thread owns one or two float4 of the row, and every
// slice of the pending sum loaded before the first is used (MAXS loads in flight per thread, slices past the last one
// re-read slice 0 and are dropped by a select), so a row costs one memory round trip instead of
// one per slice.  The additions run in slice order from +0, then the bias, then x: the same
// order, hence the same bits, as the stand-alone reduction followed by the plain kernel.
template <int NV, int WAVES, int MAXS>
__global__ __launch_bounds__(WAVES * 64) void layernorm_fewrows_kernel(float* __restrict__ x,
                                                                       const _Float16* __restrict__ g,
                                                                       const _Float16* __restrict__ b,
                                                                       _Float16* __restrict__ out, int rows, int hidden,
                                                                       const PendingSum pend) {
  __shared__ float scratch[WAVES];
  const int row = blockIdx.x;
  float4v* xr = reinterpret_cast<float4v*>(x + static_cast<int64_t>(row) * hidden);
  const int nvec = hidden / 4;
  const int64_t slice_vecs = static_cast<int64_t>(rows) * nvec;
  const float4v* prow = reinterpret_cast<const float4v*>(pend.partial) + static_cast<int64_t>(row) * nvec;
  float4v v[NV];
  half4 gg[NV], bb[NV];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = threadIdx.x + i * WAVES * 64;
    const bool ok = c < nvec;
    const int cc = ok ? c : 0;                       // always a valid address; the value is dropped below
    if constexpr (MAXS > 0) {
      float4v p[MAXS];
#pragma unroll
      for (int sl = 0; sl < MAXS; ++sl) p[sl] = prow[(sl < pend.splits ? sl : 0) * slice_vecs + cc];
      v[i] = xr[cc];
      gg[i] = reinterpret_cast<const half4*>(g)[cc];
      bb[i] = reinterpret_cast<const half4*>(b)[cc];
      const half4 pb = reinterpret_cast<const half4*>(pend.bias)[cc];
      float4v t = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int sl = 0; sl < MAXS; ++sl) t += sl < pend.splits ? p[sl] : float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int e = 0; e < 4; ++e) t[e] += static_cast<float>(pb[e]);
      v[i] += t;
      if (ok) xr[c] = v[i];
    } else {                                         // nothing pending: the plain LayerNorm of a few rows
      v[i] = xr[cc];
      gg[i] = reinterpret_cast<const half4*>(g)[cc];
      bb[i] = reinterpret_cast<const half4*>(b)[cc];
    }
    if (ok) sum += (v[i][0] + v[i][1]) + (v[i][2] + v[i][3]);
  }
  const float mean = block_sum<WAVES>(sum, scratch) / static_cast<float>(hidden);
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    if (static_cast<int>(threadIdx.x) + i * WAVES * 64 < nvec) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[i][e] -= mean;
        sq += v[i][e] * v[i][e];
      }
    }
  }
  const float var = block_sum<WAVES>(sq, scratch) / static_cast<float>(hidden);
  const float inv = 1.0f / sqrtf(var + 1e-5f);
  _Float16* orow = out + static_cast<int64_t>(row) * hidden;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = threadIdx.x + i * WAVES * 64;
    if (c < nvec) {
      half4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        o[e] = static_cast<_Float16>(v[i][e] * inv * static_cast<float>(gg[i][e]) + static_cast<float>(bb[i][e]));
      reinterpret_cast<half4*>(orow)[c] = o;
    }
  }
}

template <int NV, int WAVES>
void launch_fewrows(float* x, const _Float16* g, const _Float16* b, _Float16* out, int rows, int hidden,
                    hipStream_t s, const PendingSum& pend) {
  const dim3 grid(rows), block(WAVES * 64);
  if (pend.splits <= 0)
    hipLaunchKernelGGL((layernorm_fewrows_kernel<NV, WAVES, 0>), grid, block, 0, s, x, g, b, out, rows, hidden, pend);
  else if (pend.splits <= 4)
    hipLaunchKernelGGL((layernorm_fewrows_kernel<NV, WAVES, 4>), grid, block, 0, s, x, g, b, out, rows, hidden, pend);
  else if (pend.splits <= 8)
    hipLaunchKernelGGL((layernorm_fewrows_kernel<NV, WAVES, 8>), grid, block, 0, s, x, g, b, out, rows, hidden, pend);
  else
    hipLaunchKernelGGL((layernorm_fewrows_kernel<NV, WAVES, 16>), grid, block, 0, s, x, g, b, out, rows, hidden, pend);
}

}  // namespace

hipError_t launch_embed(const int32_t* ids, const _Float16* tok, const _Float16* pos, float* x, int M, int seq,
                        int hidden, int vocab_local, int rank, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  if (hidden % 8 || seq <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(embed_kernel, dim3(M), dim3(256), 0, s, ids, tok, pos, x, seq, hidden, vocab_local, rank);
  return hipGetLastError();
}

hipError_t launch_layernorm(float* x, const _Float16* g, const _Float16* b, _Float16* out, int rows, int hidden,
                            hipStream_t s, const PendingSum* pending) {
  if (rows <= 0) return hipSuccess;
  static_assert(kMaxHidden == 256 * 4 * 16, "registration admits exactly the widths these kernels cover");
  if (hidden % 4 || hidden <= 0 || hidden > kMaxHidden) return hipErrorInvalidValue;
  const bool fuse = pending && pending->splits > 0;
  const PendingSum pend = fuse ? *pending : PendingSum{};
  const dim3 grid(rows);
  const int nvec = hidden / 4;
  if (rows <= kFewRows && nvec > 64) {     // with or without a pending sum: both reduce the row in the same order
    if (pend.splits > 16) return hipErrorInvalidValue;
    if (nvec <= 256) launch_fewrows<1, 4>(x, g, b, out, rows, hidden, s, pend);          // up to 1024 columns
    else if (nvec <= 512) launch_fewrows<1, 8>(x, g, b, out, rows, hidden, s, pend);     // 2048
    else if (nvec <= 1024) launch_fewrows<1, 16>(x, g, b, out, rows, hidden, s, pend);   // 4096
    else if (nvec <= 1280) launch_fewrows<2, 10>(x, g, b, out, rows, hidden, s, pend);   // 5120
    else if (nvec <= 2048) launch_fewrows<2, 16>(x, g, b, out, rows, hidden, s, pend);   // up to 8192
    else if (nvec <= 3072) launch_fewrows<3, 16>(x, g, b, out, rows, hidden, s, pend);   // 9216, 12288
    else launch_fewrows<4, 16>(x, g, b, out, rows, hidden, s, pend);                     // up to 16384
    return hipGetLastError();
  }
#define CTN_LN(NV, WAVES)                                                                                     \
  do {                                                                                                        \
    if (fuse) hipLaunchKernelGGL((layernorm_kernel<NV, WAVES, true>), grid, dim3(WAVES * 64), 0, s, x, g, b, out, rows, hidden, pend);  \
    else hipLaunchKernelGGL((layernorm_kernel<NV, WAVES, false>), grid, dim3(WAVES * 64), 0, s, x, g, b, out, rows, hidden, pend); \
  } while (0)
  if (nvec <= 64) CTN_LN(1, 1);            // up to 256 columns: one wavefront
  else if (nvec <= 256) CTN_LN(1, 4);      // up to 1024 columns
  else if (nvec <= 512) CTN_LN(2, 4);      // 2048
  else if (nvec <= 1024) CTN_LN(4, 4);     // 4096
  else if (nvec <= 1536) CTN_LN(6, 4);     // 5120, 6144
  else if (nvec <= 2048) CTN_LN(8, 4);     // up to 8192
  else if (nvec <= 3072) CTN_LN(12, 4);    // 9216, 12288
  else CTN_LN(16, 4);                      // up to 16384
#undef CTN_LN
  return hipGetLastError();
}

}  // namespace ctn
