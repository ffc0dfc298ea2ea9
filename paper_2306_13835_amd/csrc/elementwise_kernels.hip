// Token/position embedding and LayerNorm of the shard forward pass.
//
// The paper only names the model (OPT, Section 5.1); these are the public OPT
// decoder's steps at the rank's shapes.  Both kernels are bound by HBM
// bandwidth: embed reads 2*hidden*2 B and writes 4*hidden B per token,
// LayerNorm reads 4*hidden B and writes 2*hidden B per row.
#include "kernels.h"

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

// One 64-lane wavefront per row, the row held in registers (NV float4 per
// lane): mean, then the mean of squared deviations (biased), both reduced
// across the wavefront, then normalise, scale, shift, round to fp16.
// FUSE: first finish a split-K product's residual update of this row (x += slices + bias, written
// back to x), in the same order of additions as the stand-alone reduction.
template <int NV, bool FUSE>
__global__ __launch_bounds__(256) void layernorm_kernel(float* __restrict__ x, const _Float16* __restrict__ g,
                                                        const _Float16* __restrict__ b,
                                                        _Float16* __restrict__ out, int rows, int hidden,
                                                        const PendingSum pend) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  float4v* xr = reinterpret_cast<float4v*>(x + static_cast<int64_t>(row) * hidden);
  const int nvec = hidden / 4;
  float4v v[NV];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = lane + i * 64;
    if (c < nvec) {
      v[i] = xr[c];
      if (FUSE) {
        float4v t = {0.f, 0.f, 0.f, 0.f};
        for (int sl = 0; sl < pend.splits; ++sl)
          t += reinterpret_cast<const float4v*>(pend.partial + (static_cast<int64_t>(sl) * rows + row) * hidden)[c];
        const half4 bb = reinterpret_cast<const half4*>(pend.bias)[c];
#pragma unroll
        for (int e = 0; e < 4; ++e) t[e] += static_cast<float>(bb[e]);
        v[i] += t;
        xr[c] = v[i];
      }
      sum += (v[i][0] + v[i][1]) + (v[i][2] + v[i][3]);
    } else {
      v[i] = float4v{0.f, 0.f, 0.f, 0.f};
    }
  }
  const float mean = wave_sum(sum) / static_cast<float>(hidden);
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = lane + i * 64;
    if (c < nvec) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[i][e] -= mean;
        sq += v[i][e] * v[i][e];
      }
    }
  }
  const float var = wave_sum(sq) / static_cast<float>(hidden);
  const float inv = 1.0f / sqrtf(var + 1e-5f);
  _Float16* orow = out + static_cast<int64_t>(row) * hidden;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = lane + i * 64;
    if (c < nvec) {
      const half4 gg = reinterpret_cast<const half4*>(g)[c];
      const half4 bb = reinterpret_cast<const half4*>(b)[c];
      half4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        o[e] = static_cast<_Float16>(v[i][e] * inv * static_cast<float>(gg[e]) + static_cast<float>(bb[e]));
      reinterpret_cast<half4*>(orow)[c] = o;
    }
  }
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
  if (hidden % 4 || hidden <= 0 || hidden > 64 * 4 * 32) return hipErrorInvalidValue;
  const dim3 grid((rows + 3) / 4), block(256);
  const int nv = (hidden / 4 + 63) / 64;
  const bool fuse = pending && pending->splits > 0;
  const PendingSum pend = fuse ? *pending : PendingSum{};
#define CTN_LN(NV)                                                                                              \
  do {                                                                                                          \
    if (fuse) hipLaunchKernelGGL((layernorm_kernel<NV, true>), grid, block, 0, s, x, g, b, out, rows, hidden, pend);  \
    else hipLaunchKernelGGL((layernorm_kernel<NV, false>), grid, block, 0, s, x, g, b, out, rows, hidden, pend); \
  } while (0)
  if (nv <= 4) CTN_LN(4);
  else if (nv <= 8) CTN_LN(8);
  else if (nv <= 16) CTN_LN(16);
  else if (nv <= 20) CTN_LN(20);
  else CTN_LN(32);
#undef CTN_LN
  return hipGetLastError();
}

}  // namespace ctn
