// Causal self-attention of one tensor-parallel rank's heads, fused:
//   out = softmax_causal((q d^-1/2) k^T) v        per (batch, head)
// with scores, probabilities and the running maximum / sum kept in fp32
// registers and never written to memory (one pass over the keys with a
// running rescale).  The paper names the model only (OPT, Section 5.1); this
// is the attention of the public OPT decoder on the heads this rank owns
// (Section 3.1: tensor parallel workers).
//
// Mapping to the matrix cores (v_mfma_f32_32x32x16_f16): a wavefront owns 32
// queries.  It forms the TRANSPOSED score tile  S^T[key, query] = K Q^T  so
// that in the accumulator layout every lane holds one query column and 16
// keys: the row-wise softmax statistics are then per-lane values plus one
// exchange with lane ^ 32.  The probabilities, rounded to fp16, are fed back
// unchanged as the B operand of  O^T[dim, query] = V^T P^T ; the contraction
// index of that product is permuted the same way for both operands, so no
// data movement is needed.
//
// K and V^T of up to 256 keys at a time are staged in LDS for the 4 wavefronts
// (128 queries) of a workgroup: every global load of the chunk is in flight
// before the first LDS write, so a sequence of 256 tokens pays the memory
// latency once and crosses two barriers, not two per 32 keys.  V is transposed
// on the way in: a thread loads 8 dims of 4 consecutive keys and writes, per
// dim, the 4 keys as one 8-byte LDS store.
//
// Share of the forward pass: ~1 % of the flops at the benchmark shapes.
#include "kernels.h"

namespace ctn {

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int QB = 128;    // queries per workgroup (4 wavefronts x 32)
constexpr int KT = 32;     // keys per score tile
constexpr int CH = 256;    // keys staged in LDS at a time
constexpr int VT_ROW = CH + 4;

template <int D>
__global__ __launch_bounds__(256) void attention_kernel(const _Float16* __restrict__ qkv,
                                                        _Float16* __restrict__ out, int seq, int heads) {
  constexpr int KS = D / 16;        // MFMA steps over the head dimension
  constexpr int DT = D / 32;        // 32-row tiles of O^T
  constexpr int K_ROW = D + 8;
  constexpr int PARTS = D / 8;      // 16-byte pieces of one key or value row
  constexpr int K_ITEMS = CH * PARTS / 256;        // per thread and chunk: rows x pieces of K
  constexpr int V_ITEMS = (CH / 4) * PARTS / 256;  // ... groups of 4 keys x pieces of V
  __shared__ __attribute__((aligned(16))) _Float16 Ks[CH][K_ROW];
  __shared__ __attribute__((aligned(16))) _Float16 Vt[D][VT_ROW];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int head = blockIdx.y, b = blockIdx.z;
  const int HL = heads * D, ld = 3 * HL;
  const int q0 = blockIdx.x * QB;
  const int qw0 = q0 + wave * 32;
  const int g = lane >> 5;
  const int qi = qw0 + (lane & 31);               // this lane's query
  const int qload = qi < seq ? qi : seq - 1;      // clamp: rows past the end are computed but not stored
  const _Float16* base = qkv + static_cast<int64_t>(b) * seq * ld + head * D;

  half8 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
    qf[ks] = *reinterpret_cast<const half8*>(base + static_cast<int64_t>(qload) * ld + ks * 16 + g * 8);

  float16v o[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[t][e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float scale = (D == 64) ? 0.125f : 0.08838834764831845f;   // d^-1/2

  const int q_last_wg = (q0 + QB - 1 < seq - 1) ? q0 + QB - 1 : seq - 1;
  const int n_tiles = q_last_wg / KT + 1;          // key tiles up to the workgroup's diagonal
  const int my_tiles = (qw0 + 31) / KT + 1;        // ... up to this wavefront's diagonal

  for (int c0 = 0; c0 < n_tiles * KT; c0 += CH) {
    const int n_keys = (n_tiles * KT - c0 < CH) ? n_tiles * KT - c0 : CH;   // a multiple of 32
    if (c0) __syncthreads();                        // previous chunk fully consumed
    // every load of the chunk first, then the LDS writes
    half8 kreg[K_ITEMS], vreg[V_ITEMS][4];
#pragma unroll
    for (int i = 0; i < K_ITEMS; ++i) {
      const int it = tid + i * 256, key = it / PARTS, part = it % PARTS;
      kreg[i] = half8{0, 0, 0, 0, 0, 0, 0, 0};
      if (key < n_keys && c0 + key < seq)
        kreg[i] = *reinterpret_cast<const half8*>(base + static_cast<int64_t>(c0 + key) * ld + HL + part * 8);
    }
#pragma unroll
    for (int i = 0; i < V_ITEMS; ++i) {
      const int it = tid + i * 256, kg = it / PARTS, part = it % PARTS;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int key = 4 * kg + j;
        vreg[i][j] = half8{0, 0, 0, 0, 0, 0, 0, 0};
        if (key < n_keys && c0 + key < seq)
          vreg[i][j] = *reinterpret_cast<const half8*>(base + static_cast<int64_t>(c0 + key) * ld + 2 * HL + part * 8);
      }
    }
#pragma unroll
    for (int i = 0; i < K_ITEMS; ++i) {
      const int it = tid + i * 256, key = it / PARTS, part = it % PARTS;
      if (key < n_keys) *reinterpret_cast<half8*>(&Ks[key][part * 8]) = kreg[i];
    }
#pragma unroll
    for (int i = 0; i < V_ITEMS; ++i) {
      const int it = tid + i * 256, kg = it / PARTS, part = it % PARTS;
      if (4 * kg < n_keys) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const half4 col = {vreg[i][0][e], vreg[i][1][e], vreg[i][2][e], vreg[i][3][e]};
          *reinterpret_cast<half4*>(&Vt[part * 8 + e][4 * kg]) = col;
        }
      }
    }
    __syncthreads();

    const int t_end = (my_tiles < (c0 + n_keys) / KT) ? my_tiles : (c0 + n_keys) / KT;   // uniform per wavefront
    for (int kt = c0 / KT; kt < t_end; ++kt) {
      const int k0 = kt * KT, kl = k0 - c0;          // first key of the tile, overall and inside the chunk
      // S^T tile: rows = keys (A operand from LDS), columns = queries (B operand in registers)
      float16v s;
#pragma unroll
      for (int e = 0; e < 16; ++e) s[e] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const half8 kf = *reinterpret_cast<const half8*>(&Ks[kl + (lane & 31)][ks * 16 + g * 8]);
        s = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, qf[ks], s, 0, 0, 0);
      }
      // accumulator element e of this lane is key  k0 + 8*(e/4) + 4*g + e%4
      float m_tile = -INFINITY;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int key = k0 + 8 * (e >> 2) + 4 * g + (e & 3);
        s[e] = (key <= qi && key < seq) ? s[e] * scale : -INFINITY;
        m_tile = fmaxf(m_tile, s[e]);
      }
      m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 32, 64));
      const float m_new = fmaxf(m_run, m_tile);       // finite from the first tile on: key 0 is never masked
      const float alpha = __expf(m_run - m_new);
      float psum = 0.f;
      half8 pf[2];
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float p = __expf(s[e] - m_new);
        psum += p;
        pf[e >> 3][e & 7] = static_cast<_Float16>(p);
      }
      psum += __shfl_xor(psum, 32, 64);
      l_run = l_run * alpha + psum;
      m_run = m_new;

      // O^T += V^T P^T.  Contraction slot (step t, group g, element e) stands for
      // key 16t + 8*(e/4) + 4g + e%4 on both operands.
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
        for (int e = 0; e < 16; ++e) o[dt][e] *= alpha;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const _Float16* vrow = &Vt[dt * 32 + (lane & 31)][kl + 16 * t + 4 * g];
          const half4 lo = *reinterpret_cast<const half4*>(vrow);
          const half4 hi = *reinterpret_cast<const half4*>(vrow + 8);
          const half8 vf = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pf[t], o[dt], 0, 0, 0);
        }
      }
    }
  }

  if (qi < seq) {
    const float inv = 1.0f / l_run;
    _Float16* orow = out + (static_cast<int64_t>(b) * seq + qi) * HL + head * D;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        half4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = static_cast<_Float16>(o[dt][4 * r + e] * inv);
        *reinterpret_cast<half4*>(orow + dt * 32 + 8 * r + 4 * g) = v;
      }
  }
}

}  // namespace

hipError_t launch_attention(const _Float16* qkv, _Float16* out, int batch, int seq, int heads, int head_dim,
                            hipStream_t s) {
  if (batch <= 0 || seq <= 0 || heads <= 0) return hipSuccess;
  if (heads > 65535 || batch > 65535) return hipErrorInvalidValue;
  const dim3 grid((seq + QB - 1) / QB, heads, batch), block(256);
  if (head_dim == 64)
    hipLaunchKernelGGL(attention_kernel<64>, grid, block, 0, s, qkv, out, seq, heads);
  else if (head_dim == 128)
    hipLaunchKernelGGL(attention_kernel<128>, grid, block, 0, s, qkv, out, seq, heads);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace ctn
