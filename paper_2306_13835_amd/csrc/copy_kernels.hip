// Copy kernels for swap-in (pinned host -> HBM arena) and swap-out (reverse).
//
// Section 5.1 of the paper attributes the gap to the link's lower bound to the
// parameters travelling as one message per tensor (alpha-beta model).  Here
// one launch moves every tensor of a transfer block: the device itself issues
// 16-byte loads against the host mapping and stores into the arena, so the
// per-message cost is paid once per block, not once per tensor.
//
// Bound: the host link.  Algorithmic traffic: each parameter byte crosses the
// link once and is written (or read) once in HBM.
#include "kernels.h"

namespace ctn {

namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 8;                          // 16-byte loads in flight per lane
constexpr uint32_t kChunk16 = kThreads * kUnroll;   // 16-byte units per chunk (32 KiB)

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// DIR only gives the two directions distinct kernel names in profiles
// (0: host -> device, 1: device -> host, 2: anything else); the code is the same.
template <int DIR>
__global__ __launch_bounds__(kThreads) void copy_table_kernel(const CopyTable t) {
  const uint32_t total = t.chunk_prefix[t.n];
  for (uint32_t chunk = blockIdx.x; chunk < total; chunk += gridDim.x) {
    int s = 0;
    while (s + 1 < t.n && chunk >= t.chunk_prefix[s + 1]) ++s;   // uniform across the workgroup
    const u32x4* __restrict__ src = static_cast<const u32x4*>(t.seg[s].src);
    u32x4* __restrict__ dst = static_cast<u32x4*>(t.seg[s].dst);
    const uint64_t n16 = t.seg[s].n16;
    const uint64_t base = static_cast<uint64_t>(chunk - t.chunk_prefix[s]) * kChunk16 + threadIdx.x;
    u32x4 v[kUnroll];
    if (base - threadIdx.x + kChunk16 <= n16) {                  // full chunk: no per-load guard
#pragma unroll
      for (int j = 0; j < kUnroll; ++j) v[j] = __builtin_nontemporal_load(src + base + j * kThreads);
#pragma unroll
      for (int j = 0; j < kUnroll; ++j) __builtin_nontemporal_store(v[j], dst + base + j * kThreads);
    } else {
#pragma unroll
      for (int j = 0; j < kUnroll; ++j) {
        const uint64_t i = base + j * kThreads;
        if (i < n16) v[j] = __builtin_nontemporal_load(src + i);
      }
#pragma unroll
      for (int j = 0; j < kUnroll; ++j) {
        const uint64_t i = base + j * kThreads;
        if (i < n16) __builtin_nontemporal_store(v[j], dst + i);
      }
    }
  }
}

}  // namespace

bool copy_table_finish(CopyTable& t) {
  if (t.n < 0 || t.n > kCopyMaxSegs) return false;
  uint64_t acc = 0;
  t.chunk_prefix[0] = 0;
  for (int i = 0; i < t.n; ++i) {
    acc += (t.seg[i].n16 + kChunk16 - 1) / kChunk16;
    if (acc > 0xFFFFFFFFull) return false;
    t.chunk_prefix[i + 1] = static_cast<uint32_t>(acc);
  }
  return true;
}

int default_copy_blocks() { return 32; }

hipError_t launch_copy_table(const CopyTable& t, int blocks, hipStream_t s, int dir) {
  if (t.n <= 0 || t.chunk_prefix[t.n] == 0) return hipSuccess;
  if (blocks <= 0) blocks = default_copy_blocks();
  uint32_t total = t.chunk_prefix[t.n];
  if (static_cast<uint32_t>(blocks) > total) blocks = static_cast<int>(total);
  if (dir == kCopyH2D) hipLaunchKernelGGL(copy_table_kernel<0>, dim3(blocks), dim3(kThreads), 0, s, t);
  else if (dir == kCopyD2H) hipLaunchKernelGGL(copy_table_kernel<1>, dim3(blocks), dim3(kThreads), 0, s, t);
  else hipLaunchKernelGGL(copy_table_kernel<2>, dim3(blocks), dim3(kThreads), 0, s, t);
  return hipGetLastError();
}

}  // namespace ctn
