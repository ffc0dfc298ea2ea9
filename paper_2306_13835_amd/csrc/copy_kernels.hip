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

constexpr int kUnroll = 8;                          // 16-byte loads in flight per lane

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// DIR only gives the two directions distinct kernel names in profiles
// (0: host -> device, 1: device -> host, 2: anything else); the code is the same.
// THREADS: workgroup size, 1, 2 or 4 wavefronts; a workgroup moves chunks of THREADS * 8 * 16 bytes,
// so the table's chunk counts are those of that chunk size (copy_table_finish).
template <int DIR, int THREADS>
__global__ __launch_bounds__(THREADS) void copy_table_kernel(const CopyTable t) {
  constexpr uint32_t kChunk16 = THREADS * kUnroll;
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
      for (int j = 0; j < kUnroll; ++j) v[j] = __builtin_nontemporal_load(src + base + j * THREADS);
#pragma unroll
      for (int j = 0; j < kUnroll; ++j) __builtin_nontemporal_store(v[j], dst + base + j * THREADS);
    } else {
#pragma unroll
      for (int j = 0; j < kUnroll; ++j) {
        const uint64_t i = base + j * THREADS;
        if (i < n16) v[j] = __builtin_nontemporal_load(src + i);
      }
#pragma unroll
      for (int j = 0; j < kUnroll; ++j) {
        const uint64_t i = base + j * THREADS;
        if (i < n16) __builtin_nontemporal_store(v[j], dst + i);
      }
    }
  }
}

template <int THREADS>
void launch_dir(const CopyTable& t, int blocks, hipStream_t s, int dir) {
  if (dir == kCopyH2D) hipLaunchKernelGGL((copy_table_kernel<0, THREADS>), dim3(blocks), dim3(THREADS), 0, s, t);
  else if (dir == kCopyD2H) hipLaunchKernelGGL((copy_table_kernel<1, THREADS>), dim3(blocks), dim3(THREADS), 0, s, t);
  else hipLaunchKernelGGL((copy_table_kernel<2, THREADS>), dim3(blocks), dim3(THREADS), 0, s, t);
}

}  // namespace

int copy_workgroup_threads(int waves) {
  if (waves <= 0 || waves % 4 == 0) return 256;
  return waves % 2 == 0 ? 128 : 64;
}

bool copy_table_finish(CopyTable& t, int threads) {
  if (t.n < 0 || t.n > kCopyMaxSegs) return false;
  if (threads != 64 && threads != 128 && threads != 256) return false;
  const uint64_t chunk16 = static_cast<uint64_t>(threads) * kUnroll;
  uint64_t acc = 0;
  t.chunk_prefix[0] = 0;
  for (int i = 0; i < t.n; ++i) {
    acc += (t.seg[i].n16 + chunk16 - 1) / chunk16;
    if (acc > 0xFFFFFFFFull) return false;
    t.chunk_prefix[i + 1] = static_cast<uint32_t>(acc);
  }
  t.threads = threads;
  return true;
}

int default_copy_waves() { return 128; }

hipError_t launch_copy_table(const CopyTable& t, int waves, hipStream_t s, int dir) {
  if (t.n <= 0 || t.chunk_prefix[t.n] == 0) return hipSuccess;
  if (waves <= 0) waves = default_copy_waves();
  const int threads = t.threads;
  if (threads != 64 && threads != 128 && threads != 256) return hipErrorInvalidValue;   // table not finished
  int blocks = waves * 64 / threads;
  if (blocks < 1) blocks = 1;
  const uint32_t total = t.chunk_prefix[t.n];
  if (static_cast<uint32_t>(blocks) > total) blocks = static_cast<int>(total);
  if (threads == 256) launch_dir<256>(t, blocks, s, dir);
  else if (threads == 128) launch_dir<128>(t, blocks, s, dir);
  else launch_dir<64>(t, blocks, s, dir);
  return hipGetLastError();
}

}  // namespace ctn
