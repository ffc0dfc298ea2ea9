// Host runtime behind the C ABI: contexts, model registration, asynchronous
// swap-in / swap-out on dedicated streams with one event per transfer block,
// LRU residency under a byte budget, and the layer-by-layer forward pass that
// waits only for the blocks it is about to read.
//
// Paper: Section 3 (demand paging of whole models), Section 3.2 (load and
// offload entries run on two extra streams next to the compute stream; a
// batch may only run on loaded parameters; host copies stay pinned),
// Section 4 (LRU), Section 5.1 (per-tensor messages and their alpha cost).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <vector>

#include "computron.h"
#include "computron_test.h"
#include "engine.hpp"
#include "kernels.h"
#include "layout.hpp"
#include "residency.hpp"

using namespace ctn;

// Scratch for ctn_op_gemm_static: callers that must not allocate (HIP graph capture, tight serving
// loops) get the split-K partial tiles from this array instead of a workspace of their own.  Every
// device the library runs on holds its own copy until the process ends.  In host code the array's
// name is only a handle for hipGetSymbolAddress: kernels receive the looked-up device address.
constexpr uint64_t kStaticScratchBytes = 64ull << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each device, once looked up

// Device address of the static scratch array on the current device (looked up once per device,
// with that device current).  hipSuccess and *out set, or the failing HIP status.
hipError_t static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

struct PendingRelease {   // arena range given back by an eviction whose offload may still be copying
  uint64_t off, len;
  hipEvent_t done;        // borrowed from the model that was evicted
  int model;
};

struct Eviction {         // blocks [b0, b1) of a model: decided, arena given back, not yet copied to the host
  int model, b0, b1;
  std::vector<uint64_t> off;   // arena offset of each of those blocks
  bool discard = false;        // no copy back: only the ordering against the last readers is enqueued
  int waves = 0;               // CTN_XFER_AUTO: width of the copy kernel for this offload (0: as wide as a load's)
};

struct Model {
  ShardLayout lay;
  std::vector<void*> host;           // per tensor, list order (host address)
  std::vector<void*> host_dev;       // the same memory as the device sees it
  // Per transfer block: maximal runs of tensors that are back to back both on
  // the host and in the arena image, so one copy can move a whole run.
  struct Run { int first; uint64_t bytes; };   // first tensor (list index) and total bytes
  std::vector<std::vector<Run>> runs;
  // Blocks [0, k) are resident (or on their way in), each at its own arena
  // offset.  Whole-model residency places all blocks in one range and k is 0
  // or the block count; block residency places every block in a slot of its own.
  int k = 0;
  std::vector<uint64_t> block_off;
  bool full() const { return k == lay.n_blocks; }
  uint64_t placement = 0;            // changes whenever blocks are placed: key of the captured graphs
  int last_load_first = 0;           // first block the last load brought in
  bool fragmented = true;            // more than 4 runs per block on average
  bool offload_enqueued = true;      // false between the eviction decision and the offload's enqueue
  std::vector<hipEvent_t> ev_block;  // recorded on the h2d stream after each block
  hipEvent_t ev_in_start = nullptr, ev_out_start = nullptr, ev_out_done = nullptr;
  hipEvent_t ev_last_use[2] = {nullptr, nullptr};   // last inference on each of the two inference lanes
  bool used[2] = {false, false};                    // that event has been recorded at least once
  bool load_recorded = false, out_recorded = false;
  bool pending_in = false, pending_out = false;

  // Captured forward passes of this placement (see forward_graph).
  struct Graph { uint64_t placement; int batch, seq; float* logits; hipGraphExec_t exec; };
  std::vector<Graph> graphs;
  void drop_graphs() {   // only when none of them can still be running
    for (Graph& g : graphs) (void)hipGraphExecDestroy(g.exec);
    graphs.clear();
  }

  Model() = default;
  Model(const Model&) = delete;
  Model& operator=(const Model&) = delete;
  ~Model() {   // also runs when registration fails half way
    drop_graphs();
    for (hipEvent_t e : ev_block)
      if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : {ev_in_start, ev_out_start, ev_out_done, ev_last_use[0], ev_last_use[1]})
      if (e) (void)hipEventDestroy(e);
  }
};

struct RetiredGraphs {   // captured forward passes of an evicted placement; destroyed once `done` has passed
  std::vector<hipGraphExec_t> execs;
  hipEvent_t done;
};

// Token ids of one inference, staged in pinned, device-mapped host memory that the context owns: the
// caller's buffer is free again when ctn_infer returns, and the embedding kernel reads the few KB
// straight over the link instead of waiting for a separate copy.
struct IdSlot {
  int32_t* host = nullptr;
  int32_t* dev = nullptr;          // the same memory as the device sees it
  size_t cap = 0;                  // ids
  hipEvent_t done = nullptr;       // recorded after the last kernel that reads the slot
  bool used = false;
};
constexpr int kIdSlots = 8;

struct Activations {   // carved from the workspace for one inference of M tokens
  int32_t* ids;
  float* x;
  _Float16 *a, *qkv, *attn, *u;
  float* logits;
  float* partial;            // split-K scratch
  uint64_t partial_floats;
  uint64_t bytes;
};

}  // namespace

struct ctn_ctx {
  ctn_config cfg{};
  hipStream_t s_compute = nullptr, s_h2d = nullptr, s_d2h = nullptr;
  bool own_streams = false;
  // Library-owned streams only: an unmasked compute stream for inferences that
  // start while the link is quiet (all compute units, no copy wavefronts to avoid).
  hipStream_t s_wide = nullptr;
  // Second inference lane (two-lane engine): a model that is still loading runs its batch here,
  // behind its transfer blocks' events, while batches of loaded models go on as before.
  hipStream_t s_lane1 = nullptr;
  bool two_lanes = false;            // each lane then works in its own half of the workspace
  hipStream_t last_compute = nullptr;
  bool use_graphs = false;           // replay captured forward passes on the unmasked stream
  hipEvent_t ev_compute_done = nullptr;
  Residency res{0};
  RangeAllocator arena;
  std::vector<std::unique_ptr<Model>> models;
  std::vector<PendingRelease> pending;
  std::vector<Eviction> deferred;    // evictions whose offload is not enqueued yet
  uint64_t placements = 0;
  std::vector<ctn_block_event> block_events;
  std::vector<RetiredGraphs> retired;
  int evict_waves = 0;               // CTN_XFER_AUTO: copy-kernel width of the offloads decided next (0: full)
  std::vector<ctn_event> events;
  ctn_stats stats{};
  int last_hip = 0;
  GemmTuning tuning;                 // test / tuning switches of this context's products (defaults: none)
  IdSlot id_slots[kIdSlots];
  int next_id_slot = 0;
};

namespace {

int g_last_hip = 0;   // HIP status of the last failing call made without a context

#define CTN_HIP(ctx, expr)                        \
  do {                                            \
    hipError_t e_ = (expr);                       \
    if (e_ != hipSuccess) {                       \
      if (ctx) (ctx)->last_hip = (int)e_;         \
      return CTN_E_HIP;                           \
    }                                             \
  } while (0)

Model* get_model(ctn_ctx* c, ctn_model m) {
  if (!c || m < 0 || m >= (ctn_model)c->models.size()) return nullptr;
  return c->models[m].get();
}

void log_event(ctn_ctx* c, int kind, int model, const std::vector<int>& victims) {
  ctn_event e{};
  e.kind = kind;
  e.model = model;
  e.n_victims = (int32_t)victims.size();
  for (size_t i = 0; i < victims.size() && i < 13; ++i) e.victims[i] = victims[i];
  c->events.push_back(e);
}

uint64_t activation_bytes(const ctn_model_desc& d, int64_t M, bool with_logits, Activations* out,
                          char* base) {
  const uint64_t h = d.hidden, hl = d.hidden / d.tp, fl = d.ffn / d.tp, vl = d.vocab / d.tp;
  uint64_t cur = 0;
  auto take = [&](uint64_t n) {
    uint64_t o = cur;
    cur = align_up(cur + n);
    return o;
  };
  const uint64_t o_ids = take(4ull * M), o_x = take(4ull * M * h), o_a = take(2ull * M * h),
                 o_qkv = take(2ull * M * 3 * hl), o_attn = take(2ull * M * hl), o_u = take(2ull * M * fl),
                 o_log = with_logits ? take(4ull * M * vl) : 0;
  // up to 16 K-slices of the widest product that is ever split (not the vocabulary head)
  const uint64_t widest = std::max<uint64_t>(std::max<uint64_t>(3 * hl, fl), h);
  // (larger batches split only the row-parallel products, N = hidden, in at most 4 slices).  Never less than a
  // smaller batch needs: a workspace sized for max_tokens must serve every batch up to it.
  const uint64_t small_m = M < 64 ? M : 64;
  const uint64_t partial_floats = std::max<uint64_t>(16ull * small_m * widest, 4ull * M * h);
  const uint64_t o_part = partial_floats ? take(4ull * partial_floats) : 0;
  if (out && base) {
    out->ids = reinterpret_cast<int32_t*>(base + o_ids);
    out->x = reinterpret_cast<float*>(base + o_x);
    out->a = reinterpret_cast<_Float16*>(base + o_a);
    out->qkv = reinterpret_cast<_Float16*>(base + o_qkv);
    out->attn = reinterpret_cast<_Float16*>(base + o_attn);
    out->u = reinterpret_cast<_Float16*>(base + o_u);
    out->logits = with_logits ? reinterpret_cast<float*>(base + o_log) : nullptr;
    out->partial = partial_floats ? reinterpret_cast<float*>(base + o_part) : nullptr;
    out->partial_floats = partial_floats;
    out->bytes = cur;
  }
  return cur;
}

// Graph executables of a placement that is being given up may still be running:
// they are parked behind an event on the stream that replays them.
void retire_graphs(ctn_ctx* c, Model* m) {
  if (m->graphs.empty()) return;
  RetiredGraphs r;
  for (Model::Graph& g : m->graphs) r.execs.push_back(g.exec);
  m->graphs.clear();
  r.done = nullptr;
  if (hipEventCreateWithFlags(&r.done, hipEventDisableTiming) != hipSuccess ||
      hipEventRecord(r.done, c->s_wide) != hipSuccess) {
    (void)hipGetLastError();
    if (r.done) (void)hipEventDestroy(r.done);
    r.done = nullptr;                // destroyed at the next full synchronisation instead
  }
  c->retired.push_back(std::move(r));
}

void purge_retired(ctn_ctx* c, bool all) {
  for (size_t i = 0; i < c->retired.size();) {
    RetiredGraphs& r = c->retired[i];
    const bool done = all || (r.done && hipEventQuery(r.done) == hipSuccess);
    if (!done) {
      (void)hipGetLastError();
      ++i;
      continue;
    }
    for (hipGraphExec_t e : r.execs) (void)hipGraphExecDestroy(e);
    if (r.done) (void)hipEventDestroy(r.done);
    c->retired.erase(c->retired.begin() + i);
  }
}

void log_blocks(ctn_ctx* c, int kind, const Residency::Move& mv, uint64_t use) {
  if (mv.b0 >= mv.b1) return;
  c->block_events.push_back(ctn_block_event{kind, mv.model, mv.b0, mv.b1, use});
}

// Bytes of arena a block occupies where it is placed.
uint64_t block_footprint(const ctn_ctx* c, const ShardLayout& L, int b) {
  return c->res.block_mode() ? L.slot_bytes : L.block_span[b];
}

// Moves transfer block b of model m between its host tensors and `base` (where the block sits,
// or will sit, in the arena) on stream s.  how: 0 = one hipMemcpyAsync per tensor (the paper's
// per-tensor messages, Section 5.1), 1 = one copy-kernel launch over the block's runs, 2 = one
// hipMemcpyAsync per run of adjacent tensors.
enum { kPerTensorDma = 0, kCopyKernel = 1, kPerRunDma = 2, kGatherSmallDmaLarge = 3 };
// kGatherSmallDmaLarge: runs of up to kSmallRunBytes travel together in one narrow copy-kernel launch per block
// (the per-message cost of Section 5.1 is paid once for all of them), the larger runs by one DMA copy each.
constexpr uint64_t kSmallRunBytes = 256 << 10;
constexpr int kSmallRunWaves = 8;
// Offloads by the copy kernel beside loads by the DMA engines (CTN_XFER_DMA_IN_KERNEL_OUT, and CTN_XFER_AUTO
// in a run of back-to-back swaps): writes to the host that a kernel issues take link capacity from the loads
// running beside them, the more the wider the kernel is.  Measured on the alternating two-model workload
// (6.7B/TP2 shard, one DMA copy per run for the loads), offload 4 / 8 / 12 / 128 wavefronts wide: load 54.5 /
// 50.2 / 44.0 / 37.5 GB/s against offload 24.2 / 44.9 / 50.0 / 50.7 GB/s.  The two directions trade places
// between 8 and 12 wavefronts, and sharply (an intermediate number of bytes in flight lands on one side or the
// other), so a balanced offload alternates its blocks between the two.
constexpr int kBalancedWavesLow = 8, kBalancedWavesHigh = 12;
constexpr int kBalancedOffload = -1;          // Eviction::waves: alternate as above

// How an offload of model m travels under the context's transfer mode.
int offload_path(const ctn_ctx* c, const Model* m) {
  switch (c->cfg.transfer_mode) {
    case CTN_XFER_DMA: return kPerTensorDma;
    case CTN_XFER_KERNEL: case CTN_XFER_DMA_IN_KERNEL_OUT: return kCopyKernel;
    case CTN_XFER_KERNEL_IN_DMA_OUT: case CTN_XFER_DMA_RUNS: return kPerRunDma;
    default: return m->fragmented ? kCopyKernel : kPerRunDma;   // CTN_XFER_AUTO
  }
}

int copy_block(ctn_ctx* c, Model* m, int b, char* base, bool to_device, int how, hipStream_t s, int waves) {
  const ShardLayout& L = m->lay;
  if (m->runs[b].empty()) return CTN_OK;        // a stage without tensors outside its layers
  if (how == kCopyKernel || how == kGatherSmallDmaLarge) {
    const bool only_small = how == kGatherSmallDmaLarge;
    if (only_small) waves = kSmallRunWaves;
    CopyTable t{};
    static_assert(kLayerTensors <= kCopyMaxSegs, "a layer block's tensors must fit one copy table");
    for (const Model::Run& r : m->runs[b]) {
      if (only_small && r.bytes > kSmallRunBytes) continue;
      if (t.n >= kCopyMaxSegs) {                 // a block 0 with more runs than one table holds: flush and go on
        if (!copy_table_finish(t, copy_workgroup_threads(waves))) return CTN_E_INVAL;
        CTN_HIP(c, launch_copy_table(t, waves, s, to_device ? kCopyH2D : kCopyD2H));
        t = CopyTable{};
      }
      char* dev = base + L.offset_in_block(r.first);
      t.seg[t.n].src = to_device ? m->host_dev[r.first] : dev;
      t.seg[t.n].dst = to_device ? dev : m->host_dev[r.first];
      t.seg[t.n].n16 = r.bytes / 16;
      ++t.n;
    }
    if (!copy_table_finish(t, copy_workgroup_threads(waves))) return CTN_E_INVAL;
    CTN_HIP(c, launch_copy_table(t, waves, s, to_device ? kCopyH2D : kCopyD2H));
    if (!only_small) return CTN_OK;
  }
  auto one = [&](int ti, uint64_t bytes) {
    char* dev = base + L.offset_in_block(ti);
    return to_device ? hipMemcpyAsync(dev, m->host[ti], bytes, hipMemcpyHostToDevice, s)
                     : hipMemcpyAsync(m->host[ti], dev, bytes, hipMemcpyDeviceToHost, s);
  };
  if (how == kPerTensorDma) {
    for (int ti : L.block_tensors[b]) CTN_HIP(c, one(ti, L.nbytes[ti]));
  } else {
    for (const Model::Run& r : m->runs[b]) {
      if (how == kGatherSmallDmaLarge && r.bytes <= kSmallRunBytes) continue;   // went with the gather launch
      CTN_HIP(c, one(r.first, r.bytes));
    }
  }
  return CTN_OK;
}

// Eviction happens in two steps so that, on a miss, the load of the requested
// model and its forward pass can be enqueued before the (latency-insensitive)
// offload of the victims: evict_logical() updates the bookkeeping and frees
// the blocks' arena ranges; enqueue_offload() issues the copies back to the
// host tensors and records the completion event the freed ranges wait on.
// The residency policy has already dropped the blocks named by `mv`.
void evict_logical(ctn_ctx* c, const Residency::Move& mv) {
  if (mv.b0 >= mv.b1) return;
  Model* m = c->models[mv.model].get();
  retire_graphs(c, m);               // they point into the blocks being given up
  m->offload_enqueued = false;
  Eviction ev{mv.model, mv.b0, mv.b1, {}};
  uint64_t run_off = 0, run_len = 0;
  auto give_back = [&]() {
    if (!run_len) return;
    c->arena.release(run_off, run_len);
    c->pending.push_back({run_off, run_len, m->ev_out_done, mv.model});
  };
  ev.discard = c->cfg.discard_on_evict != 0;
  ev.waves = c->evict_waves;
  for (int b = mv.b0; b < mv.b1; ++b) {
    const uint64_t off = m->block_off[b], len = block_footprint(c, m->lay, b);
    ev.off.push_back(off);
    if (run_len && run_off + run_len == off) {
      run_len += len;
    } else {
      give_back();
      run_off = off;
      run_len = len;
    }
  }
  give_back();
  m->k = mv.b0;
  c->deferred.push_back(std::move(ev));
}

int enqueue_offload(ctn_ctx* c, const Eviction& ev) {
  Model* m = c->models[ev.model].get();
  char* arena = static_cast<char*>(c->cfg.arena_dev);
  // The offload must see the complete device copy (blocks are loaded in order on
  // one stream, so the last block's event covers the others) and must not
  // overtake an inference that is still reading it.
  CTN_HIP(c, hipStreamWaitEvent(c->s_d2h, m->ev_block[ev.b1 - 1], 0));
  for (int lane = 0; lane < 2; ++lane)
    if (m->used[lane]) CTN_HIP(c, hipStreamWaitEvent(c->s_d2h, m->ev_last_use[lane], 0));
  CTN_HIP(c, hipEventRecord(m->ev_out_start, c->s_d2h));
  const ShardLayout& L = m->lay;
  int how = offload_path(c, m);
  // The widths that balance an offload kernel against the load beside it were measured with the kernel confined
  // to the offload stream's own compute units; on a caller's streams, where it shares the chip with the forward
  // pass, it falls behind (160 against 142 ms per alternating step), so there AUTO offloads by DMA copies.
  if (c->cfg.transfer_mode == CTN_XFER_AUTO && how == kCopyKernel && ev.waves == kBalancedOffload && !c->own_streams)
    how = kPerRunDma;
  int waves = c->cfg.copy_waves_out ? c->cfg.copy_waves_out : 4 * c->cfg.copy_blocks;
  // (an eviction that a miss decided runs beside that miss's load; an explicit swap-out has the link to itself)
  const bool balanced = !c->cfg.copy_waves_out && how == kCopyKernel && ev.waves == kBalancedOffload &&
                        (c->cfg.transfer_mode == CTN_XFER_DMA_IN_KERNEL_OUT || c->cfg.transfer_mode == CTN_XFER_AUTO);
  if (c->cfg.transfer_mode == CTN_XFER_AUTO && !c->cfg.copy_waves_out && ev.waves > 0) waves = ev.waves;
  uint64_t bytes = 0;
  // (a discarded device copy moves nothing; the stream waits above and the event below still
  // order the reuse of its blocks after the load and the inferences that were using them)
  for (int b = ev.b0; b < ev.b1 && !ev.discard; ++b) {
    bytes += L.block_bytes[b];
    // balanced: the blocks alternate between the two widths on either side of the point where the link's two
    // directions trade places, so the offload as a whole keeps pace with the DMA load beside it
    const int w = balanced ? ((b & 1) ? kBalancedWavesHigh : kBalancedWavesLow) : waves;
    const int rc = copy_block(c, m, b, arena + ev.off[b - ev.b0], false, how, c->s_d2h, w);
    if (rc) return rc;
  }
  CTN_HIP(c, hipEventRecord(m->ev_out_done, c->s_d2h));
  m->out_recorded = true;
  m->pending_out = true;
  c->stats.bytes_d2h += bytes;
  c->stats.n_swap_out += 1;
  return CTN_OK;
}

// Issues every offload that was decided but not yet enqueued.
int flush_deferred(ctn_ctx* c) {
  for (const Eviction& ev : c->deferred) {
    int rc = enqueue_offload(c, ev);
    if (rc) return rc;
  }
  for (const Eviction& ev : c->deferred) c->models[ev.model]->offload_enqueued = true;
  c->deferred.clear();
  return CTN_OK;
}

// Make model mi completely resident (a use).  On a miss: evict from the least
// recently used models while the budget (or the arena) has no room for the
// missing blocks, then enqueue their load.  Offloads of the victims stay
// deferred (see flush_deferred) unless the load has to reuse a victim's range.
int ensure_resident(ctn_ctx* c, int mi) {
  Model* m = c->models[mi].get();
  std::vector<int> victims;
  if (m->full()) {
    c->res.touch(mi);
    c->stats.n_hit += 1;
    log_event(c, 0, mi, victims);
    return CTN_OK;
  }
  const ShardLayout& L = m->lay;
  const bool by_block = c->res.block_mode();
  const uint64_t whole_footprint = by_block ? L.slot_bytes * L.n_blocks : L.arena_bytes;
  if (L.param_bytes > c->res.budget() || whole_footprint > c->cfg.arena_bytes) return CTN_E_TOO_BIG;
  int rc = flush_deferred(c);
  if (rc) return rc;
  purge_retired(c, false);
  // Forget offloads that have finished; the others still read their old ranges.
  for (size_t i = 0; i < c->pending.size();) {
    if (hipEventQuery(c->pending[i].done) == hipSuccess) {
      c->pending.erase(c->pending.begin() + i);
    } else {
      (void)hipGetLastError();   // "not ready" is an answer, not a failure to report later
      ++i;
    }
  }
  const uint64_t use = c->events.size();
  const int first = m->k;                       // blocks [first, n_blocks) are missing
  std::vector<Residency::Move> moves;           // what this use evicts, one entry per victim, in order
  while (c->res.over_budget_with(mi))
    if (c->res.evict_step(mi, moves) < 0) return CTN_E_BUSY;   // (cannot happen: the model fits the budget alone)
  // CTN_XFER_AUTO reads the link's state from the context's own record and its events, never from the clock:
  // the link is busy both ways during this load when the miss evicts (its victims' offloads run beside the
  // load) or when an offload that an earlier use enqueued has not completed.
  const bool two_way = !moves.empty() || !c->pending.empty();
  c->evict_waves = kBalancedOffload;      // (CTN_XFER_AUTO) offloads that run beside this load keep pace with it
  for (const Residency::Move& mv : moves) evict_logical(c, mv);
  auto busy_ranges = [&]() {
    std::vector<RangeAllocator::Range> b;
    for (const PendingRelease& p : c->pending) b.push_back({p.off, p.len});
    return b;
  };
  // The budget has room but no arena hole is wide enough: keep evicting.
  auto evict_for_room = [&]() -> bool {
    std::vector<Residency::Move> step;
    if (c->res.evict_step(mi, step) < 0) return false;
    evict_logical(c, step[0]);
    c->stats.n_extra_evictions += 1;
    for (Residency::Move& mv : moves)
      if (mv.model == step[0].model) {
        mv.b0 = step[0].b0;
        return true;
      }
    moves.push_back(step[0]);
    return true;
  };
  // Prefer holes no offload is reading, so load and offload overlap on the
  // two link directions (Section 3.2 / 5.1); otherwise the load waits.
  std::vector<RangeAllocator::Range> placed;    // arena ranges this load writes
  struct GiveBack {                             // every early return below hands them back to the arena
    RangeAllocator& arena;
    const std::vector<RangeAllocator::Range>& ranges;
    bool keep = false;
    ~GiveBack() {
      if (!keep)
        for (const RangeAllocator::Range& r : ranges) arena.release(r.off, r.len);
    }
  } give_back{c->arena, placed};
  if (!by_block) {
    uint64_t off = c->arena.alloc_avoiding(L.arena_bytes, busy_ranges());
    while (off == UINT64_MAX) {
      if (!evict_for_room()) return CTN_E_BUSY;
      off = c->arena.alloc_avoiding(L.arena_bytes, busy_ranges());
    }
    placed.push_back({off, L.arena_bytes});
    for (int b = 0; b < L.n_blocks; ++b) m->block_off[b] = off + L.block_start[b];
  } else {
    const int n_missing = L.n_blocks - first;
    // all missing blocks side by side when a hole that no offload is reading allows it, else slot by slot
    const uint64_t together = c->arena.alloc_avoiding(L.slot_bytes * n_missing, busy_ranges(), -1);
    if (together != UINT64_MAX) {
      placed.push_back({together, L.slot_bytes * n_missing});
      for (int b = first; b < L.n_blocks; ++b) m->block_off[b] = together + L.slot_bytes * (b - first);
    } else {
      for (int b = first; b < L.n_blocks; ++b) {
        uint64_t off = c->arena.alloc_avoiding(L.slot_bytes, busy_ranges());
        while (off == UINT64_MAX) {
          if (!evict_for_room()) return CTN_E_BUSY;
          off = c->arena.alloc_avoiding(L.slot_bytes, busy_ranges());
        }
        placed.push_back({off, L.slot_bytes});
        m->block_off[b] = off;
      }
    }
  }
  m->placement = ++c->placements;
  auto overlaps_load = [&](const PendingRelease& p) {
    for (const RangeAllocator::Range& r : placed)
      if (p.off < r.off + r.len && r.off < p.off + p.len) return true;
    return false;
  };
  bool reuses_victim_range = false;
  for (const PendingRelease& p : c->pending)
    if (overlaps_load(p) && !c->models[p.model]->offload_enqueued) reuses_victim_range = true;
  if (reuses_victim_range) {     // the completion events the load must wait on have to exist first
    rc = flush_deferred(c);
    if (rc) return rc;
  }
  for (const PendingRelease& p : c->pending)
    if (overlaps_load(p)) CTN_HIP(c, hipStreamWaitEvent(c->s_h2d, p.done, 0));
  // The load reads the host tensors this model's own offload may still be writing.
  if (m->pending_out) CTN_HIP(c, hipStreamWaitEvent(c->s_h2d, m->ev_out_done, 0));
  char* arena = static_cast<char*>(c->cfg.arena_dev);
  // AUTO: with the link's other direction idle, a host list in many pieces is gathered by one kernel launch
  // per block (no per-piece cost on the host or the device, 98.8 % of the link's peak).  Beside an offload
  // the DMA engines load it, one copy per run: host reads that a kernel issues are many small requests that
  // travel against the offload's data and slow both directions (kernel both ways at full width: 33 + 52 GB/s;
  // DMA loads beside the balanced offload kernel: 47 + 47).  A packed list always takes one DMA copy per run.
  int how = kPerRunDma;
  switch (c->cfg.transfer_mode) {
    case CTN_XFER_DMA: how = kPerTensorDma; break;
    case CTN_XFER_KERNEL: case CTN_XFER_KERNEL_IN_DMA_OUT: how = kCopyKernel; break;
    case CTN_XFER_DMA_IN_KERNEL_OUT: case CTN_XFER_DMA_RUNS: how = kPerRunDma; break;
    default:   // CTN_XFER_AUTO
      how = !m->fragmented ? kPerRunDma : (two_way ? kGatherSmallDmaLarge : kCopyKernel);
      break;
  }
  CTN_HIP(c, hipEventRecord(m->ev_in_start, c->s_h2d));
  for (int b = first; b < L.n_blocks; ++b) {
    rc = copy_block(c, m, b, arena + m->block_off[b], true, how, c->s_h2d, 4 * c->cfg.copy_blocks);
    if (rc) return rc;
    CTN_HIP(c, hipEventRecord(m->ev_block[b], c->s_h2d));
  }
  give_back.keep = true;
  m->k = L.n_blocks;
  m->last_load_first = first;
  m->load_recorded = true;
  m->pending_in = true;
  c->stats.bytes_h2d += c->res.missing_bytes(mi);
  const Residency::Move loaded = c->res.load_missing(mi);
  c->stats.n_swap_in += 1;
  c->stats.n_miss += 1;
  if (first > 0) c->stats.n_partial_miss += 1;
  c->stats.resident_bytes = c->res.resident_bytes();
  c->stats.peak_resident_bytes = c->res.peak_bytes();
  for (const Residency::Move& mv : moves) {
    victims.push_back(mv.model);
    log_blocks(c, 1, mv, use);
  }
  log_blocks(c, 0, loaded, use);
  log_event(c, 1, mi, victims);
  return CTN_OK;
}

constexpr int kDefaultCopyCus = 8;

// Three streams, each with its own hardware queue and a disjoint set of
// compute units: bits [0, n) of the CU mask for swap-in, [n, 2n) for swap-out,
// the rest for inference.  Consecutive mask bits fall on consecutive XCDs, so
// n = 8 takes one compute unit from every XCD.  A wavefront of the copy
// kernel spends microseconds waiting on each host-link load; sharing a compute
// unit's memory pipeline with it stalls the forward pass's wavefronts, which
// this partition prevents.
int create_partitioned_streams(ctn_ctx* c, int copy_cus) {
  int dev = 0;
  hipDeviceProp_t prop;
  CTN_HIP(c, hipGetDevice(&dev));
  CTN_HIP(c, hipGetDeviceProperties(&prop, dev));
  const int n_cu = prop.multiProcessorCount;
  if (n_cu < 4 * copy_cus) return CTN_E_INVAL;
  const int words = (n_cu + 31) / 32;
  auto make = [&](int lo, int hi, hipStream_t* out) -> hipError_t {
    std::vector<uint32_t> mask(words, 0u);
    for (int b = lo; b < hi; ++b) mask[b / 32] |= 1u << (b % 32);
    return hipExtStreamCreateWithCUMask(out, (uint32_t)words, mask.data());
  };
  CTN_HIP(c, make(0, copy_cus, &c->s_h2d));
  CTN_HIP(c, make(copy_cus, 2 * copy_cus, &c->s_d2h));
  CTN_HIP(c, make(2 * copy_cus, n_cu, &c->s_compute));
  CTN_HIP(c, make(2 * copy_cus, n_cu, &c->s_lane1));
  // The unmasked stream also gets an explicit mask, of every compute unit.  A plain stream may be handed a
  // hardware queue that an earlier, destroyed masked stream of this process used, and then runs on that
  // stream's compute units (measured: resident 1 x 64 requests at 7.1 ms instead of 3.0 ms in a process that
  // had created and destroyed a context before).
  CTN_HIP(c, make(0, n_cu, &c->s_wide));
  CTN_HIP(c, hipEventCreateWithFlags(&c->ev_compute_done, hipEventDisableTiming));
  c->own_streams = true;
  c->use_graphs = false;   // measured on ROCm 7.2 / MI355X: replay is no faster than direct launches (the
                           // time between the ~400 small kernels is spent on the device, not on the host)
  return CTN_OK;
}

// True when no load or offload is still running (events queried, flags refreshed).
bool link_quiet(ctn_ctx* c) {
  bool quiet = true;
  for (auto& m : c->models) {
    if (m->pending_in) {
      if (hipEventQuery(m->ev_block.back()) == hipSuccess) m->pending_in = false;
      else quiet = false;
    }
    if (m->pending_out) {
      if (hipEventQuery(m->ev_out_done) == hipSuccess) m->pending_out = false;
      else quiet = false;
    }
  }
  (void)hipGetLastError();
  return quiet;
}

template <typename T>
T* dev_tensor(ctn_ctx* c, Model* m, int ti) {
  const ShardLayout& L = m->lay;
  return reinterpret_cast<T*>(static_cast<char*>(c->cfg.arena_dev) + m->block_off[L.block_of[ti]] +
                              L.offset_in_block(ti));
}

// The launch sequence of one forward pass on stream s.  with_waits: wait for the
// transfer blocks' events (not needed, and not capturable across loads, when the
// model is known to be completely resident).
int forward_launches(ctn_ctx* c, Model* m, const Activations& act, const int32_t* ids_dev, int batch, int seq,
                     float* logits, hipStream_t s, bool with_waits) {
  const ShardLayout& L = m->lay;
  const ctn_model_desc& d = L.d;
  const int M = batch * seq;
  const int h = d.hidden, hl = L.hl(), fl = L.fl(), vl = L.vl();
  // The paper's rule (Section 3.2): a batch runs only on a fully loaded
  // model.  With pipelining the same rule is applied per transfer block.
  if (with_waits) {
    if (!c->cfg.pipeline) CTN_HIP(c, hipStreamWaitEvent(s, m->ev_block.back(), 0));
    else CTN_HIP(c, hipStreamWaitEvent(s, m->ev_block[0], 0));
  }

  const GemmTuning* tune = &c->tuning;
  // A split-K row-parallel product leaves its residual update to the LayerNorm that follows it.
  PendingSum pend;
  // Stage 0 builds the residual stream from the token ids; later pipeline stages were handed it.
  if (L.has_embed())
    CTN_HIP(c, launch_embed(ids_dev, dev_tensor<_Float16>(c, m, L.idx_tok()), dev_tensor<_Float16>(c, m, L.idx_pos()),
                            act.x, M, seq, h, vl, d.rank, s));
  const int n_layers = L.local_layers();
  for (int l = 0; l < n_layers; ++l) {
    if (with_waits && c->cfg.pipeline) CTN_HIP(c, hipStreamWaitEvent(s, m->ev_block[1 + l], 0));
    auto T = [&](int w) { return dev_tensor<_Float16>(c, m, L.layer_tensor(l, w)); };
    CTN_HIP(c, launch_layernorm(act.x, T(LN1_W), T(LN1_B), act.a, M, h, s, &pend));
    // q | k | v: three column-parallel projections of the same input in one launch
    const _Float16* const wqkv[3] = {T(Q_W), T(K_W), T(V_W)};
    const _Float16* const bqkv[3] = {T(Q_B), T(K_B), T(V_B)};
    CTN_HIP(c, launch_gemm3(act.a, wqkv, bqkv, act.qkv, M, hl, h, CTN_EPI_BIAS_F16, s, act.partial, act.partial_floats, tune));
    CTN_HIP(c, launch_attention(act.qkv, act.attn, batch, seq, L.local_heads(), L.head_dim(), s));
    // row parallel: this rank's partial sum joins the residual stream (the
    // cross-rank reduction is the identity on one GPU), bias added once
    CTN_HIP(c, launch_gemm(act.attn, T(O_W), T(O_B), act.x, M, h, hl, CTN_EPI_BIAS_RESID_F32, s, act.partial, act.partial_floats, &pend, tune));
    CTN_HIP(c, launch_layernorm(act.x, T(LN2_W), T(LN2_B), act.a, M, h, s, &pend));
    CTN_HIP(c, launch_gemm(act.a, T(FC1_W), T(FC1_B), act.u, M, fl, h, CTN_EPI_BIAS_RELU_F16, s, act.partial, act.partial_floats, nullptr, tune));
    // (a stage that ends without a final LayerNorm has nobody to finish a deferred update for it)
    PendingSum* after_fc2 = (l + 1 < n_layers || L.has_head()) ? &pend : nullptr;
    CTN_HIP(c, launch_gemm(act.u, T(FC2_W), T(FC2_B), act.x, M, h, fl, CTN_EPI_BIAS_RESID_F32, s, act.partial, act.partial_floats, after_fc2, tune));
  }
  if (!L.has_head()) return CTN_OK;            // the stage emits the residual stream act.x
  CTN_HIP(c, launch_layernorm(act.x, dev_tensor<_Float16>(c, m, L.idx_final_w()),
                              dev_tensor<_Float16>(c, m, L.idx_final_b()), act.a, M, h, s, &pend));
  // head: the token matrix (tied), or the last pipeline stage's own copy of it; vocabulary slice
  CTN_HIP(c, launch_gemm(act.a, dev_tensor<_Float16>(c, m, L.idx_head()), nullptr, logits, M, vl, h, CTN_EPI_F32, s, nullptr, 0, nullptr, tune));
  return CTN_OK;
}

// Replays (capturing on first use) the forward pass of a completely resident model.
int forward_graph(ctn_ctx* c, Model* m, const Activations& act, int batch, int seq, float* logits, hipStream_t s) {
  for (const Model::Graph& g : m->graphs)
    if (g.placement == m->placement && g.batch == batch && g.seq == seq && g.logits == logits) {
      CTN_HIP(c, hipGraphLaunch(g.exec, s));
      return CTN_OK;
    }
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
  if (hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal) != hipSuccess) {
    (void)hipGetLastError();
    c->use_graphs = false;   // this runtime cannot capture here: keep launching directly
    return forward_launches(c, m, act, act.ids, batch, seq, logits, s, true);
  }
  const int rc = forward_launches(c, m, act, act.ids, batch, seq, logits, s, false);
  const hipError_t e_end = hipStreamEndCapture(s, &graph);
  if (rc || e_end != hipSuccess || !graph) {
    if (graph) (void)hipGraphDestroy(graph);
    (void)hipGetLastError();
    if (rc) return rc;
    c->use_graphs = false;
    return forward_launches(c, m, act, act.ids, batch, seq, logits, s, true);
  }
  const hipError_t e_inst = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
  (void)hipGraphDestroy(graph);
  if (e_inst != hipSuccess || !exec) {
    (void)hipGetLastError();
    c->use_graphs = false;
    return forward_launches(c, m, act, act.ids, batch, seq, logits, s, true);
  }
  if (m->graphs.size() >= 8) {           // bounded cache: drop the oldest capture
    (void)hipGraphExecDestroy(m->graphs.front().exec);
    m->graphs.erase(m->graphs.begin());
  }
  m->graphs.push_back({m->placement, batch, seq, logits, exec});
  CTN_HIP(c, hipGraphLaunch(exec, s));
  return CTN_OK;
}

}  // namespace

extern "C" {

int ctn_create(const ctn_config* cfg, ctn_ctx** out) {
  if (!cfg || !out) return CTN_E_INVAL;
  if (!cfg->arena_dev || !cfg->workspace_dev) return CTN_E_INVAL;
  const bool own_streams = !cfg->stream_compute && !cfg->stream_h2d && !cfg->stream_d2h;
  if (!own_streams && (!cfg->stream_compute || !cfg->stream_h2d || !cfg->stream_d2h)) return CTN_E_INVAL;
  if (cfg->copy_cus < 0 || cfg->copy_cus > 64 || (cfg->copy_cus > 0 && cfg->copy_cus < 8)) return CTN_E_INVAL;
  if (reinterpret_cast<uintptr_t>(cfg->arena_dev) % kAlign || reinterpret_cast<uintptr_t>(cfg->workspace_dev) % kAlign)
    return CTN_E_INVAL;
  if (cfg->hbm_budget_bytes == 0 || cfg->arena_bytes == 0) return CTN_E_INVAL;
  if (cfg->transfer_mode < CTN_XFER_DMA || cfg->transfer_mode > CTN_XFER_DMA_RUNS) return CTN_E_INVAL;
  if (cfg->copy_blocks < 0 || cfg->copy_blocks > 4096 || cfg->copy_waves_out < 0 || cfg->copy_waves_out > 16384) return CTN_E_INVAL;
  if (cfg->block_residency != 0 && cfg->block_residency != 1) return CTN_E_INVAL;
  if (cfg->discard_on_evict != 0 && cfg->discard_on_evict != 1) return CTN_E_INVAL;
  if (!own_streams && (cfg->stream_h2d == cfg->stream_compute || cfg->stream_d2h == cfg->stream_compute ||
                       cfg->stream_h2d == cfg->stream_d2h))
    return CTN_E_INVAL;
  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || n_dev < 1) return CTN_E_HIP;   // no silent fallback
  {   // the static scratch array's address on this device, for ctn_op_gemm_static
    void* sp = nullptr;
    const hipError_t e = static_scratch(&sp);
    if (e != hipSuccess) {
      (void)hipGetLastError();
      g_last_hip = (int)e;
      return CTN_E_HIP;
    }
  }
  ctn_ctx* c = new (std::nothrow) ctn_ctx();
  if (!c) return CTN_E_NOMEM;
  c->cfg = *cfg;
  if (own_streams) {
    int rc = create_partitioned_streams(c, cfg->copy_cus ? cfg->copy_cus : kDefaultCopyCus);
    if (rc) {
      g_last_hip = c->last_hip;
      delete c;
      return rc;
    }
  } else {
    c->s_compute = static_cast<hipStream_t>(cfg->stream_compute);
    c->s_h2d = static_cast<hipStream_t>(cfg->stream_h2d);
    c->s_d2h = static_cast<hipStream_t>(cfg->stream_d2h);
  }
  c->res = Residency(cfg->hbm_budget_bytes, cfg->block_residency != 0);
  c->arena.reset(cfg->arena_bytes / kAlign * kAlign);
  c->stats.budget_bytes = cfg->hbm_budget_bytes;
  *out = c;
  return CTN_OK;
}

int ctn_sync(ctn_ctx* c) {
  if (!c) return CTN_E_INVAL;
  const int rc = flush_deferred(c);       // nothing decided may stay unissued behind a full synchronisation
  if (rc) return rc;
  CTN_HIP(c, hipStreamSynchronize(c->s_h2d));
  CTN_HIP(c, hipStreamSynchronize(c->s_d2h));
  CTN_HIP(c, hipStreamSynchronize(c->s_compute));
  if (c->s_wide) CTN_HIP(c, hipStreamSynchronize(c->s_wide));
  if (c->s_lane1) CTN_HIP(c, hipStreamSynchronize(c->s_lane1));
  purge_retired(c, true);
  for (auto& m : c->models) m->pending_in = m->pending_out = false;
  c->pending.clear();
  return CTN_OK;
}

int ctn_destroy(ctn_ctx* c) {
  if (!c) return CTN_E_INVAL;
  int rc = ctn_sync(c);
  c->models.clear();   // destroys every model's events
  for (IdSlot& sl : c->id_slots) {
    if (sl.host) (void)hipHostFree(sl.host);
    if (sl.done) (void)hipEventDestroy(sl.done);
  }
  if (c->own_streams) {
    for (hipStream_t st : {c->s_compute, c->s_h2d, c->s_d2h, c->s_wide, c->s_lane1})
      if (st) (void)hipStreamDestroy(st);
    if (c->ev_compute_done) (void)hipEventDestroy(c->ev_compute_done);
  }
  delete c;
  return rc;
}

int ctn_host_alloc(uint64_t nbytes, void** out) {
  if (!out || nbytes == 0) return CTN_E_INVAL;
  void* p = nullptr;
  hipError_t e = hipHostMalloc(&p, nbytes, hipHostMallocMapped | hipHostMallocPortable);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    g_last_hip = (int)e;
    return e == hipErrorOutOfMemory ? CTN_E_NOMEM : CTN_E_HIP;
  }
  *out = p;
  return CTN_OK;
}

int ctn_host_free(void* p) {
  if (!p) return CTN_OK;
  return hipHostFree(p) == hipSuccess ? CTN_OK : CTN_E_HIP;
}

int ctn_register_model(ctn_ctx* c, const ctn_model_desc* desc, const ctn_param* params, size_t n,
                       uint64_t hbm_budget_bytes, ctn_model* out) {
  if (!c || !desc || !params || !out) return CTN_E_INVAL;
  if (hbm_budget_bytes != 0 && hbm_budget_bytes != c->res.budget()) return CTN_E_INVAL;
  if (!desc_valid(*desc)) return CTN_E_INVAL;
  auto m = std::make_unique<Model>();
  m->lay = make_layout(*desc);
  const ShardLayout& L = m->lay;
  if (n != (size_t)L.n_tensors) return CTN_E_INVAL;
  for (int i = 0; i < L.n_tensors; ++i) {
    const ctn_param& p = params[i];
    int64_t r, cc;
    expected_shape(*desc, i, r, cc);
    if (!p.host_ptr || reinterpret_cast<uintptr_t>(p.host_ptr) % 16 || p.nbytes % 16) return CTN_E_INVAL;
    if (p.nbytes != L.nbytes[i]) return CTN_E_INVAL;
    if (cc == 0) {
      if (p.ndim != 1 || p.shape[0] != r) return CTN_E_INVAL;
    } else {
      if (p.ndim != 2 || p.shape[0] != r || p.shape[1] != cc) return CTN_E_INVAL;
    }
    m->host.push_back(p.host_ptr);
  }
  const uint64_t footprint = c->res.block_mode() ? L.slot_bytes * L.n_blocks : L.arena_bytes;
  if (L.param_bytes > c->res.budget() || footprint > c->cfg.arena_bytes) return CTN_E_TOO_BIG;
  // the device must be able to dereference the host tensors (zero-copy path)
  for (int i = 0; i < L.n_tensors; ++i) {
    void* dp = nullptr;
    hipError_t e = hipHostGetDevicePointer(&dp, m->host[i], 0);
    if (e != hipSuccess || !dp) {
      (void)hipGetLastError();
      c->last_hip = (int)e;
      return CTN_E_INVAL;
    }
    m->host_dev.push_back(dp);
  }
  m->runs.assign(L.n_blocks, {});
  for (int b = 0; b < L.n_blocks; ++b)
    for (int ti : L.block_tensors[b]) {
      auto& rs = m->runs[b];
      if (!rs.empty()) {
        Model::Run& r = rs.back();
        const bool host_adjacent = static_cast<char*>(m->host[r.first]) + r.bytes == m->host[ti];
        const bool arena_adjacent = L.offset[r.first] + r.bytes == L.offset[ti];
        if (host_adjacent && arena_adjacent) {
          r.bytes += L.nbytes[ti];
          continue;
        }
      }
      rs.push_back({ti, L.nbytes[ti]});
    }
  size_t n_runs = 0;
  for (auto& rs : m->runs) n_runs += rs.size();
  m->fragmented = n_runs > 4 * static_cast<size_t>(L.n_blocks);
  m->ev_block.assign(L.n_blocks, nullptr);
  for (auto& e : m->ev_block) CTN_HIP(c, hipEventCreate(&e));
  CTN_HIP(c, hipEventCreate(&m->ev_in_start));
  CTN_HIP(c, hipEventCreate(&m->ev_out_start));
  CTN_HIP(c, hipEventCreate(&m->ev_out_done));
  for (hipEvent_t& e : m->ev_last_use) CTN_HIP(c, hipEventCreateWithFlags(&e, hipEventDisableTiming));
  m->block_off.assign(L.n_blocks, 0);
  int idx = c->res.add_model(L.block_bytes);
  c->models.push_back(std::move(m));
  *out = idx;
  return CTN_OK;
}

int ctn_swap_in(ctn_ctx* c, ctn_model mi) {
  if (!get_model(c, mi)) return c ? CTN_E_NOMODEL : CTN_E_INVAL;
  const int rc = ensure_resident(c, mi);
  const int rc2 = flush_deferred(c);
  return rc ? rc : rc2;
}

int ctn_swap_out(ctn_ctx* c, ctn_model mi) {
  Model* m = get_model(c, mi);
  if (!m) return c ? CTN_E_NOMODEL : CTN_E_INVAL;
  std::vector<int> victims;
  if (m->k > 0) {
    victims.push_back(mi);
    const Residency::Move mv = c->res.evict_all(mi);
    c->evict_waves = 0;                // nothing competes for the link on the caller's behalf: full width
    evict_logical(c, mv);
    log_blocks(c, 1, mv, c->events.size());
  }
  int rc = flush_deferred(c);
  if (rc) return rc;
  c->stats.resident_bytes = c->res.resident_bytes();
  log_event(c, 2, mi, victims);
  return CTN_OK;
}

int ctn_wait(ctn_ctx* c, ctn_model mi) {
  Model* m = get_model(c, mi);
  if (!m) return c ? CTN_E_NOMODEL : CTN_E_INVAL;
  if (m->pending_out) {
    CTN_HIP(c, hipEventSynchronize(m->ev_out_done));
    m->pending_out = false;
  }
  if (m->pending_in) {
    CTN_HIP(c, hipEventSynchronize(m->ev_block.back()));
    m->pending_in = false;
  }
  return CTN_OK;
}

uint64_t ctn_workspace_bytes(const ctn_model_desc* desc, int64_t max_tokens, int32_t n_models) {
  (void)n_models;
  if (!desc || !desc_valid(*desc) || max_tokens <= 0) return 0;
  return activation_bytes(*desc, max_tokens, true, nullptr, nullptr);
}

uint64_t ctn_arena_bytes(const ctn_model_desc* desc) {
  if (!desc || !desc_valid(*desc)) return 0;
  return make_layout(*desc).arena_bytes;
}

uint64_t ctn_slot_bytes(const ctn_model_desc* desc) {
  if (!desc || !desc_valid(*desc)) return 0;
  return make_layout(*desc).slot_bytes;
}

// Copies n token ids into the next staging slot (waiting, on the host, for the slot's previous reader
// only when every slot's reader is still running, i.e. with kIdSlots inferences in flight).
static int stage_ids(ctn_ctx* c, const int32_t* ids_host, size_t n, IdSlot** out) {
  // the first slot, from the one after the last used, whose reader has finished: a batch that waits for its
  // model's load keeps its slot for a long time while batches of loaded models come and go
  int pick = -1;
  for (int i = 0; i < kIdSlots && pick < 0; ++i) {
    const int k = (c->next_id_slot + i) % kIdSlots;
    if (!c->id_slots[k].used || hipEventQuery(c->id_slots[k].done) == hipSuccess) pick = k;
  }
  (void)hipGetLastError();                  // "not ready" is an answer
  if (pick < 0) pick = c->next_id_slot;     // every slot busy: wait for this one
  IdSlot& sl = c->id_slots[pick];
  c->next_id_slot = (pick + 1) % kIdSlots;
  if (sl.used) CTN_HIP(c, hipEventSynchronize(sl.done));
  if (sl.cap < n) {
    if (sl.host) CTN_HIP(c, hipHostFree(sl.host));
    sl.host = nullptr;
    sl.cap = 0;
    size_t cap = 256;
    while (cap < n) cap *= 2;
    void* p = nullptr;
    hipError_t e = hipHostMalloc(&p, 4 * cap, hipHostMallocMapped | hipHostMallocPortable);
    if (e != hipSuccess) {
      (void)hipGetLastError();
      c->last_hip = (int)e;
      return e == hipErrorOutOfMemory ? CTN_E_NOMEM : CTN_E_HIP;
    }
    void* dp = nullptr;
    CTN_HIP(c, hipHostGetDevicePointer(&dp, p, 0));
    sl.host = static_cast<int32_t*>(p);
    sl.dev = static_cast<int32_t*>(dp);
    sl.cap = cap;
    if (!sl.done) CTN_HIP(c, hipEventCreateWithFlags(&sl.done, hipEventDisableTiming));
  }
  std::memcpy(sl.host, ids_host, 4 * n);
  *out = &sl;
  return CTN_OK;
}

// Enqueues one inference.  *result_dev / *result_bytes describe where the result stands on the
// device when the caller asked for it in host memory (the caller copies it down).
static int infer_enqueue(ctn_ctx* c, ctn_model mi, const int32_t* ids_host, const void* hidden_in, int32_t in_is_device,
                         int32_t batch, int32_t seq, void* logits_out, int32_t out_is_device, float** logits_dev,
                         uint64_t* logits_bytes, int lane = 0) {
  Model* m = get_model(c, mi);
  if (!m) return c ? CTN_E_NOMODEL : CTN_E_INVAL;
  if (!logits_out) return CTN_E_INVAL;
  const ShardLayout& L = m->lay;
  const ctn_model_desc& d = L.d;
  // stage 0 starts from token ids, every later pipeline stage from the residual stream
  if (L.has_embed() ? (!ids_host || hidden_in) : !hidden_in) return CTN_E_INVAL;
  // (the attention launch puts the batch entries on a grid dimension of at most 65535)
  if (batch <= 0 || batch > 65535 || seq <= 0 || seq > d.max_pos || (int64_t)batch * seq > (1 << 24)) return CTN_E_SHAPE;
  const int M = batch * seq;
  const bool own_logits = !out_is_device && L.has_head();
  Activations act{};
  // with two lanes each works in its own half of the workspace
  const uint64_t ws_half = c->cfg.workspace_bytes / 2 / kAlign * kAlign;
  const uint64_t ws_cap = c->two_lanes ? ws_half : c->cfg.workspace_bytes;
  char* ws_base = static_cast<char*>(c->cfg.workspace_dev) + (lane == 1 ? ws_half : 0);
  if (lane < 0 || lane > 1 || (lane == 1 && !c->two_lanes)) return CTN_E_INVAL;
  if (activation_bytes(d, M, own_logits, &act, ws_base) > ws_cap) return CTN_E_SHAPE;
  if (L.has_embed())
    for (int i = 0; i < M; ++i)
      if (ids_host[i] < 0 || ids_host[i] >= d.vocab) return CTN_E_INVAL;

  int rc = ensure_resident(c, mi);
  if (rc) return rc;
  c->stats.n_infer += 1;

  // With library-owned streams the masked compute stream keeps the forward pass
  // off the copy kernels' compute units; when nothing is moving, the unmasked
  // stream gives it the whole chip.  Both orders of use are chained by an event.
  hipStream_t s = c->s_compute;
  if (lane == 1) {
    s = c->s_lane1;
  } else {
    if (c->s_wide && link_quiet(c)) s = c->s_wide;
    if (c->last_compute && c->last_compute != s) CTN_HIP(c, hipStreamWaitEvent(s, c->ev_compute_done, 0));
  }
  const uint64_t x_bytes = 4ull * M * d.hidden;
  const bool replayable = c->use_graphs && lane == 0 && s == c->s_wide && !m->pending_in;
  IdSlot* slot = nullptr;
  if (L.has_embed()) {
    rc = stage_ids(c, ids_host, M, &slot);
    if (rc) return rc;
    // a captured graph reads its ids from the workspace address it was captured with
    if (replayable) CTN_HIP(c, hipMemcpyAsync(act.ids, slot->host, 4ull * M, hipMemcpyHostToDevice, s));
  } else {
    CTN_HIP(c, hipMemcpyAsync(act.x, hidden_in, x_bytes, in_is_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, s));
  }
  float* logits = out_is_device ? static_cast<float*>(logits_out) : act.logits;

  // A resident model on an idle link needs no event waits: the whole launch
  // sequence is captured once per (model placement, shape, output) as a HIP
  // graph and replayed, which removes the per-launch host cost of ~400 small kernels.
  if (replayable) {
    rc = forward_graph(c, m, act, batch, seq, logits, s);
  } else {
    rc = forward_launches(c, m, act, slot ? slot->dev : nullptr, batch, seq, logits, s, true);
  }
  if (rc) return rc;
  if (slot) {
    CTN_HIP(c, hipEventRecord(slot->done, s));
    slot->used = true;
  }
  if (!L.has_head()) {       // the stage's result is the residual stream
    if (out_is_device) CTN_HIP(c, hipMemcpyAsync(logits_out, act.x, x_bytes, hipMemcpyDeviceToDevice, s));
    logits = act.x;
  }
  CTN_HIP(c, hipEventRecord(m->ev_last_use[lane], s));
  m->used[lane] = true;
  if (c->s_wide && lane == 0) {
    CTN_HIP(c, hipEventRecord(c->ev_compute_done, s));
    c->last_compute = s;
    // whoever synchronises the primary compute stream also waits for this inference
    if (s != c->s_compute) CTN_HIP(c, hipStreamWaitEvent(c->s_compute, c->ev_compute_done, 0));
  }
  *logits_dev = logits;
  *logits_bytes = 4ull * M * L.out_features();
  return CTN_OK;
}

int ctn_infer(ctn_ctx* c, ctn_model mi, const int32_t* ids_host, int32_t batch, int32_t seq, void* logits_out,
              int32_t out_is_device) {
  return ctn_infer_stage(c, mi, ids_host, nullptr, 0, batch, seq, logits_out, out_is_device);
}

int ctn_infer_stage(ctn_ctx* c, ctn_model mi, const int32_t* ids_host, const void* hidden_in, int32_t in_is_device,
                    int32_t batch, int32_t seq, void* logits_out, int32_t out_is_device) {
  float* logits = nullptr;
  uint64_t nbytes = 0;
  const int rc = infer_enqueue(c, mi, ids_host, hidden_in, in_is_device, batch, seq, logits_out, out_is_device,
                               &logits, &nbytes);
  // the victims' offloads go out after the load and the forward pass are in their queues
  const int rc2 = c ? flush_deferred(c) : CTN_OK;
  if (rc || rc2) return rc ? rc : rc2;
  if (!out_is_device) {
    hipStream_t s = c->last_compute ? c->last_compute : c->s_compute;
    CTN_HIP(c, hipMemcpyAsync(logits_out, logits, nbytes, hipMemcpyDeviceToHost, s));
    CTN_HIP(c, hipStreamSynchronize(s));
  }
  return CTN_OK;
}

int ctn_is_resident(ctn_ctx* c, ctn_model mi, int32_t* out) {
  Model* m = get_model(c, mi);
  if (!m) return c ? CTN_E_NOMODEL : CTN_E_INVAL;
  if (!out) return CTN_E_INVAL;
  *out = m->full() ? 1 : 0;
  return CTN_OK;
}

int ctn_resident_blocks(ctn_ctx* c, ctn_model mi, int32_t* resident, int32_t* total) {
  Model* m = get_model(c, mi);
  if (!m) return c ? CTN_E_NOMODEL : CTN_E_INVAL;
  if (resident) *resident = m->k;
  if (total) *total = m->lay.n_blocks;
  return CTN_OK;
}

int ctn_get_block_events(ctn_ctx* c, uint64_t first, ctn_block_event* out, uint64_t cap, uint64_t* n_out,
                         uint64_t* total) {
  if (!c || !n_out || !total || (cap && !out)) return CTN_E_INVAL;
  *total = c->block_events.size();
  uint64_t n = 0;
  for (uint64_t i = first; i < c->block_events.size() && n < cap; ++i) out[n++] = c->block_events[i];
  *n_out = n;
  return CTN_OK;
}

int ctn_get_stats(ctn_ctx* c, ctn_stats* out) {
  if (!c || !out) return CTN_E_INVAL;
  c->stats.resident_bytes = c->res.resident_bytes();
  c->stats.peak_resident_bytes = c->res.peak_bytes();
  *out = c->stats;
  return CTN_OK;
}

int ctn_get_events(ctn_ctx* c, uint64_t first, ctn_event* out, uint64_t cap, uint64_t* n_out, uint64_t* total) {
  if (!c || !n_out || !total || (cap && !out)) return CTN_E_INVAL;
  *total = c->events.size();
  uint64_t n = 0;
  for (uint64_t i = first; i < c->events.size() && n < cap; ++i) out[n++] = c->events[i];
  *n_out = n;
  return CTN_OK;
}

int ctn_last_swap_ms(ctn_ctx* c, ctn_model mi, float* in_ms, float* out_ms, float* block_ms, int32_t cap,
                     int32_t* n_blocks) {
  Model* m = get_model(c, mi);
  if (!m) return c ? CTN_E_NOMODEL : CTN_E_INVAL;
  int rc = ctn_wait(c, mi);
  if (rc) return rc;
  if (n_blocks) *n_blocks = m->lay.n_blocks;
  if (in_ms) {
    *in_ms = -1.f;
    if (m->load_recorded) CTN_HIP(c, hipEventElapsedTime(in_ms, m->ev_in_start, m->ev_block.back()));
  }
  if (out_ms) {
    *out_ms = -1.f;
    if (m->out_recorded) {
      CTN_HIP(c, hipEventSynchronize(m->ev_out_done));
      CTN_HIP(c, hipEventElapsedTime(out_ms, m->ev_out_start, m->ev_out_done));
    }
  }
  if (block_ms && m->load_recorded)
    for (int b = 0; b < m->lay.n_blocks && b < cap; ++b) {
      block_ms[b] = 0.f;             // blocks that were already resident took no part in the last load
      if (b >= m->last_load_first) CTN_HIP(c, hipEventElapsedTime(&block_ms[b], m->ev_in_start, m->ev_block[b]));
    }
  return CTN_OK;
}

int ctn_debug_read_param(ctn_ctx* c, ctn_model mi, int32_t index, void* dst, uint64_t cap) {
  Model* m = get_model(c, mi);
  if (!m) return c ? CTN_E_NOMODEL : CTN_E_INVAL;
  if (!dst || index < 0 || index >= m->lay.n_tensors || m->lay.block_of[index] >= m->k) return CTN_E_INVAL;
  if (cap < m->lay.nbytes[index]) return CTN_E_INVAL;
  int rc = ctn_wait(c, mi);
  if (rc) return rc;
  CTN_HIP(c, hipMemcpy(dst, dev_tensor<char>(c, m, index), m->lay.nbytes[index], hipMemcpyDeviceToHost));
  return CTN_OK;
}

int ctn_get_streams(ctn_ctx* c, void** compute, void** h2d, void** d2h) {
  if (!c) return CTN_E_INVAL;
  if (compute) *compute = c->s_compute;
  if (h2d) *h2d = c->s_h2d;
  if (d2h) *d2h = c->s_d2h;
  return CTN_OK;
}

int ctn_set_graphs(ctn_ctx* c, int32_t enable) {
  if (!c) return CTN_E_INVAL;
  c->use_graphs = enable && c->s_wide != nullptr;
  return CTN_OK;
}

int ctn_set_discard(ctn_ctx* c, int32_t enable) {
  if (!c || (enable != 0 && enable != 1)) return CTN_E_INVAL;
  c->cfg.discard_on_evict = enable;
  return CTN_OK;
}

int ctn_set_mode(ctn_ctx* c, int32_t transfer_mode, int32_t pipeline, int32_t copy_blocks) {
  if (!c) return CTN_E_INVAL;
  if (transfer_mode < CTN_XFER_DMA || transfer_mode > CTN_XFER_DMA_RUNS) return CTN_E_INVAL;
  if (copy_blocks < 0 || copy_blocks > 4096) return CTN_E_INVAL;
  c->cfg.transfer_mode = transfer_mode;
  c->cfg.pipeline = pipeline ? 1 : 0;
  c->cfg.copy_blocks = copy_blocks;
  return CTN_OK;
}

int ctn_set_copy_width(ctn_ctx* c, int32_t blocks_in, int32_t waves_out) {
  if (!c || blocks_in < 0 || blocks_in > 4096 || waves_out < 0 || waves_out > 16384) return CTN_E_INVAL;
  c->cfg.copy_blocks = blocks_in;
  c->cfg.copy_waves_out = waves_out;
  return CTN_OK;
}

int ctn_last_hip_error(ctn_ctx* c) { return c ? c->last_hip : g_last_hip; }

const char* ctn_strerror(int code) {
  switch (code) {
    case CTN_OK: return "ok";
    case CTN_E_INVAL: return "invalid argument";
    case CTN_E_TOO_BIG: return "shard larger than the budget or the arena";
    case CTN_E_NOMODEL: return "unknown model";
    case CTN_E_BUSY: return "no room can be made";
    case CTN_E_HIP: return "HIP call failed";
    case CTN_E_SHAPE: return "batch/sequence outside what the model or workspace allows";
    case CTN_E_NOMEM: return "out of memory";
    default: return "unknown error";
  }
}

int ctn_residency_replay(uint64_t budget, const uint64_t* sizes, int32_t n_models, const int32_t* trace,
                         uint64_t n, ctn_event* out) {
  if (!sizes || n_models <= 0 || (n && (!trace || !out))) return CTN_E_INVAL;
  Residency res(budget);
  for (int i = 0; i < n_models; ++i) res.add_model(sizes[i]);
  for (uint64_t i = 0; i < n; ++i) {
    const int m = trace[i];
    if (m < 0 || m >= n_models) return CTN_E_NOMODEL;
    ctn_event e{};
    e.model = m;
    if (res.resident(m)) {
      res.touch(m);
      e.kind = 0;
    } else {
      if (res.size(m) > budget) return CTN_E_TOO_BIG;
      e.kind = 1;
      std::vector<Residency::Move> moves;
      while (res.over_budget_with(m))
        if (res.evict_step(m, moves) < 0) return CTN_E_BUSY;
      for (const Residency::Move& mv : moves) {
        if (e.n_victims < 13) e.victims[e.n_victims] = mv.model;
        e.n_victims += 1;
      }
      res.load_missing(m);
    }
    out[i] = e;
  }
  return CTN_OK;
}

int ctn_block_residency_replay(uint64_t budget, const int32_t* n_blocks, const uint64_t* block_bytes, int32_t n_models,
                               const int32_t* trace, uint64_t n, ctn_event* out, ctn_block_event* blocks_out,
                               uint64_t cap, uint64_t* n_blocks_out) {
  if (!n_blocks || !block_bytes || n_models <= 0 || !n_blocks_out || (n && (!trace || !out)) || (cap && !blocks_out))
    return CTN_E_INVAL;
  Residency res(budget, true);
  uint64_t at = 0;
  for (int i = 0; i < n_models; ++i) {
    if (n_blocks[i] < 1) return CTN_E_INVAL;
    res.add_model(std::vector<uint64_t>(block_bytes + at, block_bytes + at + n_blocks[i]));
    at += n_blocks[i];
  }
  uint64_t nb = 0;
  auto emit = [&](int kind, const Residency::Move& mv, uint64_t use) {
    if (mv.b0 >= mv.b1) return true;
    if (nb >= cap) return false;
    blocks_out[nb++] = ctn_block_event{kind, mv.model, mv.b0, mv.b1, use};
    return true;
  };
  for (uint64_t i = 0; i < n; ++i) {
    const int m = trace[i];
    if (m < 0 || m >= n_models) return CTN_E_NOMODEL;
    ctn_event e{};
    e.model = m;
    if (res.resident(m)) {
      res.touch(m);
      e.kind = 0;
    } else {
      if (res.size(m) > budget) return CTN_E_TOO_BIG;
      e.kind = 1;
      std::vector<Residency::Move> moves;
      while (res.over_budget_with(m))
        if (res.evict_step(m, moves) < 0) return CTN_E_BUSY;
      for (const Residency::Move& mv : moves) {
        if (e.n_victims < 13) e.victims[e.n_victims] = mv.model;
        e.n_victims += 1;
        if (!emit(1, mv, i)) return CTN_E_INVAL;
      }
      if (!emit(0, res.load_missing(m), i)) return CTN_E_INVAL;
    }
    out[i] = e;
  }
  *n_blocks_out = nb;
  return CTN_OK;
}

// ---- serving engine ------------------------------------------------------------

struct ctn_engine {
  ctn_ctx* ctx;
  int max_batch, seq;
  RequestQueues queues;
  int64_t next_id = 0;
  std::vector<int32_t> packed;   // ids of the batch being dispatched
  TransitionPredictor predictor;
  bool prefetch = false;
  // two-lane engine: the batch in flight on each lane (model -1: none) and its completion event
  bool two_lanes = false;
  int lane_model[2] = {-1, -1};
  hipEvent_t lane_done[2] = {nullptr, nullptr};
};

int ctn_engine_create(ctn_ctx* c, int32_t max_batch, int32_t seq, ctn_engine** out) {
  if (!c || !out || max_batch < 1 || seq < 1) return CTN_E_INVAL;
  ctn_engine* e = new (std::nothrow) ctn_engine{c, max_batch, seq, RequestQueues(), 0, {}, {}, false};
  if (!e) return CTN_E_NOMEM;
  *out = e;
  return CTN_OK;
}

int ctn_engine_create_async(ctn_ctx* c, int32_t max_batch, int32_t seq, ctn_engine** out) {
  if (!c || !out || max_batch < 1 || seq < 1) return CTN_E_INVAL;
  if (!c->own_streams || !c->s_lane1) return CTN_E_INVAL;     // the second lane needs the library's own streams
  ctn_engine* e = new (std::nothrow) ctn_engine{c, max_batch, seq, RequestQueues(), 0, {}, {}, false};
  if (!e) return CTN_E_NOMEM;
  e->two_lanes = true;
  for (hipEvent_t& ev : e->lane_done)
    if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) {
      c->last_hip = (int)hipGetLastError();
      for (hipEvent_t x : e->lane_done)
        if (x) (void)hipEventDestroy(x);
      delete e;
      return CTN_E_HIP;
    }
  c->two_lanes = true;          // from now on every inference stays inside its lane's half of the workspace
  *out = e;
  return CTN_OK;
}

int ctn_engine_destroy(ctn_engine* e) {
  if (!e) return CTN_OK;
  if (e->two_lanes) {
    // the context goes back to one lane over the whole workspace once nothing runs in the halves
    (void)ctn_sync(e->ctx);
    e->ctx->two_lanes = false;
  }
  for (hipEvent_t ev : e->lane_done)
    if (ev) (void)hipEventDestroy(ev);
  delete e;
  return CTN_OK;
}

// Refreshes which lanes still have a batch in flight.
static void refresh_lanes(ctn_engine* e) {
  for (int l = 0; l < 2; ++l)
    if (e->lane_model[l] >= 0 && hipEventQuery(e->lane_done[l]) == hipSuccess) e->lane_model[l] = -1;
  (void)hipGetLastError();      // "not ready" is an answer
}

int ctn_engine_lanes(ctn_engine* e, int32_t* busy) {
  if (!e || !busy || !e->two_lanes) return CTN_E_INVAL;
  refresh_lanes(e);
  for (int l = 0; l < 2; ++l) busy[l] = e->lane_model[l] >= 0 ? 1 : 0;
  return CTN_OK;
}

int ctn_engine_dispatch(ctn_engine* e, void* const logits_out[2], int64_t* served, int32_t cap, int32_t* n_served,
                        ctn_model* model, int32_t* was_miss, int32_t* lane_out) {
  if (!e || !e->two_lanes || !logits_out || !logits_out[0] || !logits_out[1] || !served || !n_served ||
      cap < e->max_batch)
    return CTN_E_INVAL;
  *n_served = 0;
  ctn_ctx* c = e->ctx;
  refresh_lanes(e);
  const bool lane_free[2] = {e->lane_model[0] < 0, e->lane_model[1] < 0};
  int lane = 0;
  // "Loaded" = every block resident and landed.  A model whose load was started ahead of its
  // request (ctn_engine_idle) and is still arriving takes the load lane like a miss, so that its
  // batch waits there and not in front of the loaded models' batches.
  auto loaded = [&](int k) {
    Model* mk = c->models[k].get();
    if (!mk->full()) return false;
    if (mk->pending_in && hipEventQuery(mk->ev_block.back()) == hipSuccess) mk->pending_in = false;
    return !mk->pending_in;
  };
  const int m = pick_two_lane(
      e->queues, loaded, [&](int k) { return e->lane_model[kLoadLane] == k; }, lane_free, &lane);
  (void)hipGetLastError();
  if (m < 0) return CTN_OK;
  const bool miss = !c->models[m]->full();
  std::vector<QueuedRequest> batch = e->queues.pop(m, e->max_batch);
  e->packed.clear();
  for (const QueuedRequest& r : batch) e->packed.insert(e->packed.end(), r.ids.begin(), r.ids.end());
  float* result = nullptr;
  uint64_t nbytes = 0;
  int rc = infer_enqueue(c, m, e->packed.data(), nullptr, 0, static_cast<int32_t>(batch.size()), e->seq,
                         logits_out[lane], 1, &result, &nbytes, lane);
  const int rc2 = flush_deferred(c);
  if (!rc) rc = rc2;
  if (!rc && hipEventRecord(e->lane_done[lane], lane == kLoadLane ? c->s_lane1 : (c->last_compute ? c->last_compute : c->s_compute)) != hipSuccess) {
    c->last_hip = (int)hipGetLastError();
    rc = CTN_E_HIP;
  }
  if (rc) {   // put the requests back in order so nothing is lost
    for (auto it = batch.rbegin(); it != batch.rend(); ++it) e->queues.push_front(m, std::move(*it));
    return rc;
  }
  e->lane_model[lane] = m;
  for (size_t i = 0; i < batch.size(); ++i) served[i] = batch[i].id;
  *n_served = static_cast<int32_t>(batch.size());
  if (model) *model = m;
  if (was_miss) *was_miss = miss ? 1 : 0;
  if (lane_out) *lane_out = lane;
  e->predictor.observe(m);
  return CTN_OK;
}

int ctn_engine_submit(ctn_engine* e, ctn_model m, const int32_t* ids, double timestamp, int64_t* request_id) {
  if (!e || !ids) return CTN_E_INVAL;
  Model* mod = get_model(e->ctx, m);
  if (!mod) return CTN_E_NOMODEL;
  if (!mod->lay.has_embed()) return CTN_E_INVAL;   // the queues hold token ids: stage 0 shards only
  if (e->seq > mod->lay.d.max_pos) return CTN_E_SHAPE;
  for (int i = 0; i < e->seq; ++i)
    if (ids[i] < 0 || ids[i] >= mod->lay.d.vocab) return CTN_E_INVAL;
  e->queues.ensure(static_cast<int>(e->ctx->models.size()));
  QueuedRequest r{e->next_id, timestamp, std::vector<int32_t>(ids, ids + e->seq)};
  e->queues.push(m, std::move(r));
  if (request_id) *request_id = e->next_id;
  e->next_id += 1;
  return CTN_OK;
}

int ctn_engine_pending(ctn_engine* e, int64_t* n) {
  if (!e || !n) return CTN_E_INVAL;
  *n = e->queues.pending();
  return CTN_OK;
}

int ctn_engine_step(ctn_engine* e, void* logits_out, int64_t* served, int32_t cap, int32_t* n_served,
                    ctn_model* model, int32_t* was_miss) {
  if (!e || e->two_lanes || !logits_out || !served || !n_served || cap < e->max_batch) return CTN_E_INVAL;
  *n_served = 0;
  const int m = e->queues.pick();
  if (m < 0) return CTN_OK;
  std::vector<QueuedRequest> batch = e->queues.pop(m, e->max_batch);
  e->packed.clear();
  for (const QueuedRequest& r : batch) e->packed.insert(e->packed.end(), r.ids.begin(), r.ids.end());
  if (model) *model = m;
  if (was_miss) *was_miss = e->ctx->models[m]->full() ? 0 : 1;
  const int rc = ctn_infer(e->ctx, m, e->packed.data(), static_cast<int32_t>(batch.size()), e->seq, logits_out, 1);
  if (rc) {   // put the requests back in order so nothing is lost
    for (auto it = batch.rbegin(); it != batch.rend(); ++it) e->queues.push_front(m, std::move(*it));
    return rc;
  }
  for (size_t i = 0; i < batch.size(); ++i) served[i] = batch[i].id;
  *n_served = static_cast<int32_t>(batch.size());
  e->predictor.observe(m);
  return CTN_OK;
}

int ctn_engine_set_prefetch(ctn_engine* e, int32_t enable, int32_t min_count, int32_t min_share_percent) {
  if (!e || min_count < 1 || min_share_percent < 0 || min_share_percent > 100) return CTN_E_INVAL;
  e->prefetch = enable != 0;
  e->predictor.configure(min_count, min_share_percent);
  return CTN_OK;
}

int ctn_engine_idle(ctn_engine* e, ctn_model* loaded) {
  if (!e || !loaded) return CTN_E_INVAL;
  *loaded = -1;
  if (!e->prefetch || e->queues.pending() > 0) return CTN_OK;
  const int p = e->predictor.predict();
  Model* m = get_model(e->ctx, p);
  if (!m || m->full()) return CTN_OK;
  const int rc = ctn_swap_in(e->ctx, p);
  if (rc) return rc;
  e->ctx->stats.n_prefetch += 1;
  *loaded = p;
  return CTN_OK;
}

int ctn_predictor_replay(int32_t n_models, int32_t min_count, int32_t min_share_percent, const int32_t* dispatches,
                         uint64_t n, int32_t* predictions) {
  if (n_models <= 0 || min_count < 1 || min_share_percent < 0 || min_share_percent > 100 ||
      (n && (!dispatches || !predictions)))
    return CTN_E_INVAL;
  TransitionPredictor p;
  p.configure(min_count, min_share_percent);
  for (uint64_t i = 0; i < n; ++i) {
    if (dispatches[i] < 0 || dispatches[i] >= n_models) return CTN_E_NOMODEL;
    p.observe(dispatches[i]);
    predictions[i] = p.predict();
  }
  return CTN_OK;
}

int ctn_engine_replay(int32_t n_models, int32_t max_batch, uint64_t budget, const uint64_t* sizes,
                      const double* arrival, const int32_t* model_of, uint64_t n, double t_base,
                      double t_per_request, double t_miss, ctn_batch_record* batches, uint64_t cap,
                      uint64_t* n_batches, uint64_t* requests) {
  if (n_models <= 0 || max_batch < 1 || !sizes || !n_batches || (n && (!arrival || !model_of || !batches || !requests)))
    return CTN_E_INVAL;
  for (uint64_t i = 0; i < n; ++i) {
    if (model_of[i] < 0 || model_of[i] >= n_models) return CTN_E_NOMODEL;
    if (i && arrival[i] < arrival[i - 1]) return CTN_E_INVAL;
  }
  Residency res(budget);
  for (int i = 0; i < n_models; ++i) {
    if (sizes[i] > budget) return CTN_E_TOO_BIG;
    res.add_model(sizes[i]);
  }
  RequestQueues queues(n_models);
  double now = 0.0;
  uint64_t nxt = 0, served = 0, nb = 0;
  while (served < n) {
    while (nxt < n && arrival[nxt] <= now) {
      queues.push(model_of[nxt], QueuedRequest{static_cast<int64_t>(nxt), arrival[nxt], {}});
      ++nxt;
    }
    const int m = queues.pick();
    if (m < 0) {
      now = arrival[nxt];
      continue;
    }
    std::vector<QueuedRequest> batch = queues.pop(m, max_batch);
    bool miss = !res.resident(m);
    if (miss) {
      std::vector<Residency::Move> moves;
      while (res.over_budget_with(m))
        if (res.evict_step(m, moves) < 0) return CTN_E_BUSY;
      res.load_missing(m);
    } else {
      res.touch(m);
    }
    if (nb >= cap) return CTN_E_INVAL;
    ctn_batch_record& b = batches[nb++];
    b.start = now;
    b.finish = now + t_base + t_per_request * static_cast<double>(batch.size()) + (miss ? t_miss : 0.0);
    b.model = m;
    b.count = static_cast<int32_t>(batch.size());
    b.miss = miss ? 1 : 0;
    b.reserved = 0;
    b.offset = served;
    for (const QueuedRequest& r : batch) requests[served++] = static_cast<uint64_t>(r.id);
    now = b.finish;
  }
  *n_batches = nb;
  return CTN_OK;
}

int ctn_engine_replay_async(int32_t n_models, int32_t max_batch, uint64_t budget, const uint64_t* sizes,
                            const double* arrival, const int32_t* model_of, uint64_t n, double t_base,
                            double t_per_request, double t_miss, ctn_batch_record* batches, uint64_t cap,
                            uint64_t* n_batches, uint64_t* requests) {
  if (n_models <= 0 || max_batch < 1 || !sizes || !n_batches || (n && (!arrival || !model_of || !batches || !requests)))
    return CTN_E_INVAL;
  for (uint64_t i = 0; i < n; ++i) {
    if (model_of[i] < 0 || model_of[i] >= n_models) return CTN_E_NOMODEL;
    if (i && arrival[i] < arrival[i - 1]) return CTN_E_INVAL;
  }
  Residency res(budget);
  for (int i = 0; i < n_models; ++i) {
    if (sizes[i] > budget) return CTN_E_TOO_BIG;
    res.add_model(sizes[i]);
  }
  RequestQueues queues(n_models);
  double now = 0.0, lane_until[2] = {0.0, 0.0};
  int loading = -1;                       // model whose miss occupies lane 1
  uint64_t nxt = 0, served = 0, nb = 0;
  while (served < n) {
    while (nxt < n && arrival[nxt] <= now) {
      queues.push(model_of[nxt], QueuedRequest{static_cast<int64_t>(nxt), arrival[nxt], {}});
      ++nxt;
    }
    if (lane_until[kLoadLane] <= now) loading = -1;
    for (;;) {
      const bool lane_free[2] = {lane_until[0] <= now, lane_until[1] <= now};
      int lane = 0;
      const int m = pick_two_lane(
          queues, [&](int k) { return res.resident(k); }, [&](int k) { return loading == k; }, lane_free, &lane);
      if (m < 0) break;
      std::vector<QueuedRequest> batch = queues.pop(m, max_batch);
      const bool miss = lane == kLoadLane;
      if (miss) {
        std::vector<Residency::Move> moves;
        while (res.over_budget_with(m))
          if (res.evict_step(m, moves) < 0) return CTN_E_BUSY;
        res.load_missing(m);
        loading = m;
      } else {
        res.touch(m);
      }
      if (nb >= cap) return CTN_E_INVAL;
      ctn_batch_record& b = batches[nb++];
      b.start = now;
      b.finish = now + t_base + t_per_request * static_cast<double>(batch.size()) + (miss ? t_miss : 0.0);
      b.model = m;
      b.count = static_cast<int32_t>(batch.size());
      b.miss = miss ? 1 : 0;
      b.reserved = lane;
      b.offset = served;
      for (const QueuedRequest& r : batch) requests[served++] = static_cast<uint64_t>(r.id);
      lane_until[lane] = b.finish;
    }
    if (served == n) break;
    double next = -1.0;
    for (double t : lane_until)
      if (t > now && (next < 0 || t < next)) next = t;
    if (nxt < n && (next < 0 || arrival[nxt] < next)) next = arrival[nxt];
    if (next < 0) return CTN_E_BUSY;      // cannot happen: requests wait only for lanes or arrivals
    now = next;
  }
  *n_batches = nb;
  return CTN_OK;
}

// ---- single operations -------------------------------------------------------

static bool aligned16(const void* p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; }
static int op_rc(hipError_t e) { return e == hipSuccess ? CTN_OK : (e == hipErrorInvalidValue ? CTN_E_INVAL : CTN_E_HIP); }

int ctn_op_copy(void* dst, const void* src, uint64_t nbytes, int32_t blocks, void* stream) {
  if (!dst || !src || nbytes % 16 || reinterpret_cast<uintptr_t>(dst) % 16 || reinterpret_cast<uintptr_t>(src) % 16)
    return CTN_E_INVAL;
  CopyTable t{};
  t.n = 1;
  t.seg[0] = {src, dst, nbytes / 16};
  if (blocks < 0 || blocks > 16384) return CTN_E_INVAL;
  if (!copy_table_finish(t, 256)) return CTN_E_INVAL;
  return op_rc(launch_copy_table(t, 4 * blocks, static_cast<hipStream_t>(stream), kCopyOther));
}

int ctn_op_dma(void* dst, const void* src, uint64_t nbytes, void* stream) {
  if (!dst || !src) return CTN_E_INVAL;
  return op_rc(hipMemcpyAsync(dst, src, nbytes, hipMemcpyDefault, static_cast<hipStream_t>(stream)));
}

int ctn_op_embed(const int32_t* ids, const void* tok, const void* pos, float* x, int32_t M, int32_t seq,
                 int32_t hidden, int32_t vocab_local, int32_t rank, void* stream) {
  if (!ids || !tok || !pos || !x || M < 0) return CTN_E_INVAL;
  if (!aligned16(tok) || !aligned16(pos) || !aligned16(x) || reinterpret_cast<uintptr_t>(ids) % 4) return CTN_E_INVAL;
  return op_rc(launch_embed(ids, static_cast<const _Float16*>(tok), static_cast<const _Float16*>(pos), x, M, seq,
                            hidden, vocab_local, rank, static_cast<hipStream_t>(stream)));
}

int ctn_op_layernorm(const float* x, const void* g, const void* b, void* out, int32_t rows, int32_t hidden,
                     void* stream) {
  if (!x || !g || !b || !out || rows < 0) return CTN_E_INVAL;
  if (!aligned16(x) || reinterpret_cast<uintptr_t>(g) % 8 || reinterpret_cast<uintptr_t>(b) % 8 ||
      reinterpret_cast<uintptr_t>(out) % 8)
    return CTN_E_INVAL;
  return op_rc(launch_layernorm(const_cast<float*>(x), static_cast<const _Float16*>(g), static_cast<const _Float16*>(b),
                                static_cast<_Float16*>(out), rows, hidden, static_cast<hipStream_t>(stream)));
}

int ctn_op_gemm(const void* A, const void* W, const void* bias, void* out, int32_t M, int32_t N, int32_t K,
                int32_t epilogue, void* stream) {
  if (!A || !W || !out || M < 0 || N < 0) return CTN_E_INVAL;
  return op_rc(launch_gemm(static_cast<const _Float16*>(A), static_cast<const _Float16*>(W),
                           static_cast<const _Float16*>(bias), out, M, N, K, epilogue,
                           static_cast<hipStream_t>(stream)));
}

int ctn_op_gemm_ws(const void* A, const void* W, const void* bias, void* out, int32_t M, int32_t N, int32_t K,
                   int32_t epilogue, void* workspace, uint64_t workspace_bytes, void* stream) {
  if (!A || !W || !out || M < 0 || N < 0) return CTN_E_INVAL;
  if (workspace && reinterpret_cast<uintptr_t>(workspace) % 16) return CTN_E_INVAL;
  return op_rc(launch_gemm(static_cast<const _Float16*>(A), static_cast<const _Float16*>(W),
                           static_cast<const _Float16*>(bias), out, M, N, K, epilogue,
                           static_cast<hipStream_t>(stream), static_cast<float*>(workspace), workspace_bytes / 4));
}

int ctn_op_gemm_static(const void* A, const void* W, const void* bias, void* out, int32_t M, int32_t N, int32_t K,
                       int32_t epilogue, void* stream) {
  if (!A || !W || !out || M < 0 || N < 0) return CTN_E_INVAL;
  // room for the largest number of K slices a product of this shape may be cut into
  const uint64_t need = 4ull * static_cast<uint64_t>(M) * static_cast<uint64_t>(N) * (M <= 256 ? 16u : 4u);
  if (need > kStaticScratchBytes) return CTN_E_TOO_BIG;
  void* sp = nullptr;
  const hipError_t e = static_scratch(&sp);      // cached after the first call on a device; allocates nothing
  if (e != hipSuccess) {
    (void)hipGetLastError();
    g_last_hip = (int)e;
    return CTN_E_HIP;
  }
  return op_rc(launch_gemm(static_cast<const _Float16*>(A), static_cast<const _Float16*>(W),
                           static_cast<const _Float16*>(bias), out, M, N, K, epilogue,
                           static_cast<hipStream_t>(stream), static_cast<float*>(sp), kStaticScratchBytes / 4));
}

uint64_t ctn_static_scratch_bytes(void) { return kStaticScratchBytes; }

int ctn_debug_gemm_tile(ctn_ctx* c, int32_t cfg) {
  if (!c) return CTN_E_INVAL;
  return gemm_tuning_set(c->tuning, cfg) == 0 ? CTN_OK : CTN_E_INVAL;
}

int ctn_test_op_gemm(const void* A, const void* W, const void* bias, void* out, int32_t M, int32_t N, int32_t K,
                     int32_t epilogue, void* workspace, uint64_t workspace_bytes, const int32_t* hooks, int32_t n_hooks,
                     void* stream) {
  if (!A || !W || !out || M < 0 || N < 0 || n_hooks < 0 || (n_hooks && !hooks)) return CTN_E_INVAL;
  if (workspace && reinterpret_cast<uintptr_t>(workspace) % 16) return CTN_E_INVAL;
  GemmTuning t;
  for (int i = 0; i < n_hooks; ++i)
    if (gemm_tuning_set(t, hooks[i]) != 0) return CTN_E_INVAL;
  return op_rc(launch_gemm(static_cast<const _Float16*>(A), static_cast<const _Float16*>(W),
                           static_cast<const _Float16*>(bias), out, M, N, K, epilogue,
                           static_cast<hipStream_t>(stream), static_cast<float*>(workspace), workspace_bytes / 4,
                           nullptr, &t));
}

int ctn_op_attention(const void* qkv, void* out, int32_t batch, int32_t seq, int32_t heads, int32_t head_dim,
                     void* stream) {
  if (!qkv || !out || batch < 0 || seq < 0 || heads < 0) return CTN_E_INVAL;
  if (!aligned16(qkv) || !aligned16(out)) return CTN_E_INVAL;
  return op_rc(launch_attention(static_cast<const _Float16*>(qkv), static_cast<_Float16*>(out), batch, seq, heads,
                                head_dim, static_cast<hipStream_t>(stream)));
}

}  // extern "C"
