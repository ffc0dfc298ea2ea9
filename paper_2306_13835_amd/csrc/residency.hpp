// Host-only residency policy and arena range bookkeeping (no HIP here).
//
// Section 3 of the paper: a request for a model that is not in device memory
// makes a replacement policy pick resident models to swap out, then the
// requested one is swapped in ("demand paging"); Section 4 names the policy:
// least recently used.  The paper caps the number of resident models; this
// manager caps parameter bytes, which is the same thing for equal sizes.
#pragma once
#include <algorithm>
#include <climits>
#include <cstdint>
#include <limits>
#include <vector>

namespace ctn {

// Least-recently-used residency under a byte budget.  A "use" stamps the
// model with a strictly increasing counter, so the order is total.
//
// A model is a list of transfer blocks and what is resident of it is a prefix
// of that list.  In whole-model mode (the paper's) the prefix is all or
// nothing.  In block mode an eviction step takes one block from the tail of
// the least recently used model, so a miss frees no more than it needs and
// the victim later reloads only its missing tail.
class Residency {
 public:
  struct Move {        // blocks [b0, b1) of `model` leave (or enter) device memory
    int model, b0, b1;
  };

  explicit Residency(uint64_t budget, bool block_mode = false) : budget_(budget), block_mode_(block_mode) {}

  int add_model(std::vector<uint64_t> block_bytes) {
    uint64_t total = 0;
    for (uint64_t b : block_bytes) total += b;
    blocks_.push_back(std::move(block_bytes));
    size_.push_back(total);
    k_.push_back(0);
    stamp_.push_back(0);
    return static_cast<int>(size_.size()) - 1;
  }
  int add_model(uint64_t bytes) { return add_model(std::vector<uint64_t>{bytes}); }

  int n_models() const { return static_cast<int>(size_.size()); }
  int n_blocks(int m) const { return static_cast<int>(blocks_[m].size()); }
  int resident_blocks(int m) const { return k_[m]; }
  bool resident(int m) const { return k_[m] == n_blocks(m); }      // completely resident
  bool block_mode() const { return block_mode_; }
  uint64_t size(int m) const { return size_[m]; }
  uint64_t budget() const { return budget_; }
  uint64_t resident_bytes() const { return resident_bytes_; }
  uint64_t peak_bytes() const { return peak_; }
  uint64_t missing_bytes(int m) const {
    uint64_t n = 0;
    for (int b = k_[m]; b < n_blocks(m); ++b) n += blocks_[m][b];
    return n;
  }

  // A use of a completely resident model.
  void touch(int m) { stamp_[m] = ++clock_; }

  // The model with resident blocks that was used longest ago, other than `except`; -1 if none.
  int oldest(int except) const {
    int best = -1;
    uint64_t best_stamp = std::numeric_limits<uint64_t>::max();
    for (int i = 0; i < n_models(); ++i)
      if (i != except && k_[i] > 0 && stamp_[i] < best_stamp) {
        best_stamp = stamp_[i];
        best = i;
      }
    return best;
  }

  // True while the missing blocks of m do not fit next to what is resident.
  bool over_budget_with(int m) const { return resident_bytes_ + missing_bytes(m) > budget_; }

  // One eviction step on behalf of m: the least recently used other model
  // loses its last block (block mode) or everything (whole-model mode).
  // The move is merged into `out` (one entry per victim, in eviction order).
  // Returns the victim, -1 when nothing is left to evict.
  int evict_step(int m, std::vector<Move>& out) {
    const int v = oldest(m);
    if (v < 0) return -1;
    const int hi = k_[v];
    const int lo = block_mode_ ? hi - 1 : 0;
    drop(v, lo);
    for (Move& mv : out)
      if (mv.model == v) {
        mv.b0 = lo;
        return v;
      }
    out.push_back({v, lo, hi});
    return v;
  }

  // Everything resident of m leaves (explicit swap-out).  Returns the move; b0 == b1 when nothing was resident.
  Move evict_all(int m) {
    const Move mv{m, 0, k_[m]};
    drop(m, 0);
    return mv;
  }

  // The missing blocks of m have been given room: m is completely resident and just used.
  Move load_missing(int m) {
    const Move mv{m, k_[m], n_blocks(m)};
    resident_bytes_ += missing_bytes(m);
    k_[m] = n_blocks(m);
    stamp_[m] = ++clock_;
    peak_ = std::max(peak_, resident_bytes_);
    return mv;
  }

 private:
  void drop(int m, int new_k) {
    for (int b = new_k; b < k_[m]; ++b) resident_bytes_ -= blocks_[m][b];
    k_[m] = new_k;
    if (new_k == 0) stamp_[m] = 0;
  }

  uint64_t budget_;
  bool block_mode_;
  uint64_t clock_ = 0, resident_bytes_ = 0, peak_ = 0;
  std::vector<std::vector<uint64_t>> blocks_;
  std::vector<uint64_t> size_, stamp_;
  std::vector<int> k_;
};

// First-fit allocator over the caller's arena, in bytes, with coalescing.
class RangeAllocator {
 public:
  struct Range {
    uint64_t off, len;
  };
  explicit RangeAllocator(uint64_t total = 0) { reset(total); }
  void reset(uint64_t total) {
    free_.clear();
    if (total) free_.push_back({0, total});
  }
  // Returns the offset or UINT64_MAX when no hole is large enough.
  uint64_t alloc(uint64_t len) {
    for (size_t i = 0; i < free_.size(); ++i)
      if (free_[i].len >= len) {
        uint64_t off = free_[i].off;
        free_[i].off += len;
        free_[i].len -= len;
        if (free_[i].len == 0) free_.erase(free_.begin() + i);
        return off;
      }
    return UINT64_MAX;
  }
  // Placement that waits least on ranges still being read by offloads.
  // `busy` lists those ranges in the order their offloads complete (oldest
  // first).  Every hole is tried at its start and slid just past each busy
  // range; the cost of a placement is the position of the last busy range it
  // overlaps (-1: none).  Lowest cost wins, then lowest offset.  A placement
  // whose cost exceeds max_cost is not taken (UINT64_MAX is returned).
  uint64_t alloc_avoiding(uint64_t len, const std::vector<Range>& busy, int max_cost = INT32_MAX - 1) {
    int best_cost = INT32_MAX;
    uint64_t best_off = UINT64_MAX;
    auto consider = [&](const Range& hole, uint64_t off) {
      if (off < hole.off || off + len < off || off + len > hole.off + hole.len) return;
      int cost = -1;
      for (size_t k = 0; k < busy.size(); ++k)
        if (busy[k].off < off + len && off < busy[k].off + busy[k].len) cost = static_cast<int>(k);
      if (cost < best_cost || (cost == best_cost && off < best_off)) {
        best_cost = cost;
        best_off = off;
      }
    };
    for (const Range& hole : free_) {
      consider(hole, hole.off);
      for (const Range& b : busy) consider(hole, b.off + b.len);
    }
    if (best_off == UINT64_MAX || best_cost > max_cost) return UINT64_MAX;
    alloc_at(best_off, len);
    return best_off;
  }
  // Carves [off, off+len) out of the hole that contains it (caller guarantees it fits).
  void alloc_at(uint64_t off, uint64_t len) {
    for (size_t i = 0; i < free_.size(); ++i) {
      const Range hole = free_[i];
      if (off >= hole.off && off + len <= hole.off + hole.len) {
        free_.erase(free_.begin() + i);
        if (off + len < hole.off + hole.len)
          free_.insert(free_.begin() + i, {off + len, hole.off + hole.len - (off + len)});
        if (off > hole.off) free_.insert(free_.begin() + i, {hole.off, off - hole.off});
        return;
      }
    }
  }
  void release(uint64_t off, uint64_t len) {
    auto it = std::lower_bound(free_.begin(), free_.end(), off,
                               [](const Range& r, uint64_t o) { return r.off < o; });
    it = free_.insert(it, {off, len});
    if (it + 1 != free_.end() && it->off + it->len == (it + 1)->off) {
      it->len += (it + 1)->len;
      free_.erase(it + 1);
    }
    if (it != free_.begin() && (it - 1)->off + (it - 1)->len == it->off) {
      (it - 1)->len += it->len;
      free_.erase(it);
    }
  }
  uint64_t largest_hole() const {
    uint64_t m = 0;
    for (const Range& r : free_) m = std::max(m, r.len);
    return m;
  }

 private:
  std::vector<Range> free_;  // sorted by offset, never adjacent
};

}  // namespace ctn
