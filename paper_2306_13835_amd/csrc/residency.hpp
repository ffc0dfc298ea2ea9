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
class Residency {
 public:
  explicit Residency(uint64_t budget) : budget_(budget) {}

  int add_model(uint64_t bytes) {
    size_.push_back(bytes);
    stamp_.push_back(0);
    return static_cast<int>(size_.size()) - 1;
  }
  int n_models() const { return static_cast<int>(size_.size()); }
  bool resident(int m) const { return stamp_[m] != 0; }
  uint64_t size(int m) const { return size_[m]; }
  uint64_t budget() const { return budget_; }
  uint64_t resident_bytes() const { return resident_bytes_; }
  uint64_t peak_bytes() const { return peak_; }

  // A use of a resident model.
  void touch(int m) { stamp_[m] = ++clock_; }

  // The resident model used longest ago, other than `except`; -1 if none.
  int oldest(int except) const {
    int best = -1;
    uint64_t best_stamp = std::numeric_limits<uint64_t>::max();
    for (int i = 0; i < n_models(); ++i)
      if (i != except && stamp_[i] != 0 && stamp_[i] < best_stamp) {
        best_stamp = stamp_[i];
        best = i;
      }
    return best;
  }

  // True while model m (not resident) does not fit next to what is resident.
  bool over_budget_with(int m) const { return resident_bytes_ + size_[m] > budget_; }

  void mark_resident(int m) {
    stamp_[m] = ++clock_;
    resident_bytes_ += size_[m];
    peak_ = std::max(peak_, resident_bytes_);
  }
  void mark_evicted(int m) {
    stamp_[m] = 0;
    resident_bytes_ -= size_[m];
  }

 private:
  uint64_t budget_;
  uint64_t clock_ = 0, resident_bytes_ = 0, peak_ = 0;
  std::vector<uint64_t> size_, stamp_;
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
  // overlaps (-1: none).  Lowest cost wins, then lowest offset.
  uint64_t alloc_avoiding(uint64_t len, const std::vector<Range>& busy) {
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
    if (best_off == UINT64_MAX) return UINT64_MAX;
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
