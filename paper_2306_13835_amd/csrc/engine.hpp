// Host-only request queues and batch selection of the serving engine (no HIP).
//
// Section 3.1 of the paper: a request is pushed with its timestamp into the
// queue of its model; the engine picks a queue, pops its oldest requests and
// packs them into one batch entry.  Section 4: batches are scheduled by the
// oldest timestamp.  Section 5.2: the maximum batch size is a parameter (8, 32).
#pragma once
#include <algorithm>
#include <cstdint>
#include <deque>
#include <vector>

namespace ctn {

struct QueuedRequest {
  int64_t id;
  double timestamp;
  std::vector<int32_t> ids;   // token ids of the request (empty in simulations)
};

class RequestQueues {
 public:
  explicit RequestQueues(int n_models = 0) : q_(n_models) {}
  void ensure(int n_models) {
    if (static_cast<int>(q_.size()) < n_models) q_.resize(n_models);
  }
  void push(int model, QueuedRequest r) { q_[model].push_back(std::move(r)); }
  void push_front(int model, QueuedRequest r) { q_[model].push_front(std::move(r)); }
  int64_t pending() const {
    int64_t n = 0;
    for (const auto& d : q_) n += static_cast<int64_t>(d.size());
    return n;
  }
  // The model whose oldest waiting request is oldest (ties: lower index); -1 when all queues are empty.
  int pick() const {
    int best = -1;
    for (int m = 0; m < static_cast<int>(q_.size()); ++m)
      if (!q_[m].empty() && (best < 0 || q_[m].front().timestamp < q_[best].front().timestamp)) best = m;
    return best;
  }
  // Models with waiting requests, the one whose oldest request is oldest first (ties: lower index).
  std::vector<int> by_oldest_head() const {
    std::vector<int> order;
    for (int m = 0; m < static_cast<int>(q_.size()); ++m)
      if (!q_[m].empty()) order.push_back(m);
    std::stable_sort(order.begin(), order.end(),
                     [&](int a, int b) { return q_[a].front().timestamp < q_[b].front().timestamp; });
    return order;
  }
  // Pops up to max_batch oldest requests of that model.
  std::vector<QueuedRequest> pop(int model, int max_batch) {
    std::vector<QueuedRequest> out;
    auto& d = q_[model];
    while (!d.empty() && static_cast<int>(out.size()) < max_batch) {
      out.push_back(std::move(d.front()));
      d.pop_front();
    }
    return out;
  }

 private:
  std::vector<std::deque<QueuedRequest>> q_;
};

// Dispatch rule of the two-lane engine (Section 3.2: load entries are
// asynchronous, so a later batch entry proceeds without waiting for a load
// entry of another model).  Lane 0 runs batches of completely loaded models,
// lane 1 one miss at a time (the model's swap-in followed by its batch); a
// model whose miss is in flight is not dispatched again until that batch is
// done.  The queues are scanned oldest head first and the first one that can
// go (its lane is free, its model is not loading) does.  Returns the model and
// sets *lane, or -1 when nothing can be dispatched now.
constexpr int kHitLane = 0, kLoadLane = 1;
template <class IsResident, class IsLoading>
int pick_two_lane(const RequestQueues& q, IsResident is_resident, IsLoading is_loading, const bool lane_free[2],
                  int* lane) {
  for (int m : q.by_oldest_head()) {
    if (is_loading(m)) continue;
    const int l = is_resident(m) ? kHitLane : kLoadLane;
    if (!lane_free[l]) continue;
    *lane = l;
    return m;
  }
  return -1;
}

// Which model to load ahead of its next request.  The paper's closing section
// proposes speculative loading for request streams with structure (a model
// requested repeatedly, models requested in a fixed order); this is a
// first-order transition table over the dispatches: after a dispatch of model
// a the prediction is the model that most often followed a (ties: lowest
// index) if it was seen at least min_count times and makes up at least
// min_share_percent per cent of the transitions out of a; -1 otherwise.
class TransitionPredictor {
 public:
  void configure(int min_count, int min_share_percent) {
    min_count_ = min_count;
    min_share_percent_ = min_share_percent;
  }
  void observe(int m) {
    const int n = static_cast<int>(count_.size());
    if (m >= n) {
      for (auto& row : count_) row.resize(m + 1, 0);
      count_.resize(m + 1, std::vector<int64_t>(m + 1, 0));
    }
    if (last_ >= 0) count_[last_][m] += 1;
    last_ = m;
  }
  int predict() const {
    if (last_ < 0) return -1;
    const std::vector<int64_t>& row = count_[last_];
    int best = 0;
    int64_t total = 0;
    for (int b = 0; b < static_cast<int>(row.size()); ++b) {
      total += row[b];
      if (row[b] > row[best]) best = b;
    }
    if (row[best] == 0 || row[best] < min_count_) return -1;
    if (100 * row[best] < static_cast<int64_t>(min_share_percent_) * total) return -1;
    return best;
  }

 private:
  std::vector<std::vector<int64_t>> count_;
  int last_ = -1;
  int min_count_ = 2, min_share_percent_ = 50;
};

}  // namespace ctn
