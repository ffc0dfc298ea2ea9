// Host-only request queues and batch selection of the serving engine (no HIP).
//
// Section 3.1 of the paper: a request is pushed with its timestamp into the
// queue of its model; the engine picks a queue, pops its oldest requests and
// packs them into one batch entry.  Section 4: batches are scheduled by the
// oldest timestamp.  Section 5.2: the maximum batch size is a parameter (8, 32).
#pragma once
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

}  // namespace ctn
