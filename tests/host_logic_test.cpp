// CPU test of the host-only bookkeeping (no HIP): the arena range allocator against a
// brute-force byte map, and the residency policy's budget invariant.
#include <cassert>
#include <cstdio>
#include <algorithm>
#include <cstdlib>
#include <random>
#include <vector>

#include "engine.hpp"
#include "layout.hpp"
#include "residency.hpp"

using ctn::RangeAllocator;

static bool overlaps(uint64_t a, uint64_t al, uint64_t b, uint64_t bl) { return a < b + bl && b < a + al; }

int main() {
  std::mt19937_64 rng(12345);
  for (int round = 0; round < 300; ++round) {
    const uint64_t total = 64 + rng() % 200;
    RangeAllocator ra(total);
    std::vector<int> map(total, 0);   // 0 free, 1 allocated
    struct Blk { uint64_t off, len; };
    std::vector<Blk> live;
    std::vector<RangeAllocator::Range> busy;   // recently released, "still being offloaded"
    for (int step = 0; step < 200; ++step) {
      if (live.empty() || rng() % 3) {
        const uint64_t len = 1 + rng() % 40;
        // brute force: does any free placement exist, and one that avoids `busy`?
        bool any = false, clean = false;
        for (uint64_t o = 0; o + len <= total; ++o) {
          bool free_here = true;
          for (uint64_t k = o; k < o + len; ++k) free_here &= map[k] == 0;
          if (!free_here) continue;
          any = true;
          bool ok = true;
          for (auto& b : busy) ok &= !overlaps(o, len, b.off, b.len);
          clean |= ok;
        }
        {   // a placement that must not touch a busy range exists exactly when brute force finds one
          RangeAllocator probe = ra;
          const uint64_t o = probe.alloc_avoiding(len, busy, -1);
          assert((o != UINT64_MAX) == clean);
          if (o != UINT64_MAX)
            for (auto& b : busy) assert(!overlaps(o, len, b.off, b.len));
        }
        const bool used_avoiding = rng() % 2;
        const uint64_t off = used_avoiding ? ra.alloc_avoiding(len, busy) : (busy.clear(), ra.alloc(len));
        if (!any) { assert(off == UINT64_MAX); continue; }
        assert(off != UINT64_MAX && off + len <= total);
        for (uint64_t k = off; k < off + len; ++k) { assert(map[k] == 0); map[k] = 1; }
        if (clean && !busy.empty())
          for (auto& b : busy) assert(!overlaps(off, len, b.off, b.len));
        if (!clean && used_avoiding && !busy.empty()) {
          // no clean placement: the one chosen must wait on the earliest-finishing set possible
          auto cost = [&](uint64_t o) {
            int c = -1;
            for (size_t k = 0; k < busy.size(); ++k) if (overlaps(o, len, busy[k].off, busy[k].len)) c = (int)k;
            return c;
          };
          // brute force over every free placement that was available before this allocation
          int best = 1 << 30;
          for (uint64_t o = 0; o + len <= total; ++o) {
            bool free_here = true;
            for (uint64_t k = o; k < o + len; ++k) free_here &= (map[k] == 0) || (k >= off && k < off + len);
            if (free_here) best = std::min(best, cost(o));
          }
          assert(cost(off) == best);
        }
        live.push_back({off, len});
      } else {
        const size_t i = rng() % live.size();
        for (uint64_t k = live[i].off; k < live[i].off + live[i].len; ++k) map[k] = 0;
        ra.release(live[i].off, live[i].len);
        busy.push_back({live[i].off, live[i].len});
        if (busy.size() > 2) busy.erase(busy.begin());
        live.erase(live.begin() + i);
      }
    }
    for (auto& b : live) ra.release(b.off, b.len);
    assert(ra.largest_hole() == total);          // everything coalesced back into one hole
  }
  // residency, whole-model mode: budget never exceeded, victims leave completely, least recently used first
  {
    ctn::Residency r(100);
    for (int i = 0; i < 5; ++i) r.add_model(30 + i);
    std::vector<uint64_t> last(5, 0);
    uint64_t clock = 0;
    for (int step = 0; step < 1000; ++step) {
      const int m = rng() % 5;
      if (r.resident(m)) { r.touch(m); }
      else {
        std::vector<ctn::Residency::Move> moves;
        while (r.over_budget_with(m)) {
          int expect = -1;
          for (int i = 0; i < 5; ++i)
            if (i != m && r.resident(i) && (expect < 0 || last[i] < last[expect])) expect = i;
          const int v = r.evict_step(m, moves);
          assert(v >= 0 && v != m && v == expect && !r.resident(v) && r.resident_blocks(v) == 0);
        }
        r.load_missing(m);
      }
      last[m] = ++clock;
      assert(r.resident(m) && r.resident_bytes() <= 100 && r.peak_bytes() <= 100);
    }
  }
  // residency, block mode: prefixes only, one block per step from the tail of the oldest model,
  // never more evicted than the missing blocks need
  for (int round = 0; round < 200; ++round) {
    const int n = 2 + rng() % 4;
    std::vector<std::vector<uint64_t>> blocks(n);
    uint64_t biggest = 0, all = 0;
    for (auto& b : blocks) {
      const int nb = 1 + rng() % 5;
      uint64_t sum = 0;
      for (int i = 0; i < nb; ++i) { b.push_back(1 + rng() % 8); sum += b.back(); }
      biggest = std::max(biggest, sum);
      all += sum;
    }
    const uint64_t budget = biggest + rng() % (all - biggest + 2);
    ctn::Residency r(budget, true);
    for (auto& b : blocks) r.add_model(b);
    for (int step = 0; step < 100; ++step) {
      const int m = rng() % n;
      if (rng() % 10 == 0) {
        const auto mv = r.evict_all(m);
        assert(mv.b0 == 0 && r.resident_blocks(m) == 0);
        continue;
      }
      if (r.resident(m)) { r.touch(m); continue; }
      std::vector<ctn::Residency::Move> moves;
      uint64_t last_dropped = 0;
      while (r.over_budget_with(m)) {
        const int v = r.evict_step(m, moves);
        assert(v >= 0 && v != m);
        last_dropped = blocks[v][r.resident_blocks(v)];
      }
      for (size_t i = 0; i < moves.size(); ++i) {
        assert(moves[i].b0 < moves[i].b1 && r.resident_blocks(moves[i].model) == moves[i].b0);
        for (size_t j = 0; j < i; ++j) assert(moves[j].model != moves[i].model);
        if (i + 1 < moves.size()) assert(moves[i].b0 == 0);      // only the last victim keeps a prefix
      }
      const uint64_t need = r.missing_bytes(m);
      if (!moves.empty()) assert(r.resident_bytes() + need + last_dropped > budget);   // minimal
      const auto ld = r.load_missing(m);
      assert(ld.model == m && ld.b1 == (int)blocks[m].size() && r.resident(m));
      assert(r.resident_bytes() <= budget);
      uint64_t sum = 0;
      for (int i = 0; i < n; ++i)
        for (int b = 0; b < r.resident_blocks(i); ++b) sum += blocks[i][b];
      assert(sum == r.resident_bytes());
    }
  }
  // request queues: oldest head first (ties: lower model), FIFO per model, pop respects the cap
  {
    ctn::RequestQueues q(3);
    assert(q.pick() == -1 && q.pending() == 0);
    int64_t id = 0;
    const double ts[] = {5.0, 1.0, 1.5, 3.0, 0.5, 7.0};
    const int model[] = {0, 2, 1, 1, 2, 0};
    for (int i = 0; i < 6; ++i) q.push(model[i], ctn::QueuedRequest{id++, ts[i], {}});
    assert(q.pending() == 6);
    assert(q.pick() == 2);                        // head of queue 2 has timestamp 1.0 (0.5 is behind it)
    auto b = q.pop(2, 8);
    assert(b.size() == 2 && b[0].id == 1 && b[1].id == 4);
    assert(q.pick() == 1);
    b = q.pop(1, 1);
    assert(b.size() == 1 && b[0].id == 2);
    q.push_front(1, std::move(b[0]));             // a failed dispatch puts requests back in order
    b = q.pop(1, 8);
    assert(b.size() == 2 && b[0].id == 2 && b[1].id == 3);
    assert(q.pick() == 0 && q.pop(0, 1)[0].id == 0 && q.pop(0, 1)[0].id == 5 && q.pick() == -1);
    q.push(2, ctn::QueuedRequest{9, 4.0, {}});
    q.push(1, ctn::QueuedRequest{10, 4.0, {}});
    assert(q.pick() == 1);                        // equal timestamps: the lower model index wins
  }
  std::puts("host logic ok");
  {   // shard descriptions: what the kernels cannot run is refused at registration, not at the first inference
    ctn_model_desc d{};
    d.layers = 2; d.hidden = 16384; d.ffn = 65536; d.heads = 128; d.vocab = 1024; d.max_pos = 64; d.tp = 2; d.rank = 1;
    assert(ctn::desc_valid(d));                       // the widest row the LayerNorm kernels hold
    ctn_model_desc wide = d;
    wide.hidden = 9216; wide.heads = 72; wide.ffn = 36864;    // the 66B and 175B members of the OPT family fit
    assert(ctn::desc_valid(wide));
    wide.hidden = 12288; wide.heads = 96; wide.ffn = 49152;
    assert(ctn::desc_valid(wide));
    wide.hidden = 16384 + 128; wide.heads = 129;      // head size 128, divisible by everything, but too wide
    assert(!ctn::desc_valid(wide));
    ctn_model_desc odd = d;
    odd.hidden = 96 * 64; odd.heads = 64;             // head size 96
    assert(!ctn::desc_valid(odd));
    // every layer block fits one copy table whatever the shape
    const ctn::ShardLayout L = ctn::make_layout(d);
    for (int b = 1; b < L.n_blocks; ++b) assert((int)L.block_tensors[b].size() == ctn::kLayerTensors);
    assert((int)L.block_tensors[0].size() <= 5);
  }
  return 0;
}
