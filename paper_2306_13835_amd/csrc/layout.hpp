// Where the tensors of one rank's OPT shard sit inside its arena range.
//
// The parameter list (Section 3.1: a worker holds its shard of every model)
// arrives as separate host tensors in forward order: 16*L+4 for a rank that
// holds all layers.  A pipeline stage (Section 5.1 splits models by tensor and
// by pipeline parallelism) holds the layers [stage*L/pp, (stage+1)*L/pp); the
// embeddings only on stage 0, the final LayerNorm only on the last stage,
// followed there (pp > 1) by that stage's own copy of the tied head matrix.
// On the device the tensors are packed into transfer blocks that follow the
// forward pass, so a load can signal "block b has landed" (Section 3.2 loads
// whole models; the block split is this library's refinement):
//   block 0      : the tensors outside the layers, in list order (embed_tokens,
//                  embed_positions, final_ln.w, final_ln.b, lm_head; may be empty)
//   block 1 + l  : the 16 tensors of the stage's l-th decoder layer, in list order
// Every tensor starts on a 256-byte boundary.  Keeping list order means that a
// caller who stores a layer's tensors back to back on the host gets a device
// image with the same spacing, so neighbouring tensors can travel as one copy.
#pragma once
#include <algorithm>
#include <cstdint>
#include <vector>

#include "computron.h"

namespace ctn {

constexpr uint64_t kAlign = 256;
constexpr int kLayerTensors = 16;
constexpr int kPosOffset = 2;  // OPT keeps position rows shifted by two
constexpr int kMaxHidden = 16384;

inline uint64_t align_up(uint64_t x, uint64_t a = kAlign) { return (x + a - 1) / a * a; }

// Index of a tensor inside a layer's 16, in list order.
enum LayerTensor {
  LN1_W = 0, LN1_B, Q_W, Q_B, K_W, K_B, V_W, V_B, O_W, O_B, LN2_W, LN2_B, FC1_W, FC1_B, FC2_W, FC2_B
};

struct ShardLayout {
  ctn_model_desc d{};
  int n_tensors = 0;
  int n_blocks = 0;
  uint64_t param_bytes = 0;               // sum of tensor sizes (what the budget counts)
  uint64_t arena_bytes = 0;               // padded size of the arena range
  std::vector<uint64_t> offset;           // per tensor (list order): byte offset in the range
  std::vector<uint64_t> nbytes;           // per tensor
  std::vector<int> block_of;              // per tensor
  std::vector<std::vector<int>> block_tensors;  // per block: tensor indices in arena order
  std::vector<uint64_t> block_bytes;      // per block: parameter bytes
  std::vector<uint64_t> block_start;      // per block: offset of its first tensor in the range
  std::vector<uint64_t> block_span;       // per block: padded bytes from its start to the next block's
  uint64_t slot_bytes = 0;                // widest block span: the unit of block-by-block placement

  int pp() const { return d.pp > 1 ? d.pp : 1; }
  bool has_embed() const { return d.stage == 0; }
  bool has_head() const { return d.stage == pp() - 1; }
  int local_layers() const { return d.layers / pp(); }
  int n_front() const { return has_embed() ? 2 : 0; }
  int n_back() const { return has_head() ? (pp() > 1 ? 3 : 2) : 0; }
  // list indices of the tensors outside the layers (valid only where the stage holds them)
  int idx_tok() const { return 0; }
  int idx_pos() const { return 1; }
  int idx_final_w() const { return n_front() + kLayerTensors * local_layers(); }
  int idx_final_b() const { return idx_final_w() + 1; }
  int idx_head() const { return pp() > 1 ? idx_final_w() + 2 : idx_tok(); }
  // features one inference emits: a vocabulary slice of logits on the last stage, else the residual stream
  int out_features() const { return has_head() ? vl() : d.hidden; }
  int hl() const { return d.hidden / d.tp; }
  int fl() const { return d.ffn / d.tp; }
  int vl() const { return d.vocab / d.tp; }
  int local_heads() const { return d.heads / d.tp; }
  int head_dim() const { return d.hidden / d.heads; }
  int layer_tensor(int layer, int which) const { return n_front() + kLayerTensors * layer + which; }
  // Offset of tensor t from the start of its own block (blocks may be placed one by one).
  uint64_t offset_in_block(int t) const { return offset[t] - block_start[block_of[t]]; }
};

inline bool desc_valid(const ctn_model_desc& d) {
  if (d.layers < 0 || d.hidden <= 0 || d.ffn <= 0 || d.heads <= 0 || d.vocab <= 0 || d.max_pos < 1 ||
      d.tp < 1 || d.rank < 0 || d.rank >= d.tp)
    return false;
  if (d.hidden % d.heads || d.heads % d.tp || d.ffn % d.tp || d.vocab % d.tp) return false;
  const int pp = d.pp > 1 ? d.pp : 1;           // 0 and 1 both mean: no pipeline split
  if (d.pp < 0 || d.layers % pp || d.stage < 0 || d.stage >= pp) return false;
  int hd = d.hidden / d.heads;
  if (hd != 64 && hd != 128) return false;
  if ((d.hidden / d.tp) % 8 || (d.ffn / d.tp) % 8 || d.hidden % 8) return false;
  if (d.hidden > kMaxHidden) return false;      // widest row the LayerNorm kernels hold in registers
  return true;
}

// Expected shape of tensor i of the list ({rows, cols}; cols == 0 for vectors).
inline void expected_shape(const ctn_model_desc& d, int i, int64_t& rows, int64_t& cols) {
  const int64_t h = d.hidden, hl = d.hidden / d.tp, fl = d.ffn / d.tp;
  const int pp = d.pp > 1 ? d.pp : 1;
  const int n_front = d.stage == 0 ? 2 : 0;
  const int n_layer = kLayerTensors * (d.layers / pp);
  if (i < n_front) {
    rows = i == 0 ? d.vocab / d.tp : d.max_pos + kPosOffset;
    cols = h;
    return;
  }
  if (i >= n_front + n_layer) {        // final_ln.w, final_ln.b, then the last stage's head matrix
    const int j = i - n_front - n_layer;
    rows = j < 2 ? h : d.vocab / d.tp;
    cols = j < 2 ? 0 : h;
    return;
  }
  switch ((i - n_front) % kLayerTensors) {
    case Q_W: case K_W: case V_W: rows = hl; cols = h; return;
    case Q_B: case K_B: case V_B: rows = hl; cols = 0; return;
    case O_W: rows = h; cols = hl; return;
    case FC1_W: rows = fl; cols = h; return;
    case FC1_B: rows = fl; cols = 0; return;
    case FC2_W: rows = h; cols = fl; return;
    default: rows = h; cols = 0; return;  // LayerNorm vectors, o.b, fc2.b
  }
}

inline ShardLayout make_layout(const ctn_model_desc& d) {
  ShardLayout L;
  L.d = d;
  L.n_tensors = L.n_front() + kLayerTensors * L.local_layers() + L.n_back();
  L.n_blocks = L.local_layers() + 1;
  L.offset.assign(L.n_tensors, 0);
  L.nbytes.assign(L.n_tensors, 0);
  L.block_of.assign(L.n_tensors, 0);
  L.block_tensors.assign(L.n_blocks, {});
  L.block_bytes.assign(L.n_blocks, 0);
  L.block_start.assign(L.n_blocks, 0);
  L.block_span.assign(L.n_blocks, 0);
  for (int i = 0; i < L.n_tensors; ++i) {
    int64_t r, c;
    expected_shape(d, i, r, c);
    L.nbytes[i] = 2ull * static_cast<uint64_t>(r) * static_cast<uint64_t>(c ? c : 1);
    L.param_bytes += L.nbytes[i];
  }
  uint64_t cur = 0;
  auto place = [&](int block, int t) {
    cur = align_up(cur);
    if (L.block_tensors[block].empty()) L.block_start[block] = cur;
    L.offset[t] = cur;
    cur += L.nbytes[t];
    L.block_of[t] = block;
    L.block_tensors[block].push_back(t);
    L.block_bytes[block] += L.nbytes[t];
  };
  for (int t = 0; t < L.n_front(); ++t) place(0, t);
  for (int t = 0; t < L.n_back(); ++t) place(0, L.idx_final_w() + t);
  if (L.block_tensors[0].empty()) L.block_start[0] = 0;
  for (int l = 0; l < L.local_layers(); ++l)
    for (int w = 0; w < kLayerTensors; ++w) place(1 + l, L.layer_tensor(l, w));
  L.arena_bytes = align_up(cur);
  for (int b = 0; b < L.n_blocks; ++b) {
    const uint64_t end = b + 1 < L.n_blocks ? L.block_start[b + 1] : L.arena_bytes;
    L.block_span[b] = end - L.block_start[b];
    L.slot_bytes = std::max(L.slot_bytes, L.block_span[b]);
  }
  return L;
}

}  // namespace ctn
