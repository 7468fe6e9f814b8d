// Host-side launch planner: turns per-sequence lengths into workgroup slots.
// Pure host code (no HIP calls) so it can be tested without a GPU.
#pragma once

#include <algorithm>
#include <cstdint>
#include <vector>

#include "common.h"

namespace medha {

// Geometry of one kernel instantiation.
struct ModeShape {
  int rows_per_wg;  // query rows a workgroup owns
  int tile_keys;    // keys staged per loop iteration (the KV split granule)
};

struct LaunchPlan {
  std::vector<SeqDesc> descs;
  std::vector<int32_t> seq_index;  // position of each descriptor in the caller's batch
  ModeShape shape{0, 0};
  int q_blocks = 1;   // 32-row blocks per wavefront (row-split mode)
  int n_slots = 0;    // grid size
  int total_rows = 0; // token rows of the launch
  bool any_split = false;
};

struct Plan {
  LaunchPlan rows;  // row-split mode: sequences with more than 32 (token, head-in-group) rows
  LaunchPlan keys;  // key-split mode: decodes and other tiny chunks
  int64_t part_rows = 0;  // token rows of split-KV partials (both launches)
  // workspace layout (byte offsets, 256-aligned)
  size_t off_part_o = 0, off_part_lse = 0, bytes = 0;
};

struct SeqInput {
  int64_t pt_off;
  int32_t q_row, out_row, chunk_len, prefix_len;
  int32_t kv_len = -1;  // keys in the page-table slice; -1: prefix_len + chunk_len
};

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Splits the KV axis of each sequence so that the launch has about
// `target_wgs` equally long workgroups; never splits below `min_tiles` KV tiles.
inline void plan_launch(LaunchPlan& lp, int h_kv, int gqa, int target_wgs, int min_tiles,
                        int64_t& part_rows) {
  const ModeShape sh = lp.shape;
  int64_t unsplit_wgs = 0, total_steps = 0;
  for (SeqDesc& sd : lp.descs) {
    sd.n_row_tiles = (int)ceil_div((int64_t)sd.chunk_len * gqa, sh.rows_per_wg);
    const int64_t kv_tiles = ceil_div((int64_t)sd.kv_len, sh.tile_keys);
    unsplit_wgs += (int64_t)h_kv * sd.n_row_tiles;
    total_steps += (int64_t)h_kv * sd.n_row_tiles * kv_tiles;
  }
  const int64_t steps_target = std::max<int64_t>(1, ceil_div(total_steps, target_wgs));
  for (SeqDesc& sd : lp.descs) {
    const int64_t kv_tiles = std::max<int64_t>(1, ceil_div((int64_t)sd.kv_len, sh.tile_keys));
    int64_t n_split = 1;
    if (unsplit_wgs < target_wgs) {
      n_split = ceil_div(kv_tiles, steps_target);
      n_split = std::min(n_split, std::max<int64_t>(1, kv_tiles / min_tiles));
      n_split = std::max<int64_t>(1, n_split);
    }
    const int64_t tps = ceil_div(kv_tiles, n_split);
    n_split = ceil_div(kv_tiles, tps);
    sd.n_split = (int)n_split;
    sd.tiles_per_split = (int)tps;
  }
  // Longest workgroups first: the hardware hands workgroups out in slot order, so the short
  // ones fill the launch's tail instead of a long one starting last (the order of the
  // sequences inside a launch is free: every descriptor carries its own rows).
  {
    std::vector<int> order(lp.descs.size());
    for (size_t i = 0; i < order.size(); ++i) order[i] = (int)i;
    auto walk = [&](int i) {
      const SeqDesc& sd = lp.descs[i];
      return std::min<int64_t>(sd.tiles_per_split, ceil_div((int64_t)sd.kv_len, sh.tile_keys));
    };
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return walk(a) > walk(b); });
    std::vector<SeqDesc> descs(order.size());
    std::vector<int32_t> index(order.size());
    for (size_t i = 0; i < order.size(); ++i) {
      descs[i] = lp.descs[order[i]];
      index[i] = lp.seq_index[order[i]];
    }
    lp.descs.swap(descs);
    lp.seq_index.swap(index);
  }
  int slot = 0, rank = 0;
  for (SeqDesc& sd : lp.descs) {
    sd.work_start = slot;
    sd.row_rank = rank;
    sd.part_row = 0;
    if (sd.n_split > 1) {
      sd.part_row = (int32_t)part_rows;
      part_rows += (int64_t)sd.n_split * sd.chunk_len;
      lp.any_split = true;
    }
    const int64_t items = (int64_t)h_kv * sd.n_split * sd.n_row_tiles;
    slot += (int)(kXcds * ceil_div(items, kXcds));
    rank += sd.chunk_len;
  }
  lp.n_slots = slot;
  lp.total_rows = rank;
}

inline Plan make_plan(const SeqInput* seqs, int batch, int h_q, int h_kv, int head_dim,
                      int num_cus) {
  Plan plan;
  const int gqa = h_q / h_kv;
  int max_rows = 0;
  for (int b = 0; b < batch; ++b) {
    SeqDesc sd{};
    sd.pt_off = seqs[b].pt_off;
    sd.q_row = seqs[b].q_row;
    sd.out_row = seqs[b].out_row;
    sd.chunk_len = seqs[b].chunk_len;
    sd.prefix_len = seqs[b].prefix_len;
    sd.kv_len = seqs[b].kv_len >= 0 ? seqs[b].kv_len : sd.prefix_len + sd.chunk_len;
    const int64_t n_rows = (int64_t)sd.chunk_len * gqa;
    LaunchPlan& lp = n_rows <= 32 ? plan.keys : plan.rows;
    lp.descs.push_back(sd);
    lp.seq_index.push_back(b);
    if (n_rows > 32) max_rows = std::max(max_rows, (int)std::min<int64_t>(n_rows, 1 << 30));
  }
  // Row-split mode: 4 wavefronts x (32 * q_blocks) rows, 64-key tiles.
  plan.rows.q_blocks = max_rows >= 256 ? 2 : 1;
  plan.rows.shape = ModeShape{kWaves * 32 * plan.rows.q_blocks, 64};
  // Key-split mode: one 32-row block, 128-key tiles (32 per wavefront).
  plan.keys.q_blocks = 1;
  plan.keys.shape = ModeShape{32, 32 * kWaves};
  if (!plan.rows.descs.empty())
    plan_launch(plan.rows, h_kv, gqa, num_cus, 4, plan.part_rows);
  if (!plan.keys.descs.empty())
    plan_launch(plan.keys, h_kv, gqa, num_cus * 8, 4, plan.part_rows);

  size_t off = 0;
  plan.off_part_o = off;
  off = align256(off + (size_t)plan.part_rows * h_q * head_dim * sizeof(float));
  plan.off_part_lse = off;
  off = align256(off + (size_t)plan.part_rows * h_q * sizeof(float));
  plan.bytes = std::max<size_t>(off, 256);
  return plan;
}

}  // namespace medha
