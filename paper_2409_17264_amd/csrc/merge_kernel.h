// Log-sum-exp merge of partial attention results over disjoint key sets
// (paper section 3.3: KV shards' partial outputs are combined with the
// online-softmax identity).  Bandwidth-bound and tiny next to attention.
#pragma once

#include "common.h"

namespace medha {

// One thread owns 4 consecutive head-dim elements of one (row, head).  Partial
// s of that row sits at row index  base + s * stride  of the partial arrays.
// The partials are taken kBatch at a time with all loads of a batch in flight
// together (the merge is a chain of memory latencies, nothing else), and batches
// are folded with the same online rescaling the attention kernels use.
__device__ __forceinline__ void merge_one(const float* __restrict__ part_o,
                                          const float* __restrict__ part_lse, int n_split,
                                          int64_t base, int64_t stride, int h_q, int head, int d,
                                          int d4, float* __restrict__ out_row,
                                          float* __restrict__ lse_out) {
  constexpr int kBatch = 8;
  float big = -INFINITY, wsum = 0.f;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int s0 = 0; s0 < n_split; s0 += kBatch) {
    float ls[kBatch];
    f32x4 ov[kBatch];
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      // past the end: the last partial again, with weight 0
      const int64_t r = (base + min(s0 + i, n_split - 1) * stride) * h_q + head;
      ls[i] = part_lse[r];
      ov[i] = *reinterpret_cast<const f32x4*>(part_o + r * d + d4 * 4);
    }
    float top = big;
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      if (s0 + i >= n_split) ls[i] = -INFINITY;
      top = fmaxf(top, ls[i]);
    }
    if (top == -INFINITY) continue;  // nothing but empty shards so far
    const float keep = fast_exp2((big - top) * kLog2e);  // 0 while big is -inf
    wsum *= keep;
    acc *= keep;
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const float w = fast_exp2((ls[i] - top) * kLog2e);
      if (w > 0.f) {  // an empty shard's O is never read into the sum
        wsum += w;
        acc += ov[i] * w;
      }
    }
    big = top;
  }
  const float inv = wsum > 0.f ? 1.f / wsum : 0.f;
  *reinterpret_cast<f32x4*>(out_row + d4 * 4) = acc * inv;
  if (d4 == 0) *lse_out = wsum > 0.f ? big + fast_log2(wsum) * kLn2 : -INFINITY;
}

// Public merge: uniform split count, partials [n_split][rows][h_q][d].
__global__ void __launch_bounds__(kThreads) lse_merge_kernel(
    const float* __restrict__ part_o, const float* __restrict__ part_lse, int n_split,
    int64_t rows, int h_q, int d, float* __restrict__ out, float* __restrict__ lse) {
  const int per_row = d / 4;
  const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  const int64_t total = rows * h_q * per_row;
  if (idx >= total) return;
  const int d4 = (int)(idx % per_row);
  const int64_t rh = idx / per_row;
  const int head = (int)(rh % h_q);
  const int64_t row = rh / h_q;
  merge_one(part_o, part_lse, n_split, row, rows, h_q, head, d, d4, out + rh * d, lse + rh);
}

// Merge of the library's own split-KV partials, laid out per sequence:
// partial s of token j of a sequence is row  part_row + s * chunk_len + j.
// Sequences that were not split wrote their result directly and are skipped.
template <int D>
__global__ void __launch_bounds__(kThreads) split_merge_kernel(const MergeArgs args) {
  constexpr int per_row = D / 4;
  const SeqDesc* descs = args.descs ? args.descs : args.inline_descs;
  const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  const int64_t total = (int64_t)args.total_rows * args.h_q * per_row;
  if (idx >= total) return;
  const int d4 = (int)(idx % per_row);
  const int64_t rh = idx / per_row;
  const int head = (int)(rh % args.h_q);
  const int row = (int)(rh / args.h_q);  // rank of the token row among the launch's rows
  // sequences are in launch order; find the one that holds this row
  int lo = 0, hi = args.n_seq - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (descs[mid].row_rank <= row) lo = mid; else hi = mid - 1;
  }
  const SeqDesc sd = descs[lo];
  if (sd.n_split == 1) return;
  const int j = row - sd.row_rank;
  const int64_t orow = ((int64_t)sd.out_row + j) * args.h_q + head;
  merge_one(args.part_o, args.part_lse, sd.n_split, (int64_t)sd.part_row + j, sd.chunk_len,
            args.h_q, head, D, d4, args.out + orow * D, args.lse + orow);
}

}  // namespace medha
