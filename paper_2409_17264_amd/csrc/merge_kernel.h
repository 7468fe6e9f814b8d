// Log-sum-exp merge of partial attention results over disjoint key sets
// (paper section 3.3: KV shards' partial outputs are combined with the
// online-softmax identity).  Bandwidth-bound and tiny next to attention.
#pragma once

#include "common.h"

namespace medha {

// Running state of a merge: reference point `big` (largest LSE seen), sum of weights and
// weighted sum of the partial outputs, both relative to `big`.
struct MergeState {
  float big = -INFINITY;
  float wsum = 0.f;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
};

// Folds partials s_first, s_first + s_step, ... < n_split of one (row, head) into `st`, for the
// 4 head-dim elements d4*4 .. +3.  Partial s of the row sits at row index base + s * stride
// of the partial arrays.  The partials are taken kBatch at a time with all loads of a batch in
// flight together (the merge is a chain of memory latencies, nothing else), and batches are
// folded with the same online rescaling the attention kernels use.
__device__ __forceinline__ void fold_partials(const float* __restrict__ part_o,
                                              const float* __restrict__ part_lse, int n_split,
                                              int s_first, int s_step, int64_t base,
                                              int64_t stride, int h_q, int head, int d, int d4,
                                              MergeState& st) {
  constexpr int kBatch = 8;
  for (int s0 = s_first; s0 < n_split; s0 += kBatch * s_step) {
    float ls[kBatch];
    f32x4 ov[kBatch];
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      // past the end: the last partial again, with weight 0
      const int64_t r = (base + min(s0 + i * s_step, n_split - 1) * stride) * h_q + head;
      ls[i] = part_lse[r];
      ov[i] = *reinterpret_cast<const f32x4*>(part_o + r * d + d4 * 4);
    }
    float top = st.big;
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      if (s0 + i * s_step >= n_split) ls[i] = -INFINITY;
      top = fmaxf(top, ls[i]);
    }
    if (top == -INFINITY) continue;  // nothing but empty shards so far
    const float keep = fast_exp2((st.big - top) * kLog2e);  // 0 while big is -inf
    st.wsum *= keep;
    st.acc *= keep;
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const float w = fast_exp2((ls[i] - top) * kLog2e);
      if (w > 0.f) {  // an empty shard's O is never read into the sum
        st.wsum += w;
        st.acc += ov[i] * w;
      }
    }
    st.big = top;
  }
}

__device__ __forceinline__ void finish_merge(const MergeState& st, int d4,
                                             float* __restrict__ out_row,
                                             float* __restrict__ lse_out) {
  const float inv = st.wsum > 0.f ? 1.f / st.wsum : 0.f;
  *reinterpret_cast<f32x4*>(out_row + d4 * 4) = st.acc * inv;
  if (d4 == 0) *lse_out = st.wsum > 0.f ? st.big + fast_log2(st.wsum) * kLn2 : -INFINITY;
}

// One thread owns 4 consecutive head-dim elements of one (row, head) and all its partials.
__device__ __forceinline__ void merge_one(const float* __restrict__ part_o,
                                          const float* __restrict__ part_lse, int n_split,
                                          int64_t base, int64_t stride, int h_q, int head, int d,
                                          int d4, float* __restrict__ out_row,
                                          float* __restrict__ lse_out) {
  MergeState st;
  fold_partials(part_o, part_lse, n_split, 0, 1, base, stride, h_q, head, d, d4, st);
  finish_merge(st, d4, out_row, lse_out);
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
  const SeqDesc* descs = args.inline_descs;
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

// The same merge for launches with many KV ranges per row (small chunks against a long
// cache are split hundreds of ways): one workgroup per (row, head); its 256 threads are
// D/4 column groups x 256/(D/4) lanes, lane l folds ranges l, l + lanes, ..., and the
// lanes' states are combined through LDS.  The chain of dependent memory latencies is
// `lanes` times shorter than with one thread per column group.
template <int D>
__global__ void __launch_bounds__(kThreads) split_merge_wide_kernel(const MergeArgs args) {
  constexpr int per_row = D / 4;
  constexpr int lanes = kThreads / per_row;
  __shared__ f32x4 sm_acc[lanes][per_row];
  __shared__ float sm_big[lanes], sm_wsum[lanes];
  const SeqDesc* descs = args.inline_descs;
  const int head = blockIdx.x % args.h_q;
  const int row = blockIdx.x / args.h_q;  // rank of the token row among the launch's rows
  int lo = 0, hi = args.n_seq - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (descs[mid].row_rank <= row) lo = mid; else hi = mid - 1;
  }
  const SeqDesc sd = descs[lo];
  if (sd.n_split == 1) return;  // the whole workgroup: written directly by the attention kernel
  const int j = row - sd.row_rank;
  const int d4 = threadIdx.x % per_row;
  const int lane = threadIdx.x / per_row;
  MergeState st;
  fold_partials(args.part_o, args.part_lse, sd.n_split, lane, lanes, (int64_t)sd.part_row + j,
                sd.chunk_len, args.h_q, head, D, d4, st);
  sm_acc[lane][d4] = st.acc;
  if (d4 == 0) {
    sm_big[lane] = st.big;
    sm_wsum[lane] = st.wsum;
  }
  __syncthreads();
  if (lane != 0) return;
  MergeState all;
#pragma unroll
  for (int l = 0; l < lanes; ++l) all.big = fmaxf(all.big, sm_big[l]);
  if (all.big != -INFINITY) {
#pragma unroll
    for (int l = 0; l < lanes; ++l) {
      const float w = fast_exp2((sm_big[l] - all.big) * kLog2e);  // 0 for a lane that saw nothing
      if (sm_wsum[l] > 0.f) {
        all.wsum += w * sm_wsum[l];
        all.acc += sm_acc[l][d4] * w;
      }
    }
  }
  const int64_t orow = ((int64_t)sd.out_row + j) * args.h_q + head;
  finish_merge(all, d4, args.out + orow * D, args.lse + orow);
}

}  // namespace medha
