// KV-cache append for gfx950: the keys and values of a chunk's tokens are written
// into the paged pools through the page table (paper section 3.1: every chunk's K/V
// joins the cache that all later chunks and decode steps read).  A pure scatter of
// 16-byte words, bound by HBM and bit-exact by construction.
#pragma once

#include "common.h"

namespace medha {

struct AppendDesc {
  int64_t pt_off;      // first entry of the sequence in the page table
  int32_t src_row;     // first token row of the sequence in k_new / v_new
  int32_t prefix_len;  // tokens already in the cache: token j goes to position prefix_len + j
  int32_t chunk_len;
  int32_t row_rank;    // rank of the sequence's first token row among the launch's rows
};
static_assert(sizeof(AppendDesc) == 24, "AppendDesc layout");

struct AppendArgs {
  const uint4* k_new;
  const uint4* v_new;
  uint4* k_pool;
  uint4* v_pool;
  const int32_t* page_table;
  int32_t n_seq;
  int32_t h_kv;
  int32_t words_per_row;  // 16-byte words per (token, head): head_dim / 8
  int32_t num_pages;
  int32_t total_rows;     // token rows of the launch
  int32_t reserved;
  AppendDesc descs[kMaxInlineSeq];
};
static_assert(sizeof(AppendArgs) <= 4096, "kernel argument block too large");

// One thread per 16-byte word of one (token, kv head), for K and for V.  A page id
// outside [0, num_pages) is skipped: nothing outside the pools is ever written.
__global__ void __launch_bounds__(kThreads) kv_append_kernel(const AppendArgs args) {
  const int per_token = args.h_kv * args.words_per_row;
  const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= (int64_t)args.total_rows * per_token) return;
  const int row = (int)(idx / per_token);
  const int rem = (int)(idx % per_token);
  const int head = rem / args.words_per_row;
  const int word = rem % args.words_per_row;
  int lo = 0, hi = args.n_seq - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (args.descs[mid].row_rank <= row) lo = mid; else hi = mid - 1;
  }
  const AppendDesc sd = args.descs[lo];
  const int j = row - sd.row_rank;
  const int t = sd.prefix_len + j;
  const int page = args.page_table[sd.pt_off + (t >> 4)];
  if ((unsigned)page >= (unsigned)args.num_pages) return;
  const int64_t src = ((int64_t)(sd.src_row + j) * args.h_kv + head) * args.words_per_row + word;
  const int64_t dst =
      (((int64_t)page * args.h_kv + head) * kPageSize + (t & 15)) * args.words_per_row + word;
  args.k_pool[dst] = args.k_new[src];
  args.v_pool[dst] = args.v_new[src];
}

}  // namespace medha
