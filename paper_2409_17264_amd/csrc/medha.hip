// C ABI of the gfx950 paged-attention library: argument validation, launch
// planning and kernel launches.  See include/medha.h for the contract.
#include "medha.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>

#include "append_kernel.h"
#include "common.h"
#include "decode_kernel.h"
#include "merge_kernel.h"
#include "planner.h"
#include "policy.h"
#include "prefill_kernel.h"

// Scratch of medha_chunked_prefill_attn_noalloc: split-KV partials of one call.  Every GPU
// the library runs on holds its own copy, at its own address, until the process ends.  In
// host code this name is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[MEDHA_NOALLOC_SCRATCH_BYTES];

namespace medha {
namespace {

// Device address of `scratch` on the current device, looked up once per device.
constexpr int kMaxDevices = 64;
void* noalloc_scratch_ptr(int* rc) {
  static std::mutex mu;
  static void* ptr[kMaxDevices] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    *rc = MEDHA_ERR_HIP;
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(mu);
  if (ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      *rc = MEDHA_ERR_HIP;
      return nullptr;
    }
    ptr[dev] = p;
  }
  *rc = MEDHA_OK;
  return ptr[dev];
}

int current_num_cus() {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
      cus <= 0) {
    (void)hipGetLastError();
    return 256;  // MI355X; used only for planning queries made without a device
  }
  return cus;
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

int check_heads(int h_q, int h_kv, int d, int page_size) {
  if (h_q <= 0 || h_kv <= 0 || h_q % h_kv != 0) return MEDHA_ERR_INVALID_ARG;
  if (page_size != kPageSize || (d != 64 && d != 128)) return MEDHA_ERR_UNSUPPORTED;
  return MEDHA_OK;
}

template <int D, int STAGES>
hipError_t launch_decode(const AttnArgs& a, int grid, hipStream_t stream) {
  hipLaunchKernelGGL((decode_kernel<D, STAGES>), dim3(grid), dim3(kThreads), 0, stream, a);
  return hipGetLastError();
}

template <int D, int NW>
hipError_t launch_prefill(const AttnArgs& a, int grid, hipStream_t stream) {
  hipLaunchKernelGGL((prefill_kernel<D, NW, kPrefillStages>), dim3(grid), dim3(NW * 64), 0,
                     stream, a);
  return hipGetLastError();
}

// Launches one mode's sequences, at most kMaxInlineSeq per kernel launch: the descriptors of
// a group travel in the kernel arguments with their workgroup slots and row ranks counted
// from the group's first sequence, followed by the merge of that group's split-KV partials.
hipError_t launch_plan(const LaunchPlan& lp, bool split_keys, int d, AttnArgs& a,
                       hipStream_t stream) {
  if (lp.descs.empty() || lp.n_slots == 0) return hipSuccess;
  const int n_all = (int)lp.descs.size();
  for (int g0 = 0; g0 < n_all; g0 += kMaxInlineSeq) {
    const int n = std::min(kMaxInlineSeq, n_all - g0);
    const int slot0 = lp.descs[g0].work_start, rank0 = lp.descs[g0].row_rank;
    const int slot1 = g0 + n < n_all ? lp.descs[g0 + n].work_start : lp.n_slots;
    const int rank1 = g0 + n < n_all ? lp.descs[g0 + n].row_rank : lp.total_rows;
    a.n_seq = n;
    int max_split = 1;
    for (int i = 0; i < n; ++i) {
      SeqDesc& sd = a.inline_descs[i];
      sd = lp.descs[g0 + i];
      sd.work_start -= slot0;
      sd.row_rank -= rank0;
      max_split = std::max(max_split, sd.n_split);
    }
    const int grid = slot1 - slot0;
    if (grid <= 0) continue;
    hipError_t e;
    if (split_keys) {
      // short walks: the small ring, two workgroups per compute unit (see decode_kernel)
      int64_t steps = 0;
      for (int i = 0; i < n; ++i)
        steps = std::max<int64_t>(steps, std::min<int64_t>(
            a.inline_descs[i].tiles_per_split,
            ceil_div(a.inline_descs[i].kv_len, lp.shape.tile_keys)));
      if (steps <= kShortWalkTiles)
        e = d == 128 ? launch_decode<128, 1>(a, grid, stream) : launch_decode<64, 1>(a, grid, stream);
      else
        e = d == 128 ? launch_decode<128, 2>(a, grid, stream) : launch_decode<64, 2>(a, grid, stream);
    } else if (lp.q_blocks == 2) {
      e = d == 128 ? launch_prefill<128, 8>(a, grid, stream)
                   : launch_prefill<64, 8>(a, grid, stream);
    } else {
      e = d == 128 ? launch_prefill<128, 4>(a, grid, stream)
                   : launch_prefill<64, 4>(a, grid, stream);
    }
    if (e != hipSuccess) return e;
    if (max_split == 1) continue;

    MergeArgs m{};
    m.part_o = a.part_o;
    m.part_lse = a.part_lse;
    m.out = a.out;
    m.lse = a.lse;
    m.n_seq = n;
    m.h_q = a.h_q;
    m.total_rows = rank1 - rank0;
    std::memcpy(m.inline_descs, a.inline_descs, n * sizeof(SeqDesc));
    if (max_split > kWideMergeSplits) {
      // many KV ranges per row: one workgroup per (row, head), ranges spread over its lanes
      const int64_t blocks = (int64_t)m.total_rows * a.h_q;
      if (d == 128)
        hipLaunchKernelGGL(split_merge_wide_kernel<128>, dim3((unsigned)blocks), dim3(kThreads),
                           0, stream, m);
      else
        hipLaunchKernelGGL(split_merge_wide_kernel<64>, dim3((unsigned)blocks), dim3(kThreads),
                           0, stream, m);
    } else {
      const int64_t threads = (int64_t)m.total_rows * a.h_q * (d / 4);
      const int grid_m = (int)ceil_div(threads, kThreads);
      if (d == 128)
        hipLaunchKernelGGL(split_merge_kernel<128>, dim3(grid_m), dim3(kThreads), 0, stream, m);
      else
        hipLaunchKernelGGL(split_merge_kernel<64>, dim3(grid_m), dim3(kThreads), 0, stream, m);
    }
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  return hipSuccess;
}

int run_plan(const Plan& plan, const void* q, const medha_kv_cache* kv, const int32_t* page_table,
             int h_q, float softmax_scale, float* out, float* lse, void* workspace,
             size_t workspace_bytes, void* hip_stream) {
  if (plan.part_rows > 0) {
    if (workspace == nullptr || !aligned(workspace, 256) || workspace_bytes < plan.bytes)
      return MEDHA_ERR_WORKSPACE;
  }
  char* ws = static_cast<char*>(workspace);
  AttnArgs a{};
  a.q = static_cast<const __bf16*>(q);
  a.k_pool = static_cast<const __bf16*>(kv->k_pool);
  a.v_pool = static_cast<const __bf16*>(kv->v_pool);
  a.page_table = page_table;
  a.out = out;
  a.lse = lse;
  a.part_o = ws ? reinterpret_cast<float*>(ws + plan.off_part_o) : nullptr;
  a.part_lse = ws ? reinterpret_cast<float*>(ws + plan.off_part_lse) : nullptr;
  a.h_q = h_q;
  a.h_kv = kv->num_kv_heads;
  a.scale_log2 = softmax_scale * kLog2e;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (launch_plan(plan.rows, false, kv->head_dim, a, stream) != hipSuccess) return MEDHA_ERR_HIP;
  if (launch_plan(plan.keys, true, kv->head_dim, a, stream) != hipSuccess) return MEDHA_ERR_HIP;
  return MEDHA_OK;
}

int check_kv(const medha_kv_cache* kv, int h_q) {
  if (kv == nullptr || kv->k_pool == nullptr || kv->v_pool == nullptr || kv->num_pages <= 0)
    return MEDHA_ERR_INVALID_ARG;
  if (!aligned(kv->k_pool, 16) || !aligned(kv->v_pool, 16)) return MEDHA_ERR_INVALID_ARG;
  return check_heads(h_q, kv->num_kv_heads, kv->head_dim, kv->page_size);
}

}  // namespace
}  // namespace medha

using namespace medha;

extern "C" {

int medha_abi_version(void) { return 1; }

const char* medha_strerror(int code) {
  switch (code) {
    case MEDHA_OK: return "ok";
    case MEDHA_ERR_INVALID_ARG: return "invalid argument";
    case MEDHA_ERR_UNSUPPORTED: return "unsupported shape (page size must be 16, head_dim 64 or 128)";
    case MEDHA_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case MEDHA_ERR_HIP: return "HIP runtime error";
    default: return "unknown error code";
  }
}

size_t medha_chunked_prefill_workspace_bytes(const int32_t* prefix_len, const int32_t* chunk_len,
                                             int32_t batch, int32_t num_q_heads,
                                             int32_t num_kv_heads, int32_t head_dim) {
  if (batch < 0 || (batch > 0 && (prefix_len == nullptr || chunk_len == nullptr))) return 0;
  if (check_heads(num_q_heads, num_kv_heads, head_dim, kPageSize) != MEDHA_OK) return 0;
  std::vector<SeqInput> seqs(batch);
  int64_t row = 0;
  for (int b = 0; b < batch; ++b) {
    if (prefix_len[b] < 0 || chunk_len[b] < 1) return 0;
    if ((int64_t)prefix_len[b] + chunk_len[b] > INT32_MAX) return 0;
    seqs[b] = SeqInput{0, (int32_t)row, (int32_t)row, chunk_len[b], prefix_len[b]};
    row += chunk_len[b];
    if (row > INT32_MAX) return 0;
  }
  return make_plan(seqs.data(), batch, num_q_heads, num_kv_heads, head_dim, current_num_cus())
      .bytes;
}

int medha_chunked_prefill_attn(const void* q, const medha_kv_cache* kv, const int32_t* page_table,
                               const int64_t* page_table_offs, const int32_t* prefix_len,
                               const int32_t* chunk_len, int32_t batch, int32_t num_q_heads,
                               float softmax_scale, float* out, float* lse, void* workspace,
                               size_t workspace_bytes, void* hip_stream) {
  if (batch < 0) return MEDHA_ERR_INVALID_ARG;
  int rc = check_kv(kv, num_q_heads);
  if (rc != MEDHA_OK) return rc;
  if (batch == 0) return MEDHA_OK;
  if (q == nullptr || page_table == nullptr || page_table_offs == nullptr ||
      prefix_len == nullptr || chunk_len == nullptr || out == nullptr || lse == nullptr)
    return MEDHA_ERR_INVALID_ARG;
  if (!aligned(q, 16) || !aligned(out, 16) || !aligned(lse, 4) || !std::isfinite(softmax_scale))
    return MEDHA_ERR_INVALID_ARG;
  std::vector<SeqInput> seqs(batch);
  int64_t row = 0;
  for (int b = 0; b < batch; ++b) {
    if (prefix_len[b] < 0 || chunk_len[b] < 1) return MEDHA_ERR_INVALID_ARG;
    const int64_t n = (int64_t)prefix_len[b] + chunk_len[b];
    if (n > INT32_MAX) return MEDHA_ERR_INVALID_ARG;
    const int64_t have = page_table_offs[b + 1] - page_table_offs[b];
    if (page_table_offs[b] < 0 || have < ceil_div(n, kPageSize)) return MEDHA_ERR_INVALID_ARG;
    seqs[b] = SeqInput{page_table_offs[b], (int32_t)row, (int32_t)row, chunk_len[b], prefix_len[b]};
    row += chunk_len[b];
    if (row > INT32_MAX) return MEDHA_ERR_INVALID_ARG;
  }
  const Plan plan = make_plan(seqs.data(), batch, num_q_heads, kv->num_kv_heads, kv->head_dim,
                              current_num_cus());
  return run_plan(plan, q, kv, page_table, num_q_heads, softmax_scale, out, lse, workspace,
                  workspace_bytes, hip_stream);
}

int medha_chunked_prefill_attn_noalloc(const void* q, const medha_kv_cache* kv,
                                       const int32_t* page_table,
                                       const int64_t* page_table_offs, const int32_t* prefix_len,
                                       const int32_t* chunk_len, int32_t batch,
                                       int32_t num_q_heads, float softmax_scale, float* out,
                                       float* lse, void* hip_stream) {
  // The size check comes first so that an oversized batch is refused whatever else is wrong
  // with it; medha_chunked_prefill_attn validates everything again.
  if (batch > 0 && kv != nullptr && prefix_len != nullptr && chunk_len != nullptr) {
    const size_t need = medha_chunked_prefill_workspace_bytes(
        prefix_len, chunk_len, batch, num_q_heads, kv->num_kv_heads, kv->head_dim);
    if (need > (size_t)MEDHA_NOALLOC_SCRATCH_BYTES) return MEDHA_ERR_WORKSPACE;
  }
  int rc = MEDHA_OK;
  void* ws = noalloc_scratch_ptr(&rc);
  if (rc != MEDHA_OK) return rc;
  return medha_chunked_prefill_attn(q, kv, page_table, page_table_offs, prefix_len, chunk_len,
                                    batch, num_q_heads, softmax_scale, out, lse, ws,
                                    (size_t)MEDHA_NOALLOC_SCRATCH_BYTES, hip_stream);
}

size_t medha_decode_partial_workspace_bytes(const int32_t* kv_len, int32_t items,
                                            int32_t num_q_heads, int32_t num_kv_heads,
                                            int32_t head_dim) {
  if (items < 0 || (items > 0 && kv_len == nullptr)) return 0;
  if (check_heads(num_q_heads, num_kv_heads, head_dim, kPageSize) != MEDHA_OK) return 0;
  std::vector<SeqInput> seqs(items);
  for (int i = 0; i < items; ++i) {
    if (kv_len[i] < 0) return 0;
    seqs[i] = SeqInput{0, 0, i, 1, kv_len[i] - 1};
  }
  return make_plan(seqs.data(), items, num_q_heads, num_kv_heads, head_dim, current_num_cus())
      .bytes;
}

int medha_decode_partial_attn(const void* q, int32_t num_queries, const medha_kv_cache* kv,
                              const int32_t* page_table, const int64_t* page_table_offs,
                              const int32_t* q_index, const int32_t* kv_len, int32_t items,
                              int32_t num_q_heads, float softmax_scale, float* out_partial,
                              float* lse_partial, void* workspace, size_t workspace_bytes,
                              void* hip_stream) {
  if (items < 0 || num_queries < 0) return MEDHA_ERR_INVALID_ARG;
  int rc = check_kv(kv, num_q_heads);
  if (rc != MEDHA_OK) return rc;
  if (items == 0) return MEDHA_OK;
  if (q == nullptr || page_table == nullptr || page_table_offs == nullptr || q_index == nullptr ||
      kv_len == nullptr || out_partial == nullptr || lse_partial == nullptr)
    return MEDHA_ERR_INVALID_ARG;
  if (!aligned(q, 16) || !aligned(out_partial, 16) || !aligned(lse_partial, 4) ||
      !std::isfinite(softmax_scale))
    return MEDHA_ERR_INVALID_ARG;
  std::vector<SeqInput> seqs(items);
  for (int i = 0; i < items; ++i) {
    if (kv_len[i] < 0 || q_index[i] < 0 || q_index[i] >= num_queries) return MEDHA_ERR_INVALID_ARG;
    const int64_t have = page_table_offs[i + 1] - page_table_offs[i];
    if (page_table_offs[i] < 0 || have < ceil_div(kv_len[i], kPageSize))
      return MEDHA_ERR_INVALID_ARG;
    seqs[i] = SeqInput{page_table_offs[i], q_index[i], i, 1, kv_len[i] - 1};
  }
  const Plan plan = make_plan(seqs.data(), items, num_q_heads, kv->num_kv_heads, kv->head_dim,
                              current_num_cus());
  return run_plan(plan, q, kv, page_table, num_q_heads, softmax_scale, out_partial, lse_partial,
                  workspace, workspace_bytes, hip_stream);
}

size_t medha_chunk_partial_workspace_bytes(const int32_t* chunk_len, const int32_t* kv_len,
                                          int32_t items, int32_t num_q_heads,
                                          int32_t num_kv_heads, int32_t head_dim) {
  if (items < 0 || (items > 0 && (chunk_len == nullptr || kv_len == nullptr))) return 0;
  if (check_heads(num_q_heads, num_kv_heads, head_dim, kPageSize) != MEDHA_OK) return 0;
  std::vector<SeqInput> seqs(items);
  int64_t row = 0;
  for (int i = 0; i < items; ++i) {
    if (chunk_len[i] < 1 || kv_len[i] < 0) return 0;
    // the plan depends on the row count and the key count only
    seqs[i] = SeqInput{0, 0, (int32_t)row, chunk_len[i], kv_len[i] - 1, kv_len[i]};
    row += chunk_len[i];
    if (row > INT32_MAX) return 0;
  }
  return make_plan(seqs.data(), items, num_q_heads, num_kv_heads, head_dim, current_num_cus())
      .bytes;
}

int medha_chunk_partial_attn(const void* q, int32_t num_tokens, const medha_kv_cache* kv,
                             const int32_t* page_table, const int64_t* page_table_offs,
                             const int32_t* q_row, const int32_t* chunk_len,
                             const int32_t* kv_len, const int32_t* visible0, int32_t items,
                             int32_t num_q_heads, float softmax_scale, float* out_partial,
                             float* lse_partial, void* workspace, size_t workspace_bytes,
                             void* hip_stream) {
  if (items < 0 || num_tokens < 0) return MEDHA_ERR_INVALID_ARG;
  int rc = check_kv(kv, num_q_heads);
  if (rc != MEDHA_OK) return rc;
  if (items == 0) return MEDHA_OK;
  if (q == nullptr || page_table == nullptr || page_table_offs == nullptr || q_row == nullptr ||
      chunk_len == nullptr || kv_len == nullptr || visible0 == nullptr ||
      out_partial == nullptr || lse_partial == nullptr)
    return MEDHA_ERR_INVALID_ARG;
  if (!aligned(q, 16) || !aligned(out_partial, 16) || !aligned(lse_partial, 4) ||
      !std::isfinite(softmax_scale))
    return MEDHA_ERR_INVALID_ARG;
  constexpr int32_t kMaxVisible = 1 << 30;
  std::vector<SeqInput> seqs(items);
  int64_t row = 0;
  for (int i = 0; i < items; ++i) {
    if (chunk_len[i] < 1 || kv_len[i] < 0 || q_row[i] < 0 ||
        (int64_t)q_row[i] + chunk_len[i] > num_tokens)
      return MEDHA_ERR_INVALID_ARG;
    if (visible0[i] < -kMaxVisible || visible0[i] > kMaxVisible || chunk_len[i] > kMaxVisible)
      return MEDHA_ERR_INVALID_ARG;
    const int64_t have = page_table_offs[i + 1] - page_table_offs[i];
    if (page_table_offs[i] < 0 || have < ceil_div(kv_len[i], kPageSize))
      return MEDHA_ERR_INVALID_ARG;
    // row j sees keys [0, visible0 + j): its last visible key is (visible0 - 1) + j
    seqs[i] = SeqInput{page_table_offs[i], q_row[i], (int32_t)row, chunk_len[i], visible0[i] - 1,
                       kv_len[i]};
    row += chunk_len[i];
    if (row > INT32_MAX) return MEDHA_ERR_INVALID_ARG;
  }
  const Plan plan = make_plan(seqs.data(), items, num_q_heads, kv->num_kv_heads, kv->head_dim,
                              current_num_cus());
  return run_plan(plan, q, kv, page_table, num_q_heads, softmax_scale, out_partial, lse_partial,
                  workspace, workspace_bytes, hip_stream);
}

int medha_describe_plan(const int32_t* prefix_len, const int32_t* chunk_len, int32_t batch,
                        int32_t num_q_heads, int32_t num_kv_heads, int32_t head_dim,
                        int32_t num_cus, medha_plan_entry* entries, int32_t* grid_rows,
                        int32_t* grid_keys, size_t* workspace_bytes) {
  if (batch < 0 || (batch > 0 && (prefix_len == nullptr || chunk_len == nullptr ||
                                  entries == nullptr)))
    return MEDHA_ERR_INVALID_ARG;
  int rc = check_heads(num_q_heads, num_kv_heads, head_dim, kPageSize);
  if (rc != MEDHA_OK) return rc;
  std::vector<SeqInput> seqs(batch);
  int64_t row = 0;
  for (int b = 0; b < batch; ++b) {
    if (prefix_len[b] < -1 || chunk_len[b] < 1) return MEDHA_ERR_INVALID_ARG;
    seqs[b] = SeqInput{0, (int32_t)row, (int32_t)row, chunk_len[b], prefix_len[b]};
    row += chunk_len[b];
  }
  const Plan plan = make_plan(seqs.data(), batch, num_q_heads, num_kv_heads, head_dim,
                              num_cus > 0 ? num_cus : current_num_cus());
  for (int mode = 0; mode < 2; ++mode) {
    const LaunchPlan& lp = mode == 0 ? plan.rows : plan.keys;
    for (size_t i = 0; i < lp.descs.size(); ++i) {
      const SeqDesc& sd = lp.descs[i];
      medha_plan_entry& e = entries[lp.seq_index[i]];
      e.mode = mode;
      e.rows_per_wg = lp.shape.rows_per_wg;
      e.tile_keys = lp.shape.tile_keys;
      e.n_row_tiles = sd.n_row_tiles;
      e.n_split = sd.n_split;
      e.tiles_per_split = sd.tiles_per_split;
      e.work_start = sd.work_start;
      e.n_slots = (i + 1 < lp.descs.size() ? lp.descs[i + 1].work_start : lp.n_slots) -
                  sd.work_start;
    }
  }
  if (grid_rows) *grid_rows = plan.rows.n_slots;
  if (grid_keys) *grid_keys = plan.keys.n_slots;
  if (workspace_bytes) *workspace_bytes = plan.bytes;
  return MEDHA_OK;
}

int medha_describe_slot(int32_t slot, int32_t num_kv_heads, int32_t n_split, int32_t n_row_tiles,
                        int32_t* kv_head, int32_t* split, int32_t* row_tile) {
  if (slot < 0 || num_kv_heads <= 0 || n_split <= 0 || n_row_tiles <= 0)
    return MEDHA_ERR_INVALID_ARG;
  const SlotItem it = decode_slot(slot, num_kv_heads, n_split, n_row_tiles);
  if (kv_head) *kv_head = it.kv_head;
  if (split) *split = it.split;
  if (row_tile) *row_tile = it.row_tile;
  return it.valid;
}

int medha_lse_merge(const float* out_partial, const float* lse_partial, int32_t num_splits,
                    int64_t rows, int32_t num_q_heads, int32_t head_dim, float* out, float* lse,
                    void* hip_stream) {
  if (num_splits < 1 || rows < 0 || num_q_heads <= 0 || head_dim <= 0)
    return MEDHA_ERR_INVALID_ARG;
  if (head_dim % 4 != 0) return MEDHA_ERR_UNSUPPORTED;
  if (rows == 0) return MEDHA_OK;
  if (out_partial == nullptr || lse_partial == nullptr || out == nullptr || lse == nullptr)
    return MEDHA_ERR_INVALID_ARG;
  if (!aligned(out_partial, 16) || !aligned(out, 16)) return MEDHA_ERR_INVALID_ARG;
  // one thread per 4 output elements; the grid has to fit 31 bits (checked without overflow)
  const int64_t per_row = (int64_t)num_q_heads * (head_dim / 4);
  if (rows > ((int64_t)INT32_MAX * kThreads) / per_row) return MEDHA_ERR_INVALID_ARG;
  const int64_t grid = ceil_div(rows * per_row, kThreads);
  if (grid > INT32_MAX) return MEDHA_ERR_INVALID_ARG;
  hipLaunchKernelGGL(lse_merge_kernel, dim3((unsigned)grid), dim3(kThreads), 0,
                     static_cast<hipStream_t>(hip_stream), out_partial, lse_partial, num_splits,
                     rows, num_q_heads, head_dim, out, lse);
  return hipGetLastError() == hipSuccess ? MEDHA_OK : MEDHA_ERR_HIP;
}

int medha_kv_append(const void* k_new, const void* v_new, const medha_kv_cache* kv,
                    const int32_t* page_table, const int64_t* page_table_offs,
                    const int32_t* prefix_len, const int32_t* chunk_len, int32_t batch,
                    void* hip_stream) {
  if (kv == nullptr || batch < 0) return MEDHA_ERR_INVALID_ARG;
  if (kv->num_kv_heads <= 0 || kv->num_pages < 0) return MEDHA_ERR_INVALID_ARG;
  if (kv->page_size != kPageSize || (kv->head_dim != 64 && kv->head_dim != 128))
    return MEDHA_ERR_UNSUPPORTED;
  if (batch == 0) return MEDHA_OK;
  if (k_new == nullptr || v_new == nullptr || kv->k_pool == nullptr || kv->v_pool == nullptr ||
      page_table == nullptr || page_table_offs == nullptr || prefix_len == nullptr ||
      chunk_len == nullptr)
    return MEDHA_ERR_INVALID_ARG;
  if (!aligned(k_new, 16) || !aligned(v_new, 16) || !aligned(kv->k_pool, 16) ||
      !aligned(kv->v_pool, 16))
    return MEDHA_ERR_INVALID_ARG;
  int64_t rows = 0;
  for (int b = 0; b < batch; ++b) {
    if (prefix_len[b] < 0 || chunk_len[b] < 1) return MEDHA_ERR_INVALID_ARG;
    const int64_t pages = ceil_div((int64_t)prefix_len[b] + chunk_len[b], kPageSize);
    if (page_table_offs[b] < 0 || page_table_offs[b + 1] - page_table_offs[b] < pages)
      return MEDHA_ERR_INVALID_ARG;
    rows += chunk_len[b];
    if (rows > INT32_MAX) return MEDHA_ERR_INVALID_ARG;
  }
  // validated in full before the first launch; up to kMaxInlineSeq sequences per launch
  int64_t src_row = 0;
  for (int b0 = 0; b0 < batch; b0 += kMaxInlineSeq) {
    AppendArgs a{};
    a.k_new = static_cast<const uint4*>(k_new);
    a.v_new = static_cast<const uint4*>(v_new);
    a.k_pool = static_cast<uint4*>(const_cast<void*>(kv->k_pool));
    a.v_pool = static_cast<uint4*>(const_cast<void*>(kv->v_pool));
    a.page_table = page_table;
    a.h_kv = kv->num_kv_heads;
    a.words_per_row = kv->head_dim / 8;
    a.num_pages = kv->num_pages;
    a.n_seq = std::min(kMaxInlineSeq, batch - b0);
    int32_t rank = 0;
    for (int i = 0; i < a.n_seq; ++i) {
      AppendDesc& sd = a.descs[i];
      sd.pt_off = page_table_offs[b0 + i];
      sd.src_row = (int32_t)src_row;
      sd.prefix_len = prefix_len[b0 + i];
      sd.chunk_len = chunk_len[b0 + i];
      sd.row_rank = rank;
      rank += sd.chunk_len;
      src_row += sd.chunk_len;
    }
    a.total_rows = rank;
    const int64_t threads = (int64_t)rank * a.h_kv * a.words_per_row;
    const int64_t grid = ceil_div(threads, kThreads);
    if (grid > INT32_MAX) return MEDHA_ERR_INVALID_ARG;
    hipLaunchKernelGGL(kv_append_kernel, dim3((unsigned)grid), dim3(kThreads), 0,
                       static_cast<hipStream_t>(hip_stream), a);
    if (hipGetLastError() != hipSuccess) return MEDHA_ERR_HIP;
  }
  return MEDHA_OK;
}

// ------------------------------------------------------------------ policy (host only)
double medha_policy_chunk_time(const medha_time_model* model, int64_t kv_size, int64_t chunk) {
  if (!policy::valid(model) || kv_size < 0 || chunk < 0 || kv_size > (1ll << 40) ||
      chunk > (1 << 24))
    return std::numeric_limits<double>::quiet_NaN();
  return policy::chunk_time(*model, kv_size, chunk);
}

int medha_policy_fit_time_model(const int64_t* kv_size, const int64_t* chunk,
                                const double* seconds, int32_t n, medha_time_model* model,
                                double* max_rel_err) {
  if (kv_size == nullptr || chunk == nullptr || seconds == nullptr || model == nullptr || n < 3)
    return -1;
  std::vector<double> x[3];
  for (int i = 0; i < n; ++i) {
    if (kv_size[i] < 0 || chunk[i] < 1 || !(seconds[i] > 0.0) || !std::isfinite(seconds[i]))
      return -1;
    if (kv_size[i] > (1ll << 40) || chunk[i] > (1 << 24)) return -1;
    x[0].push_back(1.0);
    x[1].push_back((double)chunk[i]);
    x[2].push_back((double)chunk[i] * (double)kv_size[i] +
                   (double)(chunk[i] * (chunk[i] + 1)) / 2.0);
  }
  // all three columns first; drop a column whose coefficient comes out negative and refit
  bool use[3] = {true, true, true};
  double coef[3] = {0, 0, 0};
  for (int round = 0; round < 3; ++round) {
    int cols[3], k = 0;
    for (int j = 0; j < 3; ++j)
      if (use[j]) cols[k++] = j;
    if (k == 0 || !policy::fit_columns(x, seconds, n, cols, k, coef)) return -1;
    int worst = -1;
    for (int j = 0; j < 3; ++j)
      if (use[j] && coef[j] < 0.0 && (worst < 0 || coef[j] < coef[worst])) worst = j;
    if (worst < 0) break;
    use[worst] = false;
    coef[worst] = 0.0;
  }
  for (double c : coef)
    if (!std::isfinite(c) || c < 0.0) return -1;
  *model = medha_time_model{coef[0], coef[1], coef[2], 0.0, 0.0};
  if (max_rel_err) {
    double worst = 0.0;
    for (int i = 0; i < n; ++i) {
      const double pred = model->t_fixed + policy::chunk_time(*model, kv_size[i], chunk[i]);
      worst = std::max(worst, std::fabs(pred - seconds[i]) / seconds[i]);
    }
    *max_rel_err = worst;
  }
  return 0;
}

int64_t medha_policy_max_chunk(const medha_time_model* model, int64_t kv_size, double t_budget,
                               int64_t max_chunk) {
  if (!policy::valid(model) || kv_size < 0 || max_chunk < 0 || std::isnan(t_budget)) return -1;
  if (kv_size > (1ll << 40) || max_chunk > (1 << 24)) return -1;  // products stay exact in fp64
  return policy::max_chunk(*model, kv_size, t_budget, max_chunk);
}

int64_t medha_policy_get_chunk_size(const medha_time_model* model, int64_t kv_size,
                                    int64_t remaining, int32_t is_long, int32_t batch_has_long,
                                    double rel_slack, double rho_max, double t_current,
                                    double t_target, int64_t max_chunk) {
  if (!policy::valid(model) || kv_size < 0 || remaining < 0 || max_chunk < 0) return -1;
  if (kv_size > (1ll << 40) || max_chunk > (1 << 24)) return -1;
  if (std::isnan(rel_slack) || !(rho_max >= 0.0 && rho_max <= 1.0) || std::isnan(t_current) ||
      !(t_target >= 0.0))
    return -1;
  // one long prefill per batch; otherwise the iteration's time budget, shrunk in proportion
  // to the slack the request can afford to give away (at most rho_max of it), less what the
  // batch already costs
  if (is_long && batch_has_long) return 0;
  const double yielded = rel_slack > 0.0 ? (rel_slack < rho_max ? rel_slack : rho_max) : 0.0;
  const double left = t_target * (1.0 - yielded) - t_current;
  if (!(left > 0.0)) return 0;
  return policy::max_chunk(*model, kv_size, left, max_chunk < remaining ? max_chunk : remaining);
}

double medha_policy_simulate_prefill(const medha_time_model* model, int64_t length,
                                     double t_target, int64_t max_chunk) {
  if (!policy::valid(model) || length < 0 || max_chunk < 1 || max_chunk > (1 << 24) ||
      length > (1ll << 40) || std::isnan(t_target))
    return std::numeric_limits<double>::quiet_NaN();
  return policy::simulate_prefill(*model, length, t_target, max_chunk);
}

int medha_policy_build_prefill_cache(const medha_time_model* model, int64_t l_max, int64_t delta,
                                     double t_target, int64_t max_chunk, double* cache,
                                     int64_t cache_len) {
  if (!policy::valid(model) || cache == nullptr || delta < 1 || l_max < 0 ||
      cache_len != l_max / delta + 1 || max_chunk < 1 || max_chunk > (1 << 24) ||
      l_max > (1ll << 40) || std::isnan(t_target))
    return -1;
  // One walk over the chunks of the longest prefill.  The chunks of a shorter length are the
  // same until the one that reaches its end, which is cut there: so every entry whose length
  // falls inside the current chunk is (time before the chunk) + (the cut chunk), and an entry
  // the walk never reaches (no chunk fits any more) keeps the time reached.
  const medha_time_model& m = *model;
  const double budget = t_target - m.t_fixed;
  double total = 0.0;
  int64_t done = 0, next = 0;  // next cache entry to fill
  while (next < cache_len) {
    const int64_t target = next * delta;
    if (target <= done) {  // only for target == done: a length that ends on a chunk boundary
      cache[next++] = total;
      continue;
    }
    // the chunk a prefill of exactly `target` tokens would take at `done`
    const int64_t c_here = policy::max_chunk(m, done, budget, std::min(max_chunk, target - done));
    if (c_here == 0) {  // stuck: this and every longer length stop here
      cache[next++] = total;
      continue;
    }
    if (done + c_here == target) {
      // the cut chunk ends the shorter prefill; the longest one may take a longer chunk here
      cache[next++] = total + (m.t_fixed + policy::chunk_time(m, done, c_here));
      continue;
    }
    // target lies beyond this chunk: c_here is the uncut chunk, the walk advances
    total += m.t_fixed + policy::chunk_time(m, done, c_here);
    done += c_here;
  }
  return 0;
}

double medha_policy_remaining_time(const double* cache, int64_t cache_len, int64_t delta,
                                   int64_t l_total, int64_t l_processed) {
  if (cache == nullptr || cache_len < 1 || delta < 1 || l_total < 0 || l_processed < 0)
    return std::numeric_limits<double>::quiet_NaN();
  auto lookup = [&](int64_t length) {
    const int64_t i = length / delta, r = length % delta;
    if (i >= cache_len - 1) return cache[cache_len - 1];
    return cache[i] + (cache[i + 1] - cache[i]) * ((double)r / (double)delta);
  };
  return lookup(l_total) - lookup(l_processed);
}

double medha_policy_relative_slack(double arrival, double deadline, double now,
                                   double remaining_work, double total_work) {
  return (arrival + deadline - now - remaining_work) / total_work;
}

int medha_policy_simulate_schedule(int32_t policy_id, const double* arrival, const double* work,
                                   const double* deadline, int32_t n, double quantum,
                                   double* finish, double* first_start) {
  if (arrival == nullptr || work == nullptr || deadline == nullptr || finish == nullptr ||
      n < 1 || !(quantum > 0.0) || policy_id < 0 || policy_id > 2)
    return -1;
  for (int i = 0; i < n; ++i)
    if (!(work[i] > 0.0) || !std::isfinite(work[i]) || !std::isfinite(arrival[i]) ||
        arrival[i] < 0.0 || !std::isfinite(deadline[i]))
      return -1;
  constexpr double kEps = 1e-12;
  std::vector<double> left(work, work + n);
  std::vector<char> done(n, 0), started(n, 0);
  int n_done = 0, current = -1;
  double t = 0.0;
  while (n_done < n) {
    // requests that have arrived and are not finished
    int pick = -1;
    double best = 0.0;
    bool any_ready = false;
    double next_arrival = std::numeric_limits<double>::infinity();
    for (int i = 0; i < n; ++i) {
      if (done[i]) continue;
      if (arrival[i] <= t + kEps) {
        any_ready = true;
        double key;
        if (policy_id == 0) key = arrival[i];
        else if (policy_id == 1) key = arrival[i] + deadline[i];
        else key = (arrival[i] + deadline[i] - t - left[i]) / work[i];
        if (pick < 0 || key < best) { pick = i; best = key; }
      } else {
        next_arrival = std::min(next_arrival, arrival[i]);
      }
    }
    if (!any_ready) { t = next_arrival; continue; }
    if (policy_id == 0 && current >= 0 && !done[current]) pick = current;  // no preemption
    current = pick;
    if (!started[current]) {
      started[current] = 1;
      if (first_start) first_start[current] = t;
    }
    const double run = std::min(quantum, left[current]);
    left[current] -= run;
    t += run;
    if (left[current] <= kEps) {
      done[current] = 1;
      finish[current] = t;
      ++n_done;
    }
  }
  return 0;
}

}  // extern "C"
