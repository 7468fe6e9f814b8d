// Shared definitions of the HIP attention library: work descriptors handed from
// the host planner to the kernels, vector types, small device helpers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace medha {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kPageSize = 16;     // tokens per KV page
constexpr int kThreads = 256;     // threads per workgroup (4 wavefronts of 64)
constexpr int kWaves = 4;
constexpr int kXcds = 8;          // accelerator dies; workgroup i is dispatched to die i % 8
constexpr int kPrefillStages = 4;  // K/V tiles in flight per workgroup (LDS ring)
constexpr int kMaxInlineSeq = 64; // sequence descriptors per kernel launch (they travel as kernel arguments)
constexpr int kShortWalkTiles = 24;   // key-split launches walking at most this many 128-key tiles per workgroup use the small ring
constexpr int kWideMergeSplits = 16;  // more KV ranges per row than this: the wide merge kernel
constexpr float kRescaleSlack = 8.f;  // log2 units a row maximum may exceed the softmax reference
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// One sequence of a launch.  Its page table (from pt_off) describes kv_len keys;
// query row j (0 <= j < chunk_len) attends to keys [0, min(prefix_len + j, kv_len - 1)]
// of them, to none if that is negative.  Chunked prefill: kv_len = prefix_len +
// chunk_len.  A decode item: chunk_len == 1, prefix_len == kv_len - 1.  A chunk
// against a KV shard: prefix_len + 1 = keys of the shard its first row sees, which
// may be <= 0 or exceed kv_len.  The sequence owns workgroup slots
// [work_start, work_start + 8 * ceil(h_kv * n_split * n_row_tiles / 8)).
struct SeqDesc {
  int64_t pt_off;           // first entry of the sequence in the page table
  int32_t q_row;            // first query token row in q
  int32_t out_row;          // first token row in out / lse
  int32_t chunk_len;        // query tokens
  int32_t prefix_len;       // see above
  int32_t work_start;       // first workgroup slot
  int32_t n_row_tiles;      // query-row tiles per KV head
  int32_t n_split;          // KV ranges the keys are split into (1 = write out directly)
  int32_t tiles_per_split;  // KV tiles per range
  int32_t part_row;         // first token row of this sequence in the partial workspace
  int32_t row_rank;         // rank of the sequence's first token row among the launch's rows
  int32_t kv_len;           // keys the page-table slice describes
  int32_t reserved;
};
static_assert(sizeof(SeqDesc) == 56, "SeqDesc layout");

// Kernel arguments of the attention kernels.  The sequence descriptors ride in the
// argument block itself (no host-to-device copy, no synchronisation); a batch of more
// than kMaxInlineSeq sequences takes several launches.
struct AttnArgs {
  const __bf16* q;
  const __bf16* k_pool;
  const __bf16* v_pool;
  const int32_t* page_table;
  float* out;
  float* lse;
  float* part_o;    // split-KV partial outputs  [part rows][h_q][d]
  float* part_lse;  // split-KV partial LSEs     [part rows][h_q]
  int32_t n_seq;
  int32_t h_q;
  int32_t h_kv;
  float scale_log2;  // softmax_scale * log2(e)
  SeqDesc inline_descs[kMaxInlineSeq];
};
static_assert(sizeof(AttnArgs) <= 4096, "kernel argument block too large");

// Arguments of the merge over the library's own split-KV partials.
struct MergeArgs {
  const float* part_o;
  const float* part_lse;
  float* out;
  float* lse;
  int32_t n_seq;
  int32_t h_q;
  int32_t total_rows;  // token rows of all sequences of the launch
  int32_t reserved;
  SeqDesc inline_descs[kMaxInlineSeq];
};
static_assert(sizeof(MergeArgs) <= 4096, "kernel argument block too large");

// Workgroup slot u of a sequence -> its work item.  Slot u runs on die u % 8
// (the hardware deals consecutive workgroups round-robin to the 8 dies).  The
// sequence's items, ordered (group, row tile) with group = (KV split, KV head),
// are cut into 8 equal contiguous runs, one per die: the row tiles that stream
// the same K/V range share a die and hence its L2.  Slots past a run are idle.
struct SlotItem {
  int valid, kv_head, split, row_tile;
};
__host__ __device__ inline SlotItem decode_slot(int u, int h_kv, int n_split, int n_row_tiles) {
  const int items = h_kv * n_split * n_row_tiles;
  const int per_die = (items + kXcds - 1) / kXcds;
  const int y = u / kXcds;
  const int item = (u % kXcds) * per_die + y;
  SlotItem r;
  r.valid = (y < per_die && item < items) ? 1 : 0;
  const int grp = item / n_row_tiles;
  r.row_tile = item % n_row_tiles;
  r.kv_head = grp % h_kv;
  r.split = grp / h_kv;
  return r;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// Value held by the lane 32 positions away (lane ^ 32), via the gfx950
// half-wave swap: swap(x, x) returns {x of low half, x of high half} in every lane.
__device__ __forceinline__ float other_half(float x, int hi_half) {
  unsigned u = __builtin_bit_cast(unsigned, x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  unsigned o = hi_half ? r[0] : r[1];
  return __builtin_bit_cast(float, o);
}
__device__ __forceinline__ float max_halves(float x) {
  unsigned u = __builtin_bit_cast(unsigned, x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__builtin_bit_cast(float, (unsigned)r[0]), __builtin_bit_cast(float, (unsigned)r[1]));
}
__device__ __forceinline__ float sum_halves(float x) {
  unsigned u = __builtin_bit_cast(unsigned, x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __builtin_bit_cast(float, (unsigned)r[0]) + __builtin_bit_cast(float, (unsigned)r[1]);
}

}  // namespace medha
