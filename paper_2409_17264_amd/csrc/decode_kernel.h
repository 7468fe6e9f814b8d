// Key-split attention kernel for gfx950: decode steps and other tiny row counts
// (paper section 3.3: one query token against a long KV shard is bound by the
// rate at which the KV cache streams from HBM).
//
// The <= 32 query rows of a (sequence, KV head) -- the GQA group's heads of the
// one token, or of a few tokens -- sit in one 32-row block that all 4 wavefronts
// of the workgroup share; the keys are what is split: wavefront w walks the
// 32-key blocks w, w+4, w+8, ... of the workgroup's KV range with its own
// online-softmax state, and the four states are combined through LDS at the end.
//
// Each wavefront streams its blocks HBM -> LDS with asynchronous 16-byte loads
// into a private two-stage ring (no workgroup barrier in the loop, so the four
// streams run decoupled and up to 128 KiB of loads are in flight per compute
// unit).  The arithmetic per block is the prefill kernel's: S^T = K Q^T and
// O^T += V^T P^T on the matrix cores with only `rows` of the 32 columns live,
// which costs a few percent of the matrix peak and keeps the vector ALUs out of
// the way of the memory stream.
#pragma once

#include <type_traits>

#include "common.h"
#include "prefill_kernel.h"

namespace medha {

template <int D, int STAGES = 2>
struct DecodeGeom {
  static constexpr int kBlockKeys = 32;
  static constexpr int kChunksPerRow = D / 8;
  static constexpr int kRowsPerInstr = 64 / kChunksPerRow;             // 4 or 8
  static constexpr int kInstrPerBlock = kBlockKeys / kRowsPerInstr;    // per K (or V) block
  static constexpr int kHalfBytes = kBlockKeys * D * 2;                // K (or V) block
  static constexpr int kBlockBytes = 2 * kHalfBytes;
  static constexpr int kLoadsPerBlock = 2 * kInstrPerBlock;
  static constexpr int kStagesPerWave = STAGES;
  static constexpr int kLdsBytes = kWaves * kStagesPerWave * kBlockBytes;
  static constexpr int kSplitKeys = kBlockKeys * kWaves;  // planner's KV-split granule (128)
};

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt range");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Asynchronous loads of the 32-key block starting at sequence key `key0`
// (a multiple of 32, so it spans exactly the two pages page0, page1).
template <int D>
__device__ __forceinline__ void issue_block(const AttnArgs& args, int page0, int page1, int key0,
                                            int kv_total, int kv_head, uint32_t k_lds,
                                            uint32_t v_lds, int lane) {
  using G = DecodeGeom<D>;
  const char* kp = reinterpret_cast<const char*>(args.k_pool);
  const char* vp = reinterpret_cast<const char*>(args.v_pool);
  const int r_in = lane / G::kChunksPerRow;
  const int pos = lane % G::kChunksPerRow;
#pragma unroll
  for (int j = 0; j < G::kInstrPerBlock; ++j) {
    const int row = j * G::kRowsPerInstr + r_in;  // 0..31
    const int page = (j * G::kRowsPerInstr < kPageSize) ? page0 : page1;
    // keys past the end are clamped to the last one (masked, but finite)
    const int t = min(key0 + row, kv_total - 1);
    const int64_t off =
        (((int64_t)page * args.h_kv + kv_head) * kPageSize + (t & 15)) * (D * 2);
    const uint32_t lds_off = j * G::kRowsPerInstr * (D * 2);
    async_load16(kp + off + Swz<D>::k(row, pos) * 16, k_lds + lds_off);
    async_load16(vp + off + Swz<D>::v(row, pos) * 16, v_lds + lds_off);
  }
}

// STAGES = blocks in flight per wavefront.  2 (128 KiB of LDS, one workgroup per compute unit)
// suits long walks; 1 (64 KiB, two workgroups per compute unit, so that one's start-up --
// descriptor, page ids, the first blocks' trip to HBM -- and its final combine hide behind
// the other's stream) suits launches whose workgroups walk only a few blocks each.
// (launched with 256 threads; the bound of 512 makes the compiler budget for two wavefronts
// per SIMD, i.e. at most 256 vector registers, all architectural: with more it parks the
// accumulators in AGPRs and copies them back and forth around every vector-ALU use)
template <int D, int STAGES>
__global__ void __launch_bounds__(2 * kThreads)
decode_kernel(const AttnArgs args) {
  using G = DecodeGeom<D, STAGES>;
  __shared__ __attribute__((aligned(1024))) char lds[G::kLdsBytes];

  const SeqDesc* descs = args.inline_descs;
  const SeqDesc sd = uniform(descs[find_seq_slot(descs, args.n_seq, blockIdx.x)]);
  // one row tile per sequence here, so a slot is just (KV head, split)
  const SlotItem it = decode_slot(blockIdx.x - sd.work_start, args.h_kv, sd.n_split, 1);
  if (!it.valid) return;
  const int kv_head = it.kv_head, split = it.split;

  const int gqa = args.h_q / args.h_kv;
  const int n_rows = sd.chunk_len * gqa;  // <= 32
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const int col = lane & 31, half = lane >> 5;

  RowBlock<D> rb;
  rb.init(fabsf(args.scale_log2), lane);
  const bool valid = col < n_rows;
  const int rr = valid ? col : (n_rows - 1);
  const int tok = rr / gqa;
  const int hq = kv_head * gqa + rr % gqa;
  const int kv_total = sd.kv_len;  // keys that exist
  rb.limit = min(sd.prefix_len + tok, kv_total - 1);
  {
    const unsigned flip = args.scale_log2 < 0.f ? 0x80008000u : 0u;
    const __bf16* qp = args.q + ((int64_t)(sd.q_row + tok) * args.h_q + hq) * D + half * 8;
#pragma unroll
    for (int sl = 0; sl < RowBlock<D>::kSlices; ++sl) {
      uint4 raw = make_uint4(0, 0, 0, 0);
      if (valid) raw = *reinterpret_cast<const uint4*>(qp + sl * 16);
      raw.x ^= flip; raw.y ^= flip; raw.z ^= flip; raw.w ^= flip;
      rb.q[sl] = __builtin_bit_cast(bf16x8, raw);
    }
  }

  // This workgroup's key range and its 32-key blocks.
  const int keys_needed = max(0, min(kv_total, sd.prefix_len + sd.chunk_len));  // last row's
  const int k_begin = split * sd.tiles_per_split * G::kSplitKeys;
  const int k_end = min(keys_needed, k_begin + sd.tiles_per_split * G::kSplitKeys);
  const int n_blocks = k_end > k_begin ? (k_end - k_begin + G::kBlockKeys - 1) / G::kBlockKeys : 0;
  const int unmasked_keys = max(0, min(kv_total, sd.prefix_len + 1));  // visible to every row
  const int last_page = (kv_total - 1) >> 4;
  ConstI32Ptr pt = (ConstI32Ptr)(args.page_table + sd.pt_off);

  const uint32_t ring_lds = lds_address(lds) + wave * (G::kStagesPerWave * G::kBlockBytes);
  const char* ring = lds + wave * (G::kStagesPerWave * G::kBlockBytes);

  // issue block b into stage st (both wave-uniform)
  auto issue = [&](int b, int st) {
    const int key0 = k_begin + b * G::kBlockKeys;
    const int pi = __builtin_amdgcn_readfirstlane(key0 >> 4);
    const int page0 = pt[pi];
    const int page1 = pt[min(pi + 1, last_page)];
    const uint32_t base = ring_lds + st * G::kBlockBytes;
    issue_block<D>(args, page0, page1, key0, kv_total, kv_head, base, base + G::kHalfBytes, lane);
  };
  // Walks this wavefront's blocks b0, b0+4, ... < b_end with two in flight.
  // Self-contained: starts and ends with no load in flight.  MASK applies the
  // per-row key limit (only the last blocks of a sequence need it).
  auto run_blocks = [&](int b0, int b_end, auto mask_tag) {
    constexpr bool MASK = decltype(mask_tag)::value;
    if (b0 < b_end) issue(b0, 0);
    if (STAGES == 2 && b0 + kWaves < b_end) issue(b0 + kWaves, 1);
    int st = 0;
    for (int b = b0; b < b_end; b += kWaves, st ^= (STAGES - 1)) {
      if (STAGES == 2 && b + kWaves < b_end)
        wait_vmcnt<G::kLoadsPerBlock>();  // the younger block may still fly
      else
        wait_vmcnt<0>();
      const char* base = ring + st * G::kBlockBytes;
      rb.template step<1, MASK>(base, base + G::kHalfBytes, k_begin + b * G::kBlockKeys, half);
      // every LDS read of the stage has returned (its data fed the matrix cores)
      if (b + STAGES * kWaves < b_end) issue(b + STAGES * kWaves, st);
    }
  };
  // blocks below n_unmasked are visible to every row; this wavefront's first block at or
  // above it is the smallest wave + 4i >= n_unmasked
  const int n_unmasked = min(n_blocks, max(0, unmasked_keys - k_begin) / G::kBlockKeys);
  const int first_masked = wave + ((max(0, n_unmasked - wave) + kWaves - 1) / kWaves) * kWaves;
  run_blocks(wave, n_unmasked, std::false_type{});
  run_blocks(first_masked, n_blocks, std::true_type{});

  // Combine the 4 wavefronts' (m, l, O) over their disjoint keys through LDS.
  const bool direct = sd.n_split == 1;
  float* o_base = direct ? args.out : args.part_o;
  float* l_base = direct ? args.lse : args.part_lse;
  const int64_t row_base =
      direct ? (int64_t)sd.out_row : (int64_t)sd.part_row + (int64_t)split * sd.chunk_len;
  __syncthreads();  // all rings are drained and read
  // (the buffer holds kCombineRows rows of every wavefront: 32 with the large ring, 16 with
  // the small one, whose launches then take two passes if they have more rows)
  constexpr int kCombineRows = STAGES == 2 ? 32 : 16;
  float* sm_o = reinterpret_cast<float*>(lds);           // [wave][kCombineRows][D]
  float* sm_ml = sm_o + kWaves * kCombineRows * D;       // [wave][kCombineRows][2]
  static_assert(kWaves * kCombineRows * (D + 2) * 4 <= G::kLdsBytes, "combine buffer fits");
  const float lt = rb.row_sum();
  for (int row0 = 0; row0 < n_rows; row0 += kCombineRows) {
    const int in_pass = col - row0;
    if (valid && in_pass >= 0 && in_pass < kCombineRows) {
      float* op = sm_o + (wave * kCombineRows + in_pass) * D + 4 * half;
#pragma unroll
      for (int db = 0; db < RowBlock<D>::kDBlocks; ++db)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          f32x4 v;
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] = rb.o[db][4 * i + j];
          *reinterpret_cast<f32x4*>(op + db * 32 + 8 * i) = v;
        }
      if (half == 0) {
        sm_ml[(wave * kCombineRows + in_pass) * 2 + 0] = rb.m;
        sm_ml[(wave * kCombineRows + in_pass) * 2 + 1] = lt;
      }
    }
    __syncthreads();
    const int rows_here = min(kCombineRows, n_rows - row0);
    for (int e = threadIdx.x; e < rows_here * (D / 4); e += kThreads) {
      const int rl = e / (D / 4);
      const int r = row0 + rl;
      const int d4 = e % (D / 4);
      float mw[kWaves], lw[kWaves], mm = -INFINITY;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        mw[w] = sm_ml[(w * kCombineRows + rl) * 2 + 0];
        lw[w] = sm_ml[(w * kCombineRows + rl) * 2 + 1];
        mm = fmaxf(mm, mw[w]);
      }
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
      float lt_all = 0.f;
      if (mm != -INFINITY) {
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
          const float a = fast_exp2(mw[w] - mm);
          lt_all += a * lw[w];
          const f32x4 ov =
              *reinterpret_cast<const f32x4*>(sm_o + (w * kCombineRows + rl) * D + d4 * 4);
          if (lw[w] > 0.f) acc += ov * a;
        }
      }
      const float inv = lt_all > 0.f ? 1.f / lt_all : 0.f;
      const int64_t orow = (row_base + r / gqa) * args.h_q + kv_head * gqa + r % gqa;
      *reinterpret_cast<f32x4*>(o_base + orow * D + d4 * 4) = acc * inv;
      if (d4 == 0) l_base[orow] = lt_all > 0.f ? (mm + fast_log2(lt_all)) * kLn2 : -INFINITY;
    }
    if (row0 + kCombineRows < n_rows) __syncthreads();  // before the next pass refills
  }
}

}  // namespace medha
