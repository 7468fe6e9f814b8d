// Row-split chunked-prefill attention kernel for gfx950 (paper section 3.1).
//
// A workgroup of NW wavefronts owns NW*32 query rows of one KV head's GQA group
// (row = (token, head-in-group), token-major) and walks 64-key tiles of the paged
// KV sequence.  Every wavefront owns 32 rows for the whole walk:
//     S^T = K Q^T      (MFMA 32x32x16 bf16, K from LDS, Q^T resident in registers)
//     online softmax   (a lane owns one row: statistics are lane-local)
//     O^T += V^T P^T   (MFMA, V^T through the transposing LDS read, P^T straight
//                       from the S^T accumulators)
// With two wavefronts per SIMD the matrix-core phase of one overlaps the softmax
// phase of the other.
//
// K/V tiles go HBM -> LDS directly (no registers) with asynchronous 16-byte
// global loads into a ring of NS stages, gathered page by page through the page
// table.  Each page row is 16*D*2 contiguous bytes, so every 1 KiB load
// instruction reads whole rows.  Rows are stored unpadded; bank conflicts are
// avoided by XOR-swizzling the 16-byte column index with the row index (one
// pattern for the 16-byte K reads, another for the 8-byte transposing V reads).
#pragma once

#include "common.h"

namespace medha {

template <int D>
struct Swz {
  static constexpr int kChunksPerRow = D / 8;  // 16-byte chunks per key row
  // K rows are read 16 bytes per lane by 16 consecutive rows at one logical chunk.
  __device__ static __forceinline__ int k(int row, int chunk) {
    return D == 128 ? (chunk ^ (row & 15)) : (chunk ^ ((row >> 1) & 7));
  }
  // V rows are read 8 bytes per lane: 4 consecutive rows x 64 bytes per half-wave.
  __device__ static __forceinline__ int v(int row, int chunk) {
    return D == 128 ? (chunk ^ ((row & 3) << 2)) : (chunk ^ (((row >> 1) & 1) << 2));
  }
};

// Asynchronous 16-byte-per-lane load HBM -> LDS: lane i's 16 bytes land at
// lds_uniform + 16*i (the LDS base travels in M0, so it is wave-uniform), the
// global address is per lane.  Completion is counted by vmcnt only.  Written by
// hand, like ring_barrier() below: the ring's ordering is enforced by explicit
// counter waits, whereas the compiler, when it sees such loads, drains the whole
// load queue before the next LDS read that might alias them.
__device__ __forceinline__ void async_load16(const void* gptr, uint32_t lds_addr_uniform) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
               :
               : "s"(lds_addr_uniform), "v"(gptr)
               : "m0", "memory");
}
// Same, with the global address split into a wave-uniform base (scalar registers)
// and a 32-bit per-lane byte offset: no vector-ALU address arithmetic per load.
__device__ __forceinline__ void async_load16(const void* base_uniform, uint32_t lane_off,
                                             uint32_t lds_addr_uniform) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_addr_uniform), "v"(lane_off), "s"(base_uniform)
               : "m0", "memory");
}

// Byte address of a __shared__ object inside the workgroup's LDS allocation.
__device__ __forceinline__ uint32_t lds_address(const void* p) {
  return (uint32_t)(uintptr_t)((__attribute__((address_space(3))) const char*)p);
}

// Workgroup barrier for the K/V ring: waits until at most N of this wavefront's
// vector-memory operations (the asynchronous tile loads) are still in flight,
// then meets the other wavefronts.  Written by hand because the generic
// barrier drains every outstanding load, which would serialise the ring.  The
// memory clobber keeps the compiler from moving LDS accesses across it.
template <int N>
__device__ __forceinline__ void ring_barrier() {
  static_assert(N >= 0 && N < 64, "vmcnt range");
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

template <int D, int NW>
struct TileGeom {
  static constexpr int kTileKeys = 64;
  static constexpr int kChunksPerRow = D / 8;
  static constexpr int kRowsPerInstr = 64 / kChunksPerRow;       // rows one wave-wide load covers
  static constexpr int kInstrPerTile = kTileKeys / kRowsPerInstr;  // per K (or V) tile
  static constexpr int kInstrPerWave = kInstrPerTile / NW;
  static constexpr int kRowsPerWave = kTileKeys / NW;              // 8 or 16: inside one page
  static constexpr int kTileBytes = kTileKeys * D * 2;             // K (or V) tile
  static constexpr int kLoadsPerWaveTile = 2 * kInstrPerWave;      // K and V
  static_assert(kInstrPerTile % NW == 0 && kInstrPerWave >= 1, "tile must divide over waves");
  static_assert(kRowsPerWave <= kPageSize, "a wave's rows of a tile stay inside one page");
};

// Id of the page holding this wavefront's rows of a tile.  The page table is
// read through the constant address space with a wave-uniform index, i.e. by a
// scalar load: it stays out of the vector-memory queue, which then holds nothing
// but the K/V tile loads that ring_barrier() counts.  Keys past the end are
// clamped to the last one: they are masked, but must be finite.
typedef const int32_t __attribute__((address_space(4))) * ConstI32Ptr;

template <int D, int NW>
__device__ __forceinline__ int tile_page(ConstI32Ptr pt, int tile, int kv_total, int wave) {
  using G = TileGeom<D, NW>;
  const int idx = min(tile * G::kTileKeys + wave * G::kRowsPerWave, kv_total - 1) >> 4;
  return pt[__builtin_amdgcn_readfirstlane(idx)];
}

// This wavefront's share of the asynchronous loads of a 64-key tile: which rows
// (all inside one page) and, per lane, which 16-byte chunk of which row.  The
// per-lane byte offsets inside the page are the same for every tile that lies
// wholly inside the sequence, so they are computed once.
template <int D, int NW>
struct TileLoader {
  using G = TileGeom<D, NW>;
  uint32_t k_off[G::kInstrPerWave];  // byte offset inside the (page, KV head) block
  uint32_t v_off[G::kInstrPerWave];
  int row0;                          // first row of the tile this wavefront loads (uniform)
  int r_in, pos;

  __device__ __forceinline__ void init(int wave, int lane) {
    row0 = wave * G::kRowsPerWave;
    r_in = lane / G::kChunksPerRow;
    pos = lane % G::kChunksPerRow;
#pragma unroll
    for (int j = 0; j < G::kInstrPerWave; ++j) {
      const int row = row0 + j * G::kRowsPerInstr + r_in;
      k_off[j] = (row & 15) * (D * 2) + Swz<D>::k(row, pos) * 16;
      v_off[j] = (row & 15) * (D * 2) + Swz<D>::v(row, pos) * 16;
    }
  }

  // page = id of the page holding rows row0.. of tile `tile` (see tile_page()).
  __device__ __forceinline__ void issue(const AttnArgs& args, int page, int tile, int kv_total,
                                        int kv_head, uint32_t k_stage, uint32_t v_stage) const {
    const int64_t page_off = ((int64_t)page * args.h_kv + kv_head) * (kPageSize * D * 2);
    const char* kp = reinterpret_cast<const char*>(args.k_pool) + page_off;  // wave-uniform
    const char* vp = reinterpret_cast<const char*>(args.v_pool) + page_off;
    if ((tile + 1) * G::kTileKeys <= kv_total) {
#pragma unroll
      for (int j = 0; j < G::kInstrPerWave; ++j) {
        const uint32_t lds_off = (row0 + j * G::kRowsPerInstr) * (D * 2);  // wave-uniform
        async_load16(kp, k_off[j], k_stage + lds_off);
        async_load16(vp, v_off[j], v_stage + lds_off);
      }
    } else {
      // last, ragged tile: keys past the end are clamped to the last one (masked, but finite)
#pragma unroll
      for (int j = 0; j < G::kInstrPerWave; ++j) {
        const int row = row0 + j * G::kRowsPerInstr + r_in;
        const int t = min(tile * G::kTileKeys + row, kv_total - 1);
        const uint32_t lds_off = (row0 + j * G::kRowsPerInstr) * (D * 2);
        async_load16(kp, (uint32_t)((t & 15) * (D * 2) + Swz<D>::k(row, pos) * 16),
                     k_stage + lds_off);
        async_load16(vp, (uint32_t)((t & 15) * (D * 2) + Swz<D>::v(row, pos) * 16),
                     v_stage + lds_off);
      }
    }
  }
};

// Softmax state and accumulators of one wavefront (32 query rows).
template <int D>
struct RowBlock {
  static constexpr int kSlices = D / 16;
  static constexpr int kDBlocks = D / 32;
  bf16x8 q[kSlices];
  f32x16 o[kDBlocks];
  float m;        // running maximum of scale_log2 * score
  float l;        // this lane's share of the running sum
  int limit;      // last visible key index of the lane's row
  float scale_log2;
  // per-lane LDS byte offsets of the operand reads inside a stage
  int k_off[kSlices];
  int v_off[kDBlocks];

  __device__ __forceinline__ void init(float scale, int lane) {
    scale_log2 = scale;
    m = -INFINITY;
    l = 0.f;
#pragma unroll
    for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[db][e] = 0.f;
    const int col = lane & 31, half = lane >> 5;
#pragma unroll
    for (int sl = 0; sl < kSlices; ++sl)
      k_off[sl] = col * (D * 2) + Swz<D>::k(col, 2 * sl + half) * 16;
    const int l16 = lane & 15, dhalf = (lane >> 4) & 1;
    const int vrow = 4 * half + (l16 >> 2);
#pragma unroll
    for (int db = 0; db < kDBlocks; ++db) {
      const int chunk = 4 * db + 2 * dhalf + ((l16 & 3) >> 1);
      v_off[db] = vrow * (D * 2) + Swz<D>::v(vrow, chunk) * 16 + (l16 & 1) * 8;
    }
  }

  // V^T operands of 16-key slice g (keys 16g .. 16g+15 of the tile) for all D/32
  // head-dim blocks: for this lane's half, keys 16g + 4*half + {0..3} and the
  // same + 8, through the transposing LDS read of row-major V.
  __device__ __forceinline__ void read_v_slice(const char* v_lds, int g,
                                               bf16x8 (&vop)[kDBlocks]) const {
    const char* vrow = v_lds + g * 16 * (D * 2);
#pragma unroll
    for (int db = 0; db < kDBlocks; ++db) {
      const char* vp = vrow + v_off[db];
      const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (s16x4 __attribute__((address_space(3)))*)(vp));
      const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (s16x4 __attribute__((address_space(3)))*)(vp + 8 * (D * 2)));
      vop[db] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7));
    }
  }

  // One tile of NKB blocks of 32 keys (2*NKB slices of 16 keys).  The instruction
  // order is laid out by hand as a software pipeline, and fenced so that it
  // stays that way: LDS operand reads are issued two steps before the MFMAs that
  // consume them (their latency would otherwise stall every MFMA), and the
  // exponentials of slice g+1 sit between the MFMAs of slice g.
  //   S^T = K Q^T:    A = 32 keys x 16 dims from LDS, B = Q^T from registers.
  //   softmax:        mask on diagonal tiles, row maximum (lane-local + one
  //                   half-wave exchange), accumulator rescale only if some
  //                   row's maximum moved, p = exp2(s*scale_log2 - m), row sum.
  //   O^T += V^T P^T: B = P^T slice taken from the S^T registers of the same
  //                   keys (bf16, round to nearest even), A = V^T slice.
  // key0 = sequence index of the tile's first key.
  template <int NKB, bool MASK>
  __device__ __forceinline__ void step(const char* k_lds, const char* v_lds, int key0, int half) {
    constexpr int kGroups = 2 * NKB;
    bf16x8 vop[2][kDBlocks];
    read_v_slice(v_lds, 0, vop[0]);
    read_v_slice(v_lds, 1, vop[1]);

    f32x16 s[NKB];
    {
      bf16x8 a[3][NKB];
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
        for (int e = 0; e < 16; ++e) s[kb][e] = 0.f;
        // rows kb*32 + col: the swizzle only looks at row bits below 32
        a[0][kb] = *reinterpret_cast<const bf16x8*>(k_lds + kb * 32 * (D * 2) + k_off[0]);
        a[1][kb] = *reinterpret_cast<const bf16x8*>(k_lds + kb * 32 * (D * 2) + k_off[1]);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int sl = 0; sl < kSlices; ++sl) {
        if (sl + 2 < kSlices) {
#pragma unroll
          for (int kb = 0; kb < NKB; ++kb)
            a[(sl + 2) % 3][kb] =
                *reinterpret_cast<const bf16x8*>(k_lds + kb * 32 * (D * 2) + k_off[sl + 2]);
        }
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
          s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[sl % 3][kb], q[sl], s[kb], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    }

    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        if (MASK) {
          const int t = key0 + kb * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
          s[kb][e] = (t <= limit) ? s[kb][e] : -INFINITY;
        }
        mx = fmaxf(mx, s[kb][e]);
      }
    mx = max_halves(mx) * scale_log2;  // scale_log2 >= 0
    // m is the reference point of the exponentials, not necessarily the true running
    // maximum: it is moved up (and the accumulators rescaled) only when some row's maximum
    // exceeds it by more than kRescaleSlack, so that p <= 2^kRescaleSlack.  The common factor
    // cancels in O = acc / l and LSE = m + log2(l); after the first few tiles of a long
    // sequence the rescale practically never runs.
    if (__any(mx > m + kRescaleSlack)) {
      const float m_new = fmaxf(m, mx);
      // a row that has seen no key yet keeps m = -inf: nothing to rescale
      const float alpha = (m_new == -INFINITY) ? 1.f : fast_exp2(m - m_new);
      l *= alpha;
#pragma unroll
      for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[db][e] *= alpha;
      m = m_new;
    }
    // exponentiate against 0 while the row has no key
    const float m_use = (MASK && m == -INFINITY) ? 0.f : m;

    float ls = 0.f;
    // P^T operand of slice g: elements 8*(g%2) .. +7 of S^T block g/2.  The row sum is
    // taken over the fp32 values (a sum of the bf16-rounded ones, two per instruction with
    // the bf16 dot product, costs up to 4e-3 in LSE on short rows).
    auto probs = [&](int g) -> bf16x8 {
      f32x8 pe;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float sv = s[g >> 1][8 * (g & 1) + e];
        pe[e] = fast_exp2(__builtin_fmaf(sv, scale_log2, -m_use));
        // the select is also right when scale_log2 == 0 (-inf * 0 is not a number)
        if (MASK) pe[e] = (sv == -INFINITY) ? 0.f : pe[e];
        ls += pe[e];
      }
      return __builtin_convertvector(pe, bf16x8);
    };
    bf16x8 pg[2];
    pg[0] = probs(0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int g = 0; g < kGroups; ++g) {
      if (g + 1 < kGroups) pg[(g + 1) & 1] = probs(g + 1);
#pragma unroll
      for (int db = 0; db < kDBlocks; ++db)
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop[g & 1][db], pg[g & 1], o[db], 0, 0, 0);
      if (g + 2 < kGroups) read_v_slice(v_lds, g + 2, vop[g & 1]);
      __builtin_amdgcn_sched_barrier(0);
    }
    l += ls;
  }
};

// The descriptor is the same for the whole workgroup: say so, so that everything
// derived from it lives in scalar registers.
__device__ __forceinline__ SeqDesc uniform(const SeqDesc& d) {
  SeqDesc u;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)(uint64_t)d.pt_off);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)d.pt_off >> 32));
  u.pt_off = (int64_t)(((uint64_t)hi << 32) | lo);
  u.q_row = __builtin_amdgcn_readfirstlane(d.q_row);
  u.out_row = __builtin_amdgcn_readfirstlane(d.out_row);
  u.chunk_len = __builtin_amdgcn_readfirstlane(d.chunk_len);
  u.prefix_len = __builtin_amdgcn_readfirstlane(d.prefix_len);
  u.work_start = __builtin_amdgcn_readfirstlane(d.work_start);
  u.n_row_tiles = __builtin_amdgcn_readfirstlane(d.n_row_tiles);
  u.n_split = __builtin_amdgcn_readfirstlane(d.n_split);
  u.tiles_per_split = __builtin_amdgcn_readfirstlane(d.tiles_per_split);
  u.part_row = __builtin_amdgcn_readfirstlane(d.part_row);
  u.row_rank = __builtin_amdgcn_readfirstlane(d.row_rank);
  return u;
}

// Largest i with descs[i].work_start <= slot.
__device__ __forceinline__ int find_seq_slot(const SeqDesc* descs, int n_seq, int slot) {
  int lo = 0, hi = n_seq - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (descs[mid].work_start <= slot) lo = mid; else hi = mid - 1;
  }
  return lo;
}

template <int D, int NW, int NS>
struct PrefillShape {
  static constexpr int kRowsPerWg = NW * 32;
  static constexpr int kStageBytes = 2 * TileGeom<D, NW>::kTileBytes;  // K tile then V tile
  static constexpr int kLdsBytes = NS * kStageBytes;
};

// The ring: NS stages of (K tile, V tile), contiguous from `base`.
struct Ring {
  char* base;         // for operand reads
  uint32_t lds_addr;  // the same place as an LDS byte address, for the tile loads
};

// Walks tiles [kt_a, kt_b) through the NS-stage ring.  Self-contained: starts
// with no load in flight and ends with none.  Tile loads run NS-1 tiles ahead.
template <int D, int NW, int NS, bool MASK>
__device__ __forceinline__ void run_tiles(RowBlock<D>& rb, const AttnArgs& args, ConstI32Ptr pt,
                                          int kt_a, int kt_b, int kv_total, int kv_head,
                                          const Ring& ring, const TileLoader<D, NW>& ld,
                                          int wave, int lane) {
  using G = TileGeom<D, NW>;
  constexpr int kStage = PrefillShape<D, NW, NS>::kStageBytes;
  constexpr int kAhead = NS - 1;  // tiles in flight beyond the current one, plus one
  if (kt_a >= kt_b) return;
  const int half = lane >> 5;
  const int last = kt_b - 1;
  // prologue: tiles kt_a .. kt_a+NS-2 (clamped: a repeated tile is loaded again, harmlessly)
#pragma unroll
  for (int s = 0; s < kAhead; ++s) {
    const int tile = min(kt_a + s, last);
    const int page = tile_page<D, NW>(pt, tile, kv_total, wave);
    ld.issue(args, page, tile, kv_total, kv_head, ring.lds_addr + s * kStage,
             ring.lds_addr + s * kStage + G::kTileBytes);
  }
  // page id of the next tile to issue, fetched one step ahead of its use
  int page_next = tile_page<D, NW>(pt, min(kt_a + kAhead, last), kv_total, wave);
  for (int kt = kt_a; kt < kt_b; kt += NS) {
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int cur = kt + s;
      if (cur < kt_b) {
        // this wavefront's loads of tile `cur` have landed (the younger tiles may fly); after
        // the barrier everyone's have, and everyone is done with the stage refilled next
        ring_barrier<(kAhead - 1) * G::kLoadsPerWaveTile>();
        const uint32_t nxt = ring.lds_addr + ((s + kAhead) % NS) * kStage;
        ld.issue(args, page_next, min(cur + kAhead, last), kv_total, kv_head, nxt,
                 nxt + G::kTileBytes);
        page_next = tile_page<D, NW>(pt, min(cur + kAhead + 1, last), kv_total, wave);
        const char* st = ring.base + s * kStage;
        rb.template step<2, MASK>(st, st + G::kTileBytes, cur * G::kTileKeys, half);
      }
    }
  }
  ring_barrier<0>();
}

// (the launch bound is 512 also for the 4-wavefront variant: it makes the compiler budget
// for two wavefronts per SIMD, at most 256 vector registers, all architectural)
template <int D, int NW, int NS>
__global__ void __launch_bounds__(512) prefill_kernel(const AttnArgs args) {
  using Shape = PrefillShape<D, NW, NS>;
  __shared__ __attribute__((aligned(1024))) char lds[Shape::kLdsBytes];
  const Ring stages{lds, lds_address(lds)};

  const SeqDesc* descs = args.descs ? args.descs : args.inline_descs;
  const SeqDesc sd = uniform(descs[find_seq_slot(descs, args.n_seq, blockIdx.x)]);

  const SlotItem it =
      decode_slot(blockIdx.x - sd.work_start, args.h_kv, sd.n_split, sd.n_row_tiles);
  if (!it.valid) return;
  const int row_tile = it.row_tile, kv_head = it.kv_head, split = it.split;

  const int gqa = args.h_q / args.h_kv;
  const int n_rows = sd.chunk_len * gqa;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const int col = lane & 31, half = lane >> 5;

  RowBlock<D> rb;
  rb.init(fabsf(args.scale_log2), lane);

  const int wg_row0 = row_tile * Shape::kRowsPerWg;
  const int r = wg_row0 + wave * 32 + col;
  const bool valid = r < n_rows;
  const int rr = valid ? r : (n_rows - 1);
  const int tok = rr / gqa;
  const int hq = kv_head * gqa + rr % gqa;
  rb.limit = sd.prefix_len + tok;
  {
    // a negative scale is folded into the sign of Q (exact), so the kernel's scale is >= 0
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

  // Keys this row tile needs: up to the limit of its last row.
  const int last_row = min(n_rows, wg_row0 + Shape::kRowsPerWg) - 1;
  const int keys_needed = sd.prefix_len + last_row / gqa + 1;
  const int kv_total = sd.prefix_len + sd.chunk_len;
  const int tiles_needed = (keys_needed + 63) / 64;
  const int kt_begin = split * sd.tiles_per_split;
  const int kt_end = min(tiles_needed, kt_begin + sd.tiles_per_split);
  // tiles below kt_mid are fully visible to every row of the workgroup
  const int unmasked_keys = sd.prefix_len + min(wg_row0, n_rows - 1) / gqa + 1;
  const int kt_mid = max(kt_begin, min(kt_end, unmasked_keys / 64));

  ConstI32Ptr pt = (ConstI32Ptr)(args.page_table + sd.pt_off);
  TileLoader<D, NW> loader;
  loader.init(wave, lane);
  run_tiles<D, NW, NS, false>(rb, args, pt, kt_begin, kt_mid, kv_total, kv_head, stages, loader,
                              wave, lane);
  run_tiles<D, NW, NS, true>(rb, args, pt, kt_mid, kt_end, kv_total, kv_head, stages, loader,
                             wave, lane);

  const bool direct = sd.n_split == 1;
  float* o_base = direct ? args.out : args.part_o;
  float* l_base = direct ? args.lse : args.part_lse;
  const int64_t row_base =
      direct ? (int64_t)sd.out_row : (int64_t)sd.part_row + (int64_t)split * sd.chunk_len;
  const float lt = sum_halves(rb.l);
  const float inv = lt > 0.f ? 1.f / lt : 0.f;
  const float lse = lt > 0.f ? (rb.m + fast_log2(lt)) * kLn2 : -INFINITY;
  if (valid) {
    const int64_t orow = (row_base + tok) * args.h_q + hq;
    float* op = o_base + orow * D + 4 * half;
#pragma unroll
    for (int db = 0; db < RowBlock<D>::kDBlocks; ++db)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        f32x4 v;
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = rb.o[db][4 * i + j] * inv;
        *reinterpret_cast<f32x4*>(op + db * 32 + 8 * i) = v;
      }
    if (half == 0) l_base[orow] = lse;
  }
}

}  // namespace medha
