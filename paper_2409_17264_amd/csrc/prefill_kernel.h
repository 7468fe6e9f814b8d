// Row-split chunked-prefill attention kernel for gfx950 (paper section 3.1).
//
// A workgroup of NW wavefronts owns NW*32 query rows of one KV head's GQA group
// (row = (token, head-in-group), token-major) and walks 64-key tiles of the paged
// KV sequence.  Every wavefront owns 32 rows for the whole walk:
//     S^T = K Q^T      (MFMA 32x32x16 bf16, K from LDS, Q^T resident in registers)
//     online softmax   (a lane owns one row: statistics are lane-local)
//     O^T += V^T P^T   (MFMA, V^T through the transposing LDS read, P^T straight
//                       from the S^T accumulators)
// The tile walk is software-pipelined inside every wavefront: the S^T MFMAs of tile
// j+1 and the O^T MFMAs of tile j form one instruction stream with the softmax
// arithmetic of tile j spread between them (RowBlock::fused), because the matrix
// pipe and the vector ALU share an issue port and neither should wait for the other.
//
// K/V tiles go HBM -> LDS directly (no registers) with asynchronous 16-byte
// global loads into a ring of NS stages (K tiles in its low half, V tiles in its
// high half), gathered page by page through the page table.  Each page row is 16*D*2 contiguous bytes, so every 1 KiB load
// instruction reads whole rows.  Rows are stored unpadded; bank conflicts are
// avoided by XOR-swizzling the 16-byte column index with the row index (one
// pattern for the 16-byte K reads, another for the 8-byte transposing V reads).
#pragma once

#include <type_traits>
#include <utility>

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
// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), in order.
template <int... Is, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, Is...>, F& f) {
  (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

template <int D>
struct RowBlock {
  static constexpr int kSlices = D / 16;
  static constexpr int kDBlocks = D / 32;
  bf16x8 q[kSlices];
  f32x16 o[kDBlocks];
  float m;        // reference point of the exponentials (log2 domain), see update_reference()
  float l;        // kSpecShare * (this lane's share of the running sum), see add_to_sum()
  int limit;      // last visible key index of the lane's row
  float scale_log2;
  // per-lane LDS byte offsets of the operand reads inside a stage
  int k_off[kSlices];
  int v_off[kDBlocks];

  // v_bias: constant added to the V^T read offsets (the caller subtracts it from the V tile
  // pointers it passes; with it the pointers' constant parts fit the LDS instructions'
  // 16-bit immediate offset and cost no address arithmetic).
  __device__ __forceinline__ void init(float scale, int lane, int v_bias = 0) {
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
      v_off[db] = vrow * (D * 2) + Swz<D>::v(vrow, chunk) * 16 + (l16 & 1) * 8 + v_bias;
      asm volatile("" : "+v"(v_off[db]));  // opaque: stays one register, constants stay immediates
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

  // A tile of NKB blocks of 32 keys (2*NKB slices of 16 keys) is two phases:
  //   qk():         S^T = K Q^T.  A = 32 keys x 16 dims from LDS, B = Q^T from registers.
  //   softmax_pv(): mask on diagonal tiles, row maximum (lane-local + one half-wave
  //                 exchange), p = exp2(s*scale_log2 - m), row sum, then
  //                 O^T += V^T P^T with B = P^T slice taken from the S^T registers
  //                 of the same keys (bf16, round to nearest even), A = V^T slice.
  // The instruction order of both is laid out by hand as a software pipeline and
  // fenced so that it stays that way: LDS operand reads are issued a few steps
  // before the MFMAs that consume them (their latency would otherwise stall every
  // MFMA), and exponentials sit between MFMAs.  fused() below interleaves the
  // qk() of the next tile with the softmax_pv() of the current one.
  template <int NKB>
  __device__ __forceinline__ void qk(const char* k_lds, f32x16 (&s)[NKB]) const {
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

  // Moves the reference point m of the exponentials up to the row maximum of the
  // (masked) scores just seen, if that exceeds it, and rescales the accumulators.
  // m is the point the exponentials are taken against, not necessarily the running
  // maximum: unmasked tiles are exponentiated against it as it stands (see fused()),
  // and any common factor cancels in O = acc / l and LSE = m + log2(l).  Whenever this
  // routine runs, the largest probability of the row so far becomes exactly 1 and so
  // loses nothing in the bf16 rounding of P, which is what rows carried by one or two
  // keys need.  Returns the value to exponentiate against (0 while the row has seen
  // no key).
  template <bool MASK>
  __device__ __forceinline__ float update_reference(float mx_raw) {
    const float mx = max_halves(mx_raw) * scale_log2;  // scale_log2 >= 0
    if (__any(mx > m)) {
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
    return (MASK && m == -INFINITY) ? 0.f : m;
  }

  // One probability: exp2(s*scale_log2 - m_use), 0 for a masked score (the select is
  // also right when scale_log2 == 0, where -inf * 0 is not a number).
  template <bool MASK>
  __device__ __forceinline__ float prob(float sv, float m_use) const {
    const float p = fast_exp2(__builtin_fmaf(sv, scale_log2, -m_use));
    return (MASK && sv == -INFINITY) ? 0.f : p;
  }

  // vop holds the V^T operands of slices 0 and 1, already requested by the caller.
  // key0 = sequence index of the tile's first key.
  template <int NKB, bool MASK>
  __device__ __forceinline__ void softmax_pv(f32x16 (&s)[NKB], const char* v_lds,
                                             bf16x8 (&vop)[2][kDBlocks], int key0, int half) {
    constexpr int kGroups = 2 * NKB;
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
    const float m_use = update_reference<MASK>(mx);

    float ls = 0.f;
    // P^T operand of slice g: elements 8*(g%2) .. +7 of S^T block g/2.  The row sum is
    // taken over the fp32 values (a sum of the bf16-rounded ones, two per instruction with
    // the bf16 dot product, costs up to 4e-3 in LSE on short rows).
    auto probs = [&](int g) -> bf16x8 {
      f32x8 pe;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        pe[e] = prob<MASK>(s[g >> 1][8 * (g & 1) + e], m_use);
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
    add_to_sum(ls);
  }

  // One whole tile: the first V^T operands are requested ahead of phase 1.
  template <int NKB, bool MASK>
  __device__ __forceinline__ void step(const char* k_lds, const char* v_lds, int key0, int half) {
    bf16x8 vop[2][kDBlocks];
    read_v_slice(v_lds, 0, vop[0]);
    read_v_slice(v_lds, 1, vop[1]);
    f32x16 s[NKB];
    qk<NKB>(k_lds, s);
    softmax_pv<NKB, MASK>(s, v_lds, vop, key0, half);
  }

  // Steady state of the 64-key tile walk: softmax_pv() of the current tile (scores
  // sc, V tile v_cur, first key key0) and qk() of the next tile (K tile k_next, scores
  // into sn) as ONE stream of kSlots slots.  Slot i holds one MFMA -- first the
  // next tile's S^T = K Q^T, then the current tile's O^T += V^T P^T, slice by slice --
  // the LDS read of the operand of slot i+3, and a share of the current tile's softmax
  // arithmetic, spread so that every slice's P^T is complete before its MFMAs.  The
  // vector ALU is the scarce unit here (an exponential costs two issue slots, and the
  // matrix instructions go through the same issue port), so the count of its
  // instructions per tile decides the speed.
  //
  // Tiles that every row sees in full (MASK false) are therefore exponentiated
  // SPECULATIVELY against the reference point m as it stands, without looking for the
  // row maximum first.  What the speculation must not do is round a probability that
  // carries a large share of its row: P goes to the matrix cores as bf16 (relative
  // rounding error up to 2^-8), the row sum is taken over the unrounded values, so the
  // error of one key's weight reaches O undamped unless that probability is exactly 1
  // (the row maximum, taken against itself) or small next to the row sum.  The
  // speculation is therefore checked on the row sums, twice per tile and before any
  // MFMA consumes the probabilities in question: the lane's sum over the two slices
  // just exponentiated (all p >= 0, so it bounds each of them; an overflow to +inf or a
  // NaN shows as well) must not exceed kSpecShare times the lane's sum so far.  The
  // lane keeps its sum pre-multiplied by kSpecShare (a power of two: exact), so the
  // check is one comparison of two registers.  A failed check takes the exact route for
  // those two slices -- maximum, move of the reference point, rescale, new
  // probabilities -- and evens out the sums of the two lanes that share a row (a lane
  // whose keys so far happen to weigh little would otherwise keep failing).  Keys that
  // bring a sizeable share of their row take that route; everything else -- nearly all
  // of a long walk -- passes.  While the sum is still small (the head of a walk) every
  // check would fail: those tiles do not speculate at all (SPEC false, see run_tiles()).
  // Diagonal tiles (MASK true) always take the exact route.
  static constexpr float kSpecShare = 1.f / 16.f;

  __device__ __forceinline__ void add_to_sum(float ls) { l = __builtin_fmaf(ls, kSpecShare, l); }
  // The row's sum of probabilities relative to the reference point (both lanes of the row).
  __device__ __forceinline__ float row_sum() const { return sum_halves(l) * (1.f / kSpecShare); }

  // Exact recomputation of slices 2*KB and 2*KB+1 (score block KB) after a failed check.
  template <int KB>
  __device__ __forceinline__ void respeculate(const f32x16 (&sc)[2], uint32_t (&pw)[4][4], float& ls) {
    float mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sc[KB][e]);
    const float m_use = update_reference<false>(mx);
    ls = 0.f;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      f32x8 pe;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        pe[e] = prob<false>(sc[KB][8 * h + e], m_use);
        ls += pe[e];
      }
      const uint4 w = __builtin_bit_cast(uint4, __builtin_convertvector(pe, bf16x8));
      pw[2 * KB + h][0] = w.x; pw[2 * KB + h][1] = w.y;
      pw[2 * KB + h][2] = w.z; pw[2 * KB + h][3] = w.w;
    }
  }

  //
  // QK false leaves the next tile out (the walk's last tile): the same slots without
  // their K reads and S^T MFMAs; k_next and sn are not touched.  SPEC false takes the
  // exact route (row maximum first) also on an unmasked tile: for the first tiles of a
  // walk, whose speculation would fail anyway, it is the cheaper of the two.
  template <bool MASK, bool QK = true, bool SPEC = true>
  __device__ __forceinline__ void fused(const char* k_next, const char* v_cur, f32x16 (&sc)[2],
                                        f32x16 (&sn)[2], int key0, int half) {
    constexpr bool kSpec = SPEC && !MASK;
    constexpr int kQk = 2 * kSlices;       // MFMAs of the next tile's S^T
    constexpr int kPv = 4 * kDBlocks;      // MFMAs of the current tile's O^T
    constexpr int kSlots = kQk + kPv;
    constexpr int kMaxSlots = kSpec ? 0 : kSlots / 8;  // slots that share the row maximum
    constexpr int kSpan = 3 * kSlots / 16; // slots over which a slice's exponentials spread
    // slice g: exponentials in slots [kMaxSlots + g*kSpan, +kSpan), MFMAs from kQk + g*kDBlocks
    static_assert(kMaxSlots + 4 * kSpan <= kQk + 3 * kDBlocks, "P^T ready before its MFMAs");
    // the speculation checks close slots 2*kSpan-1 and 4*kSpan-1
    static_assert(2 * kSpan <= kQk && 4 * kSpan <= kQk + 2 * kDBlocks, "checked before consumed");
    bf16x8 ka[4], va[4];
    uint32_t pw[4][4];  // P^T operands of the 4 slices as packed bf16 pairs
    float mx = -INFINITY, m_use = m, ls = 0.f;
    float pe_prev = 0.f;

    auto read_operand = [&](int i) {
      if (i < kQk) {
        if (QK)
          ka[i & 3] = *reinterpret_cast<const bf16x8*>(k_next + (i & 1) * 32 * (D * 2) + k_off[i >> 1]);
      } else if (i < kSlots) {
        const int j = i - kQk, g = j / kDBlocks, db = j % kDBlocks;
        const char* vp = v_cur + g * 16 * (D * 2) + v_off[db];
        const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (s16x4 __attribute__((address_space(3)))*)(vp));
        const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (s16x4 __attribute__((address_space(3)))*)(vp + 8 * (D * 2)));
        va[i & 3] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7));
      }
    };
    read_operand(0);
    read_operand(1);
    read_operand(2);
    if (QK) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e) sn[kb][e] = 0.f;
    }
    __builtin_amdgcn_sched_barrier(0);

    auto slot = [&](auto slot_index) {
      constexpr int i = decltype(slot_index)::value;
      // The wavefront's issue priority falls as it advances through the tile (3, 2, 1, 0 by
      // quarters).  Two wavefronts share a SIMD and meet at a barrier after every tile; with
      // equal priorities the arbiter serves the older one first, which then finishes its
      // tile early and idles at the barrier (measured: a quarter of its time) while the
      // other runs on alone -- and one wavefront alone cannot keep the matrix pipe full.
      // This way whichever is behind wins the arbitration and both arrive together.
      if constexpr (i % (kSlots / 4) == 0) __builtin_amdgcn_s_setprio(3 - i / (kSlots / 4));
      read_operand(i + 3);
      if constexpr (i < kQk) {
        if constexpr (QK)
          sn[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[i & 3], q[i >> 1], sn[i & 1], 0, 0, 0);
      } else {
        constexpr int j = i - kQk, g = j / kDBlocks, db = j % kDBlocks;
        const uint4 w = make_uint4(pw[g][0], pw[g][1], pw[g][2], pw[g][3]);
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[i & 3], __builtin_bit_cast(bf16x8, w),
                                                        o[db], 0, 0, 0);
      }
      // this slot's share of the softmax of the current tile
      if constexpr (!kSpec && i < kMaxSlots) {
        constexpr int per = 32 / (kSpec ? 1 : kMaxSlots);
#pragma unroll
        for (int f = i * per; f < (i + 1) * per; ++f) {
          if (MASK) {
            const int t = key0 + (f >> 4) * 32 + 8 * ((f & 15) >> 2) + 4 * half + (f & 3);
            sc[f >> 4][f & 15] = (t <= limit) ? sc[f >> 4][f & 15] : -INFINITY;
          }
          mx = fmaxf(mx, sc[f >> 4][f & 15]);
        }
      }
      if constexpr (!kSpec && i == kMaxSlots) m_use = update_reference<MASK>(mx);
      if constexpr (i >= kMaxSlots && i < kMaxSlots + 4 * kSpan) {
        constexpr int g = (i - kMaxSlots) / kSpan, r = (i - kMaxSlots) % kSpan;
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if ((e * kSpan) / 8 == r) {
            const float pe = prob<MASK>(sc[g >> 1][8 * (g & 1) + e], m_use);
            // (the first term after a check starts the sum: no addition to zero)
            if (kSpec && (g & 1) == 0 && e == 0) ls = pe; else ls += pe;
            if (e & 1) {
              const f32x2 pair = {pe_prev, pe};
              pw[g][e >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pair, bf16x2));
            } else {
              pe_prev = pe;
            }
          }
      }
      asm volatile("" : "+v"(ls));  // keeps the additions in their slots
      if constexpr (kSpec && (i == 2 * kSpan - 1 || i == 4 * kSpan - 1)) {
        // ls covers the two slices just finished
        if (__builtin_expect(__any(!(ls <= l)), 0)) {
          respeculate<(i == 2 * kSpan - 1) ? 0 : 1>(sc, pw, ls);
          m_use = m;
          add_to_sum(ls);
          l = 0.5f * sum_halves(l);
          ls = 0.f;
        }
        // (one common addition after the branch: with an addition on each side of it the
        // register allocation of the whole loop degrades badly)
        add_to_sum(ls);
        ls = 0.f;
      }
      __builtin_amdgcn_sched_barrier(0);
    };
    static_for<kSlots>(slot);
    if (!kSpec) add_to_sum(ls);  // (the speculative route adds at its checks)
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
  u.kv_len = __builtin_amdgcn_readfirstlane(d.kv_len);
  u.reserved = 0;
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

// Tiles at the head of an unmasked walk that take the exact route without speculating
// first (a multiple of the ring's stage count).  Measured on walks of 65 to 4100 tiles:
// 24 to 32 is best; 8 and 12 leave failed checks behind, with every tile exact the long
// walks take 4 % longer.
constexpr int kWarmTiles = 24;

// The ring: NS stages of (K tile, V tile), contiguous from `base`.
struct Ring {
  char* base;         // for operand reads
  uint32_t lds_addr;  // the same place as an LDS byte address, for the tile loads
};

// Walks tiles [kt_a, kt_b) through the 4-stage ring.  Self-contained: starts with
// no load in flight and ends with none.
//
// Iteration `cur` runs RowBlock::fused(): the softmax and P*V of tile cur together
// with the Q*K^T of tile cur+1, whose scores it hands to the next iteration in
// registers (two score sets, used alternately).  So at the barrier that opens
// iteration cur, tile cur+1 must have landed, tile cur+2 is in flight, and tile cur+3
// is issued into the stage of tile cur-1, which everybody left at that barrier.
template <int D, int NW, int NS, bool MASK>
__device__ __forceinline__ void run_tiles(RowBlock<D>& rb, const AttnArgs& args, ConstI32Ptr pt,
                                          int kt_a, int kt_b, int kv_total, int kv_head,
                                          const Ring& ring, const TileLoader<D, NW>& ld,
                                          int wave, int lane) {
  using G = TileGeom<D, NW>;
  static_assert(NS == 4, "stages: tile cur, cur+1, cur+2 (in flight), cur+3 (being issued)");
  static_assert(kWarmTiles % NS == 0, "the walk's head is a whole number of ring rounds");
  constexpr int kTile = G::kTileBytes;  // K tiles fill the low half of the ring, V tiles the high
  if (kt_a >= kt_b) return;
  const int half = lane >> 5;
  const int last = kt_b - 1;
  // prologue: tiles kt_a .. kt_a+2 (clamped: a repeated tile is loaded again, harmlessly)
#pragma unroll
  for (int s = 0; s < 3; ++s) {
    const int tile = min(kt_a + s, last);
    const int page = tile_page<D, NW>(pt, tile, kv_total, wave);
    ld.issue(args, page, tile, kv_total, kv_head, ring.lds_addr + s * kTile,
             ring.lds_addr + (NS + s) * kTile);
  }
  // page id of the next tile to issue
  int page_next = tile_page<D, NW>(pt, min(kt_a + 3, last), kv_total, wave);
  f32x16 s0[2], s1[2];  // scores of the even / odd tiles (counted from kt_a)
  ring_barrier<2 * G::kLoadsPerWaveTile>();  // tile kt_a has landed, for everyone
  rb.template qk<2>(ring.base, s0);
  if (!MASK) {
    float mx = -INFINITY;
#pragma unroll
    for (int f = 0; f < 32; ++f) mx = fmaxf(mx, s0[f >> 4][f & 15]);
    rb.template update_reference<false>(mx);
  }
  // One group of NS iterations starting at tile kt (stage numbers are compile-time).
  auto group = [&](int kt, auto spec) {
    constexpr bool kSpeculate = decltype(spec)::value;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int cur = kt + s;
      if (cur < last) {
        // this wavefront's loads of tile cur+1 have landed (tile cur+2 may fly); after the
        // barrier everyone's have, and everyone is done with the stage refilled next
        ring_barrier<G::kLoadsPerWaveTile>();
        asm volatile("" : "+s"(page_next));  // the page id is first needed here, not before
        const uint32_t nxt = ring.lds_addr + ((s + 3) % NS) * kTile;
        ld.issue(args, page_next, min(cur + 3, last), kv_total, kv_head, nxt, nxt + NS * kTile);
        const char* k_next = ring.base + ((s + 1) % NS) * kTile;
        const char* v_cur = ring.base + s * kTile;  // + the bias in rb.v_off
        if (s & 1)
          rb.template fused<MASK, true, kSpeculate>(k_next, v_cur, s1, s0, cur * G::kTileKeys,
                                                    half);
        else
          rb.template fused<MASK, true, kSpeculate>(k_next, v_cur, s0, s1, cur * G::kTileKeys,
                                                    half);
        // The scalar load of the next page id goes HERE, after the tile's last LDS read has
        // been consumed and before the barrier: scalar loads and LDS reads share one
        // counter and scalar loads return out of order, so with one in flight every wait for
        // an LDS operand becomes a wait for everything -- a stall of a scalar-load latency in
        // front of the tile's first MFMA.  Here its latency hides behind the barrier.
        __builtin_amdgcn_sched_barrier(0);
        page_next = tile_page<D, NW>(pt, min(cur + 4, last), kv_total, wave);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  int kt = kt_a;
  if constexpr (!MASK) {
    // The speculation check of fused() cannot pass before a lane's sum is 16 times what two
    // slices bring: not in the first 8 tiles of a walk of diffuse rows, and with 64 lanes
    // voting and the odd large score, rarely in the first twenty.  A failed check costs a
    // multiple of what the row maximum costs when it is taken up front, so the head of the
    // walk takes it up front.
    for (; kt < last && kt < kt_a + kWarmTiles; kt += NS) group(kt, std::false_type{});
  }
  for (; kt < last; kt += NS) group(kt, std::true_type{});
  // the last tile: its scores are in registers, its V tile landed with its K tile
  {
    const char* v_last = ring.base + ((last - kt_a) % NS) * kTile;  // + the bias in rb.v_off
    if ((last - kt_a) & 1)
      rb.template fused<MASK, false>(nullptr, v_last, s1, s0, last * G::kTileKeys, half);
    else
      rb.template fused<MASK, false>(nullptr, v_last, s0, s1, last * G::kTileKeys, half);
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

  const SeqDesc* descs = args.inline_descs;
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
  // V tiles sit NS K-tiles above the ring's base
  rb.init(fabsf(args.scale_log2), lane, NS * TileGeom<D, NW>::kTileBytes);

  const int wg_row0 = row_tile * Shape::kRowsPerWg;
  const int r = wg_row0 + wave * 32 + col;
  const bool valid = r < n_rows;
  const int rr = valid ? r : (n_rows - 1);
  const int tok = rr / gqa;
  const int hq = kv_head * gqa + rr % gqa;
  const int kv_total = sd.kv_len;  // keys that exist
  rb.limit = min(sd.prefix_len + tok, kv_total - 1);
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
  const int keys_needed = max(0, min(kv_total, sd.prefix_len + last_row / gqa + 1));
  const int tiles_needed = (keys_needed + 63) / 64;
  const int kt_begin = split * sd.tiles_per_split;
  const int kt_end = min(tiles_needed, kt_begin + sd.tiles_per_split);
  // tiles below kt_mid are fully visible to every row of the workgroup
  const int unmasked_keys =
      max(0, min(kv_total, sd.prefix_len + min(wg_row0, n_rows - 1) / gqa + 1));
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
  const float lt = rb.row_sum();
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
