// Paged attention kernels for gfx950 (wave64, MFMA 32x32x16 bf16).
//
// One kernel template serves both shapes of the method:
//   - row-split mode (prefill chunks, paper section 3.1): a workgroup owns a
//     tile of query rows (a row = one (token, query head) pair of one KV head's
//     group, so a K/V tile is shared by the whole GQA group), its 4 wavefronts
//     each own 32*QB rows and all walk the same KV tiles staged in LDS;
//   - key-split mode (decode and other tiny row counts, section 3.3): the <=32
//     rows are shared by the 4 wavefronts, which split every 128-key tile
//     between them and combine their running statistics at the end.
// In both modes the KV axis may also be split across workgroups; then partial
// (O, LSE) go to a workspace and a merge kernel finishes the job.
//
// Register mapping (lane l: col = l % 32, half = l / 32):
//   S^T = K Q^T  : A = K rows (32 keys x 16 dims), B = Q^T; a lane owns query
//                  row `col` and 16 of the 32 keys, so softmax row statistics
//                  are lane-local plus one half-wave exchange.
//   O^T = V^T P^T: A = V^T (32 dims x 16 keys) read from row-major V in LDS
//                  with the transposing LDS read, B = P^T taken straight from
//                  the S^T accumulator registers (the key order inside a
//                  16-key slice is permuted identically on both operands).
#pragma once

#include "common.h"

namespace medha {

template <int D>
struct Lds {
  // Row strides (bytes) chosen so that the 16-byte K operand reads of 16
  // consecutive rows, and the 8-byte transposing V reads of 4 rows x 64 bytes,
  // fall on distinct banks.
  static constexpr int kRowK = D * 2 + 16;
  static constexpr int kRowV = D * 2 + 64;
};

__device__ __forceinline__ bf16x8 lds_read_k(const char* p) {
  return *reinterpret_cast<const bf16x8*>(p);
}

// Transposing LDS read: a 16-lane block that points at 4 rows x 16 columns of
// 16-bit data (lane i at row i/4, columns 4*(i%4)..+3) receives, in lane i,
// column i of the 4 rows.
__device__ __forceinline__ s16x4 lds_read_tr(const char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (s16x4 __attribute__((address_space(3)))*)(p));
}

// Cooperative global -> register -> LDS staging of one KV tile of BN keys.
template <int D, int BN>
struct TileStage {
  static constexpr int kChunksPerRow = D / 8;  // 16-byte pieces per key row
  static constexpr int kIter = BN * kChunksPerRow / kThreads;
  static_assert(BN * kChunksPerRow % kThreads == 0, "tile must divide over the workgroup");
  uint4 k[kIter];
  uint4 v[kIter];

  // Loads keys [key0, key0 + BN) of the sequence; keys >= kv_total are zeros
  // (their pages may not exist and their slots may hold anything).
  __device__ __forceinline__ void load(const __bf16* __restrict__ k_pool,
                                       const __bf16* __restrict__ v_pool,
                                       const int32_t* __restrict__ pt, int key0, int kv_total,
                                       int h_kv, int kv_head) {
#pragma unroll
    for (int it = 0; it < kIter; ++it) {
      const int ci = it * kThreads + threadIdx.x;
      const int key = ci / kChunksPerRow;
      const int chunk = ci % kChunksPerRow;
      const int t = key0 + key;
      if (t < kv_total) {
        const int page = pt[t >> 4];
        const int64_t off =
            (((int64_t)page * h_kv + kv_head) * kPageSize + (t & 15)) * D + chunk * 8;
        k[it] = *reinterpret_cast<const uint4*>(k_pool + off);
        v[it] = *reinterpret_cast<const uint4*>(v_pool + off);
      } else {
        k[it] = make_uint4(0, 0, 0, 0);
        v[it] = make_uint4(0, 0, 0, 0);
      }
    }
  }

  __device__ __forceinline__ void store(char* k_lds, char* v_lds) const {
#pragma unroll
    for (int it = 0; it < kIter; ++it) {
      const int ci = it * kThreads + threadIdx.x;
      const int key = ci / kChunksPerRow;
      const int chunk = ci % kChunksPerRow;
      *reinterpret_cast<uint4*>(k_lds + key * Lds<D>::kRowK + chunk * 16) = k[it];
      *reinterpret_cast<uint4*>(v_lds + key * Lds<D>::kRowV + chunk * 16) = v[it];
    }
  }
};

// Per-wavefront attention state over QB blocks of 32 query rows.
template <int D, int QB>
struct WaveAttn {
  static constexpr int kSlices = D / 16;   // contraction slices of Q K^T
  static constexpr int kDBlocks = D / 32;  // 32-wide blocks of the head dimension
  bf16x8 q[QB][kSlices];
  f32x16 o[QB][kDBlocks];
  float m[QB];      // running row maximum (log2 domain), same in both half-wave lanes of a row
  float l[QB];      // this lane's share of the running row sum
  int limit[QB];    // last key index the lane's row may attend to
  float scale_log2;
  int col, half;

  __device__ __forceinline__ void init(float scale) {
    scale_log2 = scale;
    col = threadIdx.x & 31;
    half = (threadIdx.x >> 5) & 1;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      m[qb] = -INFINITY;
      l[qb] = 0.f;
#pragma unroll
      for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[qb][db][e] = 0.f;
    }
  }

  // One step over NKB blocks of 32 keys starting at LDS rows k_lds / v_lds whose
  // first row is key index key0 of the sequence.  MASK applies the causal /
  // length limit per row; without it every key of the tile is visible.
  template <int NKB, bool MASK>
  __device__ __forceinline__ void step(const char* k_lds, const char* v_lds, int key0) {
    f32x16 s[QB][NKB];
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int e = 0; e < 16; ++e) s[qb][kb][e] = 0.f;
      const char* krow = k_lds + (kb * 32 + col) * Lds<D>::kRowK + half * 16;
#pragma unroll
      for (int sl = 0; sl < kSlices; ++sl) {
        const bf16x8 a = lds_read_k(krow + sl * 32);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
          s[qb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, q[qb][sl], s[qb][kb], 0, 0, 0);
      }
    }

    bf16x8 p[QB][NKB][2];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      float mx = -INFINITY;
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          float x = s[qb][kb][e] * scale_log2;
          if (MASK) {
            const int t = key0 + kb * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
            x = (t <= limit[qb]) ? x : -INFINITY;
          }
          s[qb][kb][e] = x;
          mx = fmaxf(mx, x);
        }
      mx = max_halves(mx);
      const float m_old = m[qb];
      const float m_new = fmaxf(m_old, mx);
      // a row that has seen no key yet keeps m = -inf; exponentiate against 0 then
      const float m_use = (MASK && m_new == -INFINITY) ? 0.f : m_new;
      if (__any(m_new != m_old)) {
        const float alpha = fast_exp2(m_old - m_use);
        l[qb] *= alpha;
#pragma unroll
        for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
          for (int e = 0; e < 16; ++e) o[qb][db][e] *= alpha;
      }
      m[qb] = m_new;
      float ls = 0.f;
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb) {
        f32x8 lo, hi;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          lo[e] = fast_exp2(s[qb][kb][e] - m_use);
          hi[e] = fast_exp2(s[qb][kb][8 + e] - m_use);
          ls += lo[e] + hi[e];
        }
        p[qb][kb][0] = __builtin_convertvector(lo, bf16x8);
        p[qb][kb][1] = __builtin_convertvector(hi, bf16x8);
      }
      l[qb] += ls;
    }

    // O^T += V^T P^T.  Slice t of key block kb holds, for this lane's half,
    // keys kb*32 + 16t + 4*half + {0..3} and the same + 8.
    const int l16 = threadIdx.x & 15;
    const int dhalf = (threadIdx.x >> 4) & 1;
    const char* vbase =
        v_lds + (4 * half + (l16 >> 2)) * Lds<D>::kRowV + (16 * dhalf + 4 * (l16 & 3)) * 2;
#pragma unroll
    for (int db = 0; db < kDBlocks; ++db) {
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const char* vp = vbase + (kb * 32 + 16 * t) * Lds<D>::kRowV + db * 64;
          const s16x4 v0 = lds_read_tr(vp);
          const s16x4 v1 = lds_read_tr(vp + 8 * Lds<D>::kRowV);
          const s16x8 v8 = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
          const bf16x8 a = __builtin_bit_cast(bf16x8, v8);
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
            o[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, p[qb][kb][t], o[qb][db], 0, 0, 0);
        }
      }
    }
  }
};

// Largest i with descs[i].work_start <= slot.
__device__ __forceinline__ int find_seq(const SeqDesc* descs, int n_seq, int slot) {
  int lo = 0, hi = n_seq - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (descs[mid].work_start <= slot) lo = mid; else hi = mid - 1;
  }
  return lo;
}

template <int D, int QB, bool SPLIT_KEYS>
struct KernelShape {
  static constexpr int kRowsPerWave = 32 * QB;
  static constexpr int kRowsPerWg = SPLIT_KEYS ? 32 : kRowsPerWave * kWaves;
  static constexpr int kTileKeys = SPLIT_KEYS ? 32 * kWaves : 64;   // keys staged per iteration
  static constexpr int kKeyBlocksPerWave = SPLIT_KEYS ? 1 : kTileKeys / 32;
  static constexpr int kStageBytes = kTileKeys * (Lds<D>::kRowK + Lds<D>::kRowV);
  static constexpr int kLdsBytes = 2 * kStageBytes;
};

template <int D, int QB, bool SPLIT_KEYS>
__global__ void __launch_bounds__(kThreads) attn_kernel(const AttnArgs args) {
  using Shape = KernelShape<D, QB, SPLIT_KEYS>;
  static_assert(!SPLIT_KEYS || QB == 1, "key-split mode shares one 32-row block");
  constexpr int BN = Shape::kTileKeys;
  constexpr int NKB = Shape::kKeyBlocksPerWave;
  __shared__ __attribute__((aligned(16))) char lds[Shape::kLdsBytes];

  const SeqDesc* descs = args.descs ? args.descs : args.inline_descs;
  const SeqDesc sd = descs[find_seq(descs, args.n_seq, blockIdx.x)];

  // Slot -> (KV head, KV split, row tile).  Slot s runs on die s % 8.  The
  // sequence's work items, ordered (group, row tile) with group = (split, KV
  // head), are cut into 8 equal contiguous runs, one per die: the row tiles that
  // stream the same K/V range share a die and hence its L2.
  const int u = blockIdx.x - sd.work_start;
  const int groups = args.h_kv * sd.n_split;
  const int items = groups * sd.n_row_tiles;
  const int per_die = (items + kXcds - 1) / kXcds;
  const int y = u / kXcds;
  const int item = (u % kXcds) * per_die + y;
  if (y >= per_die || item >= items) return;
  const int grp = item / sd.n_row_tiles;
  const int row_tile = item % sd.n_row_tiles;
  const int kv_head = grp % args.h_kv;
  const int split = grp / args.h_kv;

  const int gqa = args.h_q / args.h_kv;
  const int n_rows = sd.chunk_len * gqa;
  const int wave = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const int col = lane & 31, half = lane >> 5;

  WaveAttn<D, QB> st;
  st.init(args.scale_log2);

  const int row0 = row_tile * Shape::kRowsPerWg + (SPLIT_KEYS ? 0 : wave * Shape::kRowsPerWave);
  int tok[QB];
  bool valid[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int r = row0 + qb * 32 + col;
    valid[qb] = r < n_rows;
    const int rr = valid[qb] ? r : (n_rows - 1);
    tok[qb] = rr / gqa;
    st.limit[qb] = sd.prefix_len + tok[qb];
    const int hq = kv_head * gqa + rr % gqa;
    const __bf16* qp = args.q + ((int64_t)(sd.q_row + tok[qb]) * args.h_q + hq) * D + half * 8;
#pragma unroll
    for (int sl = 0; sl < WaveAttn<D, QB>::kSlices; ++sl) {
      uint4 raw = make_uint4(0, 0, 0, 0);
      if (valid[qb]) raw = *reinterpret_cast<const uint4*>(qp + sl * 16);
      st.q[qb][sl] = __builtin_bit_cast(bf16x8, raw);
    }
  }

  // Keys this row tile needs: up to the limit of its last row.
  const int last_row = min(n_rows, (row_tile + 1) * Shape::kRowsPerWg) - 1;
  const int keys_needed = sd.prefix_len + last_row / gqa + 1;  // may be 0
  const int kv_total = sd.prefix_len + sd.chunk_len;           // keys that exist
  const int tiles_needed = (keys_needed + BN - 1) / BN;
  const int kt_begin = split * sd.tiles_per_split;
  const int kt_end = min(tiles_needed, kt_begin + sd.tiles_per_split);
  // first key index at which some row of this wavefront needs the mask
  const int wave_first_tok = min(row0, n_rows - 1) / gqa;
  const int unmasked_keys = sd.prefix_len + wave_first_tok + 1;

  const int32_t* pt = args.page_table + sd.pt_off;
  TileStage<D, BN> stage;
  if (kt_begin < kt_end)
    stage.load(args.k_pool, args.v_pool, pt, kt_begin * BN, kv_total, args.h_kv, kv_head);
  int buf = 0;
  for (int kt = kt_begin; kt < kt_end; ++kt) {
    char* k_lds = lds + buf * Shape::kStageBytes;
    char* v_lds = k_lds + BN * Lds<D>::kRowK;
    stage.store(k_lds, v_lds);
    __syncthreads();
    if (kt + 1 < kt_end)
      stage.load(args.k_pool, args.v_pool, pt, (kt + 1) * BN, kv_total, args.h_kv, kv_head);
    const int wave_rows = SPLIT_KEYS ? wave * 32 : 0;  // this wavefront's rows of the stage
    const int key0 = kt * BN + wave_rows;
    const char* kw = k_lds + wave_rows * Lds<D>::kRowK;
    const char* vw = v_lds + wave_rows * Lds<D>::kRowV;
    if (key0 + NKB * 32 <= unmasked_keys)
      st.template step<NKB, false>(kw, vw, key0);
    else
      st.template step<NKB, true>(kw, vw, key0);
    buf ^= 1;
  }

  const bool direct = sd.n_split == 1;
  float* o_base = direct ? args.out : args.part_o;
  float* l_base = direct ? args.lse : args.part_lse;
  const int64_t row_base =
      direct ? (int64_t)sd.out_row : (int64_t)sd.part_row + (int64_t)split * sd.chunk_len;

  if (!SPLIT_KEYS) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const float lt = sum_halves(st.l[qb]);
      const float inv = lt > 0.f ? 1.f / lt : 0.f;
      const float lse = lt > 0.f ? (st.m[qb] + fast_log2(lt)) * kLn2 : -INFINITY;
      if (valid[qb]) {
        const int r = row0 + qb * 32 + col;
        const int hq = kv_head * gqa + r % gqa;
        const int64_t orow = (row_base + tok[qb]) * args.h_q + hq;
        float* op = o_base + orow * D + 4 * half;
#pragma unroll
        for (int db = 0; db < WaveAttn<D, QB>::kDBlocks; ++db)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            f32x4 v;
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = st.o[qb][db][4 * i + j] * inv;
            *reinterpret_cast<f32x4*>(op + db * 32 + 8 * i) = v;
          }
        if (half == 0) l_base[orow] = lse;
      }
    }
  } else {
    // Combine the 4 wavefronts' (m, l, O) over their disjoint keys through LDS.
    __syncthreads();  // every wavefront is done reading K/V
    float* sm_o = reinterpret_cast<float*>(lds);                  // [wave][32][D]
    float* sm_ml = sm_o + kWaves * 32 * D;                        // [wave][32][2]
    static_assert(kWaves * 32 * (D + 2) * 4 <= Shape::kLdsBytes, "combine buffer fits");
    const float lt = sum_halves(st.l[0]);
    if (col < n_rows - row0) {
      float* op = sm_o + (wave * 32 + col) * D + 4 * half;
#pragma unroll
      for (int db = 0; db < WaveAttn<D, QB>::kDBlocks; ++db)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          f32x4 v;
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] = st.o[0][db][4 * i + j];
          *reinterpret_cast<f32x4*>(op + db * 32 + 8 * i) = v;
        }
      if (half == 0) {
        sm_ml[(wave * 32 + col) * 2 + 0] = st.m[0];
        sm_ml[(wave * 32 + col) * 2 + 1] = lt;
      }
    }
    __syncthreads();
    const int rows_here = min(32, n_rows - row0);
    for (int e = threadIdx.x; e < rows_here * (D / 4); e += kThreads) {
      const int r = e / (D / 4);
      const int d4 = e % (D / 4);
      float mw[kWaves], lw[kWaves], mm = -INFINITY;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        mw[w] = sm_ml[(w * 32 + r) * 2 + 0];
        lw[w] = sm_ml[(w * 32 + r) * 2 + 1];
        mm = fmaxf(mm, mw[w]);
      }
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
      float lt_all = 0.f;
      if (mm != -INFINITY) {
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
          const float a = fast_exp2(mw[w] - mm);
          lt_all += a * lw[w];
          const f32x4 ov = *reinterpret_cast<const f32x4*>(sm_o + (w * 32 + r) * D + d4 * 4);
          if (lw[w] > 0.f) acc += ov * a;
        }
      }
      const float inv = lt_all > 0.f ? 1.f / lt_all : 0.f;
      const int rr = row0 + r;
      const int hq = kv_head * gqa + rr % gqa;
      const int64_t orow = (row_base + rr / gqa) * args.h_q + hq;
      *reinterpret_cast<f32x4*>(o_base + orow * D + d4 * 4) = acc * inv;
      if (d4 == 0)
        l_base[orow] = lt_all > 0.f ? (mm + fast_log2(lt_all)) * kLn2 : -INFINITY;
    }
  }
}

}  // namespace medha
