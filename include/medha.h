/*
 * medha.h — C ABI of the MI355X (gfx950) paged-attention library.
 *
 * Three operations, the data-parallel hot path of preemptive long-context
 * serving with chunked prefills and KV-cache parallelism:
 *
 *   medha_chunked_prefill_attn  attention of prefill chunks against a long
 *                               paged KV-cache prefix, causal inside the chunk,
 *                               giving O and the log-sum-exp (LSE) per head;
 *   medha_decode_partial_attn   one query token against one KV shard, giving
 *                               a partial (O, LSE);
 *   medha_lse_merge             exact combination of partials over disjoint
 *                               key sets.
 *
 * Common conventions
 *   - "dev" pointers are device (HBM) memory, "host" pointers ordinary host
 *     memory.  The caller owns every buffer.  The library allocates no device
 *     memory, keeps no state between calls, never synchronises the device, and
 *     enqueues work only on `hip_stream` (a hipStream_t passed as void*; NULL
 *     is the default stream).  Host arrays are fully read before the call
 *     returns; device buffers must stay valid until the stream reaches the end
 *     of the enqueued work.
 *   - All tensors are dense, row-major (C order), without padding.
 *     bf16 = the upper 16 bits of an IEEE fp32.
 *   - KV cache: a pool of pages, k_pool and v_pool both
 *         bf16 [num_pages][num_kv_heads][page_size][head_dim],
 *     page_size == 16, head_dim in {64, 128}.  Token t of a sequence lives in
 *     physical page  page_table[t / 16]  at slot  t % 16.  Pool slots that no
 *     token occupies are never read into a result.  Page ids are trusted: they
 *     are NOT range-checked on the device.
 *   - Grouped-query attention: query head h uses KV head h / (num_q_heads /
 *     num_kv_heads).
 *   - Scores are softmax_scale * <q, k>; LSE is the natural logarithm of the sum
 *     of exp(score) over the keys attended to.  A row that attends to no key
 *     gets O = 0 and LSE = -inf.
 *   - Arithmetic: bf16 operands, fp32 accumulation (matrix cores), fp32 softmax
 *     statistics; probabilities are rounded to bf16 before the P*V product.
 *     For one input and one device the result is bitwise reproducible.
 *   - Return value: MEDHA_OK (0) or a negative error code.  On an error
 *     detected by argument validation nothing is enqueued and no output byte
 *     is written.
 */
#ifndef MEDHA_H_
#define MEDHA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MEDHA_OK 0
#define MEDHA_ERR_INVALID_ARG (-1)  /* null pointer, bad length, bad head counts, misalignment */
#define MEDHA_ERR_UNSUPPORTED (-2)  /* page_size != 16, head_dim not 64/128                     */
#define MEDHA_ERR_WORKSPACE (-3)    /* workspace missing, misaligned or too small              */
#define MEDHA_ERR_HIP (-4)          /* a HIP runtime call failed                               */

/* Paged KV cache descriptor (host struct holding device pointers).  The pools are read-only
 * for every call except medha_kv_append. */
typedef struct medha_kv_cache {
  const void* k_pool; /* dev bf16 [num_pages][num_kv_heads][page_size][head_dim], 16-byte aligned */
  const void* v_pool; /* dev bf16, same shape                                                    */
  int32_t num_pages;
  int32_t page_size;    /* must be 16 */
  int32_t num_kv_heads;
  int32_t head_dim;     /* 64 or 128 */
} medha_kv_cache;

/*
 * Chunked-prefill attention (paper section 3.1: a chunk of c new tokens attends
 * to the whole KV cache of the earlier chunks and causally to itself; section
 * 2.6: the prefix is re-read for every chunk).  Batched and variable-length:
 * sequence b contributes chunk_len[b] consecutive query rows; row j of it
 * attends to keys 0 .. prefix_len[b] + j of its own paged sequence.  The chunk's
 * own K/V must already be in the cache.  A decode step is a sequence with
 * chunk_len == 1, so one call serves a mixed batch of one long prefill chunk
 * and many decodes (section 2.6 "Latency Interference", section 4 batch packing).
 *
 *   q                dev  bf16 [sum chunk_len][num_q_heads][head_dim], 16-byte aligned
 *   page_table       dev  int32, the per-sequence tables concatenated
 *   page_table_offs  host int64 [batch + 1]; sequence b owns
 *                    page_table[offs[b] .. offs[b+1]) which must hold at least
 *                    ceil((prefix_len[b] + chunk_len[b]) / 16) entries
 *   prefix_len       host int32 [batch], >= 0
 *   chunk_len        host int32 [batch], >= 1
 *   out              dev  fp32 [sum chunk_len][num_q_heads][head_dim], 16-byte aligned
 *   lse              dev  fp32 [sum chunk_len][num_q_heads]
 *   workspace        dev, 256-byte aligned, at least
 *                    medha_chunked_prefill_workspace_bytes(...) bytes; contents
 *                    are scratch (split-KV partials); may be NULL when that
 *                    size is <= 256 (nothing is split).
 *
 * Work is split over query tiles and, when those are too few to fill the GPU,
 * also over KV ranges whose partials are merged on the same stream.  Sequence
 * descriptors travel in the kernel arguments, 64 per launch: a larger batch takes
 * several launches, and no call ever copies from host memory or blocks the host.
 */
int medha_chunked_prefill_attn(const void* q, const medha_kv_cache* kv, const int32_t* page_table,
                               const int64_t* page_table_offs, const int32_t* prefix_len,
                               const int32_t* chunk_len, int32_t batch, int32_t num_q_heads,
                               float softmax_scale, float* out, float* lse, void* workspace,
                               size_t workspace_bytes, void* hip_stream);

/* Workspace size for the call above with the same host arrays, head counts and
 * the current device.  Returns 0 for invalid arguments. */
size_t medha_chunked_prefill_workspace_bytes(const int32_t* prefix_len, const int32_t* chunk_len,
                                             int32_t batch, int32_t num_q_heads,
                                             int32_t num_kv_heads, int32_t head_dim);

/*
 * medha_chunked_prefill_attn for callers that cannot allocate device memory or hand
 * over a workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, results and error codes, without the workspace:
 * the split-KV partials go to a scratch array of MEDHA_NOALLOC_SCRATCH_BYTES that is
 * part of the library's device image (every GPU the library runs on holds its own copy
 * until the process ends).  The call allocates nothing and calls no allocating routine;
 * its first call on a device looks the array's address up (make that call outside a
 * graph capture).  A batch whose workspace need, as reported by
 * medha_chunked_prefill_workspace_bytes, exceeds MEDHA_NOALLOC_SCRATCH_BYTES is
 * refused with MEDHA_ERR_WORKSPACE and nothing is enqueued.  All calls on one GPU share
 * that GPU's array: calls that overlap on one GPU (different streams, or graphs
 * replayed concurrently) race on it and must be serialised by the caller.  Nothing in
 * the array has to start at zero: every partial is written before it is read.
 */
#define MEDHA_NOALLOC_SCRATCH_BYTES (64u << 20)
int medha_chunked_prefill_attn_noalloc(const void* q, const medha_kv_cache* kv,
                                       const int32_t* page_table,
                                       const int64_t* page_table_offs, const int32_t* prefix_len,
                                       const int32_t* chunk_len, int32_t batch,
                                       int32_t num_q_heads, float softmax_scale, float* out,
                                       float* lse, void* hip_stream);

/*
 * Split-KV decode partial (paper section 3.3 "Bounding Decode Latency": the
 * query is replicated to every KV shard, each computes a partial attention
 * output over its local keys).  Item i takes query token q_index[i] and
 * attends, without a mask, to tokens [0, kv_len[i]) of the paged sequence given
 * by its page-table slice.  A KV-parallel shard is an item whose slice starts
 * at the shard's first page (shards start on page boundaries).  kv_len 0 is
 * allowed and yields O = 0, LSE = -inf.
 *
 *   q                dev  bf16 [num_queries][num_q_heads][head_dim], 16-byte aligned
 *   page_table       dev  int32, concatenated slices
 *   page_table_offs  host int64 [items + 1]
 *   q_index          host int32 [items], each in [0, num_queries)
 *   kv_len           host int32 [items], >= 0
 *   out_partial      dev  fp32 [items][num_q_heads][head_dim], 16-byte aligned
 *   lse_partial      dev  fp32 [items][num_q_heads]
 *   workspace        as above, size from medha_decode_partial_workspace_bytes
 */
int medha_decode_partial_attn(const void* q, int32_t num_queries, const medha_kv_cache* kv,
                              const int32_t* page_table, const int64_t* page_table_offs,
                              const int32_t* q_index, const int32_t* kv_len, int32_t items,
                              int32_t num_q_heads, float softmax_scale, float* out_partial,
                              float* lse_partial, void* workspace, size_t workspace_bytes,
                              void* hip_stream);

size_t medha_decode_partial_workspace_bytes(const int32_t* kv_len, int32_t items,
                                            int32_t num_q_heads, int32_t num_kv_heads,
                                            int32_t head_dim);

/*
 * KV-cache-parallel partial of a prefill chunk (paper section 3.3: the query that
 * is replicated to the KV shards is a decode token or a prefill chunk; each shard
 * computes a partial attention output over its local keys).  Item i is (chunk,
 * shard): query rows q_row[i] .. q_row[i] + chunk_len[i] - 1 of q against the
 * kv_len[i] keys of the item's page-table slice (a shard starts on a page
 * boundary).  Row j of the chunk sees the first
 *     min(kv_len[i], max(0, visible0[i] + j))
 * keys of the slice: a shard that lies wholly before the chunk has
 * visible0 >= kv_len (no mask); for the shard that holds the chunk's own keys,
 * visible0 = (position of the chunk's first token) - (position of the shard's
 * first token) + 1.  Rows that see no key of a shard get O = 0, LSE = -inf.
 * The items' outputs follow each other in item order, so S shards of one chunk
 * of c rows produce exactly the [S][c][num_q_heads][head_dim] / [S][c][num_q_heads]
 * arrays medha_lse_merge takes.
 *
 *   q                dev  bf16 [num_tokens][num_q_heads][head_dim], 16-byte aligned
 *   page_table       dev  int32, concatenated slices
 *   page_table_offs  host int64 [items + 1]; slice i holds >= ceil(kv_len[i] / 16) entries
 *   q_row            host int32 [items], q_row[i] + chunk_len[i] <= num_tokens
 *   chunk_len        host int32 [items], >= 1
 *   kv_len           host int32 [items], >= 0
 *   visible0         host int32 [items], |visible0| <= 2^30
 *   out_partial      dev  fp32 [sum chunk_len][num_q_heads][head_dim], 16-byte aligned
 *   lse_partial      dev  fp32 [sum chunk_len][num_q_heads]
 *   workspace        as above, size from medha_chunk_partial_workspace_bytes
 */
int medha_chunk_partial_attn(const void* q, int32_t num_tokens, const medha_kv_cache* kv,
                             const int32_t* page_table, const int64_t* page_table_offs,
                             const int32_t* q_row, const int32_t* chunk_len,
                             const int32_t* kv_len, const int32_t* visible0, int32_t items,
                             int32_t num_q_heads, float softmax_scale, float* out_partial,
                             float* lse_partial, void* workspace, size_t workspace_bytes,
                             void* hip_stream);

size_t medha_chunk_partial_workspace_bytes(const int32_t* chunk_len, const int32_t* kv_len,
                                           int32_t items, int32_t num_q_heads,
                                           int32_t num_kv_heads, int32_t head_dim);

/*
 * LSE merge (paper section 3.3: the partial outputs of the KV shards are
 * combined with the online-softmax identity).  For every (row, head):
 *     LSE = ln sum_s exp(LSE_s)        O = sum_s exp(LSE_s - LSE) * O_s
 * Partials with LSE_s = -inf weigh zero; if all are -inf, O = 0, LSE = -inf.
 *
 *   out_partial  dev fp32 [num_splits][rows][num_q_heads][head_dim], 16-byte aligned
 *   lse_partial  dev fp32 [num_splits][rows][num_q_heads]
 *   out          dev fp32 [rows][num_q_heads][head_dim]   (may not alias the inputs)
 *   lse          dev fp32 [rows][num_q_heads]
 * head_dim must be a multiple of 4; num_splits >= 1.
 */
int medha_lse_merge(const float* out_partial, const float* lse_partial, int32_t num_splits,
                    int64_t rows, int32_t num_q_heads, int32_t head_dim, float* out, float* lse,
                    void* hip_stream);

/*
 * KV-cache append (paper section 3.1: the keys and values of every chunk join
 * the paged cache that all later chunks and decode steps read; the attention
 * calls above expect them there).  Token j of sequence b, row
 * sum(chunk_len[0..b)) + j of k_new / v_new, is written to position
 * prefix_len[b] + j of the sequence: page page_table[offs[b] + position / 16],
 * slot position % 16, all KV heads.  A bit-exact copy; nothing else in the pools
 * is touched.  This is the one call that WRITES kv->k_pool / kv->v_pool.
 *
 *   k_new, v_new     dev  bf16 [sum chunk_len][num_kv_heads][head_dim], 16-byte aligned
 *   page_table, page_table_offs, prefix_len, chunk_len, batch: as for
 *                    medha_chunked_prefill_attn (same arrays can be passed to both)
 *
 * A page-table entry outside [0, kv->num_pages) is skipped on the device (that
 * token is not written); pages shared by two sequences of the batch are the
 * caller's error and give an unspecified winner.  No workspace, no allocation;
 * batches of more than 64 sequences take several kernel launches.
 */
int medha_kv_append(const void* k_new, const void* v_new, const medha_kv_cache* kv,
                    const int32_t* page_table, const int64_t* page_table_offs,
                    const int32_t* prefix_len, const int32_t* chunk_len, int32_t batch,
                    void* hip_stream);

/*
 * Introspection of the launch plan (host only; needs no GPU).  How the library
 * would lay a chunked-prefill batch out over workgroups on a device with
 * num_cus compute units (0 = the current device, or 256 if there is none):
 * per sequence the kernel it goes to, its query-row tiling and its KV split.
 * A decode item of kv_len n is the sequence (prefix_len n - 1, chunk_len 1),
 * so prefix_len may be -1 here.  medha_describe_slot maps a workgroup slot of
 * a sequence (0 <= slot < n_slots) to its work item and returns 1, or 0 for an
 * idle padding slot.  These two calls exist for tests and tuning; they launch
 * nothing.
 */
typedef struct medha_plan_entry {
  int32_t mode;            /* 0: row-split prefill kernel, 1: key-split decode kernel */
  int32_t rows_per_wg;     /* (token, head-in-group) query rows per workgroup          */
  int32_t tile_keys;       /* granule of the KV split, in keys                         */
  int32_t n_row_tiles;     /* row tiles per KV head                                    */
  int32_t n_split;         /* KV ranges; > 1 means partials + merge                    */
  int32_t tiles_per_split; /* granules per range                                       */
  int32_t work_start;      /* first workgroup slot inside its kernel launch            */
  int32_t n_slots;         /* slots owned: 8 * ceil(kv_heads * n_split * n_row_tiles / 8) */
} medha_plan_entry;

int medha_describe_plan(const int32_t* prefix_len, const int32_t* chunk_len, int32_t batch,
                        int32_t num_q_heads, int32_t num_kv_heads, int32_t head_dim,
                        int32_t num_cus, medha_plan_entry* entries /* host [batch] */,
                        int32_t* grid_rows, int32_t* grid_keys, size_t* workspace_bytes);

int medha_describe_slot(int32_t slot, int32_t num_kv_heads, int32_t n_split, int32_t n_row_tiles,
                        int32_t* kv_head, int32_t* split, int32_t* row_tile);

/* Static, human-readable text for a return code. */
const char* medha_strerror(int code);

/* ABI version of this header (bumped on incompatible change). */
int medha_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MEDHA_H_ */
