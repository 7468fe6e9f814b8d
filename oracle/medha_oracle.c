/*
 * Parity oracle for paged chunked-prefill / split-KV decode attention and the
 * log-sum-exp merge.  TEST INFRASTRUCTURE ONLY: nothing on the product path may
 * call into this file.  It shares no code, header or table with the HIP kernels.
 *
 * What is computed is the plain definition of softmax attention, because the
 * method only re-associates it:
 *   - a prefill chunk attends to the whole cached prefix plus, causally, to
 *     itself (paper section 2.6 "KV-Cache Read Amplification", section 3.1);
 *     chunk i+1 needs only the K/V of earlier chunks, never their outputs
 *     (section 3.3, stream pipeline paragraph), so every row is independent;
 *   - several query heads share one KV head (section 3.1, GQA remark);
 *   - for KV-cache parallelism the query is replicated, each shard yields a
 *     partial attention output over its own keys and the partials are combined
 *     by the online-softmax identity (section 3.3 "Bounding Decode Latency").
 *
 * Arithmetic: inputs are bf16 bit patterns widened exactly to fp64; every sum is
 * a plain left-to-right fp64 loop; softmax is two-pass (max, then exp/sum); no
 * tiling, no running rescale, no fused steps.
 *
 * Layouts (all row-major, C order):
 *   q        bf16  [tokens][h_q][d]
 *   k_pool   bf16  [num_pages][h_kv][page_size][d]      (v_pool alike)
 *   token t of a sequence lives in physical page page_table[t / page_size],
 *   slot t % page_size.
 *
 * Return value: 0 on success, -1 bad argument, -2 page id out of range,
 * -3 out of memory.
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double bf16_to_f64(uint16_t bits) {
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* One (query row, head): scores against keys [0, n_keys) of one paged sequence,
 * two-pass softmax, weighted sum of values.  scratch holds n_keys doubles.
 * n_keys == 0 gives O = 0 and LSE = -inf. */
static int attend_one(const uint16_t *q_row /* [d] */, const uint16_t *k_pool,
                      const uint16_t *v_pool, int32_t num_pages, int32_t page_size,
                      int32_t h_kv, int32_t d, int32_t kv_head, const int32_t *pt,
                      int64_t n_keys, double scale, double *scratch, double *out /* [d] */,
                      double *lse) {
    for (int32_t x = 0; x < d; ++x) out[x] = 0.0;
    if (n_keys == 0) {
        *lse = -INFINITY;
        return 0;
    }
    double m = -INFINITY;
    for (int64_t t = 0; t < n_keys; ++t) {
        int32_t page = pt[t / page_size];
        int32_t slot = (int32_t)(t % page_size);
        if (page < 0 || page >= num_pages) return -2;
        const uint16_t *k_row =
            k_pool + (((int64_t)page * h_kv + kv_head) * page_size + slot) * (int64_t)d;
        double dot = 0.0;
        for (int32_t x = 0; x < d; ++x) dot += bf16_to_f64(q_row[x]) * bf16_to_f64(k_row[x]);
        double s = scale * dot;
        scratch[t] = s;
        if (s > m) m = s;
    }
    double l = 0.0;
    for (int64_t t = 0; t < n_keys; ++t) {
        int32_t page = pt[t / page_size];
        int32_t slot = (int32_t)(t % page_size);
        const uint16_t *v_row =
            v_pool + (((int64_t)page * h_kv + kv_head) * page_size + slot) * (int64_t)d;
        double p = exp(scratch[t] - m);
        l += p;
        for (int32_t x = 0; x < d; ++x) out[x] += p * bf16_to_f64(v_row[x]);
    }
    for (int32_t x = 0; x < d; ++x) out[x] /= l;
    *lse = m + log(l);
    return 0;
}

/*
 * Chunked-prefill attention for a batch of sequences.  Sequence b contributes
 * chunk_len[b] query rows (concatenated in q); row j of it sees keys
 * 0 .. prefix_len[b] + j of its paged sequence (the chunk's own K/V are already
 * in the cache).  rows == NULL: compute every row, out is [tokens][h_q][d].
 * Otherwise rows[0..n_rows) are indices into the concatenated token axis and
 * out is [n_rows][h_q][d], lse [n_rows][h_q].
 */
int medha_oracle_chunked_prefill(const uint16_t *q, const uint16_t *k_pool,
                                 const uint16_t *v_pool, int32_t num_pages, int32_t page_size,
                                 int32_t h_kv, int32_t d, const int32_t *page_table,
                                 const int64_t *page_table_offs, const int32_t *prefix_len,
                                 const int32_t *chunk_len, int32_t batch, int32_t h_q,
                                 double scale, const int64_t *rows, int64_t n_rows, double *out,
                                 double *lse) {
    if (batch < 0 || h_q <= 0 || h_kv <= 0 || d <= 0 || page_size <= 0 || h_q % h_kv != 0)
        return -1;
    int64_t total = 0, max_keys = 0;
    for (int32_t b = 0; b < batch; ++b) {
        if (prefix_len[b] < 0 || chunk_len[b] < 0) return -1;
        int64_t n = (int64_t)prefix_len[b] + chunk_len[b];
        int64_t pages_needed = (n + page_size - 1) / page_size;
        if (page_table_offs[b + 1] - page_table_offs[b] < pages_needed) return -1;
        if (n > max_keys) max_keys = n;
        total += chunk_len[b];
    }
    if (rows == NULL) n_rows = total;
    int32_t group = h_q / h_kv;
    int status = 0;
    int64_t n_items = n_rows * h_q;
#pragma omp parallel
    {
        double *scratch = (double *)malloc(sizeof(double) * (size_t)(max_keys > 0 ? max_keys : 1));
        /* every thread reaches the loop below; one without scratch only reports */
        {
#pragma omp for schedule(dynamic, 1)
            for (int64_t it = 0; it < n_items; ++it) {
                int64_t r = it / h_q;
                int32_t h = (int32_t)(it % h_q);
                int64_t tok = rows ? rows[r] : r;
                int rc = 0;
                if (scratch == NULL) {
                    rc = -3;
                } else if (tok < 0 || tok >= total) {
                    rc = -1;
                } else {
                    int32_t b = 0;
                    int64_t start = 0;
                    while (tok >= start + chunk_len[b]) {
                        start += chunk_len[b];
                        ++b;
                    }
                    int64_t j = tok - start;
                    int64_t n_keys = (int64_t)prefix_len[b] + j + 1;
                    rc = attend_one(q + (tok * h_q + h) * (int64_t)d, k_pool, v_pool, num_pages,
                                    page_size, h_kv, d, h / group,
                                    page_table + page_table_offs[b], n_keys, scale, scratch,
                                    out + (r * h_q + h) * (int64_t)d, lse + r * h_q + h);
                }
                if (rc != 0) {
#pragma omp atomic write
                    status = rc;
                }
            }
        }
        free(scratch);
    }
    return status;
}

/*
 * Split-KV decode partial: item i takes query token q_index[i] and attends,
 * without a mask, to keys [0, kv_len[i]) of the paged sequence described by its
 * page-table slice (a KV shard is an item whose slice starts at the shard's
 * first page).  out_partial [items][h_q][d], lse_partial [items][h_q].
 */
int medha_oracle_decode_partial(const uint16_t *q, int32_t num_queries, const uint16_t *k_pool,
                                const uint16_t *v_pool, int32_t num_pages, int32_t page_size,
                                int32_t h_kv, int32_t d, const int32_t *page_table,
                                const int64_t *page_table_offs, const int32_t *q_index,
                                const int32_t *kv_len, int32_t items, int32_t h_q, double scale,
                                double *out_partial, double *lse_partial) {
    if (items < 0 || h_q <= 0 || h_kv <= 0 || d <= 0 || page_size <= 0 || h_q % h_kv != 0)
        return -1;
    int64_t max_keys = 0;
    for (int32_t i = 0; i < items; ++i) {
        if (kv_len[i] < 0 || q_index[i] < 0 || q_index[i] >= num_queries) return -1;
        int64_t pages_needed = ((int64_t)kv_len[i] + page_size - 1) / page_size;
        if (page_table_offs[i + 1] - page_table_offs[i] < pages_needed) return -1;
        if (kv_len[i] > max_keys) max_keys = kv_len[i];
    }
    int32_t group = h_q / h_kv;
    int status = 0;
    int64_t n_items = (int64_t)items * h_q;
#pragma omp parallel
    {
        double *scratch = (double *)malloc(sizeof(double) * (size_t)(max_keys > 0 ? max_keys : 1));
        /* every thread reaches the loop below; one without scratch only reports */
        {
#pragma omp for schedule(dynamic, 1)
            for (int64_t it = 0; it < n_items; ++it) {
                int64_t i = it / h_q;
                int32_t h = (int32_t)(it % h_q);
                int rc = -3;
                if (scratch != NULL)
                    rc = attend_one(q + ((int64_t)q_index[i] * h_q + h) * d, k_pool, v_pool,
                                    num_pages, page_size, h_kv, d, h / group,
                                    page_table + page_table_offs[i], kv_len[i], scale, scratch,
                                    out_partial + (i * h_q + h) * (int64_t)d,
                                    lse_partial + i * h_q + h);
                if (rc != 0) {
#pragma omp atomic write
                    status = rc;
                }
            }
        }
        free(scratch);
    }
    return status;
}

/*
 * KV-cache-parallel partial of a prefill CHUNK (paper section 3.3: the query that is
 * replicated to the KV shards is "either a decode token or a prefill chunk").  Item i is
 * (chunk, shard): query rows q_row[i] .. q_row[i] + chunk_len[i] - 1 of q against the
 * paged key slice of kv_len[i] keys given by the item's page-table slice.  Row j of the
 * chunk sees the first  min(kv_len, max(0, visible0[i] + j))  keys of the slice: a shard
 * that lies wholly before the chunk has visible0 >= kv_len (no mask); the shard that
 * holds the chunk's own keys has visible0 = (chunk's first position) - (shard's first
 * position) + 1; rows with no visible key yield O = 0, LSE = -inf.
 * out_partial [sum chunk_len][h_q][d], lse_partial [sum chunk_len][h_q], items in order.
 */
int medha_oracle_chunk_partial(const uint16_t *q, int32_t num_tokens, const uint16_t *k_pool,
                               const uint16_t *v_pool, int32_t num_pages, int32_t page_size,
                               int32_t h_kv, int32_t d, const int32_t *page_table,
                               const int64_t *page_table_offs, const int32_t *q_row,
                               const int32_t *chunk_len, const int32_t *kv_len,
                               const int32_t *visible0, int32_t items, int32_t h_q,
                               double scale, double *out_partial, double *lse_partial) {
    if (items < 0 || h_q <= 0 || h_kv <= 0 || d <= 0 || page_size <= 0 || h_q % h_kv != 0)
        return -1;
    int64_t max_keys = 0, total_rows = 0;
    for (int32_t i = 0; i < items; ++i) {
        if (kv_len[i] < 0 || chunk_len[i] < 1 || q_row[i] < 0 ||
            (int64_t)q_row[i] + chunk_len[i] > num_tokens)
            return -1;
        int64_t pages_needed = ((int64_t)kv_len[i] + page_size - 1) / page_size;
        if (page_table_offs[i + 1] - page_table_offs[i] < pages_needed) return -1;
        if (kv_len[i] > max_keys) max_keys = kv_len[i];
        total_rows += chunk_len[i];
    }
    /* (item, row in chunk) of every output row */
    int32_t *row_item = (int32_t *)malloc(sizeof(int32_t) * (size_t)(total_rows > 0 ? total_rows : 1));
    int32_t *row_j = (int32_t *)malloc(sizeof(int32_t) * (size_t)(total_rows > 0 ? total_rows : 1));
    if (row_item == NULL || row_j == NULL) {
        free(row_item);
        free(row_j);
        return -3;
    }
    int64_t r = 0;
    for (int32_t i = 0; i < items; ++i)
        for (int32_t j = 0; j < chunk_len[i]; ++j, ++r) {
            row_item[r] = i;
            row_j[r] = j;
        }
    int32_t group = h_q / h_kv;
    int status = 0;
    int64_t n_units = total_rows * h_q;
#pragma omp parallel
    {
        double *scratch = (double *)malloc(sizeof(double) * (size_t)(max_keys > 0 ? max_keys : 1));
        /* every thread reaches the loop below; one without scratch only reports */
        {
#pragma omp for schedule(dynamic, 1)
            for (int64_t u = 0; u < n_units; ++u) {
                int64_t row = u / h_q;
                int32_t h = (int32_t)(u % h_q);
                int32_t i = row_item[row], j = row_j[row];
                int64_t n_keys = (int64_t)visible0[i] + j;
                if (n_keys < 0) n_keys = 0;
                if (n_keys > kv_len[i]) n_keys = kv_len[i];
                int rc = -3;
                if (scratch != NULL)
                    rc = attend_one(q + ((int64_t)(q_row[i] + j) * h_q + h) * d, k_pool, v_pool,
                                    num_pages, page_size, h_kv, d, h / group,
                                    page_table + page_table_offs[i], n_keys, scale, scratch,
                                    out_partial + (row * h_q + h) * (int64_t)d,
                                    lse_partial + row * h_q + h);
                if (rc != 0) {
#pragma omp atomic write
                    status = rc;
                }
            }
        }
        free(scratch);
    }
    free(row_item);
    free(row_j);
    return status;
}

/*
 * Merge of num_splits partial results over disjoint key sets:
 *   LSE = ln sum_s exp(LSE_s),   O = sum_s exp(LSE_s - LSE) O_s.
 * Partials with LSE_s = -inf (no keys) carry weight zero; if every partial is
 * empty the result is O = 0, LSE = -inf.
 * out_partial [num_splits][rows][h_q][d], lse_partial [num_splits][rows][h_q].
 */
int medha_oracle_lse_merge(const double *out_partial, const double *lse_partial,
                           int32_t num_splits, int64_t rows, int32_t h_q, int32_t d, double *out,
                           double *lse) {
    if (num_splits <= 0 || rows < 0 || h_q <= 0 || d <= 0) return -1;
    int64_t n = rows * h_q;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n; ++r) {
        double big = -INFINITY;
        for (int32_t s = 0; s < num_splits; ++s) {
            double v = lse_partial[(int64_t)s * n + r];
            if (v > big) big = v;
        }
        double *o = out + r * d;
        for (int32_t x = 0; x < d; ++x) o[x] = 0.0;
        if (big == -INFINITY) {
            lse[r] = -INFINITY;
            continue;
        }
        double wsum = 0.0;
        for (int32_t s = 0; s < num_splits; ++s) {
            double w = exp(lse_partial[(int64_t)s * n + r] - big);
            wsum += w;
            const double *os = out_partial + ((int64_t)s * n + r) * d;
            if (w != 0.0)
                for (int32_t x = 0; x < d; ++x) o[x] += w * os[x];
        }
        for (int32_t x = 0; x < d; ++x) o[x] /= wsum;
        lse[r] = big + log(wsum);
    }
    return 0;
}

/* Number of OpenMP threads a parallel region uses here (for reporting). */
int medha_oracle_num_threads(void) {
    int n = 1;
#pragma omp parallel
    {
#pragma omp single
        n =
#ifdef _OPENMP
            omp_get_num_threads();
#else
            1;
#endif
    }
    return n;
}
