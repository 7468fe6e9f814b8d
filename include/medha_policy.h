/*
 * medha_policy.h -- host-side scheduling helpers that sit on top of the attention
 * kernels' measured timings: the paper's adaptive chunk-size selection, its
 * prefill-time estimation, and relative-slack (LARS) priorities.  Plain C, host
 * memory only, no GPU needed, no allocation that outlives a call, thread-safe
 * (no state).  Exported by the same shared library as medha.h.
 *
 * Runtime model.  The paper predicts iteration times with an external simulator
 * (section 4.3 "Runtime Prediction"); here the model is five coefficients, in
 * seconds, fitted to times measured on the device at hand:
 *     chunk of c tokens on a cache of kv tokens:
 *         t_token * c + t_pair * (c * kv + c * (c + 1) / 2)
 *     (linear layers per token; attention per visible (query, key) pair -- the
 *     exact causal count, which is what the attention kernels' time follows);
 *     an iteration adds t_fixed once, t_decode per decode request and
 *     t_decode_key per cached key of the decodes.
 * All coefficients must be finite and >= 0, so that time grows with the chunk.
 */
#ifndef MEDHA_POLICY_H_
#define MEDHA_POLICY_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct medha_time_model {
  double t_fixed;
  double t_token;
  double t_pair;
  double t_decode;
  double t_decode_key;
} medha_time_model;

/* Predicted time of one chunk (see above).  Sizes are limited to kv_size <= 2^40 and
 * chunk <= 2^24 in every call of this header (the pair count stays exact in fp64).
 * NaN for a null or invalid model or sizes outside that range. */
double medha_policy_chunk_time(const medha_time_model* model, int64_t kv_size, int64_t chunk);

/* Least-squares fit, in relative error (sum of ((predicted - measured) / measured)^2),
 * of (t_fixed, t_token, t_pair) to n >= 3 measured (kv_size, chunk, seconds)
 * samples; t_decode and t_decode_key are set to 0.
 * A coefficient that comes out negative is clamped to 0 and the others refitted.
 * max_rel_err (optional) receives max |predicted - measured| / measured.
 * Returns 0, or -1 for bad arguments / a singular system. */
int medha_policy_fit_time_model(const int64_t* kv_size, const int64_t* chunk,
                                const double* seconds, int32_t n, medha_time_model* model,
                                double* max_rel_err);

/* The chunk search of Algorithm 2 (appendix "Adaptive Chunk Size Selection"):
 * the largest c in [0, max_chunk] whose predicted chunk time is <= t_budget
 * (the time is a quadratic in c: closed form, corrected by exact evaluation).
 * Returns -1 for bad arguments. */
int64_t medha_policy_max_chunk(const medha_time_model* model, int64_t kv_size, double t_budget,
                               int64_t max_chunk);

/* Algorithm 2, GetChunkSize.  A long prefill is refused (0) when the batch
 * already holds one; a request with relative slack rho yields the fraction
 * min(rho_max, max(0, rho)) of t_target (section 4.3 "Space Sharing"); the chunk
 * is the largest that fits  t_target * (1 - rho) - t_current, at most
 * min(max_chunk, remaining) tokens; 0 if nothing fits.  -1 for bad arguments. */
int64_t medha_policy_get_chunk_size(const medha_time_model* model, int64_t kv_size,
                                    int64_t remaining, int32_t is_long, int32_t batch_has_long,
                                    double rel_slack, double rho_max, double t_current,
                                    double t_target, int64_t max_chunk);

/* Algorithm 3 (appendix "Prefill Time Estimation"), SimulatePrefill: total time to
 * prefill `length` tokens chunk after chunk, each chunk the largest whose
 * iteration (t_fixed + chunk time) stays within t_target; stops early when no
 * chunk fits.  NaN for bad arguments. */
double medha_policy_simulate_prefill(const medha_time_model* model, int64_t length,
                                     double t_target, int64_t max_chunk);

/* Algorithm 3, BuildPrefillCache: cache[i] = SimulatePrefill(i * delta) for
 * i = 0 .. l_max / delta (cache_len must be l_max / delta + 1; caller's memory).
 * One walk over the chunks of the longest length, same values as entry-by-entry.
 * Returns 0, or -1 for bad arguments. */
int medha_policy_build_prefill_cache(const medha_time_model* model, int64_t l_max, int64_t delta,
                                     double t_target, int64_t max_chunk, double* cache,
                                     int64_t cache_len);

/* Algorithm 3, GetRemainingTime: cache(l_total) - cache(l_processed), lengths
 * between entries interpolated linearly, lengths past the end take the last
 * entry.  NaN for bad arguments. */
double medha_policy_remaining_time(const double* cache, int64_t cache_len, int64_t delta,
                                   int64_t l_total, int64_t l_processed);

/* Section 4 "Length-Aware Relative Slack": (arrival + deadline - now - remaining_work)
 * / total_work, the priority key (smallest first). */
double medha_policy_relative_slack(double arrival, double deadline, double now,
                                   double remaining_work, double total_work);

/* The paper's single-server scenario (section 4 "Illustrative Scenario"), for any
 * request list: decisions every `quantum` seconds; policy 0 = first come first
 * served (runs to completion), 1 = earliest deadline first, 2 = smallest relative
 * slack (both re-decided every quantum; ties go to the lower index).  finish and
 * first_start (host, [n], first_start optional) receive the times.  Returns 0, or
 * -1 for bad arguments (n < 1, work <= 0, quantum <= 0, unknown policy). */
int medha_policy_simulate_schedule(int32_t policy, const double* arrival, const double* work,
                                   const double* deadline, int32_t n, double quantum,
                                   double* finish, double* first_start);

#ifdef __cplusplus
}
#endif
#endif /* MEDHA_POLICY_H_ */
