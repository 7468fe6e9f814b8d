// Host-side scheduling helpers on top of the attention kernels' measured timings:
// adaptive chunk-size selection (paper appendix, Algorithm 2), prefill-time
// estimation (Algorithm 3) and relative-slack priorities (section 4).  No GPU code.
#pragma once

#include <cmath>
#include <cstdint>
#include <limits>
#include <vector>

#include "medha_policy.h"

namespace medha {
namespace policy {

inline bool valid(const medha_time_model* m) {
  if (m == nullptr) return false;
  const double c[5] = {m->t_fixed, m->t_token, m->t_pair, m->t_decode, m->t_decode_key};
  for (double x : c)
    if (!std::isfinite(x) || x < 0.0) return false;
  return true;
}

// t_token * c + t_pair * (c * kv + c (c + 1) / 2), for kv <= 2^40 and c <= 2^24 (the callers
// check): c * kv can pass 2^63, so that product is taken in floating point (both factors are
// exact there and the product is correctly rounded); c (c + 1) stays below 2^49.
inline double chunk_time(const medha_time_model& m, int64_t kv, int64_t c) {
  const double pairs = (double)c * (double)kv + (double)(c * (c + 1)) / 2.0;
  return m.t_token * (double)c + m.t_pair * pairs;
}

// Largest c in [0, hi] with chunk_time(kv, c) <= budget.  The time is a quadratic in c,
//     (t_pair / 2) c^2 + (t_token + t_pair (kv + 1/2)) c,
// so the answer is the floor of its positive root at `budget`, taken in closed form and then
// walked by the one or two steps the rounding of the root may be off, with chunk_time itself
// as the judge (it grows with c, so the walk ends at the exact answer).
inline int64_t max_chunk(const medha_time_model& m, int64_t kv, double budget, int64_t hi) {
  if (hi < 1 || !(budget >= 0.0)) return 0;
  const double a = 0.5 * m.t_pair;
  const double b = m.t_token + m.t_pair * ((double)kv + 0.5);
  double root;
  if (a > 0.0) {
    // the form without cancellation: 2 budget / (b + sqrt(b^2 + 4 a budget))
    root = 2.0 * budget / (b + std::sqrt(b * b + 4.0 * a * budget));
  } else if (b > 0.0) {
    root = budget / b;
  } else {
    root = (double)hi;  // every chunk is free
  }
  int64_t c = root >= (double)hi ? hi : (root > 0.0 ? (int64_t)root : 0);
  while (c < hi && chunk_time(m, kv, c + 1) <= budget) ++c;
  while (c > 0 && !(chunk_time(m, kv, c) <= budget)) --c;
  return c;
}

// Time of a whole prefill of `length` tokens when every iteration takes the largest chunk
// that fits t_target (Algorithm 3's estimate): a walk over chunk boundaries.  A position
// where not even one token fits ends the estimate there.
inline double simulate_prefill(const medha_time_model& m, int64_t length, double t_target,
                               int64_t max_c) {
  const double per_iteration = t_target - m.t_fixed;  // what is left for the chunk itself
  double elapsed = 0.0;
  for (int64_t pos = 0; pos < length;) {
    const int64_t room = length - pos;
    const int64_t c = max_chunk(m, pos, per_iteration, room < max_c ? room : max_c);
    if (c == 0) break;
    elapsed += m.t_fixed + chunk_time(m, pos, c);
    pos += c;
  }
  return elapsed;
}

// Solves the k x k system a x = b in place (partial pivoting); false if singular.
inline bool solve(double a[3][3], double b[3], int k) {
  for (int i = 0; i < k; ++i) {
    int p = i;
    for (int r = i + 1; r < k; ++r)
      if (std::fabs(a[r][i]) > std::fabs(a[p][i])) p = r;
    if (!(std::fabs(a[p][i]) > 0.0)) return false;
    for (int c = 0; c < k; ++c) std::swap(a[i][c], a[p][c]);
    std::swap(b[i], b[p]);
    for (int r = i + 1; r < k; ++r) {
      const double f = a[r][i] / a[i][i];
      for (int c = i; c < k; ++c) a[r][c] -= f * a[i][c];
      b[r] -= f * b[i];
    }
  }
  for (int i = k - 1; i >= 0; --i) {
    for (int c = i + 1; c < k; ++c) b[i] -= a[i][c] * b[c];
    b[i] /= a[i][i];
  }
  return true;
}

// Least squares in RELATIVE error -- minimises sum ((prediction - y) / y)^2, i.e. every row
// is weighted by 1 / y, so that a 0.5 ms sample counts like a 30 ms one -- over the columns
// listed in `cols` (0: constant, 1: tokens, 2: pairs), each column scaled to unit maximum so
// that the normal equations stay well conditioned.
inline bool fit_columns(const std::vector<double> (&x)[3], const double* y, int n,
                        const int* cols, int k, double out[3]) {
  double scale[3] = {1.0, 1.0, 1.0};
  for (int j = 0; j < k; ++j) {
    double mx = 0.0;
    for (int i = 0; i < n; ++i) mx = std::max(mx, std::fabs(x[cols[j]][i]));
    if (!(mx > 0.0)) return false;
    scale[j] = mx;
  }
  double a[3][3] = {{0}}, b[3] = {0, 0, 0};
  for (int i = 0; i < n; ++i)
    for (int r = 0; r < k; ++r) {
      const double xr = x[cols[r]][i] / scale[r] / y[i];
      b[r] += xr;  // the weighted target is y / y = 1
      for (int c = 0; c < k; ++c) a[r][c] += xr * (x[cols[c]][i] / scale[c] / y[i]);
    }
  if (!solve(a, b, k)) return false;
  out[0] = out[1] = out[2] = 0.0;
  for (int j = 0; j < k; ++j) out[cols[j]] = b[j] / scale[j];
  return true;
}

}  // namespace policy
}  // namespace medha
