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

// t_token * c + t_pair * (c * kv + c (c + 1) / 2); sizes stay below 2^53 in the products
inline double chunk_time(const medha_time_model& m, int64_t kv, int64_t c) {
  const double pairs = (double)(c * kv) + (double)(c * (c + 1)) / 2.0;
  return m.t_token * (double)c + m.t_pair * pairs;
}

// Largest c in [0, hi] with chunk_time(kv, c) <= budget (the time grows with c).
inline int64_t max_chunk(const medha_time_model& m, int64_t kv, double budget, int64_t hi) {
  int64_t lo = 0;  // always fits when budget >= 0 ... checked by the caller for c >= 1 below
  if (hi < 1 || !(chunk_time(m, kv, 1) <= budget)) return 0;
  lo = 1;
  while (lo < hi) {
    const int64_t mid = lo + (hi - lo + 1) / 2;
    if (chunk_time(m, kv, mid) <= budget) lo = mid; else hi = mid - 1;
  }
  return lo;
}

inline double simulate_prefill(const medha_time_model& m, int64_t length, double t_target,
                               int64_t max_c) {
  double total = 0.0;
  int64_t done = 0;
  while (done < length) {
    const int64_t c = max_chunk(m, done, t_target - m.t_fixed, std::min(max_c, length - done));
    if (c == 0) break;
    total += m.t_fixed + chunk_time(m, done, c);
    done += c;
  }
  return total;
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
