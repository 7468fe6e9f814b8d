// Host-side hardening driver: the library's host code (argument validation, launch planner,
// scheduling helpers) and the C oracle, built with -fsanitize=address,undefined and run on the
// CPU.  No kernel is launched: every call either only plans, or is refused by validation, or
// (attention calls with well-formed arguments) fails at launch for want of a GPU, after the
// planner has run.  Exit code 0 = no finding; the sanitizers abort on their own findings.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <algorithm>
#include <random>
#include <utility>
#include <vector>

#include "medha.h"
#include "medha_policy.h"

extern "C" {
int medha_oracle_chunked_prefill(const uint16_t*, const uint16_t*, const uint16_t*, int32_t,
                                 int32_t, int32_t, int32_t, const int32_t*, const int64_t*,
                                 const int32_t*, const int32_t*, int32_t, int32_t, double,
                                 const int64_t*, int64_t, double*, double*);
int medha_oracle_decode_partial(const uint16_t*, int32_t, const uint16_t*, const uint16_t*,
                                int32_t, int32_t, int32_t, int32_t, const int32_t*,
                                const int64_t*, const int32_t*, const int32_t*, int32_t, int32_t,
                                double, double*, double*);
int medha_oracle_chunk_partial(const uint16_t*, int32_t, const uint16_t*, const uint16_t*,
                               int32_t, int32_t, int32_t, int32_t, const int32_t*,
                               const int64_t*, const int32_t*, const int32_t*, const int32_t*,
                               const int32_t*, int32_t, int32_t, double, double*, double*);
int medha_oracle_lse_merge(const double*, const double*, int32_t, int64_t, int32_t, int32_t,
                           double*, double*);
}

#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
      std::exit(1);                                                        \
    }                                                                      \
  } while (0)

static int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Every (KV head, KV range, row tile) of every sequence is owned by exactly one workgroup slot,
// the ranges cover the keys, and the grids are the sums of the slots.
static void check_plan(const std::vector<int32_t>& prefix, const std::vector<int32_t>& chunk,
                       int h_q, int h_kv, int d, int cus, bool walk_slots) {
  const int n = (int)prefix.size();
  std::vector<medha_plan_entry> e(n);
  int32_t grid_rows = -1, grid_keys = -1;
  size_t ws = 0;
  CHECK(medha_describe_plan(prefix.data(), chunk.data(), n, h_q, h_kv, d, cus, e.data(),
                            &grid_rows, &grid_keys, &ws) == MEDHA_OK);
  const int gqa = h_q / h_kv;
  int64_t total[2] = {0, 0}, part_rows = 0;
  std::vector<std::pair<int32_t, int32_t>> spans[2];  // (work_start, n_slots) per launch
  for (int i = 0; i < n; ++i) {
    const int64_t rows = (int64_t)chunk[i] * gqa;
    CHECK(e[i].mode == (rows <= 32 ? 1 : 0));
    CHECK(e[i].n_row_tiles == ceil_div(rows, e[i].rows_per_wg));
    const int64_t keys = (int64_t)prefix[i] + chunk[i];
    const int64_t kv_tiles = std::max<int64_t>(1, ceil_div(keys, e[i].tile_keys));
    CHECK(e[i].n_split >= 1 && e[i].tiles_per_split >= 1);
    CHECK((int64_t)e[i].n_split * e[i].tiles_per_split >= kv_tiles);
    CHECK((int64_t)(e[i].n_split - 1) * e[i].tiles_per_split < kv_tiles);
    const int64_t items = (int64_t)h_kv * e[i].n_split * e[i].n_row_tiles;
    CHECK(e[i].n_slots == 8 * ceil_div(items, 8));
    spans[e[i].mode].push_back({e[i].work_start, e[i].n_slots});
    total[e[i].mode] += e[i].n_slots;
    if (e[i].n_split > 1) part_rows += (int64_t)e[i].n_split * chunk[i];
    if (walk_slots) {
      std::vector<char> seen((size_t)items, 0);
      for (int u = 0; u < e[i].n_slots; ++u) {
        int32_t kh = -1, sp = -1, rt = -1;
        const int valid = medha_describe_slot(u, h_kv, e[i].n_split, e[i].n_row_tiles, &kh, &sp, &rt);
        if (!valid) continue;
        CHECK(kh >= 0 && kh < h_kv && sp >= 0 && sp < e[i].n_split && rt >= 0 &&
              rt < e[i].n_row_tiles);
        const size_t id = ((size_t)sp * h_kv + kh) * e[i].n_row_tiles + rt;
        CHECK(!seen[id]);
        seen[id] = 1;
      }
      for (char c : seen) CHECK(c);
    }
  }
  // the sequences of a launch tile its grid (in the planner's own order)
  for (int mode = 0; mode < 2; ++mode) {
    std::sort(spans[mode].begin(), spans[mode].end());
    int64_t end = 0;
    for (const auto& sp : spans[mode]) {
      CHECK(sp.first == end);
      end += sp.second;
    }
    CHECK(end == total[mode]);
  }
  CHECK(grid_rows == total[0] && grid_keys == total[1]);
  CHECK(ws >= (size_t)part_rows * h_q * (d + 1) * 4);
  CHECK(ws == medha_chunked_prefill_workspace_bytes(prefix.data(), chunk.data(), n, h_q, h_kv, d) ||
        cus != 0);
}

static void planner_fuzz(std::mt19937_64& rng) {
  const int heads[][2] = {{1, 1}, {2, 1}, {8, 1}, {8, 2}, {32, 8}, {64, 1}, {128, 8}, {7, 7}};
  for (int it = 0; it < 300; ++it) {
    const auto& hh = heads[rng() % 8];
    const int d = (rng() & 1) ? 64 : 128;
    const int cus = (int)(rng() % 4 == 0 ? 1 + rng() % 400 : 256);
    int n;
    switch (rng() % 4) {
      case 0: n = 1; break;
      case 1: n = 1 + (int)(rng() % 70); break;
      case 2: n = 1 + (int)(rng() % 1000); break;
      default: n = it % 50 == 3 ? 10000 : 1 + (int)(rng() % 300);
    }
    std::vector<int32_t> prefix(n), chunk(n);
    int64_t rows = 0;
    for (int i = 0; i < n; ++i) {
      const int kind = (int)(rng() % 8);
      chunk[i] = kind < 4 ? 1 : (kind < 7 ? 1 + (int)(rng() % 300) : 1 + (int)(rng() % 20000));
      if (n == 1 && it % 7 == 0) chunk[i] = 1 + (int)(rng() % 100000);
      const uint64_t span = kind == 0 ? 64 : (kind < 6 ? 100000 : (uint64_t)INT32_MAX);
      int64_t p = (int64_t)(rng() % span);
      if (it % 11 == 0 && i == 0) p = (int64_t)INT32_MAX - chunk[i];  // the largest sequence
      p = std::min<int64_t>(p, (int64_t)INT32_MAX - chunk[i]);
      prefix[i] = (int32_t)p;
      rows += chunk[i];
    }
    if (rows > INT32_MAX) continue;
    check_plan(prefix, chunk, hh[0], hh[1], d, cus, n <= 300);
  }
}

static void validation_paths() {
  // fake but well-aligned "device" addresses: the host code never dereferences them
  void* dev = reinterpret_cast<void*>(0x7f0000000000ull);
  medha_kv_cache kv{dev, dev, 1000, 16, 2, 128};
  const int64_t offs[3] = {0, 10, 20};
  const int32_t prefix[2] = {100, 50}, chunk[2] = {20, 1};
  float* out = reinterpret_cast<float*>(dev);
  // bad arguments: refused before anything else happens
  CHECK(medha_chunked_prefill_attn(dev, &kv, (const int32_t*)dev, offs, prefix, chunk, -1, 8, .1f,
                                   out, out, nullptr, 0, nullptr) == MEDHA_ERR_INVALID_ARG);
  CHECK(medha_chunked_prefill_attn(nullptr, &kv, (const int32_t*)dev, offs, prefix, chunk, 2, 8,
                                   .1f, out, out, nullptr, 0, nullptr) == MEDHA_ERR_INVALID_ARG);
  CHECK(medha_chunked_prefill_attn(dev, &kv, (const int32_t*)dev, offs, prefix, chunk, 2, 7, .1f,
                                   out, out, nullptr, 0, nullptr) == MEDHA_ERR_INVALID_ARG);
  CHECK(medha_chunked_prefill_attn(dev, nullptr, (const int32_t*)dev, offs, prefix, chunk, 2, 8,
                                   .1f, out, out, nullptr, 0, nullptr) == MEDHA_ERR_INVALID_ARG);
  medha_kv_cache kv96 = kv;
  kv96.head_dim = 96;
  CHECK(medha_chunked_prefill_attn(dev, &kv96, (const int32_t*)dev, offs, prefix, chunk, 2, 8, .1f,
                                   out, out, nullptr, 0, nullptr) == MEDHA_ERR_UNSUPPORTED);
  const int32_t bad_prefix[2] = {INT32_MAX, 50};
  CHECK(medha_chunked_prefill_attn(dev, &kv, (const int32_t*)dev, offs, bad_prefix, chunk, 2, 8,
                                   .1f, out, out, nullptr, 0, nullptr) == MEDHA_ERR_INVALID_ARG);
  CHECK(medha_chunked_prefill_attn(dev, &kv, (const int32_t*)dev, offs, prefix, chunk, 2, 8, NAN,
                                   out, out, nullptr, 0, nullptr) == MEDHA_ERR_INVALID_ARG);
  CHECK(medha_chunked_prefill_attn_noalloc(dev, &kv, (const int32_t*)dev, offs, prefix, chunk, -1,
                                           8, .1f, out, out, nullptr) != MEDHA_OK);
  // a batch that needs a workspace, without one
  const int32_t long_prefix[1] = {5000000}, one[1] = {64};
  const int64_t long_offs[2] = {0, 400000};
  CHECK(medha_chunked_prefill_workspace_bytes(long_prefix, one, 1, 8, 2, 128) > 256);
  CHECK(medha_chunked_prefill_attn(dev, &kv, (const int32_t*)dev, long_offs, long_prefix, one, 1,
                                   8, .1f, out, out, nullptr, 0, nullptr) == MEDHA_ERR_WORKSPACE);
  // well-formed, more than 64 sequences in both kernels: the planner and the grouping of the
  // launches run; with no GPU the launch itself fails (with one, this driver is not run)
  {
    const int n = 300;
    std::vector<int32_t> p(n), c(n);
    std::vector<int64_t> o(n + 1, 0);
    for (int i = 0; i < n; ++i) {
      p[i] = 100 + 37 * i;
      c[i] = i % 3 == 0 ? 40 : 1;
      o[i + 1] = o[i] + ceil_div(p[i] + c[i], 16);
    }
    const int rc = medha_chunked_prefill_attn(dev, &kv, (const int32_t*)dev, o.data(), p.data(),
                                              c.data(), n, 8, .1f, out, out, dev, (size_t)1 << 30,
                                              nullptr);
    CHECK(rc == MEDHA_ERR_HIP || rc == MEDHA_OK);
  }
  // decode / chunk partial / merge / append validation
  const int32_t qi[2] = {0, 5}, kl[2] = {100, 50};
  CHECK(medha_decode_partial_attn(dev, 2, &kv, (const int32_t*)dev, offs, qi, kl, 2, 8, .1f, out,
                                  out, nullptr, 0, nullptr) == MEDHA_ERR_INVALID_ARG);
  const int32_t neg[2] = {-1, 50};
  CHECK(medha_decode_partial_attn(dev, 8, &kv, (const int32_t*)dev, offs, qi, neg, 2, 8, .1f, out,
                                  out, nullptr, 0, nullptr) == MEDHA_ERR_INVALID_ARG);
  CHECK(medha_decode_partial_workspace_bytes(neg, 2, 8, 2, 128) == 0);
  const int32_t q_row[1] = {0}, c20[1] = {20}, k120[1] = {120}, vis[1] = {(1 << 30) + 1};
  CHECK(medha_chunk_partial_attn(dev, 20, &kv, (const int32_t*)dev, offs, q_row, c20, k120, vis, 1,
                                 8, .1f, out, out, nullptr, 0, nullptr) == MEDHA_ERR_INVALID_ARG);
  CHECK(medha_lse_merge(out, out, 0, 10, 8, 128, out, out, nullptr) == MEDHA_ERR_INVALID_ARG);
  CHECK(medha_lse_merge(out, out, 2, 10, 8, 126, out, out, nullptr) == MEDHA_ERR_UNSUPPORTED);
  CHECK(medha_lse_merge(out, out, 2, INT64_MAX / 4, 8, 128, out, out, nullptr) ==
        MEDHA_ERR_INVALID_ARG);
  CHECK(medha_kv_append(dev, dev, &kv, (const int32_t*)dev, offs, neg, chunk, 2, nullptr) ==
        MEDHA_ERR_INVALID_ARG);
  CHECK(medha_strerror(-3) != nullptr && medha_strerror(12345) != nullptr);
}

static void policy_paths(std::mt19937_64& rng) {
  std::uniform_real_distribution<double> u(0.0, 1.0);
  for (int it = 0; it < 2000; ++it) {
    medha_time_model m{1e-4 * u(rng), 1e-8 * u(rng) * (it % 5 != 0), 1e-11 * u(rng) * (it % 7 != 0),
                       0.0, 0.0};
    const int64_t kv = (int64_t)(u(rng) * (it % 3 ? 2e6 : 1e12));
    const int64_t hi = 1 + (int64_t)(u(rng) * (it % 4 ? 20000 : (1 << 24) - 1));
    const double budget = it % 13 == 0 ? -1.0 : 0.05 * u(rng);
    const int64_t c = medha_policy_max_chunk(&m, kv, budget, hi);
    CHECK(c >= 0 && c <= hi);
    if (c > 0) CHECK(medha_policy_chunk_time(&m, kv, c) <= budget);
    if (c < hi && budget >= 0.0) CHECK(!(medha_policy_chunk_time(&m, kv, c + 1) <= budget));
    const int64_t g = medha_policy_get_chunk_size(&m, kv, 1 + (int64_t)(u(rng) * 1e6), it & 1, 0,
                                                  2.0 * u(rng) - 0.5, 0.4, 1e-3 * u(rng), 0.02, hi);
    CHECK(g >= 0 && g <= hi);
  }
  medha_time_model m{1e-4, 1e-8, 4e-12, 0.0, 0.0};
  const double t = medha_policy_simulate_prefill(&m, 1 << 20, 0.02, 16384);
  CHECK(std::isfinite(t) && t > 0.0);
  const int64_t l_max = 1 << 20, delta = 4096, len = l_max / delta + 1;
  std::vector<double> cache((size_t)len);
  CHECK(medha_policy_build_prefill_cache(&m, l_max, delta, 0.02, 16384, cache.data(), len) == 0);
  CHECK(medha_policy_build_prefill_cache(&m, l_max, delta, 0.02, 16384, cache.data(), len - 1) != 0);
  for (int64_t i = 1; i < len; ++i) CHECK(cache[(size_t)i] >= cache[(size_t)i - 1]);
  CHECK(std::fabs(cache.back() - t) <= 1e-9 * t);
  CHECK(medha_policy_remaining_time(cache.data(), len, delta, l_max, 0) == cache.back());
  CHECK(medha_policy_remaining_time(cache.data(), len, delta, 5 * l_max, l_max) == 0.0);
  const double arrival[3] = {0, 5, 5}, work[3] = {10, 0.5, 0.5}, deadline[3] = {20, 1, 1};
  double finish[3], start[3];
  for (int pol = 0; pol < 3; ++pol)
    CHECK(medha_policy_simulate_schedule(pol, arrival, work, deadline, 3, 0.1, finish, start) == 0);
  CHECK(medha_policy_simulate_schedule(3, arrival, work, deadline, 3, 0.1, finish, start) != 0);
  int64_t kvs[5] = {0, 1000, 50000, 100000, 1000000}, cs[5] = {512, 1024, 2048, 4096, 8192};
  double secs[5];
  for (int i = 0; i < 5; ++i) secs[i] = 1e-4 + medha_policy_chunk_time(&m, kvs[i], cs[i]);
  medha_time_model fit{};
  double err = 1.0;
  CHECK(medha_policy_fit_time_model(kvs, cs, secs, 5, &fit, &err) == 0 && err < 1e-6);
  CHECK(medha_policy_fit_time_model(kvs, cs, secs, 2, &fit, &err) != 0);
}

static void oracle_paths(std::mt19937_64& rng) {
  // tiny random cases through every oracle entry, including empty and ragged ones; the
  // sanitizers watch the indexing
  for (int it = 0; it < 40; ++it) {
    const int h_kv = 1 + (int)(rng() % 2), gqa = 1 + (int)(rng() % 3), h_q = h_kv * gqa;
    const int d = 8 * (1 + (int)(rng() % 3)), batch = 1 + (int)(rng() % 3);
    std::vector<int32_t> prefix(batch), chunk(batch), pt;
    std::vector<int64_t> offs(batch + 1, 0);
    int tokens = 0;
    for (int b = 0; b < batch; ++b) {
      prefix[b] = (int32_t)(rng() % 40);
      chunk[b] = (int32_t)(rng() % 20) + (it % 5 == 0 ? 0 : 1);
      offs[b + 1] = offs[b] + ceil_div(prefix[b] + chunk[b], 16);
      tokens += chunk[b];
    }
    const int num_pages = (int)offs[batch] + 2;
    for (int i = 0; i < offs[batch]; ++i) pt.push_back((int32_t)((i * 7 + 1) % num_pages));
    std::vector<uint16_t> q((size_t)std::max(1, tokens) * h_q * d),
        k((size_t)num_pages * h_kv * 16 * d), v(k.size());
    for (auto& x : q) x = (uint16_t)(0x3c00 + rng() % 0x400);
    for (auto& x : k) x = (uint16_t)(0x3c00 + rng() % 0x400) | (uint16_t)((rng() & 1) << 15);
    for (auto& x : v) x = (uint16_t)(0x3c00 + rng() % 0x400);
    std::vector<double> out((size_t)std::max(2, tokens) * h_q * d),
        lse((size_t)std::max(2, tokens) * h_q);
    CHECK(medha_oracle_chunked_prefill(q.data(), k.data(), v.data(), num_pages, 16, h_kv, d,
                                       pt.data(), offs.data(), prefix.data(), chunk.data(), batch,
                                       h_q, 0.3, nullptr, 0, out.data(), lse.data()) == 0);
    if (tokens > 0) {
      const int64_t rows[2] = {0, tokens - 1};
      CHECK(medha_oracle_chunked_prefill(q.data(), k.data(), v.data(), num_pages, 16, h_kv, d,
                                         pt.data(), offs.data(), prefix.data(), chunk.data(),
                                         batch, h_q, 0.3, rows, 2, out.data(), lse.data()) == 0);
      const int64_t bad_rows[1] = {tokens};
      CHECK(medha_oracle_chunked_prefill(q.data(), k.data(), v.data(), num_pages, 16, h_kv, d,
                                         pt.data(), offs.data(), prefix.data(), chunk.data(),
                                         batch, h_q, 0.3, bad_rows, 1, out.data(), lse.data()) != 0);
    }
    // decode partials over the same sequences (kv_len = prefix, may be 0), then a merge
    std::vector<int32_t> q_index(batch, 0);
    std::vector<double> po((size_t)batch * h_q * d), pl((size_t)batch * h_q);
    if (tokens > 0) {
      CHECK(medha_oracle_decode_partial(q.data(), tokens, k.data(), v.data(), num_pages, 16, h_kv,
                                        d, pt.data(), offs.data(), q_index.data(), prefix.data(),
                                        batch, h_q, 0.3, po.data(), pl.data()) == 0);
      std::vector<double> mo((size_t)h_q * d), ml((size_t)h_q);
      CHECK(medha_oracle_lse_merge(po.data(), pl.data(), batch, 1, h_q, d, mo.data(), ml.data()) == 0);
      // chunk partial: each sequence's chunk against its own keys, partly masked
      std::vector<int32_t> q_row(batch), kv_len(batch), vis(batch), c1(batch);
      int row = 0, total = 0;
      for (int b = 0; b < batch; ++b) {
        q_row[b] = row;
        c1[b] = std::max(1, (int)chunk[b]);
        if (row + c1[b] > tokens) c1[b] = tokens - row;
        if (c1[b] < 1) { c1[b] = 1; q_row[b] = 0; }
        kv_len[b] = prefix[b] + chunk[b];
        vis[b] = prefix[b] + 1 - (int)(rng() % 5);
        row += chunk[b];
        total += c1[b];
      }
      std::vector<double> co((size_t)total * h_q * d), cl((size_t)total * h_q);
      CHECK(medha_oracle_chunk_partial(q.data(), tokens, k.data(), v.data(), num_pages, 16, h_kv,
                                       d, pt.data(), offs.data(), q_row.data(), c1.data(),
                                       kv_len.data(), vis.data(), batch, h_q, 0.3, co.data(),
                                       cl.data()) == 0);
    }
  }
}

int main() {
  std::mt19937_64 rng(20240917);
  planner_fuzz(rng);
  std::puts("planner fuzz ok");
  validation_paths();
  std::puts("validation paths ok");
  policy_paths(rng);
  std::puts("policy paths ok");
  oracle_paths(rng);
  std::puts("oracle paths ok");
  return 0;
}
