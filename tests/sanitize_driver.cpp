// Host-only exercise of the library's host code under AddressSanitizer and
// UndefinedBehaviorSanitizer (built and run by tests/test_host_sanitizers.py): coarsening of
// random graphs with every accessor, plans, pair orders, schedules, the tuning record,
// argument checks.  No device call is made, so it runs without a GPU.
#include <cstdio>
#include <cstdlib>
#include <random>
#include <set>
#include <vector>
#include "gosh.h"
int main() {
  std::mt19937_64 rng(7);
  for (int trial = 0; trial < 60; ++trial) {
    const int64_t n = 2 + rng() % (trial < 40 ? 300 : 20000);
    const int64_t m = rng() % (6 * n);
    std::vector<std::set<int32_t>> rows(n);
    for (int64_t e = 0; e < m; ++e) {
      int32_t a = rng() % n, b = rng() % n;
      if (trial % 7 == 0) b = std::min<int64_t>(n - 1, a + 1 + rng() % 3);  // chains
      if (a == b) continue;
      rows[a].insert(b); rows[b].insert(a);
    }
    std::vector<int64_t> x64(n + 1, 0); std::vector<int32_t> x32(n + 1, 0), adj;
    for (int64_t v = 0; v < n; ++v) { for (int32_t u : rows[v]) adj.push_back(u); x64[v + 1] = adj.size(); x32[v + 1] = (int32_t)adj.size(); }
    gosh_csr g{n, (int64_t)adj.size(), trial % 2 ? (const void*)x64.data() : (const void*)x32.data(), adj.data(), trial % 2};
    if (gosh_csr_validate(&g) != 0) { printf("validate failed: %s\n", gosh_last_error()); return 1; }
    gosh_hierarchy* h = nullptr;
    const int threads = 1 + trial % 6;
    if (gosh_coarsen(&g, 1 + rng() % 50, trial % 3 ? 1.0 : 0.8, 2 + rng() % 20, threads, &h) != 0) { printf("coarsen failed: %s\n", gosh_last_error()); return 1; }
    const int D = gosh_hierarchy_levels(h);
    int64_t total = g.nnz;
    for (int i = 0; i < D; ++i) {
      gosh_csr v; gosh_hierarchy_graph(h, i, &v);
      if (gosh_csr_validate(&v) != 0) { printf("level %d invalid: %s\n", i, gosh_last_error()); return 1; }
      const int64_t* mult; int64_t len; gosh_hierarchy_mult(h, i, &mult, &len);
      if (i > 0) { int64_t s = 0; for (int64_t e = 0; e < len; ++e) s += mult[e]; if (s > total || len != v.nnz) { printf("weights\n"); return 1; } total = s; }
      if (i + 1 < D) { const int32_t* map; int64_t ml; gosh_hierarchy_map(h, i, &map, &ml); gosh_csr nx; gosh_hierarchy_graph(h, i + 1, &nx); for (int64_t q = 0; q < ml; ++q) if (map[q] < 0 || map[q] >= nx.n) { printf("map\n"); return 1; } double ms[3]; gosh_hierarchy_times(h, i, ms); }
    }
    gosh_hierarchy_release_device(h);
    gosh_hierarchy_free(h);
    int32_t K; int64_t rot; uint64_t bytes;
    gosh_parts_plan(n, 32, 10 + trial, 1 << 20, 3, 4, 5, &K, &rot, &bytes);
    std::vector<int32_t> a(K * (K + 1) / 2), b(K * (K + 1) / 2);
    gosh_pair_order(K, a.data(), b.data());
    std::vector<int64_t> e(5); gosh_epoch_split(100 + trial, 0.3, 5, e.data());
    const int32_t R = 1 + trial % 4;
    gosh_pair_order_blocked(K, R, a.data(), b.data());
    for (size_t q = 0; q < a.size(); ++q) if (a[q] < b[q] || a[q] >= K) { printf("blocked order\n"); return 1; }
    if (gosh_pair_level_parts(10 + trial, n, 1 + trial, 5) > 16) { printf("pair level parts\n"); return 1; }
    if (gosh_lr(0.05f, trial, 100) <= 0.f) { printf("lr\n"); return 1; }
  }
  gosh_tuning t;
  gosh_tuning_defaults(&t);
  t.hot_min_degree = 9;
  if (gosh_set_tuning(&t) != 0 || gosh_get_tuning(&t) != 0 || t.hot_min_degree != 9) { printf("tuning\n"); return 1; }
  t.max_waves = 0;
  if (gosh_set_tuning(&t) == 0 || gosh_set_tuning(nullptr) != 0) { printf("tuning range\n"); return 1; }
  // argument checks that fail before any device call
  gosh_csr bad{0, 0, nullptr, nullptr, 0};
  float dummy[4] = {0, 0, 0, 0};
  if (gosh_train_epoch(&bad, dummy, 6, 3, 0.1f, 1, 0, 0, 0, nullptr) == 0) { printf("argument check\n"); return 1; }
  if (gosh_train_epoch_static(&bad, dummy, 6, 3, 0.1f, 1, 0, 0, 0, nullptr) == 0) { printf("argument check\n"); return 1; }
  if (gosh_row_probe(dummy, 1, 4, 1, 1, 9, nullptr) == 0) { printf("argument check\n"); return 1; }
  if (gosh_epoch_split(3, 0.5, 5, nullptr) == 0) { printf("argument check\n"); return 1; }
  printf("asan driver ok\n");
  return 0;
}
