// MultiEdgeCollapse coarsening hierarchy (Alg. 4 of the paper) on the host.
//
// The marking sweep keeps the sequential semantics of Alg. 4 (its result depends on
// the visiting order, and the maps have to be reproducible bit for bit), but the
// stages around it -- degree counting sort, grouping by cluster, rebuilding the CSR
// of the coarse graph -- are parallel with OpenMP in a way that cannot change the
// output: every thread owns a contiguous range and writes to precomputed offsets.
#include <omp.h>

#include <algorithm>
#include <cstring>
#include <new>
#include <numeric>
#include <vector>

#include "gosh_common.h"

struct gosh_hierarchy {
  struct Level {
    // Level 0 borrows the caller's arrays; coarser levels own theirs (64-bit offsets).
    gosh_csr view{};
    std::vector<int64_t> xadj;
    std::vector<int32_t> adj;
    std::vector<int64_t> mult;  // fine entries merged into each entry (empty at level 0)
    std::vector<int32_t> map;   // this level -> next coarser level (empty on the last)
  };
  std::vector<Level> levels;
};

namespace {

template <typename OffT>
struct Csr {
  int64_t n;
  const OffT *xadj;
  const int32_t *adj;
  int64_t degree(int64_t v) const { return static_cast<int64_t>(xadj[v + 1] - xadj[v]); }
};

// Vertices by degree, largest first, ties by ascending id (stable counting sort).
template <typename OffT>
void degree_order(const Csr<OffT> &g, int threads, std::vector<int32_t> &order) {
  const int64_t n = g.n;
  int64_t max_deg = 0;
#pragma omp parallel for num_threads(threads) reduction(max : max_deg) schedule(static)
  for (int64_t v = 0; v < n; ++v) max_deg = std::max(max_deg, g.degree(v));
  order.resize(static_cast<size_t>(n));
  // Per-thread histograms over contiguous id ranges; bucket b = max_deg - degree.
  // Huge maximum degrees with many threads would make the histograms large, so the
  // thread count is bounded by the memory they need.
  int t_used = threads;
  while (t_used > 1 && static_cast<int64_t>(t_used) * (max_deg + 1) > (int64_t{1} << 28)) t_used /= 2;
  std::vector<std::vector<int64_t>> hist(static_cast<size_t>(t_used),
                                         std::vector<int64_t>(static_cast<size_t>(max_deg) + 1, 0));
  auto range = [&](int t, int64_t &lo, int64_t &hi) {
    lo = n * t / t_used;
    hi = n * (t + 1) / t_used;
  };
#pragma omp parallel num_threads(t_used)
  {
    const int t = omp_get_thread_num();
    int64_t lo, hi;
    range(t, lo, hi);
    auto &h = hist[static_cast<size_t>(t)];
    for (int64_t v = lo; v < hi; ++v) ++h[static_cast<size_t>(max_deg - g.degree(v))];
  }
  // Exclusive scan in (bucket, thread) order gives every thread its write cursor.
  int64_t running = 0;
  for (int64_t b = 0; b <= max_deg; ++b)
    for (int t = 0; t < t_used; ++t) {
      int64_t c = hist[static_cast<size_t>(t)][static_cast<size_t>(b)];
      hist[static_cast<size_t>(t)][static_cast<size_t>(b)] = running;
      running += c;
    }
#pragma omp parallel num_threads(t_used)
  {
    const int t = omp_get_thread_num();
    int64_t lo, hi;
    range(t, lo, hi);
    auto &h = hist[static_cast<size_t>(t)];
    for (int64_t v = lo; v < hi; ++v)
      order[static_cast<size_t>(h[static_cast<size_t>(max_deg - g.degree(v))]++)] = static_cast<int32_t>(v);
  }
}

// The marking sweep of Alg. 4.  Returns the number of clusters.
template <typename OffT>
int64_t mark_clusters(const Csr<OffT> &g, int64_t nnz, const std::vector<int32_t> &order,
                      std::vector<int32_t> &map) {
  const int64_t n = g.n;
  map.assign(static_cast<size_t>(n), -1);
  // deg <= |E|/|V|  <=>  deg * n <= nnz (exact, no rounding)
  std::vector<uint8_t> low(static_cast<size_t>(n));
  for (int64_t v = 0; v < n; ++v) low[static_cast<size_t>(v)] = g.degree(v) * n <= nnz;
  int32_t next_cluster = 0;
  for (int64_t t = 0; t < n; ++t) {
    const int32_t hub = order[static_cast<size_t>(t)];
    if (map[static_cast<size_t>(hub)] != -1) continue;
    const int32_t cluster = next_cluster++;
    map[static_cast<size_t>(hub)] = cluster;
    const bool hub_low = low[static_cast<size_t>(hub)];
    const OffT end = g.xadj[hub + 1];
    for (OffT e = g.xadj[hub]; e < end; ++e) {
      const int32_t u = g.adj[e];
      if ((hub_low || low[static_cast<size_t>(u)]) && map[static_cast<size_t>(u)] == -1)
        map[static_cast<size_t>(u)] = cluster;
    }
  }
  return next_cluster;
}

// Quotient graph of g under map: entry (a, b) for every fine entry (x, y) with
// a = map[x] != map[y] = b, parallel entries merged (their multiplicities added),
// rows ascending.
template <typename OffT>
void build_coarse(const Csr<OffT> &g, const int64_t *mult_in, const std::vector<int32_t> &map,
                  int64_t n_coarse, int threads, gosh_hierarchy::Level &out) {
  const int64_t n = g.n;
  // members of every cluster, by counting sort on the cluster id (stable: ascending id)
  std::vector<int64_t> first(static_cast<size_t>(n_coarse) + 1, 0);
  for (int64_t v = 0; v < n; ++v) ++first[static_cast<size_t>(map[static_cast<size_t>(v)]) + 1];
  for (int64_t a = 0; a < n_coarse; ++a) first[static_cast<size_t>(a) + 1] += first[static_cast<size_t>(a)];
  std::vector<int32_t> members(static_cast<size_t>(n));
  {
    std::vector<int64_t> cursor(first.begin(), first.end() - 1);
    for (int64_t v = 0; v < n; ++v)
      members[static_cast<size_t>(cursor[static_cast<size_t>(map[static_cast<size_t>(v)])]++)] = static_cast<int32_t>(v);
  }

  // Pass 1 builds each coarse row in a thread-private buffer and records its length;
  // pass 2 (after a scan of the lengths) copies the rows to their final place.  Rows
  // are produced by the same code in both passes, so only their order in memory, not
  // their content, depends on the schedule.
  out.xadj.assign(static_cast<size_t>(n_coarse) + 1, 0);
  struct Entry {
    int32_t to;
    int64_t mult;
  };
  auto make_row = [&](int64_t a, std::vector<Entry> &row) {
    row.clear();
    for (int64_t m = first[static_cast<size_t>(a)]; m < first[static_cast<size_t>(a) + 1]; ++m) {
      const int32_t x = members[static_cast<size_t>(m)];
      for (OffT e = g.xadj[x]; e < g.xadj[x + 1]; ++e) {
        const int32_t b = map[static_cast<size_t>(g.adj[e])];
        if (b != a) row.push_back(Entry{b, mult_in ? mult_in[e] : 1});
      }
    }
    std::sort(row.begin(), row.end(), [](const Entry &p, const Entry &q) { return p.to < q.to; });
    size_t w = 0;
    for (size_t r = 0; r < row.size(); ++r) {
      if (w > 0 && row[w - 1].to == row[r].to) row[w - 1].mult += row[r].mult;
      else row[w++] = row[r];
    }
    row.resize(w);
  };
#pragma omp parallel num_threads(threads)
  {
    std::vector<Entry> row;
#pragma omp for schedule(dynamic, 256)
    for (int64_t a = 0; a < n_coarse; ++a) {
      make_row(a, row);
      out.xadj[static_cast<size_t>(a) + 1] = static_cast<int64_t>(row.size());
    }
  }
  for (int64_t a = 0; a < n_coarse; ++a) out.xadj[static_cast<size_t>(a) + 1] += out.xadj[static_cast<size_t>(a)];
  const int64_t nnz_coarse = out.xadj[static_cast<size_t>(n_coarse)];
  out.adj.resize(static_cast<size_t>(nnz_coarse));
  out.mult.resize(static_cast<size_t>(nnz_coarse));
#pragma omp parallel num_threads(threads)
  {
    std::vector<Entry> row;
#pragma omp for schedule(dynamic, 256)
    for (int64_t a = 0; a < n_coarse; ++a) {
      make_row(a, row);
      int64_t pos = out.xadj[static_cast<size_t>(a)];
      for (const Entry &en : row) {
        out.adj[static_cast<size_t>(pos)] = en.to;
        out.mult[static_cast<size_t>(pos)] = en.mult;
        ++pos;
      }
    }
  }
  out.view.n = n_coarse;
  out.view.nnz = nnz_coarse;
  out.view.xadj = out.xadj.data();
  out.view.adj = out.adj.data();
  out.view.xadj_is64 = 1;
}

// One level: map of `fine` and the next level appended to h.  Returns |V_{i+1}|.
template <typename OffT>
int64_t coarsen_level(gosh_hierarchy &h, int threads) {
  gosh_hierarchy::Level &fine = h.levels.back();
  const Csr<OffT> g{fine.view.n, static_cast<const OffT *>(fine.view.xadj), fine.view.adj};
  std::vector<int32_t> order;
  degree_order(g, threads, order);
  const int64_t n_coarse = mark_clusters(g, fine.view.nnz, order, fine.map);
  gosh_hierarchy::Level next;
  const int64_t *mult_in = fine.mult.empty() ? nullptr : fine.mult.data();
  build_coarse(g, mult_in, fine.map, n_coarse, threads, next);
  h.levels.push_back(std::move(next));
  // the move kept the vectors' heap blocks, but re-point the view to be explicit
  gosh_hierarchy::Level &stored = h.levels.back();
  stored.view.xadj = stored.xadj.data();
  stored.view.adj = stored.adj.data();
  return n_coarse;
}

template <typename OffT>
int validate(const gosh_csr *g) {
  const OffT *xadj = static_cast<const OffT *>(g->xadj);
  if (xadj[0] != 0) return gosh::fail(GOSH_EINVAL, "xadj[0] = %lld, expected 0", (long long)xadj[0]);
  if (static_cast<int64_t>(xadj[g->n]) != g->nnz)
    return gosh::fail(GOSH_EINVAL, "xadj[n] = %lld but nnz = %lld", (long long)xadj[g->n], (long long)g->nnz);
  for (int64_t v = 0; v < g->n; ++v) {
    if (xadj[v + 1] < xadj[v]) return gosh::fail(GOSH_EINVAL, "xadj decreases at vertex %lld", (long long)v);
    for (OffT e = xadj[v]; e < xadj[v + 1]; ++e) {
      const int32_t u = g->adj[e];
      if (u < 0 || u >= g->n) return gosh::fail(GOSH_EINVAL, "neighbour %d of vertex %lld out of range", u, (long long)v);
      if (u == v) return gosh::fail(GOSH_EINVAL, "self loop at vertex %lld", (long long)v);
      if (e > xadj[v] && g->adj[e - 1] >= u)
        return gosh::fail(GOSH_EINVAL, "row of vertex %lld is not strictly ascending", (long long)v);
    }
  }
  return GOSH_OK;
}

}  // namespace

extern "C" {

int gosh_csr_validate(const gosh_csr *g_host) {
  if (int rc = gosh::check_csr(g_host)) return rc;
  return g_host->xadj_is64 ? validate<int64_t>(g_host) : validate<int32_t>(g_host);
}

int gosh_coarsen(const gosh_csr *g0_host, int64_t threshold, double min_shrink, int32_t max_levels,
                 int32_t n_threads, gosh_hierarchy **out) {
  if (out == nullptr) return gosh::fail(GOSH_EINVAL, "out is null");
  *out = nullptr;
  if (int rc = gosh::check_csr(g0_host)) return rc;
  if (threshold < 1) return gosh::fail(GOSH_EINVAL, "threshold = %lld: must be >= 1", (long long)threshold);
  if (!(min_shrink > 0.0 && min_shrink <= 1.0))
    return gosh::fail(GOSH_EINVAL, "min_shrink = %g: must be in (0, 1]", min_shrink);
  if (max_levels < 1) return gosh::fail(GOSH_EINVAL, "max_levels = %d: must be >= 1", max_levels);
  int threads = n_threads > 0 ? n_threads : omp_get_max_threads();
  if (threads < 1) threads = 1;
  try {
    gosh_hierarchy *h = new gosh_hierarchy();
    h->levels.reserve(static_cast<size_t>(std::min<int32_t>(max_levels, 64)));
    h->levels.emplace_back();
    h->levels[0].view = *g0_host;
    while (h->levels.back().view.n > threshold && static_cast<int32_t>(h->levels.size()) < max_levels) {
      const int64_t n_fine = h->levels.back().view.n;
      const int64_t n_coarse = h->levels.back().view.xadj_is64 ? coarsen_level<int64_t>(*h, threads)
                                                               : coarsen_level<int32_t>(*h, threads);
      if (static_cast<double>(n_coarse) > min_shrink * static_cast<double>(n_fine) || n_coarse == n_fine) break;
    }
    *out = h;
    return GOSH_OK;
  } catch (const std::bad_alloc &) {
    return gosh::fail(GOSH_ENOMEM, "out of host memory while coarsening");
  }
}

int gosh_hierarchy_levels(const gosh_hierarchy *h) { return h ? static_cast<int>(h->levels.size()) : 0; }

int gosh_hierarchy_graph(const gosh_hierarchy *h, int32_t i, gosh_csr *view) {
  if (h == nullptr || view == nullptr) return gosh::fail(GOSH_EINVAL, "null argument");
  if (i < 0 || i >= static_cast<int32_t>(h->levels.size()))
    return gosh::fail(GOSH_EINVAL, "level %d out of range [0, %zu)", i, h->levels.size());
  *view = h->levels[static_cast<size_t>(i)].view;
  return GOSH_OK;
}

int gosh_hierarchy_map(const gosh_hierarchy *h, int32_t i, const int32_t **map, int64_t *len) {
  if (h == nullptr || map == nullptr || len == nullptr) return gosh::fail(GOSH_EINVAL, "null argument");
  if (i < 0 || i + 1 >= static_cast<int32_t>(h->levels.size()))
    return gosh::fail(GOSH_EINVAL, "map %d out of range [0, %zu)", i, h->levels.size() - 1);
  *map = h->levels[static_cast<size_t>(i)].map.data();
  *len = static_cast<int64_t>(h->levels[static_cast<size_t>(i)].map.size());
  return GOSH_OK;
}

int gosh_hierarchy_mult(const gosh_hierarchy *h, int32_t i, const int64_t **mult, int64_t *len) {
  if (h == nullptr || mult == nullptr || len == nullptr) return gosh::fail(GOSH_EINVAL, "null argument");
  if (i < 0 || i >= static_cast<int32_t>(h->levels.size()))
    return gosh::fail(GOSH_EINVAL, "level %d out of range [0, %zu)", i, h->levels.size());
  const auto &m = h->levels[static_cast<size_t>(i)].mult;
  *mult = m.empty() ? nullptr : m.data();
  *len = static_cast<int64_t>(m.size());
  return GOSH_OK;
}

void gosh_hierarchy_free(gosh_hierarchy *h) { delete h; }

}  // extern "C"
