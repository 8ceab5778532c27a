// MultiEdgeCollapse coarsening hierarchy (Alg. 4 of the paper) on the host.
//
// The result is that of the sequential Alg. 4 (its maps depend on the visiting order and
// have to be reproducible bit for bit), but every stage -- degree counting sort, marking,
// grouping by cluster, rebuilding the CSR of the coarse graph -- runs in parallel with
// OpenMP in a way that cannot change the output.
#include <omp.h>

#include <algorithm>
#include <atomic>
#include <climits>
#include <cstring>
#include <new>
#include <numeric>
#include <vector>

#include "gosh_coarsen_internal.h"
#include "gosh_common.h"

struct gosh_hierarchy {
  struct Level {
    // Level 0 borrows the caller's arrays; coarser levels own theirs (64-bit offsets).
    // A hierarchy built on the device keeps every level there (dev) and fills the host
    // arrays only when an accessor asks for them (host_* say which are filled).
    int64_t n = 0, nnz = 0;
    gosh_csr view{};  // host view, valid once host_graph is set
    gosh::RawVector<int64_t> xadj;
    gosh::RawVector<int32_t> xadj32;  // host copy of a device-resident G_0 with 32-bit offsets
    gosh::RawVector<int32_t> adj;
    gosh::RawVector<int64_t> mult;  // fine entries merged into each entry (none at level 0)
    std::vector<int32_t> map;       // this level -> next coarser level (none on the last)
    bool has_mult = false, has_map = false;
    bool host_graph = false, host_mult = false, host_map = false;
    gosh::DeviceLevel dev;
    double sort_ms = 0, mark_ms = 0, build_ms = 0;  // stages of coarsening THIS level
  };
  std::vector<Level> levels;
  gosh::DeviceCoarsener *dc = nullptr;  // device-built hierarchies: staging for downloads
  ~gosh_hierarchy() {
    for (Level &l : levels) gosh::device_level_free(l.dev);
    gosh::device_coarsener_free(dc);
  }
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

// The marking sweep of Alg. 4, with the result of the sequential sweep but computed in
// parallel.  Returns the number of clusters.
//
// In the sequential sweep a vertex becomes a hub iff it is still unmarked when its turn
// comes, i.e. iff none of the neighbours that precede it in the order and may take it
// (deg(u) <= delta or deg(v) <= delta) is itself a hub; a non-hub belongs to the first
// such hub in the order.  That is a greedy independent-set recurrence over the order, and
// it can be resolved out of order:
//   * a vertex with deg > delta is always a hub (whoever precedes it has a degree at least
//     as large, so the merge condition fails);
//   * a low-degree vertex with a high-degree neighbour is never a hub;
//   * the remaining low-degree vertices are decided in rounds: hub once every preceding
//     neighbour is decided and none is a hub, non-hub as soon as one is.  Rounds stop when
//     they no longer pay (long chains of equal degrees), and what is left is swept
//     sequentially in order.
// Cluster ids are the hubs' positions among the hubs in the order, as in Alg. 4.
template <typename OffT>
int64_t mark_clusters(const Csr<OffT> &g, int64_t nnz, const std::vector<int32_t> &order,
                      int threads, std::vector<int32_t> &map) {
  const int64_t n = g.n;
  enum : uint8_t { kUndecided = 0, kHub = 1, kTaken = 2 };
  std::vector<int32_t> rank(static_cast<size_t>(n));
  std::vector<uint8_t> low(static_cast<size_t>(n));
  std::vector<std::atomic<uint8_t>> status(static_cast<size_t>(n));
#pragma omp parallel for num_threads(threads) schedule(static)
  for (int64_t t = 0; t < n; ++t) rank[static_cast<size_t>(order[static_cast<size_t>(t)])] = static_cast<int32_t>(t);
  // deg <= |E|/|V|  <=>  deg * n <= nnz (exact, no rounding)
#pragma omp parallel for num_threads(threads) schedule(static)
  for (int64_t v = 0; v < n; ++v) low[static_cast<size_t>(v)] = g.degree(v) * n <= nnz;

  // first classification: needs no knowledge of other decisions
#pragma omp parallel for num_threads(threads) schedule(dynamic, 4096)
  for (int64_t v = 0; v < n; ++v) {
    uint8_t st = kUndecided;
    if (!low[static_cast<size_t>(v)]) {
      st = kHub;
    } else {
      bool has_predecessor = false;
      for (OffT e = g.xadj[v]; e < g.xadj[v + 1]; ++e) {
        const int32_t u = g.adj[e];
        if (!low[static_cast<size_t>(u)]) { st = kTaken; break; }
        if (rank[static_cast<size_t>(u)] < rank[static_cast<size_t>(v)]) has_predecessor = true;
      }
      if (st == kUndecided && !has_predecessor) st = kHub;
    }
    status[static_cast<size_t>(v)].store(st, std::memory_order_relaxed);
  }

  // rounds over the undecided low-degree vertices
  std::vector<int32_t> pending;
  for (int64_t v = 0; v < n; ++v)
    if (status[static_cast<size_t>(v)].load(std::memory_order_relaxed) == kUndecided) pending.push_back(static_cast<int32_t>(v));
  for (int round = 0; round < 64 && pending.size() > 4096; ++round) {
    const int64_t before = static_cast<int64_t>(pending.size());
#pragma omp parallel for num_threads(threads) schedule(dynamic, 1024)
    for (int64_t i = 0; i < before; ++i) {
      const int32_t v = pending[static_cast<size_t>(i)];
      bool blocked = false, taken = false;
      for (OffT e = g.xadj[v]; e < g.xadj[v + 1]; ++e) {
        const int32_t u = g.adj[e];
        if (rank[static_cast<size_t>(u)] >= rank[static_cast<size_t>(v)]) continue;
        const uint8_t su = status[static_cast<size_t>(u)].load(std::memory_order_relaxed);
        if (su == kHub) { taken = true; break; }
        if (su == kUndecided) blocked = true;
      }
      // A decision, once made, is final and equals the sequential one, so reading a
      // neighbour decided in this same round can only save a round.
      if (taken) status[static_cast<size_t>(v)].store(kTaken, std::memory_order_relaxed);
      else if (!blocked) status[static_cast<size_t>(v)].store(kHub, std::memory_order_relaxed);
    }
    std::vector<int32_t> still;
    for (int32_t v : pending)
      if (status[static_cast<size_t>(v)].load(std::memory_order_relaxed) == kUndecided) still.push_back(v);
    pending.swap(still);
    if (static_cast<int64_t>(pending.size()) * 10 > before * 9) break;  // rounds stopped paying
  }
  // whatever is left: the sequential sweep, in order
  std::sort(pending.begin(), pending.end(), [&](int32_t p, int32_t q) {
    return rank[static_cast<size_t>(p)] < rank[static_cast<size_t>(q)];
  });
  for (int32_t v : pending) {
    bool taken = false;
    for (OffT e = g.xadj[v]; e < g.xadj[v + 1] && !taken; ++e) {
      const int32_t u = g.adj[e];
      taken = rank[static_cast<size_t>(u)] < rank[static_cast<size_t>(v)] &&
              status[static_cast<size_t>(u)].load(std::memory_order_relaxed) == kHub;
    }
    status[static_cast<size_t>(v)].store(taken ? kTaken : kHub, std::memory_order_relaxed);
  }

  // hubs are numbered in the order; every other vertex joins its first hub in the order
  map.assign(static_cast<size_t>(n), -1);
  int32_t next_cluster = 0;
  for (int64_t t = 0; t < n; ++t) {
    const int32_t v = order[static_cast<size_t>(t)];
    if (status[static_cast<size_t>(v)].load(std::memory_order_relaxed) == kHub) map[static_cast<size_t>(v)] = next_cluster++;
  }
#pragma omp parallel for num_threads(threads) schedule(dynamic, 4096)
  for (int64_t v = 0; v < n; ++v) {
    if (status[static_cast<size_t>(v)].load(std::memory_order_relaxed) != kTaken) continue;
    int32_t best_rank = INT32_MAX, best = -1;
    for (OffT e = g.xadj[v]; e < g.xadj[v + 1]; ++e) {
      const int32_t u = g.adj[e];
      const int32_t ru = rank[static_cast<size_t>(u)];
      if (ru < best_rank && ru < rank[static_cast<size_t>(v)] &&
          status[static_cast<size_t>(u)].load(std::memory_order_relaxed) == kHub) {
        best_rank = ru;
        best = u;
      }
    }
    map[static_cast<size_t>(v)] = map[static_cast<size_t>(best)];
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

  // Every thread builds whole coarse rows into a private buffer (the paper's thread-private
  // edge regions, Sec. 3.2.2) and records where each row went; a scan of the row lengths
  // then fixes the final offsets and the rows are copied to their place.  A row's content
  // does not depend on which thread built it, so the output is schedule-independent.
  //
  // Inside a row, parallel entries are merged with a per-thread stamp array over the
  // coarse ids (stamp[b] == a  <=>  b already seen in row a), so only distinct neighbours
  // are sorted; a row that reaches a large share of all coarse vertices is emitted by
  // scanning the stamp array in id order instead of sorting.
  out.xadj.assign(static_cast<size_t>(n_coarse) + 1, 0);
  struct Entry {
    int32_t to;
    int64_t mult;
  };
  struct Placed {
    int32_t thread;
    int64_t offset;
  };
  std::vector<Placed> placed(static_cast<size_t>(n_coarse));
  std::vector<std::vector<Entry>> built(static_cast<size_t>(threads));
#pragma omp parallel num_threads(threads)
  {
    const int tid = omp_get_thread_num();
    std::vector<Entry> &mine = built[static_cast<size_t>(tid)];
    std::vector<int32_t> stamp(static_cast<size_t>(n_coarse), -1);
    std::vector<int64_t> where(static_cast<size_t>(n_coarse));
    std::vector<Entry> row;
    // cluster ids follow the degree order of their hubs, so the largest rows come first;
    // small dynamic chunks keep them on different threads
#pragma omp for schedule(dynamic, 4)
    for (int64_t a = 0; a < n_coarse; ++a) {
      row.clear();
      for (int64_t m = first[static_cast<size_t>(a)]; m < first[static_cast<size_t>(a) + 1]; ++m) {
        const int32_t x = members[static_cast<size_t>(m)];
        for (OffT e = g.xadj[x]; e < g.xadj[x + 1]; ++e) {
          const int32_t b = map[static_cast<size_t>(g.adj[e])];
          if (b == a) continue;
          const int64_t w = mult_in ? mult_in[e] : 1;
          if (stamp[static_cast<size_t>(b)] != a) {
            stamp[static_cast<size_t>(b)] = static_cast<int32_t>(a);
            where[static_cast<size_t>(b)] = static_cast<int64_t>(row.size());
            row.push_back(Entry{b, w});
          } else {
            row[static_cast<size_t>(where[static_cast<size_t>(b)])].mult += w;
          }
        }
      }
      placed[static_cast<size_t>(a)] = Placed{tid, static_cast<int64_t>(mine.size())};
      out.xadj[static_cast<size_t>(a) + 1] = static_cast<int64_t>(row.size());
      if (static_cast<int64_t>(row.size()) * 16 > n_coarse) {
        for (int64_t b = 0; b < n_coarse; ++b)
          if (stamp[static_cast<size_t>(b)] == a) mine.push_back(row[static_cast<size_t>(where[static_cast<size_t>(b)])]);
      } else {
        std::sort(row.begin(), row.end(), [](const Entry &p, const Entry &q) { return p.to < q.to; });
        mine.insert(mine.end(), row.begin(), row.end());
      }
    }
  }
  for (int64_t a = 0; a < n_coarse; ++a) out.xadj[static_cast<size_t>(a) + 1] += out.xadj[static_cast<size_t>(a)];
  const int64_t nnz_coarse = out.xadj[static_cast<size_t>(n_coarse)];
  // left uninitialised: the loop below writes every element, faulting the pages in from
  // all threads
  out.adj.resize(static_cast<size_t>(nnz_coarse));
  out.mult.resize(static_cast<size_t>(nnz_coarse));
#pragma omp parallel for num_threads(threads) schedule(dynamic, 64)
  for (int64_t a = 0; a < n_coarse; ++a) {
    const Placed &pl = placed[static_cast<size_t>(a)];
    const Entry *src = built[static_cast<size_t>(pl.thread)].data() + pl.offset;
    const int64_t begin = out.xadj[static_cast<size_t>(a)], len = out.xadj[static_cast<size_t>(a) + 1] - begin;
    for (int64_t r = 0; r < len; ++r) {
      out.adj[static_cast<size_t>(begin + r)] = src[r].to;
      out.mult[static_cast<size_t>(begin + r)] = src[r].mult;
    }
  }
  out.n = n_coarse;
  out.nnz = nnz_coarse;
  out.view.n = n_coarse;
  out.view.nnz = nnz_coarse;
  out.view.xadj = out.xadj.data();
  out.view.adj = out.adj.data();
  out.view.xadj_is64 = 1;
  out.has_mult = out.host_mult = true;
  out.host_graph = true;
}

// The marking of one host graph: fills level.map, returns |V_{i+1}|.
template <typename OffT>
int64_t mark_on_host(gosh_hierarchy::Level &level, int threads) {
  const Csr<OffT> g{level.view.n, static_cast<const OffT *>(level.view.xadj), level.view.adj};
  std::vector<int32_t> order;
  const double t0 = omp_get_wtime();
  degree_order(g, threads, order);
  const double t1 = omp_get_wtime();
  const int64_t n_coarse = mark_clusters(g, level.view.nnz, order, threads, level.map);
  level.sort_ms = (t1 - t0) * 1e3;
  level.mark_ms = (omp_get_wtime() - t1) * 1e3;
  level.has_map = level.host_map = true;
  return n_coarse;
}

// One level on the host: map of the last level and the next level appended to h.
// Returns |V_{i+1}|.
template <typename OffT>
int64_t coarsen_level(gosh_hierarchy &h, int threads) {
  gosh_hierarchy::Level &fine = h.levels.back();
  const int64_t n_coarse = mark_on_host<OffT>(fine, threads);
  const double t2 = omp_get_wtime();
  const Csr<OffT> g{fine.view.n, static_cast<const OffT *>(fine.view.xadj), fine.view.adj};
  gosh_hierarchy::Level next;
  build_coarse(g, fine.mult.empty() ? nullptr : fine.mult.data(), fine.map, n_coarse, threads, next);
  fine.build_ms = (omp_get_wtime() - t2) * 1e3;
  h.levels.push_back(std::move(next));
  // the move kept the vectors' heap blocks; point the view at them
  gosh_hierarchy::Level &stored = h.levels.back();
  stored.view.xadj = stored.xadj.data();
  stored.view.adj = stored.adj.data();
  return n_coarse;
}

// Host copies of a device-built level, made on first request.
int ensure_host_graph_impl(gosh_hierarchy &h, gosh_hierarchy::Level &l);
int ensure_host_map_impl(gosh_hierarchy &h, gosh_hierarchy::Level &l);
int ensure_host_mult_impl(gosh_hierarchy &h, gosh_hierarchy::Level &l);

// The accessors that call these are C entry points: an allocation failure becomes a status.
template <typename F>
int no_throw(F &&f) {
  try {
    return f();
  } catch (const std::bad_alloc &) {
    return gosh::fail(GOSH_ENOMEM, "out of host memory while copying a level to the host");
  }
}
int ensure_host_graph(gosh_hierarchy &h, gosh_hierarchy::Level &l) {
  return no_throw([&] { return ensure_host_graph_impl(h, l); });
}
int ensure_host_map(gosh_hierarchy &h, gosh_hierarchy::Level &l) {
  return no_throw([&] { return ensure_host_map_impl(h, l); });
}
int ensure_host_mult(gosh_hierarchy &h, gosh_hierarchy::Level &l) {
  return no_throw([&] { return ensure_host_mult_impl(h, l); });
}

int ensure_host_graph_impl(gosh_hierarchy &h, gosh_hierarchy::Level &l) {
  if (l.host_graph) return GOSH_OK;
  if (!l.dev.present()) return gosh::fail(GOSH_EINVAL, "level has neither a host nor a device copy");
  void *offsets = nullptr;
  if (l.dev.xadj_is64) {
    l.xadj.resize(static_cast<size_t>(l.n) + 1);
    offsets = l.xadj.data();
  } else {
    l.xadj32.resize(static_cast<size_t>(l.n) + 1);
    offsets = l.xadj32.data();
  }
  l.adj.resize(static_cast<size_t>(l.nnz));
  if (int rc = gosh::device_download(h.dc, offsets, l.dev.xadj,
                                     (static_cast<size_t>(l.n) + 1) * (l.dev.xadj_is64 ? 8 : 4)))
    return rc;
  if (int rc = gosh::device_download(h.dc, l.adj.data(), l.dev.adj, static_cast<size_t>(l.nnz) * 4)) return rc;
  l.view.n = l.n;
  l.view.nnz = l.nnz;
  l.view.xadj = offsets;
  l.view.adj = l.adj.data();
  l.view.xadj_is64 = l.dev.xadj_is64;
  l.host_graph = true;
  return GOSH_OK;
}

int ensure_host_map_impl(gosh_hierarchy &h, gosh_hierarchy::Level &l) {
  if (l.host_map || !l.has_map) return GOSH_OK;
  if (l.dev.map == nullptr) return gosh::fail(GOSH_EINVAL, "map has neither a host nor a device copy");
  l.map.resize(static_cast<size_t>(l.n));
  if (int rc = gosh::device_download(h.dc, l.map.data(), l.dev.map, static_cast<size_t>(l.n) * 4)) return rc;
  l.host_map = true;
  return GOSH_OK;
}

int ensure_host_mult_impl(gosh_hierarchy &h, gosh_hierarchy::Level &l) {
  if (l.host_mult || !l.has_mult) return GOSH_OK;
  if (l.dev.mult == nullptr) return gosh::fail(GOSH_EINVAL, "multiplicities have neither a host nor a device copy");
  l.mult.resize(static_cast<size_t>(l.nnz));
  if (int rc = gosh::device_download(h.dc, l.mult.data(), l.dev.mult, static_cast<size_t>(l.nnz) * 8)) return rc;
  l.host_mult = true;
  return GOSH_OK;
}

// One level on the device.  *n_coarse = |V_{i+1}|; the next level is appended unless
// nothing merged.
int coarsen_level_on_device(gosh_hierarchy &h, int threads, int64_t *n_coarse) {
  gosh_hierarchy::Level &fine = h.levels.back();
  bool done = false;
  const double t0 = omp_get_wtime();
  if (int rc = gosh::device_mark(h.dc, fine.dev, n_coarse, &done, &fine.sort_ms)) return rc;
  if (done) {
    fine.mark_ms = (omp_get_wtime() - t0) * 1e3 - fine.sort_ms;
    fine.has_map = true;
  } else {
    // a chain of equal degrees: the in-order sweep of the host finishes it
    if (int rc = ensure_host_graph(h, fine)) return rc;
    *n_coarse = fine.view.xadj_is64 ? mark_on_host<int64_t>(fine, threads) : mark_on_host<int32_t>(fine, threads);
    if (int rc = gosh::device_level_set_map(fine.dev, fine.map.data())) return rc;
  }
  if (*n_coarse == fine.n) return GOSH_OK;
  const double t2 = omp_get_wtime();
  gosh_hierarchy::Level next;
  if (int rc = gosh::device_rebuild(h.dc, fine.dev, *n_coarse, next.dev)) {
    gosh::device_level_free(next.dev);
    return rc;
  }
  fine.build_ms = (omp_get_wtime() - t2) * 1e3;
  next.n = next.dev.n;
  next.nnz = next.dev.nnz;
  next.has_mult = true;
  h.levels.push_back(std::move(next));
  return GOSH_OK;
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
  if (gosh::is_device_pointer(g_host->xadj) || gosh::is_device_pointer(g_host->adj))
    return gosh::fail(GOSH_EINVAL, "gosh_csr_validate takes a host graph");
  return g_host->xadj_is64 ? validate<int64_t>(g_host) : validate<int32_t>(g_host);
}

static int coarsen_impl(const gosh_csr *g0_host, int64_t threshold, double min_shrink,
                        int32_t max_levels, int32_t n_threads, bool on_device, gosh_hierarchy **out) {
  if (out == nullptr) return gosh::fail(GOSH_EINVAL, "out is null");
  *out = nullptr;
  if (int rc = gosh::check_csr(g0_host)) return rc;
  if (threshold < 1) return gosh::fail(GOSH_EINVAL, "threshold = %lld: must be >= 1", (long long)threshold);
  if (!(min_shrink > 0.0 && min_shrink <= 1.0))
    return gosh::fail(GOSH_EINVAL, "min_shrink = %g: must be in (0, 1]", min_shrink);
  if (max_levels < 1) return gosh::fail(GOSH_EINVAL, "max_levels = %d: must be >= 1", max_levels);
  int threads = n_threads > 0 ? n_threads : omp_get_max_threads();
  if (threads < 1) threads = 1;
  gosh_hierarchy *h = nullptr;
  try {
    h = new gosh_hierarchy();
    h->levels.reserve(static_cast<size_t>(std::min<int32_t>(max_levels, 64)));
    h->levels.emplace_back();
    h->levels[0].n = g0_host->n;
    h->levels[0].nnz = g0_host->nnz;
    const bool g0_on_device = gosh::is_device_pointer(g0_host->xadj);
    if (g0_on_device && !on_device) {
      delete h;
      return gosh::fail(GOSH_EINVAL, "gosh_coarsen takes a host graph (gosh_coarsen_device takes either)");
    }
    const bool wants_levels = g0_host->n > threshold && max_levels > 1;
    if (g0_on_device) {
      // a device-resident G_0 is adopted as it is; its host copy is made if someone asks
      if (g0_host->nnz > 0 && !gosh::is_device_pointer(g0_host->adj)) {
        delete h;
        return gosh::fail(GOSH_EINVAL, "xadj is device memory but adj is not");
      }
      h->dc = gosh::device_coarsener_new(threads);
      if (int rc = gosh::device_level_borrow(*g0_host, h->levels[0].dev)) {
        delete h;
        return rc;
      }
    } else {
      h->levels[0].view = *g0_host;
      h->levels[0].host_graph = true;
      if (on_device && wants_levels) {
        h->dc = gosh::device_coarsener_new(threads);
        if (int rc = gosh::device_level_upload(h->dc, *g0_host, h->levels[0].dev)) {
          delete h;
          return rc;
        }
      }
    }
    while (h->levels.back().n > threshold && static_cast<int32_t>(h->levels.size()) < max_levels) {
      const int64_t n_fine = h->levels.back().n;
      int64_t n_coarse = 0;
      if (on_device) {
        if (int rc = coarsen_level_on_device(*h, threads, &n_coarse)) {
          delete h;
          return rc;
        }
      } else {
        n_coarse = h->levels.back().view.xadj_is64 ? coarsen_level<int64_t>(*h, threads)
                                                   : coarsen_level<int32_t>(*h, threads);
      }
      if (n_coarse == n_fine) {
        // nothing merged (e.g. only isolated vertices are left): G_{i+1} would repeat G_i
        if (!on_device) h->levels.pop_back();
        gosh_hierarchy::Level &last = h->levels.back();
        last.map.clear();
        last.has_map = last.host_map = false;
        gosh::device_level_drop_map(last.dev);
        break;
      }
      if (static_cast<double>(n_coarse) > min_shrink * static_cast<double>(n_fine)) break;
    }
    // The scratch blocks of the run stay with the hierarchy (gosh_hierarchy_trim_scratch or
    // freeing it returns them): the driver clears freed device memory in the background for
    // seconds, and host<->device copies that run meanwhile -- those of a rotation that
    // follows the coarsening at once -- make half their rate.
    *out = h;
    return GOSH_OK;
  } catch (const std::bad_alloc &) {
    delete h;
    return gosh::fail(GOSH_ENOMEM, "out of host memory while coarsening");
  }
}

int gosh_coarsen(const gosh_csr *g0_host, int64_t threshold, double min_shrink, int32_t max_levels,
                 int32_t n_threads, gosh_hierarchy **out) {
  return coarsen_impl(g0_host, threshold, min_shrink, max_levels, n_threads, false, out);
}

int gosh_coarsen_device(const gosh_csr *g0_host, int64_t threshold, double min_shrink,
                        int32_t max_levels, int32_t n_threads, gosh_hierarchy **out) {
  return coarsen_impl(g0_host, threshold, min_shrink, max_levels, n_threads, true, out);
}

int gosh_hierarchy_levels(const gosh_hierarchy *h) { return h ? static_cast<int>(h->levels.size()) : 0; }

int gosh_hierarchy_shape(const gosh_hierarchy *h, int32_t i, int64_t *n, int64_t *nnz) {
  if (h == nullptr) return gosh::fail(GOSH_EINVAL, "null argument");
  if (i < 0 || i >= static_cast<int32_t>(h->levels.size()))
    return gosh::fail(GOSH_EINVAL, "level %d out of range [0, %zu)", i, h->levels.size());
  if (n) *n = h->levels[static_cast<size_t>(i)].n;
  if (nnz) *nnz = h->levels[static_cast<size_t>(i)].nnz;
  return GOSH_OK;
}

int gosh_hierarchy_graph(const gosh_hierarchy *h, int32_t i, gosh_csr *view) {
  if (h == nullptr || view == nullptr) return gosh::fail(GOSH_EINVAL, "null argument");
  if (i < 0 || i >= static_cast<int32_t>(h->levels.size()))
    return gosh::fail(GOSH_EINVAL, "level %d out of range [0, %zu)", i, h->levels.size());
  gosh_hierarchy &hm = *const_cast<gosh_hierarchy *>(h);  // filling a host copy is not a visible change
  if (int rc = ensure_host_graph(hm, hm.levels[static_cast<size_t>(i)])) return rc;
  *view = h->levels[static_cast<size_t>(i)].view;
  return GOSH_OK;
}

int gosh_hierarchy_map(const gosh_hierarchy *h, int32_t i, const int32_t **map, int64_t *len) {
  if (h == nullptr || map == nullptr || len == nullptr) return gosh::fail(GOSH_EINVAL, "null argument");
  if (i < 0 || i + 1 >= static_cast<int32_t>(h->levels.size()))
    return gosh::fail(GOSH_EINVAL, "map %d out of range [0, %zu)", i, h->levels.size() - 1);
  gosh_hierarchy &hm = *const_cast<gosh_hierarchy *>(h);
  if (int rc = ensure_host_map(hm, hm.levels[static_cast<size_t>(i)])) return rc;
  *map = h->levels[static_cast<size_t>(i)].map.data();
  *len = static_cast<int64_t>(h->levels[static_cast<size_t>(i)].map.size());
  return GOSH_OK;
}

int gosh_hierarchy_mult(const gosh_hierarchy *h, int32_t i, const int64_t **mult, int64_t *len) {
  if (h == nullptr || mult == nullptr || len == nullptr) return gosh::fail(GOSH_EINVAL, "null argument");
  if (i < 0 || i >= static_cast<int32_t>(h->levels.size()))
    return gosh::fail(GOSH_EINVAL, "level %d out of range [0, %zu)", i, h->levels.size());
  gosh_hierarchy &hm = *const_cast<gosh_hierarchy *>(h);
  if (int rc = ensure_host_mult(hm, hm.levels[static_cast<size_t>(i)])) return rc;
  const auto &m = h->levels[static_cast<size_t>(i)].mult;
  *mult = m.empty() ? nullptr : m.data();
  *len = static_cast<int64_t>(m.size());
  return GOSH_OK;
}

int gosh_hierarchy_trim_scratch(gosh_hierarchy *h) {
  if (h != nullptr) gosh::device_coarsener_trim(h->dc);
  return GOSH_OK;
}

int gosh_hierarchy_release_device(gosh_hierarchy *h) {
  if (h == nullptr) return GOSH_OK;
  gosh::device_coarsener_trim(h->dc);
  for (gosh_hierarchy::Level &l : h->levels) {
    if (int rc = ensure_host_graph(*h, l)) return rc;
    if (int rc = ensure_host_map(*h, l)) return rc;
    if (int rc = ensure_host_mult(*h, l)) return rc;
    gosh::device_level_free(l.dev);
  }
  return GOSH_OK;
}

int gosh_hierarchy_times(const gosh_hierarchy *h, int32_t i, double *ms3) {
  if (h == nullptr || ms3 == nullptr) return gosh::fail(GOSH_EINVAL, "null argument");
  if (i < 0 || i + 1 >= static_cast<int32_t>(h->levels.size()))
    return gosh::fail(GOSH_EINVAL, "level %d out of range [0, %zu)", i, h->levels.size() - 1);
  const auto &l = h->levels[static_cast<size_t>(i)];
  ms3[0] = l.sort_ms;
  ms3[1] = l.mark_ms;
  ms3[2] = l.build_ms;
  return GOSH_OK;
}

void gosh_hierarchy_free(gosh_hierarchy *h) { delete h; }

}  // extern "C"

namespace gosh {

int hierarchy_shape(const gosh_hierarchy *h, int32_t i, gosh_csr *shape) {
  if (h == nullptr || shape == nullptr) return fail(GOSH_EINVAL, "null argument");
  if (i < 0 || i >= static_cast<int32_t>(h->levels.size()))
    return fail(GOSH_EINVAL, "level %d out of range [0, %zu)", i, h->levels.size());
  const gosh_hierarchy::Level &l = h->levels[static_cast<size_t>(i)];
  *shape = gosh_csr{};
  shape->n = l.n;
  shape->nnz = l.nnz;
  shape->xadj_is64 = l.host_graph ? l.view.xadj_is64 : l.dev.xadj_is64;
  return GOSH_OK;
}

const DeviceLevel *hierarchy_device_level(const gosh_hierarchy *h, int32_t i) {
  if (h == nullptr || i < 0 || i >= static_cast<int32_t>(h->levels.size())) return nullptr;
  const DeviceLevel &dev = h->levels[static_cast<size_t>(i)].dev;
  return dev.present() ? &dev : nullptr;
}

}  // namespace gosh
