// Multilevel driver (Alg. 2 of the paper): train the coarsest graph, project the
// embedding to the next finer graph, train that, ... until the embedding of G_0 exists.
// A level whose graph and matrix fit the device budget is trained with the epoch kernel
// (CopyToDevice + TrainInGPU); a level that does not is trained with the part-pair
// rotation on a host-resident matrix (LargeGraphGPU).  Host orchestration only: every
// numerical step is one of the library's kernels, except the row gather between two
// levels that both live on the host.
#include <hip/hip_runtime.h>
#include <omp.h>

#include <algorithm>
#include <chrono>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "gosh_coarsen_internal.h"
#include "gosh_common.h"

namespace {

struct DeviceBuffer {
  void *ptr = nullptr;
  DeviceBuffer() = default;
  DeviceBuffer(const DeviceBuffer &) = delete;
  DeviceBuffer &operator=(const DeviceBuffer &) = delete;
  ~DeviceBuffer() { reset(); }
  int alloc(size_t bytes, const char *what) {
    reset();
    if (bytes == 0) bytes = 16;
    if (hipMalloc(&ptr, bytes) != hipSuccess) {
      (void)hipGetLastError();
      ptr = nullptr;
      return gosh::fail(GOSH_ENOMEM, "cannot allocate %zu device bytes for %s", bytes, what);
    }
    return GOSH_OK;
  }
  void reset() {
    if (ptr) (void)hipFree(ptr);
    ptr = nullptr;
  }
  void swap(DeviceBuffer &o) { std::swap(ptr, o.ptr); }
};

struct PinnedBuffer {
  void *ptr = nullptr;
  PinnedBuffer() = default;
  PinnedBuffer(const PinnedBuffer &) = delete;
  PinnedBuffer &operator=(const PinnedBuffer &) = delete;
  ~PinnedBuffer() { reset(); }
  int alloc(size_t bytes, const char *what) {
    reset();
    if (bytes == 0) bytes = 16;
    if (hipHostMalloc(&ptr, bytes, hipHostMallocDefault) != hipSuccess) {
      (void)hipGetLastError();
      ptr = nullptr;
      return gosh::fail(GOSH_ENOMEM, "cannot allocate %zu pinned host bytes for %s", bytes, what);
    }
    return GOSH_OK;
  }
  void reset() {
    if (ptr) (void)hipHostFree(ptr);
    ptr = nullptr;
  }
  void swap(PinnedBuffer &o) { std::swap(ptr, o.ptr); }
};

double ms_since(std::chrono::steady_clock::time_point t0) {
  return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
}

size_t level_bytes(const gosh_csr &g, int32_t d) {
  return static_cast<size_t>(g.n + 1) * (g.xadj_is64 ? 8 : 4) + static_cast<size_t>(g.nnz) * 4 +
         static_cast<size_t>(g.n) * d * 4;
}

// Rows of a slice that a staging buffer on the device may hold: the budget left beside
// `resident` bytes, at least 64 rows' worth.
int chunk_rows(uint64_t budget, size_t resident, int32_t d, int64_t n, int64_t *rows) {
  const size_t per_row = static_cast<size_t>(d) * 4 + 4;
  size_t room = budget == 0 ? (size_t{1} << 30) : (budget > resident ? budget - resident : 0);
  int64_t r = static_cast<int64_t>(room / per_row);
  if (r < std::min<int64_t>(n, 64))
    return gosh::fail(GOSH_EBUDGET, "device budget leaves no room for a staging slice of 64 rows");
  *rows = std::min<int64_t>(r, n);
  return GOSH_OK;
}

struct Plan {
  int32_t d, k_neg;
  float lr0;
  uint64_t seed;
  uint32_t flags;  // for the epoch kernel calls
  uint32_t parts_flags;  // for the rotation calls: the same plus GOSH_FLAG_BLOCKED_ORDER if asked
  bool edge_epochs;
  bool pair_levels;  // resident levels large enough run Alg. 5 in place
  uint64_t budget;
  bool budget_is_free_memory;  // measured, not given: graphs already on the device are outside it
  int32_t P_gpu, S_gpu, B;
};

// One run of Alg. 2 over a hierarchy.  The matrix of the current level lives either on the
// device (cur_dev) or on the host (cur_host); the buffers own it unless it is the caller's
// output array.
class MultilevelRun {
 public:
  MultilevelRun(const gosh_hierarchy *h, const Plan &pl, float *M0_dev, float *M0_host, hipStream_t st)
      : h(h), pl(pl), d(pl.d), M0_dev(M0_dev), M0_host(M0_host), st(st) {}
  MultilevelRun(const MultilevelRun &) = delete;
  MultilevelRun &operator=(const MultilevelRun &) = delete;
  ~MultilevelRun() {
    if (ev0) (void)hipEventDestroy(ev0);
    if (ev1) (void)hipEventDestroy(ev1);
  }

  int run(int64_t epochs, double p, gosh_level_stats *stats) {
    const int D = gosh_hierarchy_levels(h);
    if (D < 1) return gosh::fail(GOSH_EINVAL, "hierarchy is null or empty");
    std::vector<int64_t> e_i(static_cast<size_t>(D));
    if (int rc = gosh_epoch_split(epochs, p, D, e_i.data())) return rc;
    // shapes only: the arrays of a level are fetched where the level is trained (a hierarchy
    // built on the device has no host copies until someone asks)
    G.resize(static_cast<size_t>(D));
    for (int i = 0; i < D; ++i)
      if (int rc = gosh::hierarchy_shape(h, i, &G[static_cast<size_t>(i)])) return rc;
    GOSH_TRY_HIP(hipGetDevice(&current_device), "hipGetDevice");
    if (M0_dev != nullptr && !fits(0))
      return gosh::fail(GOSH_EBUDGET,
                        "level 0 needs %zu bytes on the device, budget is %llu: use gosh_embed_host",
                        level_bytes(G[0], d), (unsigned long long)pl.budget);
    GOSH_TRY_HIP(hipEventCreate(&ev0), "hipEventCreate");
    GOSH_TRY_HIP(hipEventCreate(&ev1), "hipEventCreate");

    for (int i = D - 1; i >= 0; --i) {
      const gosh_csr &g = G[static_cast<size_t>(i)];
      gosh_level_stats ls{};
      ls.level = i;
      ls.n = g.n;
      ls.nnz = g.nnz;
      ls.epochs = e_i[static_cast<size_t>(i)];
      if (pl.edge_epochs) {
        // an epoch of the experiments samples |E_i| sources; one pass of Alg. 3 samples |V_i|
        const int64_t edges = g.nnz / 2;
        ls.epochs *= std::max<int64_t>(1, (edges + g.n - 1) / g.n);
      }
      if (i == D - 1)
        if (int rc = init_coarsest(i)) return rc;
      const int32_t in_place_parts = (cur_dev && pl.pair_levels)
                                         ? gosh_pair_level_parts(ls.epochs, g.n, gosh::tuning().pair_level_min_n, kPairLevelB)
                                         : 0;
      if (int rc = !cur_dev         ? train_by_rotation(i, ls)
                   : in_place_parts ? train_in_place(i, ls, in_place_parts)
                                    : train_on_device(i, ls))
        return rc;
      if (cur_dev) {
        gosh::CheckResult *result = nullptr;
        if (int rc = gosh::check_scratch(&result)) return rc;
        if (int rc = gosh::matrix_check_clear(result, st)) return rc;
        if (int rc = gosh::matrix_check_add(cur_dev, g.n * d, result, st)) return rc;
        if (int rc = gosh::matrix_check_read(result, &ls.max_abs, &ls.nonfinite, st)) return rc;
      }
      if (ls.nonfinite > 0 && diverged_level < 0) diverged_level = i;
      if (i > 0)
        if (int rc = project(i, ls)) return rc;
      if (stats) stats[i] = ls;
    }
    // Deliver M_0 where the caller wants it.
    if (M0_host && cur_dev) {
      GOSH_TRY_HIP(hipMemcpyAsync(M0_host, cur_dev, static_cast<size_t>(G[0].n) * d * 4, hipMemcpyDeviceToHost, st),
               "download M_0");
      GOSH_TRY_HIP(hipStreamSynchronize(st), "download M_0");
    }
    if (diverged_level >= 0)
      return gosh::fail(GOSH_EDIVERGED, "training diverged: the matrix of level %d holds non-finite values",
                        diverged_level);
    return GOSH_OK;
  }

 private:
  static constexpr int32_t kPairLevelB = 5;
  const gosh_hierarchy *h;
  const Plan &pl;
  const int32_t d;
  float *const M0_dev, *const M0_host;
  const hipStream_t st;
  std::vector<gosh_csr> G;
  int current_device = -1;
  hipEvent_t ev0 = nullptr, ev1 = nullptr;
  DeviceBuffer dev_own, dev_next;
  PinnedBuffer host_own, host_next;
  float *cur_dev = nullptr, *cur_host = nullptr;
  int diverged_level = -1;  // first (coarsest) level whose training left non-finite entries

  // The device-resident arrays of level i, if the hierarchy holds them on this device.
  const gosh::DeviceLevel *resident(int i) const {
    const gosh::DeviceLevel *dl = gosh::hierarchy_device_level(h, i);
    return dl != nullptr && dl->device == current_device ? dl : nullptr;
  }
  bool fits(int i) const {
    if (pl.budget == 0) return true;
    const gosh_csr &g = G[static_cast<size_t>(i)];
    if (pl.budget_is_free_memory && resident(i) != nullptr) return static_cast<size_t>(g.n) * d * 4 <= pl.budget;
    return level_bytes(g, d) <= pl.budget;
  }

  // "Randomly initialize M_{D-1}"
  int init_coarsest(int i) {
    const gosh_csr &g = G[static_cast<size_t>(i)];
    const size_t mat_bytes = static_cast<size_t>(g.n) * d * 4;
    if (fits(i)) {
      if (i == 0 && M0_dev) cur_dev = M0_dev;
      else {
        if (int rc = dev_own.alloc(mat_bytes, "coarsest embedding")) return rc;
        cur_dev = static_cast<float *>(dev_own.ptr);
      }
      return gosh_init_embedding(cur_dev, g.n, d, pl.seed, static_cast<uint32_t>(i), st);
    }
    if (i == 0) cur_host = M0_host;
    else {
      if (int rc = host_own.alloc(mat_bytes, "coarsest embedding")) return rc;
      cur_host = static_cast<float *>(host_own.ptr);
    }
    int64_t rows = 0;
    if (int rc = chunk_rows(pl.budget, 0, d, g.n, &rows)) return rc;
    DeviceBuffer slice;
    if (int rc = slice.alloc(static_cast<size_t>(rows) * d * 4, "initialisation slice")) return rc;
    for (int64_t lo = 0; lo < g.n; lo += rows) {
      const int64_t cnt = std::min(rows, g.n - lo);
      if (int rc = gosh::init_rows(static_cast<float *>(slice.ptr), lo, cnt, d, pl.seed, static_cast<uint32_t>(i), st))
        return rc;
      GOSH_TRY_HIP(hipMemcpyAsync(cur_host + lo * d, slice.ptr, static_cast<size_t>(cnt) * d * 4, hipMemcpyDeviceToHost,
                              st),
               "copy initial rows");
      GOSH_TRY_HIP(hipStreamSynchronize(st), "initialise on host");
    }
    return GOSH_OK;
  }

  // CopyToDevice(G_i): the arrays of level i in device memory -- where the hierarchy keeps
  // them, else uploaded into the two buffers.
  int graph_on_device(int i, DeviceBuffer &xadj_dev, DeviceBuffer &adj_dev, gosh_csr *dev) {
    gosh_csr &g = G[static_cast<size_t>(i)];
    *dev = g;
    if (const gosh::DeviceLevel *dl = resident(i)) {
      dev->xadj = dl->xadj;
      dev->adj = dl->adj;
      dev->xadj_is64 = dl->xadj_is64;
      return GOSH_OK;
    }
    if (int rc = gosh_hierarchy_graph(h, i, &g)) return rc;
    const size_t off_bytes = static_cast<size_t>(g.n + 1) * (g.xadj_is64 ? 8 : 4);
    const size_t adj_bytes = static_cast<size_t>(g.nnz) * 4;
    if (int rc = xadj_dev.alloc(off_bytes, "xadj")) return rc;
    if (int rc = adj_dev.alloc(adj_bytes, "adj")) return rc;
    GOSH_TRY_HIP(hipMemcpyAsync(xadj_dev.ptr, g.xadj, off_bytes, hipMemcpyHostToDevice, st), "copy xadj");
    if (adj_bytes)
      GOSH_TRY_HIP(hipMemcpyAsync(adj_dev.ptr, g.adj, adj_bytes, hipMemcpyHostToDevice, st), "copy adj");
    GOSH_TRY_HIP(hipStreamSynchronize(st), "upload graph");
    *dev = g;
    dev->xadj = xadj_dev.ptr;
    dev->adj = static_cast<const int32_t *>(adj_dev.ptr);
    return GOSH_OK;
  }

  // TrainInGPU
  int train_on_device(int i, gosh_level_stats &ls) {
    auto t0 = std::chrono::steady_clock::now();
    DeviceBuffer xadj_dev, adj_dev;
    gosh_csr dev{};
    if (int rc = graph_on_device(i, xadj_dev, adj_dev, &dev)) return rc;
    ls.upload_ms = ms_since(t0);
    GOSH_TRY_HIP(hipEventRecord(ev0, st), "hipEventRecord");
    for (int64_t j = 0; j < ls.epochs; ++j) {
      const float lr = gosh_lr(pl.lr0, j, ls.epochs);
      if (int rc = gosh_train_epoch(&dev, cur_dev, d, pl.k_neg, lr, pl.seed, static_cast<uint32_t>(j),
                                    static_cast<uint32_t>(i), pl.flags, st))
        return rc;
    }
    GOSH_TRY_HIP(hipEventRecord(ev1, st), "hipEventRecord");
    GOSH_TRY_HIP(hipEventSynchronize(ev1), "train level");
    float ms = 0.f;
    GOSH_TRY_HIP(hipEventElapsedTime(&ms, ev0, ev1), "hipEventElapsedTime");
    ls.train_ms = ms;
    return GOSH_OK;
  }

  // The same level trained in place with the pair order and the sampling rule of Alg. 5
  // (no part moves: the matrix is on the device); the streams are the rotation's own.
  // The part count comes from gosh_pair_level_parts: parts of at least 2^22 vertices by
  // default, because on smaller parts the scheme gains little or loses (2.4 M vertices in 16
  // parts trained at half the rate of Alg. 3, in 2 parts a fifth slower).
  int train_in_place(int i, gosh_level_stats &ls, int32_t K) {
    auto t0 = std::chrono::steady_clock::now();
    DeviceBuffer xadj_dev, adj_dev;
    gosh_csr dev{};
    if (int rc = graph_on_device(i, xadj_dev, adj_dev, &dev)) return rc;
    ls.upload_ms = ms_since(t0);
    GOSH_TRY_HIP(hipStreamSynchronize(st), "before the rotation");
    gosh_parts_stats ps{};
    const int rc = gosh_train_parts(&dev, cur_dev, d, pl.k_neg, ls.epochs, pl.lr0, pl.seed, static_cast<uint32_t>(i),
                                    0, pl.P_gpu, 1, kPairLevelB, K, pl.parts_flags, &ps);
    if (rc != GOSH_OK && rc != GOSH_EDIVERGED) return rc;  // divergence is reported at the end of the run
    ls.parts_K = ps.K;
    ls.train_ms = ps.wall_ms;
    return GOSH_OK;
  }

  // LargeGraphGPU.  A graph that already lives on the device is sampled there; otherwise
  // the host copy is used (and made, if the hierarchy has none yet).
  int train_by_rotation(int i, gosh_level_stats &ls) {
    gosh_csr &g = G[static_cast<size_t>(i)];
    if (const gosh::DeviceLevel *dl = resident(i)) {
      g.xadj = dl->xadj;
      g.adj = dl->adj;
      g.xadj_is64 = dl->xadj_is64;
    } else if (int rc = gosh_hierarchy_graph(h, i, &g)) {
      return rc;
    }
    gosh_parts_stats ps{};
    const int rc = gosh_train_parts(&g, cur_host, d, pl.k_neg, ls.epochs, pl.lr0, pl.seed, static_cast<uint32_t>(i),
                                    pl.budget, pl.P_gpu, pl.S_gpu, pl.B, 0, pl.parts_flags, &ps);
    if (rc != GOSH_OK && rc != GOSH_EDIVERGED) return rc;  // divergence is reported at the end of the run
    ls.parts_K = ps.K;
    ls.train_ms = ps.wall_ms;
    ls.max_abs = ps.max_abs;
    ls.nonfinite = ps.nonfinite;
    return GOSH_OK;
  }

  // ExpandEmbedding(M_i, map_{i-1}): the matrix of level i-1 becomes the current one.
  int project(int i, gosh_level_stats &ls) {
    const gosh_csr &g = G[static_cast<size_t>(i)];
    const size_t mat_bytes = static_cast<size_t>(g.n) * d * 4;
    auto t0 = std::chrono::steady_clock::now();
    const int64_t n_fine = G[static_cast<size_t>(i - 1)].n;
    const gosh::DeviceLevel *fine_dev = resident(i - 1);
    const int32_t *map_dev_resident = fine_dev ? fine_dev->map : nullptr;
    const int32_t *map_host = nullptr;
    if (map_dev_resident == nullptr) {
      int64_t len = 0;
      if (int rc = gosh_hierarchy_map(h, i - 1, &map_host, &len)) return rc;
    }
    const size_t fine_bytes = static_cast<size_t>(n_fine) * d * 4;
    float *next_dev = nullptr, *next_host = nullptr;
    if (fits(i - 1)) {
      if (i - 1 == 0 && M0_dev) next_dev = M0_dev;
      else {
        if (int rc = dev_next.alloc(fine_bytes, "finer embedding")) return rc;
        next_dev = static_cast<float *>(dev_next.ptr);
      }
    } else {
      if (i - 1 == 0) next_host = M0_host;
      else {
        if (int rc = host_next.alloc(fine_bytes, "finer embedding")) return rc;
        next_host = static_cast<float *>(host_next.ptr);
      }
    }
    // A coarse matrix that lives on the host only because its GRAPH did not fit may
    // still visit the device for the projection, which needs no graph.
    const float *src_dev = cur_dev;
    DeviceBuffer src_visit;
    if (src_dev == nullptr && next_host != nullptr) {
      const size_t smallest_slice = 64 * (static_cast<size_t>(d) * 4 + 4);
      if (pl.budget == 0 || mat_bytes + smallest_slice <= pl.budget) {
        if (int rc = src_visit.alloc(mat_bytes, "coarse embedding (projection)")) return rc;
        GOSH_TRY_HIP(hipMemcpyAsync(src_visit.ptr, cur_host, mat_bytes, hipMemcpyHostToDevice, st),
                 "upload coarse embedding");
        src_dev = static_cast<const float *>(src_visit.ptr);
      }
    }
    if (src_dev && next_dev) {
      DeviceBuffer map_dev;
      const int32_t *map_on_device = map_dev_resident;
      if (map_on_device == nullptr) {
        if (int rc = map_dev.alloc(static_cast<size_t>(n_fine) * 4, "map")) return rc;
        GOSH_TRY_HIP(hipMemcpyAsync(map_dev.ptr, map_host, static_cast<size_t>(n_fine) * 4, hipMemcpyHostToDevice, st),
                 "copy map");
        map_on_device = static_cast<const int32_t *>(map_dev.ptr);
      }
      if (int rc = gosh_project(src_dev, g.n, map_on_device, n_fine, d, next_dev, st)) return rc;
      GOSH_TRY_HIP(hipStreamSynchronize(st), "project");
    } else if (src_dev && next_host) {
      // project slice by slice through a device staging buffer
      int64_t rows = 0;
      if (int rc = chunk_rows(pl.budget, mat_bytes, d, n_fine, &rows)) return rc;
      DeviceBuffer slice, map_dev;
      if (int rc = slice.alloc(static_cast<size_t>(rows) * d * 4, "projection slice")) return rc;
      if (map_dev_resident == nullptr)
        if (int rc = map_dev.alloc(static_cast<size_t>(rows) * 4, "map slice")) return rc;
      for (int64_t lo = 0; lo < n_fine; lo += rows) {
        const int64_t cnt = std::min(rows, n_fine - lo);
        const int32_t *map_slice =
            map_dev_resident ? map_dev_resident + lo : static_cast<const int32_t *>(map_dev.ptr);
        if (map_dev_resident == nullptr)
          GOSH_TRY_HIP(hipMemcpyAsync(map_dev.ptr, map_host + lo, static_cast<size_t>(cnt) * 4, hipMemcpyHostToDevice, st),
                   "copy map slice");
        if (int rc = gosh_project(src_dev, g.n, map_slice, cnt, d, static_cast<float *>(slice.ptr), st)) return rc;
        GOSH_TRY_HIP(hipMemcpyAsync(next_host + lo * d, slice.ptr, static_cast<size_t>(cnt) * d * 4,
                                hipMemcpyDeviceToHost, st),
                 "copy projected slice");
        GOSH_TRY_HIP(hipStreamSynchronize(st), "project slice");
      }
    } else {
      // the coarse matrix is on the host and too large to visit the device: gather its
      // rows there, then upload if the finer level happens to fit
      if (map_host == nullptr) {
        int64_t len = 0;
        if (int rc = gosh_hierarchy_map(h, i - 1, &map_host, &len)) return rc;
      }
      float *target = next_host;
      PinnedBuffer temp;
      if (next_dev) {
        if (int rc = temp.alloc(fine_bytes, "projection staging")) return rc;
        target = static_cast<float *>(temp.ptr);
      }
      const size_t row_bytes = static_cast<size_t>(d) * 4;
      const float *coarse = cur_host;
      const int32_t row_len = d;
#pragma omp parallel for schedule(static)
      for (int64_t v = 0; v < n_fine; ++v)
        std::memcpy(target + v * row_len, coarse + static_cast<int64_t>(map_host[v]) * row_len, row_bytes);
      if (next_dev) {
        GOSH_TRY_HIP(hipMemcpyAsync(next_dev, target, fine_bytes, hipMemcpyHostToDevice, st), "upload");
        GOSH_TRY_HIP(hipStreamSynchronize(st), "upload projected level");
      }
    }
    ls.project_ms = ms_since(t0);
    dev_own.swap(dev_next);
    dev_next.reset();
    host_own.swap(host_next);
    host_next.reset();
    cur_dev = next_dev;
    cur_host = next_host;
    return GOSH_OK;
  }
};

int embed_impl(const gosh_hierarchy *h, const Plan &pl, int64_t epochs, double p, float *M0_dev,
               float *M0_host, gosh_level_stats *stats, hipStream_t st) {
  MultilevelRun run(h, pl, M0_dev, M0_host, st);
  return run.run(epochs, p, stats);
}

int check_common(int32_t d, int32_t k_neg) {
  if (int rc = gosh::check_dim(d)) return rc;
  if (k_neg < 0 || k_neg > GOSH_MAX_NEG)
    return gosh::fail(GOSH_EINVAL, "k_neg = %d: must be in [0, %d]", k_neg, GOSH_MAX_NEG);
  return GOSH_OK;
}

}  // namespace

extern "C" {

int gosh_embed(const gosh_hierarchy *h, int32_t d, int32_t k_neg, int64_t epochs, double p, float lr0,
               uint64_t seed, uint32_t flags, uint64_t device_budget_bytes, float *M0_dev,
               gosh_level_stats *stats, void *hip_stream) {
  if (int rc = check_common(d, k_neg)) return rc;
  if (int rc = gosh::check_matrix(M0_dev, d, "M0")) return rc;
  {
    gosh_csr g0{};
    if (int rc = gosh::hierarchy_shape(h, 0, &g0)) return rc;
    if (int rc = gosh::check_device_span(M0_dev, static_cast<size_t>(g0.n) * d * 4, "M0")) return rc;
  }
  // A level above level 0 can only exceed the budget if level 0 does too, which is refused.
  const uint32_t train_flags = flags & ~(GOSH_FLAG_EDGE_EPOCHS | GOSH_FLAG_BLOCKED_ORDER | GOSH_FLAG_PAIR_LEVELS);
  const Plan pl{d, k_neg, lr0, seed, train_flags, train_flags, (flags & GOSH_FLAG_EDGE_EPOCHS) != 0,
                (flags & GOSH_FLAG_PAIR_LEVELS) != 0, device_budget_bytes, false, 3, 4, 5};
  return embed_impl(h, pl, epochs, p, M0_dev, nullptr, stats, gosh::as_stream(hip_stream));
}

int gosh_embed_host(const gosh_hierarchy *h, int32_t d, int32_t k_neg, int64_t epochs, double p,
                    float lr0, uint64_t seed, uint32_t flags, uint64_t device_budget_bytes,
                    int32_t P_gpu, int32_t S_gpu, int32_t B, float *M0_host, gosh_level_stats *stats,
                    void *hip_stream) {
  if (int rc = check_common(d, k_neg)) return rc;
  if (int rc = gosh::check_matrix(M0_host, d, "M0")) return rc;
  if (P_gpu < 2 || S_gpu < 1 || B < 1)
    return gosh::fail(GOSH_EINVAL, "need P_gpu >= 2, S_gpu >= 1, B >= 1");
  const uint32_t train_flags = flags & ~(GOSH_FLAG_EDGE_EPOCHS | GOSH_FLAG_BLOCKED_ORDER | GOSH_FLAG_PAIR_LEVELS);
  // No budget given: Alg. 2's "fits into the GPU" is asked of the device itself -- what it has
  // free now, less a sixteenth for the staging buffers and pools of the calls below.
  const bool measure = device_budget_bytes == 0;
  if (measure) {
    size_t free_bytes = 0, total_bytes = 0;
    GOSH_TRY_HIP(hipMemGetInfo(&free_bytes, &total_bytes), "hipMemGetInfo");
    device_budget_bytes = free_bytes - free_bytes / 16;
    if (device_budget_bytes == 0) return gosh::fail(GOSH_ENOMEM, "the device has no free memory");
  }
  const Plan pl{d, k_neg, lr0, seed, train_flags, train_flags | (flags & GOSH_FLAG_BLOCKED_ORDER),
                (flags & GOSH_FLAG_EDGE_EPOCHS) != 0, (flags & GOSH_FLAG_PAIR_LEVELS) != 0, device_budget_bytes, measure,
                P_gpu, S_gpu, B};
  return embed_impl(h, pl, epochs, p, nullptr, M0_host, stats, gosh::as_stream(hip_stream));
}

}  // extern "C"
