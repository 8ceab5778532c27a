// Multilevel driver (Alg. 2 of the paper): train the coarsest graph, project the
// embedding to the next finer graph, train that, ... until the embedding of G_0 exists.
// Host orchestration only: every numerical step is one of the library's kernels.
#include <hip/hip_runtime.h>

#include <chrono>
#include <vector>

#include "gosh_common.h"

namespace {

struct DeviceBuffer {
  void *ptr = nullptr;
  ~DeviceBuffer() { reset(); }
  DeviceBuffer() = default;
  DeviceBuffer(const DeviceBuffer &) = delete;
  DeviceBuffer &operator=(const DeviceBuffer &) = delete;
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

double ms_since(std::chrono::steady_clock::time_point t0) {
  return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
}

#define GOSH_HIP(call, what)                                                           \
  do {                                                                                 \
    hipError_t e_ = (call);                                                            \
    if (e_ != hipSuccess) return gosh::fail(GOSH_EHIP, "%s: %s", what, hipGetErrorString(e_)); \
  } while (0)

}  // namespace

extern "C" int gosh_embed(const gosh_hierarchy *h, int32_t d, int32_t k_neg, int64_t epochs, double p,
                          float lr0, uint64_t seed, uint32_t flags, uint64_t device_budget_bytes,
                          float *M0_dev, gosh_level_stats *stats, void *hip_stream) {
  const int D = gosh_hierarchy_levels(h);
  if (D < 1) return gosh::fail(GOSH_EINVAL, "hierarchy is null or empty");
  if (int rc = gosh::check_matrix(M0_dev, d, "M0")) return rc;
  std::vector<int64_t> e_i(static_cast<size_t>(D));
  if (int rc = gosh_epoch_split(epochs, p, D, e_i.data())) return rc;
  hipStream_t st = gosh::as_stream(hip_stream);

  DeviceBuffer m_cur, m_next;  // matrix of the level being trained / of the next finer one
  float *M_i = nullptr;
  hipEvent_t ev0, ev1;
  GOSH_HIP(hipEventCreate(&ev0), "hipEventCreate");
  GOSH_HIP(hipEventCreate(&ev1), "hipEventCreate");
  struct EventGuard {
    hipEvent_t a, b;
    ~EventGuard() {
      (void)hipEventDestroy(a);
      (void)hipEventDestroy(b);
    }
  } guard{ev0, ev1};

  for (int i = D - 1; i >= 0; --i) {
    gosh_csr host{};
    if (int rc = gosh_hierarchy_graph(h, i, &host)) return rc;
    const size_t off_bytes = static_cast<size_t>(host.n + 1) * (host.xadj_is64 ? 8 : 4);
    const size_t adj_bytes = static_cast<size_t>(host.nnz) * 4;
    const size_t mat_bytes = static_cast<size_t>(host.n) * d * 4;
    if (device_budget_bytes != 0 && off_bytes + adj_bytes + mat_bytes > device_budget_bytes)
      return gosh::fail(GOSH_EBUDGET,
                        "level %d needs %zu bytes on the device, budget is %llu: train it with "
                        "gosh_train_parts",
                        i, off_bytes + adj_bytes + mat_bytes, (unsigned long long)device_budget_bytes);

    // CopyToDevice(G_i): the graph arrays of this level.
    auto t0 = std::chrono::steady_clock::now();
    DeviceBuffer xadj_dev, adj_dev;
    if (int rc = xadj_dev.alloc(off_bytes, "xadj")) return rc;
    if (int rc = adj_dev.alloc(adj_bytes, "adj")) return rc;
    GOSH_HIP(hipMemcpyAsync(xadj_dev.ptr, host.xadj, off_bytes, hipMemcpyHostToDevice, st), "copy xadj");
    if (adj_bytes)
      GOSH_HIP(hipMemcpyAsync(adj_dev.ptr, host.adj, adj_bytes, hipMemcpyHostToDevice, st), "copy adj");
    GOSH_HIP(hipStreamSynchronize(st), "upload graph");
    const double upload_ms = ms_since(t0);

    if (i == D - 1) {
      // "Randomly initialize M_{D-1}"
      if (i == 0) {
        M_i = M0_dev;
      } else {
        if (int rc = m_cur.alloc(mat_bytes, "coarsest embedding")) return rc;
        M_i = static_cast<float *>(m_cur.ptr);
      }
      if (int rc = gosh_init_embedding(M_i, host.n, d, seed, static_cast<uint32_t>(i), st)) return rc;
    }

    gosh_csr dev = host;
    dev.xadj = xadj_dev.ptr;
    dev.adj = static_cast<const int32_t *>(adj_dev.ptr);
    GOSH_HIP(hipEventRecord(ev0, st), "hipEventRecord");
    for (int64_t j = 0; j < e_i[static_cast<size_t>(i)]; ++j) {
      const float lr = gosh_lr(lr0, j, e_i[static_cast<size_t>(i)]);
      if (int rc = gosh_train_epoch(&dev, M_i, d, k_neg, lr, seed, static_cast<uint32_t>(j),
                                    static_cast<uint32_t>(i), flags, st))
        return rc;
    }
    GOSH_HIP(hipEventRecord(ev1, st), "hipEventRecord");
    GOSH_HIP(hipEventSynchronize(ev1), "train level");
    float train_ms = 0.f;
    GOSH_HIP(hipEventElapsedTime(&train_ms, ev0, ev1), "hipEventElapsedTime");

    double project_ms = 0.0;
    if (i > 0) {
      // ExpandEmbedding(M_i, map_{i-1})
      t0 = std::chrono::steady_clock::now();
      const int32_t *map_host = nullptr;
      int64_t n_fine = 0;
      if (int rc = gosh_hierarchy_map(h, i - 1, &map_host, &n_fine)) return rc;
      DeviceBuffer map_dev;
      if (int rc = map_dev.alloc(static_cast<size_t>(n_fine) * 4, "map")) return rc;
      GOSH_HIP(hipMemcpyAsync(map_dev.ptr, map_host, static_cast<size_t>(n_fine) * 4,
                              hipMemcpyHostToDevice, st), "copy map");
      float *M_fine = M0_dev;
      if (i - 1 > 0) {
        if (int rc = m_next.alloc(static_cast<size_t>(n_fine) * d * 4, "finer embedding")) return rc;
        M_fine = static_cast<float *>(m_next.ptr);
      }
      if (int rc = gosh_project(M_i, host.n, static_cast<const int32_t *>(map_dev.ptr), n_fine, d,
                                M_fine, st))
        return rc;
      GOSH_HIP(hipStreamSynchronize(st), "project");
      project_ms = ms_since(t0);
      m_cur.swap(m_next);
      m_next.reset();
      M_i = M_fine;
    }
    if (stats) {
      gosh_level_stats &s = stats[i];
      s.level = i;
      s.n = host.n;
      s.nnz = host.nnz;
      s.epochs = e_i[static_cast<size_t>(i)];
      s.upload_ms = upload_ms;
      s.train_ms = train_ms;
      s.project_ms = project_ms;
    }
  }
  return GOSH_OK;
}
