// Host-side pieces of libgosh that need no device code: error state, schedule helpers.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <mutex>

#include "gosh_common.h"

namespace gosh {

static thread_local char g_error[512] = "";

int fail(int code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
  return code;
}

int check_dim(int32_t d) {
  if (d < 4 || d > GOSH_MAX_DIM || (d % 4) != 0)
    return fail(GOSH_EINVAL, "d = %d: must be a multiple of 4 in [4, %d]", d, GOSH_MAX_DIM);
  return GOSH_OK;
}

int check_matrix(const float *M, int32_t d, const char *what) {
  if (int rc = check_dim(d)) return rc;
  if (M == nullptr) return fail(GOSH_EINVAL, "%s is null", what);
  if (reinterpret_cast<uintptr_t>(M) % 16 != 0)
    return fail(GOSH_EINVAL, "%s must be 16-byte aligned", what);
  return GOSH_OK;
}

int check_csr(const gosh_csr *g) {
  if (g == nullptr) return fail(GOSH_EINVAL, "graph is null");
  if (g->n < 1 || g->n >= 2147483647LL)
    return fail(GOSH_EINVAL, "n = %lld: must be in [1, 2^31-1)", (long long)g->n);
  if (g->nnz < 0) return fail(GOSH_EINVAL, "nnz = %lld is negative", (long long)g->nnz);
  if (g->xadj == nullptr) return fail(GOSH_EINVAL, "xadj is null");
  if (g->nnz > 0 && g->adj == nullptr) return fail(GOSH_EINVAL, "adj is null but nnz > 0");
  if (!g->xadj_is64 && g->nnz > 2147483647LL)
    return fail(GOSH_EINVAL, "nnz = %lld needs 64-bit offsets", (long long)g->nnz);
  return GOSH_OK;
}

int check_device_span(const void *p, size_t bytes, const char *what) {
  // A matrix of gosh_matrix_place is stitched from several mappings, which the runtime
  // reports one by one: the library knows its extent itself.
  if (inside_placed_matrix(p, bytes)) return GOSH_OK;
  // The runtime answers for every address: memory it does not know (pageable host memory,
  // a stale or made-up pointer) comes back as "unregistered", not as an error.
  hipPointerAttribute_t attr;
  if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
    (void)hipGetLastError();
    return fail(GOSH_EINVAL, "%s is not memory a kernel can reach (device or pinned host memory is needed)", what);
  }
  if (attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeHost && attr.type != hipMemoryTypeManaged)
    return fail(GOSH_EINVAL, "%s is not memory a kernel can reach (device or pinned host memory is needed)", what);
  hipDeviceptr_t base = nullptr;
  size_t size = 0;
  if (hipMemGetAddressRange(&base, &size, const_cast<void *>(p)) == hipSuccess) {
    const char *end = static_cast<const char *>(p) + bytes;
    if (end > static_cast<const char *>(base) + size)
      return fail(GOSH_EINVAL, "%s: %zu bytes do not fit the allocation they start in", what, bytes);
  } else {
    (void)hipGetLastError();
  }
  return GOSH_OK;
}

int check_device_csr(const gosh_csr *g) {
  if (int rc = check_device_span(g->xadj, static_cast<size_t>(g->n + 1) * (g->xadj_is64 ? 8 : 4), "xadj")) return rc;
  if (g->nnz > 0)
    if (int rc = check_device_span(g->adj, static_cast<size_t>(g->nnz) * 4, "adj")) return rc;
  return GOSH_OK;
}

int hip_fail(hipError_t e, const char *what) {
  (void)hipGetLastError();  // the runtime keeps the error until it is read
  const int code = (e == hipErrorOutOfMemory || e == hipErrorMemoryAllocation) ? GOSH_ENOMEM : GOSH_EHIP;
  return fail(code, "%s: %s", what, hipGetErrorString(e));
}

int check_launch(const char *kernel) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(GOSH_EHIP, "%s: %s", kernel, hipGetErrorString(e));
  return GOSH_OK;
}

namespace {
std::mutex g_tuning_mutex;
constexpr gosh_tuning kDefaultTuning{0, int64_t{1} << 18, 64, 4, 0, int64_t{1} << 22};
gosh_tuning g_tuning = kDefaultTuning;
}  // namespace

gosh_tuning tuning() {
  std::lock_guard<std::mutex> lock(g_tuning_mutex);
  return g_tuning;
}

int resident_waves() {
  static const int value = [] {
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) {
      int v = 0;
      if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
        cus = v;
    }
    return cus * 32;
  }();
  return value;
}

namespace {
struct HotScratch {
  void *ptr = nullptr;
  size_t bytes = 0;
};
constexpr int kMaxDevices = 64;
HotScratch g_hot_scratch[kMaxDevices];
std::mutex g_hot_scratch_mutex;  // guards the table, not the use of the buffers
}  // namespace

int hot_scratch(size_t bytes, void **out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
    return fail(GOSH_EHIP, "cannot identify the current device");
  std::lock_guard<std::mutex> lock(g_hot_scratch_mutex);
  HotScratch &h = g_hot_scratch[dev];
  if (h.bytes < bytes) {
    if (h.ptr) (void)hipFree(h.ptr);
    h.ptr = nullptr;
    h.bytes = 0;
    const size_t want = bytes + bytes / 4 + 4096;
    if (hipMalloc(&h.ptr, want) != hipSuccess) {
      (void)hipGetLastError();
      return fail(GOSH_ENOMEM, "cannot allocate %zu bytes for the hot-row bitmap", want);
    }
    h.bytes = want;
  }
  *out = h.ptr;
  return GOSH_OK;
}

int check_scratch(CheckResult **out) {
  static CheckResult *table[kMaxDevices] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
    return fail(GOSH_EHIP, "cannot identify the current device");
  std::lock_guard<std::mutex> lock(g_hot_scratch_mutex);
  if (table[dev] == nullptr) {
    void *p = nullptr;
    if (hipMalloc(&p, sizeof(CheckResult)) != hipSuccess) {
      (void)hipGetLastError();
      return fail(GOSH_ENOMEM, "cannot allocate the result of the divergence check");
    }
    table[dev] = static_cast<CheckResult *>(p);
  }
  *out = table[dev];
  return GOSH_OK;
}

}  // namespace gosh

extern "C" {

const char *gosh_last_error(void) { return gosh::g_error; }

void gosh_tuning_defaults(gosh_tuning *t) {
  if (t) *t = gosh::kDefaultTuning;
}

int gosh_set_tuning(const gosh_tuning *t) {
  const gosh_tuning v = t ? *t : gosh::kDefaultTuning;
  if (v.max_waves < 1) return gosh::fail(GOSH_EINVAL, "max_waves = %lld: must be positive", (long long)v.max_waves);
  if (v.hot_inv_eps < 1) return gosh::fail(GOSH_EINVAL, "hot_inv_eps = %lld: must be positive", (long long)v.hot_inv_eps);
  if (v.hot_all_inv_eps < 0)
    return gosh::fail(GOSH_EINVAL, "hot_all_inv_eps = %lld: must not be negative", (long long)v.hot_all_inv_eps);
  if (v.hot_min_degree < 0)
    return gosh::fail(GOSH_EINVAL, "hot_min_degree = %lld: must not be negative", (long long)v.hot_min_degree);
  if (v.pair_level_min_n < 1)
    return gosh::fail(GOSH_EINVAL, "pair_level_min_n = %lld: must be positive", (long long)v.pair_level_min_n);
  std::lock_guard<std::mutex> lock(gosh::g_tuning_mutex);
  gosh::g_tuning = v;
  return GOSH_OK;
}

int gosh_get_tuning(gosh_tuning *t) {
  if (t == nullptr) return gosh::fail(GOSH_EINVAL, "tuning record is null");
  *t = gosh::tuning();
  return GOSH_OK;
}

int32_t gosh_pair_level_parts(int64_t epochs, int64_t n, int64_t min_n, int32_t B) {
  if (epochs < 1 || n < 1 || B < 1) return 0;
  if (min_n < 1) min_n = 1;
  for (int32_t K = 16; K >= 1; K /= 2) {
    if (K * min_n > n) continue;
    const int64_t per = static_cast<int64_t>(B) * K;
    const int64_t run = (epochs + per - 1) / per * per;
    if ((run - epochs) * 8 <= epochs) return K;
  }
  return 0;
}

float gosh_lr(float lr0, int64_t j, int64_t e_i) {
  if (e_i <= 0) return 0.0f;
  double frac = 1.0 - static_cast<double>(j) / static_cast<double>(e_i);
  frac = std::fmax(frac, 1e-4);
  return static_cast<float>(static_cast<double>(lr0) * frac);
}

int gosh_epoch_split(int64_t e, double p, int32_t D, int64_t *e_i) {
  if (e_i == nullptr) return gosh::fail(GOSH_EINVAL, "e_i is null");
  if (D < 1 || D > 62) return gosh::fail(GOSH_EINVAL, "D = %d: must be in [1, 62]", D);
  if (!(p >= 0.0 && p <= 1.0)) return gosh::fail(GOSH_EINVAL, "p = %g outside [0, 1]", p);
  if (e < D) return gosh::fail(GOSH_EINVAL, "e = %lld cannot cover %d levels", (long long)e, D);
  const double uniform_share = p * static_cast<double>(e) / static_cast<double>(D);
  const double geometric_pool = (1.0 - p) * static_cast<double>(e);
  const double weight_sum = static_cast<double>((uint64_t{1} << D) - 1);
  int64_t remaining = e;
  for (int32_t level = 1; level < D; ++level) {
    double weight = static_cast<double>(uint64_t{1} << level);
    int64_t epochs = static_cast<int64_t>(std::floor(uniform_share + geometric_pool * weight / weight_sum));
    e_i[level] = epochs < 1 ? 1 : epochs;
    remaining -= e_i[level];
  }
  if (remaining < 1)
    return gosh::fail(GOSH_EINVAL, "e = %lld leaves no epoch for level 0", (long long)e);
  e_i[0] = remaining;
  return GOSH_OK;
}

}  // extern "C"
