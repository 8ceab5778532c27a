// Placement of an embedding matrix in device memory.
//
// The memory of this device answers in three classes of addresses (96 GB each; in a large
// allocation they come in runs of 16-64 GiB), and random row traffic confined to one class
// is slower than traffic spread over two: 5.2 against 6.2 TB/s for the epoch kernel.  A
// plain allocation of a few GB lies inside one class.  gosh_matrix_place builds an arena out
// of 1 GiB pieces of physical memory mapped back to back (the virtual-memory API), times the
// row probe on windows of it, keeps the pieces under the fastest window -- in practice one
// that straddles a border between two classes -- and gives all the others back.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <map>
#include <mutex>
#include <vector>

#include "gosh_common.h"

namespace {

struct Arena {
  const char *kept_begin = nullptr, *kept_end = nullptr;  // the pieces that stay mapped
  char *va = nullptr;      // reserved range
  size_t va_bytes = 0;
  size_t piece = 0;        // bytes per piece
  std::vector<hipMemGenericAllocationHandle_t> handle;  // per piece
  std::vector<char> mapped;                             // per piece

  // Unmaps and releases piece i (idempotent).
  void drop(size_t i) {
    if (!mapped[i]) return;
    (void)hipMemUnmap(va + i * piece, piece);
    (void)hipMemRelease(handle[i]);
    mapped[i] = 0;
  }
  ~Arena() {
    if (va == nullptr) return;
    (void)hipDeviceSynchronize();
    for (size_t i = 0; i < mapped.size(); ++i) drop(i);
    (void)hipMemAddressFree(va, va_bytes);
  }
};

std::mutex g_mutex;
std::map<const void *, Arena *> g_placed;  // matrix pointer -> what backs it

hipMemAllocationProp device_memory(int device) {
  hipMemAllocationProp prop = {};
  prop.type = hipMemAllocationTypePinned;
  prop.location.type = hipMemLocationTypeDevice;
  prop.location.id = device;
  return prop;
}

}  // namespace

namespace gosh {

bool inside_placed_matrix(const void *p, size_t bytes) {
  const char *lo = static_cast<const char *>(p);
  std::lock_guard<std::mutex> lock(g_mutex);
  for (const auto &entry : g_placed)
    if (lo >= entry.second->kept_begin && lo + bytes <= entry.second->kept_end) return true;
  return false;
}

}  // namespace gosh

extern "C" {

int gosh_matrix_place(int64_t n, int32_t d, uint64_t arena_bytes, float **M_dev, gosh_placement_info *info) {
  if (M_dev == nullptr) return gosh::fail(GOSH_EINVAL, "M_dev is null");
  *M_dev = nullptr;
  if (int rc = gosh::check_dim(d)) return rc;
  if (n < 1 || n >= 2147483647LL) return gosh::fail(GOSH_EINVAL, "n = %lld out of range", (long long)n);
  const auto t0 = std::chrono::steady_clock::now();
  const size_t row_bytes = static_cast<size_t>(d) * 4, need = static_cast<size_t>(n) * row_bytes;
  int device = 0;
  GOSH_TRY_HIP(hipGetDevice(&device), "hipGetDevice");
  const hipMemAllocationProp prop = device_memory(device);
  size_t granularity = 0;
  GOSH_TRY_HIP(hipMemGetAllocationGranularity(&granularity, &prop, hipMemAllocationGranularityRecommended),
               "hipMemGetAllocationGranularity");
  const size_t piece = std::max<size_t>(size_t{1} << 30, granularity) / granularity * granularity;
  size_t free_bytes = 0, total_bytes = 0;
  GOSH_TRY_HIP(hipMemGetInfo(&free_bytes, &total_bytes), "hipMemGetInfo");
  const size_t keep_free = size_t{8} << 30;
  size_t want = arena_bytes == 0 ? (size_t{120} << 30) : static_cast<size_t>(arena_bytes);
  want = std::min(want, free_bytes > keep_free ? free_bytes - keep_free : 0);
  const size_t pieces = want / piece;
  if (pieces * piece < 3 * need + piece)
    return gosh::fail(GOSH_ENOMEM, "no room for an arena of three times the matrix (%zu bytes) beside what is allocated",
                      need);

  Arena *arena = new (std::nothrow) Arena();
  if (arena == nullptr) return gosh::fail(GOSH_ENOMEM, "out of host memory");
  struct Guard {
    Arena *a;
    ~Guard() { delete a; }
  } guard{arena};
  arena->piece = piece;
  arena->va_bytes = pieces * piece;
  void *va = nullptr;
  GOSH_TRY_HIP(hipMemAddressReserve(&va, arena->va_bytes, 0, nullptr, 0), "hipMemAddressReserve");
  arena->va = static_cast<char *>(va);
  arena->handle.resize(pieces);
  arena->mapped.assign(pieces, 0);
  hipMemAccessDesc access = {};
  access.location = prop.location;
  access.flags = hipMemAccessFlagsProtReadWrite;
  for (size_t i = 0; i < pieces; ++i) {
    GOSH_TRY_HIP(hipMemCreate(&arena->handle[i], piece, &prop, 0), "hipMemCreate");
    hipError_t e = hipMemMap(arena->va + i * piece, piece, 0, arena->handle[i], 0);
    if (e != hipSuccess) {
      (void)hipMemRelease(arena->handle[i]);
      return gosh::hip_fail(e, "hipMemMap");
    }
    arena->mapped[i] = 1;
    GOSH_TRY_HIP(hipMemSetAccess(arena->va + i * piece, piece, &access, 1), "hipMemSetAccess");
  }

  // Time the row probe on windows of the arena.  A window gains only while it straddles a
  // border, i.e. within its own length of one: scan at half the window's length (at most
  // 4 GiB, at most about a thousand windows), then four times finer around the best, then at
  // the centre of gravity of the gains (they fall off linearly on both sides of the border).
  hipEvent_t start = nullptr, stop = nullptr;
  GOSH_TRY_HIP(hipEventCreate(&start), "hipEventCreate");
  struct EventGuard {
    hipEvent_t &a, &b;
    ~EventGuard() {
      if (a) (void)hipEventDestroy(a);
      if (b) (void)hipEventDestroy(b);
    }
  } events{start, stop};
  GOSH_TRY_HIP(hipEventCreate(&stop), "hipEventCreate");
  const int64_t rows_total = static_cast<int64_t>(arena->va_bytes / row_bytes);
  const int64_t last = rows_total - n;
  std::map<int64_t, float> timed;
  auto probe = [&](int64_t first_row) -> int {
    if (timed.count(first_row)) return GOSH_OK;
    float *window = reinterpret_cast<float *>(arena->va + static_cast<size_t>(first_row) * row_bytes);
    GOSH_TRY_HIP(hipEventRecord(start, nullptr), "hipEventRecord");
    if (int rc = gosh::row_probe(window, n, d, 4 * n, 1, GOSH_PROBE_READ_WRITE, nullptr)) return rc;
    GOSH_TRY_HIP(hipEventRecord(stop, nullptr), "hipEventRecord");
    GOSH_TRY_HIP(hipEventSynchronize(stop), "row probe");
    float ms = 0.f;
    GOSH_TRY_HIP(hipEventElapsedTime(&ms, start, stop), "hipEventElapsedTime");
    timed[first_row] = ms;
    return GOSH_OK;
  };
  auto fastest = [&] {
    return std::min_element(timed.begin(), timed.end(),
                            [](const auto &x, const auto &y) { return x.second < y.second; })->first;
  };
  const int64_t rows_per_gib = std::max<int64_t>(1, static_cast<int64_t>((size_t{1} << 30) / row_bytes));
  const int64_t coarse = std::max<int64_t>(1, std::min<int64_t>(4 * rows_per_gib, std::max<int64_t>(n / 2, last / 1000)));
  const int64_t fine = std::max<int64_t>(1, coarse / 4);
  for (int64_t r = 0; r <= last; r += coarse)
    if (int rc = probe(r)) return rc;
  int64_t best = fastest();
  for (int64_t r = std::max<int64_t>(0, best - 3 * fine); r <= std::min(last, best + 3 * fine); r += fine)
    if (int rc = probe(r)) return rc;
  best = fastest();
  std::vector<float> all;
  for (const auto &t : timed) all.push_back(t.second);
  std::nth_element(all.begin(), all.begin() + all.size() / 2, all.end());
  const float median = all[all.size() / 2];
  double weight = 0, moment = 0;
  for (const auto &t : timed)
    if (std::llabs(t.first - best) <= coarse && t.second < median) {
      weight += median - t.second;
      moment += (median - t.second) * static_cast<double>(t.first);
    }
  if (weight > 0) {
    const int64_t centre = std::max<int64_t>(0, std::min(last, static_cast<int64_t>(moment / weight)));
    if (int rc = probe(centre)) return rc;
    if (timed[centre] <= timed[best] * 1.01f) best = centre;
  }
  // rows start at multiples of 16 bytes anyway (d is a multiple of 4)
  const size_t begin = static_cast<size_t>(best) * row_bytes, end = begin + need;
  const size_t first_piece = begin / piece, end_piece = (end + piece - 1) / piece;
  GOSH_TRY_HIP(hipDeviceSynchronize(), "before releasing the arena");
  for (size_t i = 0; i < pieces; ++i)
    if (i < first_piece || i >= end_piece) arena->drop(i);
  float *M = reinterpret_cast<float *>(arena->va + begin);
  arena->kept_begin = arena->va + first_piece * piece;
  arena->kept_end = arena->va + end_piece * piece;
  {
    std::lock_guard<std::mutex> lock(g_mutex);
    g_placed[M] = arena;
  }
  guard.a = nullptr;
  *M_dev = M;
  if (info) {
    info->arena_bytes = pieces * piece;
    info->window_offset_bytes = begin;
    info->kept_bytes = (end_piece - first_piece) * piece;
    info->probes = static_cast<int32_t>(timed.size());
    info->probe_ms_best = timed[best];
    info->probe_ms_median = median;
    info->search_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
  }
  return GOSH_OK;
}

int gosh_matrix_release(float *M_dev) {
  Arena *arena = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_mutex);
    auto it = g_placed.find(M_dev);
    if (it == g_placed.end()) return gosh::fail(GOSH_EINVAL, "not a matrix of gosh_matrix_place");
    arena = it->second;
    g_placed.erase(it);
  }
  delete arena;  // waits for the device, unmaps, releases
  return GOSH_OK;
}

}  // extern "C"
