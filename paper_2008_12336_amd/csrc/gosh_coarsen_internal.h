// Internal interface between the coarsening driver and the device-side CSR rebuild.
#pragma once

#include <sys/mman.h>

#include <cstdint>
#include <cstdlib>
#include <new>
#include <utility>
#include <vector>

#include "gosh.h"

namespace gosh {

// Allocator for the multi-gigabyte arrays of a coarse level, which are written exactly
// once: resize() leaves trivially constructible elements uninitialised (value-initialising
// them would fault every page in on one thread), and large blocks are aligned to 2 MiB and
// marked for transparent huge pages, which cuts the number of page faults of the first
// write by 512.
template <typename T>
struct NoInitAlloc {
  using value_type = T;
  NoInitAlloc() = default;
  template <typename U>
  NoInitAlloc(const NoInitAlloc<U> &) {}
  T *allocate(size_t count) {
    constexpr size_t kHuge = size_t(2) << 20;
    const size_t bytes = count * sizeof(T);
    void *p = nullptr;
    if (bytes >= 4 * kHuge) {
      const size_t rounded = (bytes + kHuge - 1) / kHuge * kHuge;
      p = aligned_alloc(kHuge, rounded);
      if (p != nullptr) (void)madvise(p, rounded, MADV_HUGEPAGE);  // advisory: failure is harmless
    } else {
      p = malloc(bytes > 0 ? bytes : 1);
    }
    if (p == nullptr) throw std::bad_alloc();
    return static_cast<T *>(p);
  }
  void deallocate(T *p, size_t) { free(p); }
  template <typename U>
  void construct(U *p) {
    ::new (static_cast<void *>(p)) U;
  }
  template <typename U, typename... Args>
  void construct(U *p, Args &&...args) {
    ::new (static_cast<void *>(p)) U(std::forward<Args>(args)...);
  }
  template <typename U>
  bool operator==(const NoInitAlloc<U> &) const {
    return true;
  }
  template <typename U>
  bool operator!=(const NoInitAlloc<U> &) const {
    return false;
  }
};
template <typename T>
using RawVector = std::vector<T, NoInitAlloc<T>>;

// One graph of the hierarchy in device memory (all arrays exact-sized hipMalloc blocks on
// `device`; null when absent).
struct DeviceLevel {
  int device = -1;
  int64_t n = 0, nnz = 0;
  int32_t xadj_is64 = 1;
  void *xadj = nullptr;     // n + 1 offsets
  int32_t *adj = nullptr;   // nnz neighbours
  int64_t *mult = nullptr;  // nnz multiplicities (coarse levels only)
  int32_t *map = nullptr;   // n cluster ids (every level but the last)
  bool borrowed_graph = false;  // xadj and adj belong to the caller (a device-resident G_0)
  bool present() const { return xadj != nullptr; }
};
void device_level_free(DeviceLevel &level);

// State of one coarsening run: device blocks recycled over the levels and pinned staging
// for downloads.
struct DeviceCoarsener;
DeviceCoarsener *device_coarsener_new(int threads);
void device_coarsener_free(DeviceCoarsener *);
// Returns the recycled device blocks; the staging stays (later downloads use it).
void device_coarsener_trim(DeviceCoarsener *);

// Copies a host graph to the current device and range-checks it there.
int device_level_upload(DeviceCoarsener *dc, const gosh_csr &host, DeviceLevel &out);
// Adopts a graph that already lives on the current device (not freed with the level) and
// range-checks it.
int device_level_borrow(const gosh_csr &on_device, DeviceLevel &out);
// Offsets run from 0 to nnz without decreasing, neighbour ids lie in [0, n): GOSH_EINVAL if not.
int device_level_check(const DeviceLevel &level);
// True for memory allocated on a device (hipMalloc); false for host memory of any kind.
bool is_device_pointer(const void *p);
// Replaces level.map with a copy of the host array (n entries).
int device_level_set_map(DeviceLevel &level, const int32_t *map_host);
// Drops level.map.
void device_level_drop_map(DeviceLevel &level);

// The marking sweep of Alg. 4 on the device: writes fine.map and *n_coarse and sets *done.
// Chains of equal-degree vertices can make the parallel resolution take too many rounds;
// then *done is false, nothing was written, and the caller marks on the host.
// *order_ms receives the time of the degree sort.
int device_mark(DeviceCoarsener *dc, DeviceLevel &fine, int64_t *n_coarse, bool *done, double *order_ms);

// "Coarsen(G_i, map_i)" on the device: the quotient graph of `fine` under fine.map (entry
// (a, b), a != b, for every fine entry (x, y) with map[x] = a, map[y] = b; parallel entries
// merged and their multiplicities added; rows ascending).
int device_rebuild(DeviceCoarsener *dc, const DeviceLevel &fine, int64_t n_coarse, DeviceLevel &coarse);

// Copies between pageable host memory and the device through the run's pinned staging,
// the host side of every piece shared by all threads.
int device_download(DeviceCoarsener *dc, void *dst, const void *src_dev, size_t bytes);
int device_upload(DeviceCoarsener *dc, void *dst_dev, const void *src, size_t bytes);

// What the multilevel driver needs of a hierarchy without forcing host copies: the shape
// of G_i (n, nnz, xadj_is64; pointers null) and its device copy (null if there is none).
int hierarchy_shape(const gosh_hierarchy *h, int32_t i, gosh_csr *shape);
const DeviceLevel *hierarchy_device_level(const gosh_hierarchy *h, int32_t i);

}  // namespace gosh
