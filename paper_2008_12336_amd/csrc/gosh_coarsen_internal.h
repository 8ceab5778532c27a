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

// State one coarsening run keeps on the device between levels: the coarse graph of the
// last level (the next level reads it there instead of uploading it again) and pinned
// staging for the downloads.
struct DeviceCarry;
DeviceCarry *device_carry_new();
void device_carry_free(DeviceCarry *);

// "Coarsen(G_i, map_i)" on the current device: the quotient graph of the host graph
// `fine` under `map` (entry (a, b), a != b, for every fine entry (x, y) with map[x] = a,
// map[y] = b; parallel entries merged and their multiplicities added; rows ascending).
// mult_in may be null (every fine entry counts once).  Outputs are host vectors.  If
// `carry` holds the graph this very call sequence produced last (same n and nnz as
// `fine`), it is used in place of the host arrays.
int build_coarse_on_device(const gosh_csr &fine, const int64_t *mult_in, const int32_t *map,
                           int64_t n_coarse, int threads, DeviceCarry *carry,
                           RawVector<int64_t> &xadj_out, RawVector<int32_t> &adj_out,
                           RawVector<int64_t> &mult_out);

}  // namespace gosh
