// Shared by the translation units of libgosh: error reporting and argument checks.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>

#include "gosh.h"

namespace gosh {

// Records a printf-style message for gosh_last_error() and returns `code`.
int fail(int code, const char *fmt, ...);

// Argument checks common to the device entry points.  Return GOSH_OK or record an
// error and return GOSH_EINVAL.
int check_dim(int32_t d);
int check_matrix(const float *M, int32_t d, const char *what);
int check_csr(const gosh_csr *g);
// The span [p, p + bytes) must be memory a kernel can reach: a device allocation that holds
// all of it, or pinned host memory.  GOSH_EINVAL otherwise (pageable host memory, a span
// running past its allocation) -- a kernel would fault on it.
int check_device_span(const void *p, size_t bytes, const char *what);
int check_device_csr(const gosh_csr *g);  // both arrays of a device-resident graph

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

// Turns a failed launch into GOSH_EHIP.
int check_launch(const char *kernel);

// Records the failure of a HIP call for gosh_last_error() and returns its status:
// GOSH_ENOMEM when device or pinned memory ran out, GOSH_EHIP otherwise.
int hip_fail(hipError_t e, const char *what);

// Returns from the enclosing function with that status if the call fails.
#define GOSH_TRY_HIP(call, what)                                 \
  do {                                                           \
    hipError_t e_ = (call);                                      \
    if (e_ != hipSuccess) return gosh::hip_fail(e_, what);       \
  } while (0)

// The process-wide tuning record behind gosh_set_tuning / gosh_get_tuning (fields documented
// in gosh.h).  Read at the start of every call that launches a training kernel.
gosh_tuning tuning();

// Wavefronts the device keeps resident (8 on each of the 4 SIMDs of every CU).
int resident_waves();

// Rows first_row .. first_row+count-1 of the initial matrix of a level, written to
// rows_dev (count x d): the arithmetic of gosh_init_embedding for a slice.
int init_rows(float *rows_dev, int64_t first_row, int64_t count, int32_t d, uint64_t seed,
              uint32_t level, hipStream_t st);

// True if [p, p + bytes) lies inside the mapped part of a matrix of gosh_matrix_place.
bool inside_placed_matrix(const void *p, size_t bytes);

// The launch behind gosh_row_probe, without its argument checks (the caller has made them).
int row_probe(float *M_dev, int64_t n, int32_t d, int64_t accesses, uint64_t seed, int32_t mode, hipStream_t st);

// Divergence check: largest finite |entry| (as the bits of the float) and the number of
// non-finite entries, accumulated on the device.  clear, then add any number of row ranges
// (all on one stream, or ordered by events), then read (copies the result and waits for the
// stream).
struct CheckResult {
  uint32_t max_bits;
  uint32_t pad;
  unsigned long long nonfinite;
};
int matrix_check_clear(CheckResult *result_dev, hipStream_t st);
int matrix_check_add(const float *rows_dev, int64_t floats, CheckResult *result_dev, hipStream_t st);
int matrix_check_read(const CheckResult *result_dev, float *max_abs, int64_t *nonfinite, hipStream_t st);
// A per-device CheckResult owned by the library (allocated on first use, kept).
int check_scratch(CheckResult **out);

// Per-device scratch for the hot-row bitmap (one bit per vertex), grown on demand and
// kept until the process ends.  Calls on one device must not overlap on different
// streams.
int hot_scratch(size_t bytes, void **out);

}  // namespace gosh
