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

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

// Turns a failed launch into GOSH_EHIP.
int check_launch(const char *kernel);

}  // namespace gosh
