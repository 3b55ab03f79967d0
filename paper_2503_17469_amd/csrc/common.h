// Shared host-side helpers for the omnistep library: error reporting and the
// by-value segment table handed to ragged kernels.
#pragma once
#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "../../include/omnistep.h"

namespace omni {

// Records a thread-local message and returns `code` so call sites can `return fail(...)`.
int fail(int code, const char* fmt, ...);

// Worker row ranges of the concatenated batch, passed to kernels by value
// (260 bytes of kernel arguments; no device-side table to upload or keep alive).
struct Segments {
  int32_t K;
  int32_t off[OMNI_MAX_WORKERS + 1];
};

}  // namespace omni

#define OMNI_HIP_CHECK(expr)                                                        \
  do {                                                                              \
    hipError_t _e = (expr);                                                         \
    if (_e != hipSuccess)                                                           \
      return ::omni::fail(OMNI_EHIP, "%s failed: %s", #expr, hipGetErrorString(_e)); \
  } while (0)
