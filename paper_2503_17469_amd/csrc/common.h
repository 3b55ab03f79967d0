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

// Integer batch sizes b[K] proportional to the weights T[K] with sum B inside [b_min, b_max]
// (largest remainder, ties to the lowest index; bound violators clamped and the rest
// re-apportioned).  Returns OMNI_OK or OMNI_EINFEASIBLE (message prefixed with `who`).
int apportion_bounded(const uint64_t* T, int K, int64_t B, int64_t b_min, int64_t b_max, int64_t* b,
                      const char* who);

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
