// Shared host-side helpers of the C-ABI library: status plumbing and the
// thread-local error string behind as_last_error().
#pragma once

#include <cstdarg>
#include <cstdio>

#include "alignedserve.h"

namespace als {

char* error_buffer();  // thread-local, 512 bytes

inline as_status fail(as_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(error_buffer(), 512, fmt, ap);
  va_end(ap);
  return st;
}

}  // namespace als

#define ALS_HIP_CHECK(expr)                                                          \
  do {                                                                               \
    hipError_t _e = (expr);                                                          \
    if (_e != hipSuccess)                                                            \
      return als::fail(AS_EHIP, "%s failed: %s", #expr, hipGetErrorString(_e));      \
  } while (0)
