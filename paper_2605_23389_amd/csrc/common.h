// Shared host-side helpers of the C-ABI library: status plumbing and the
// thread-local error string behind as_last_error().
#pragma once

#include <cstdarg>
#include <cstdio>
#include <new>

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

// No C++ exception may cross the C ABI: entry points that allocate run their
// body between these two.  The bodies are written so that everything that can
// throw happens before the first change to the object they work on.
#define ALS_TRY try {
#define ALS_CATCH(name)                                                              \
  }                                                                                  \
  catch (const std::bad_alloc&) {                                                    \
    return als::fail(AS_ENOMEM, name ": out of host memory");                        \
  }                                                                                  \
  catch (...) {                                                                      \
    return als::fail(AS_ENOMEM, name ": unexpected C++ exception");                  \
  }

#define ALS_HIP_CHECK(expr)                                                          \
  do {                                                                               \
    hipError_t _e = (expr);                                                          \
    if (_e != hipSuccess)                                                            \
      return als::fail(AS_EHIP, "%s failed: %s", #expr, hipGetErrorString(_e));      \
  } while (0)
