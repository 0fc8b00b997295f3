// Internal helpers shared by the translation units of libexpertweave (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "expertweave.h"

namespace ew {

// Records a printf-style message for ew_last_error() and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

inline int hip_fail(hipError_t e, const char* what) {
  return fail(e == hipErrorOutOfMemory ? EW_ERR_OOM : EW_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

#define EW_HIP(call)                                    \
  do {                                                  \
    hipError_t _e = (call);                             \
    if (_e != hipSuccess) return ::ew::hip_fail(_e, #call); \
  } while (0)

// Checks the launch that was just enqueued.
#define EW_LAUNCH_CHECK(name)                                   \
  do {                                                          \
    hipError_t _e = hipGetLastError();                          \
    if (_e != hipSuccess) return ::ew::hip_fail(_e, "launch " name); \
  } while (0)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline int ilog2_ceil(int v) {  // smallest b with (1<<b) >= v, at least 1
  int b = 1;
  while ((1 << b) < v) ++b;
  return b;
}

}  // namespace ew
