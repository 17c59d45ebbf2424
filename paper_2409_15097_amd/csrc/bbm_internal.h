// Internal helpers shared by the translation units of libbbm (host side only; no kernels live here).
#pragma once
#include <hip/hip_runtime.h>
#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "bbm.h"

namespace bbm {

// Records a thread-local message and returns `code` so call sites can `return fail(...)`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Checks the launch status of the kernel just enqueued.
inline int launch_status(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(BBM_EHIP, "%s: %s", what, hipGetErrorString(e));
  return BBM_OK;
}

}  // namespace bbm
