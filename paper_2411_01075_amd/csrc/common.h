// Shared host-side helpers of the library: error reporting and argument checks.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include "../../include/cephalo.h"

namespace cephalo {

// Thread-local text of the last error; set by fail(), read by cephalo_last_error().
char* error_buffer();
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Checks the launch that was just issued; kernels are enqueued, never waited for.
#define CEPHALO_CHECK_LAUNCH(what)                                                          \
  do {                                                                                      \
    hipError_t e__ = hipGetLastError();                                                     \
    if (e__ != hipSuccess) return ::cephalo::fail(CEPHALO_EHIP, "%s: %s", what, hipGetErrorString(e__)); \
  } while (0)

typedef __bf16 bf16;

}  // namespace cephalo
