// Internal helpers shared by the host side of libroll_decode (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "roll_decode.h"

namespace roll {

// Thread-local error text returned by roll_last_error().
char* error_buffer();
constexpr int kErrorBufferBytes = 512;

inline int fail(int status, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(error_buffer(), kErrorBufferBytes, fmt, ap);
    va_end(ap);
    return status;
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

}  // namespace roll

#define ROLL_HIP_CHECK(expr)                                                          \
    do {                                                                              \
        hipError_t e_ = (expr);                                                       \
        if (e_ != hipSuccess)                                                         \
            return roll::fail(ROLL_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
    } while (0)
