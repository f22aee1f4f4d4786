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

// Page stride of the KV pools in head blocks (one head block = page_size * head_dim elements, the
// part of a page that belongs to one KV head; K's and V's are the same size): num_kv_heads for
// dense pools (page_stride 0), twice that when K and V of a page sit side by side in one
// allocation.  Returns 0 for a stride that is not a whole number of head blocks or too small.
inline int32_t page_stride_heads(int64_t page_stride, int32_t num_kv_heads, int32_t page_size, int32_t head_dim) {
    if (page_stride == 0) return num_kv_heads;
    const int64_t block = (int64_t)page_size * head_dim;
    if (page_stride < 0 || page_stride % block != 0) return 0;
    const int64_t n = page_stride / block;
    return (n < num_kv_heads || n > (1 << 20)) ? 0 : (int32_t)n;
}

}  // namespace roll

#define ROLL_HIP_CHECK(expr)                                                          \
    do {                                                                              \
        hipError_t e_ = (expr);                                                       \
        if (e_ != hipSuccess)                                                         \
            return roll::fail(ROLL_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
    } while (0)
