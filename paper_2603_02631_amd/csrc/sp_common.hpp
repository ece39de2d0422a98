// Shared host-side helpers of the library: thread-local error text and HIP
// status checking. Nothing here runs on the device.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstddef>
#include <cstdint>
#include <cstdio>

#include "sp.h"

namespace sp {

char *error_buffer();                       // thread-local, 512 bytes
sp_status fail(sp_status code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ceil(n / d) for n >= 0, d > 0 without the overflow of n + d - 1
inline int64_t ceil_div(int64_t n, int64_t d) { return n / d + (n % d != 0 ? 1 : 0); }

}  // namespace sp

// Evaluates a HIP call; on failure records the text and returns SP_ERR_DEVICE.
#define SP_HIP_CHECK(expr)                                                           \
    do {                                                                             \
        hipError_t sp_hip_err_ = (expr);                                             \
        if (sp_hip_err_ != hipSuccess)                                               \
            return sp::fail(SP_ERR_DEVICE, "%s failed: %s", #expr,                   \
                            hipGetErrorString(sp_hip_err_));                         \
    } while (0)
