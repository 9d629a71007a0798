// Host-side helpers shared by the entry points of libqnn: error reporting and argument checks.
// Nothing here touches the GPU, so every check runs (and is testable) on a machine without one.
#pragma once

#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/qnn.h"

namespace qnn {

// Thread-local message buffer behind qnn_last_error().
char *error_buffer();
constexpr int kErrorBufferSize = 256;

inline int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(error_buffer(), kErrorBufferSize, fmt, ap);
    va_end(ap);
    return code;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// n (2^w_bits - 1)(2^a_bits - 1) must stay below 2^31 so the int32 accumulator is exact.
inline bool acc_fits_int32(int64_t n, int w_bits, int a_bits)
{
    const int64_t top = (int64_t)((1 << w_bits) - 1) * (int64_t)((1 << a_bits) - 1);
    return n <= ((int64_t)INT32_MAX) / top;
}

inline int check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(QNN_ERR_LAUNCH, "%s: %s", what, hipGetErrorString(e));
    return QNN_OK;
}

} // namespace qnn
