// Division by a divisor fixed per launch: the host derives a multiplier and a shift, the device
// divides with one multiply-high, one add and one shift.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qnn {

// n / d for n < 2^31: q = (mulhi(n, mul) + n) >> shift.
struct FastDiv {
    uint32_t mul, shift, d;
};

inline FastDiv make_fastdiv(uint32_t d)
{
    uint32_t l = 0;
    while (((uint64_t)1 << l) < d) ++l;
    FastDiv f;
    f.shift = l;
    f.mul = (uint32_t)(((((uint64_t)1) << 32) * ((((uint64_t)1) << l) - d)) / d + 1);
    f.d = d;
    return f;
}

__device__ __forceinline__ uint32_t fdiv(uint32_t n, const FastDiv &f) { return (__umulhi(n, f.mul) + n) >> f.shift; }

} // namespace qnn
