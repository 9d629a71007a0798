// The linear quantizer of the encode step, shared by qnn_encode_pack and the fused epilogue of
// qnn_conv2d so that both produce the same code for the same fp32 value.
#pragma once

#include <hip/hip_runtime.h>

namespace qnn {

// Paper: Table 1 (HTanh) then Eq. 15 with round-half-up; returns the code u in [0, top],
// top = 2^bits - 1, level = 2u - top (Eq. 10).  Each step is one IEEE fp32 operation: the fma
// is explicit and the translation units are compiled with floating-point contraction off, so
// the trailing add stays an add.
__device__ __forceinline__ int quantize_code(float x, float inv_clip, float half_top, int top)
{
    float t = x * inv_clip;
    t = fmaxf(t, -1.0f);
    t = fminf(t, 1.0f);
    float r = __builtin_fmaf(t, half_top, half_top);
    r = r + 0.5f;
    // t lies in [-1, 1], so fma(t, h, h) lies in [0, 2h] = [0, top] (both ends exact) and floor(r + 0.5) in
    // [0, top]: no integer clamp is needed.  (A NaN converts to 0, also inside the range.)
    (void)top;
    return (int)floorf(r);
}

} // namespace qnn
