// The terms a residual block adds between the scale factor and the next quantizer, as the two
// convolution kernels take them: a per-channel shift (a folded batch-norm) and a shortcut held
// either as quantized codes or in fp32.  The paper's derivation drops the bias; its ResNet-18
// experiments need both.  Order and rounding are fixed (one fp32 operation per step):
//   y = (float)acc * scale[c];  y = y + bias[c];  y = y + ((float)level * res_scale);  y = y + res_f32;
//   y = max(y, 0) (relu: HReLU's lower limit, Table 1).
#pragma once

#include <math.h>

#include "qnn_host.h"

namespace qnn {

struct BlockTerms {
    const float *bias = nullptr;    // [Cout]
    const void *res_q = nullptr;    // planes [res_bits][pixels][ceil(Cout/32)] or int8 levels [pixels][Cout]
    const float *res_f32 = nullptr; // [pixels][Cout]
    int res_bits = 0, res_top = 0;  // level = 2 code - res_top
    float res_scale = 0.0f;
    int relu = 0;
    bool any() const { return bias || res_q || res_f32 || relu; }
};

// Host-side check and translation of the caller's struct (NULL: no terms).
inline int block_terms(const char *who, const qnn_block_epilogue *epi, const float *scale, int max_bits, BlockTerms &t)
{
    t = BlockTerms();
    if (!epi) return QNN_OK;
    if (!scale) return fail(QNN_ERR_INVALID_ARG, "%s: block terms given without scale", who);
    if (epi->res_q) {
        if (epi->res_bits < 1 || epi->res_bits > max_bits)
            return fail(QNN_ERR_INVALID_ARG, "%s: res_bits=%d outside [1,%d]", who, epi->res_bits, max_bits);
        if (!isfinite(epi->res_scale)) return fail(QNN_ERR_INVALID_ARG, "%s: res_scale must be finite", who);
    }
    if (!aligned16(epi->bias) || !aligned16(epi->res_q) || !aligned16(epi->res_f32))
        return fail(QNN_ERR_ALIGNMENT, "%s: block-term pointers must be 16-byte aligned", who);
    t.bias = epi->bias, t.res_q = epi->res_q, t.res_f32 = epi->res_f32, t.relu = epi->relu ? 1 : 0;
    if (epi->res_q) t.res_bits = epi->res_bits, t.res_top = (1 << epi->res_bits) - 1, t.res_scale = epi->res_scale;
    return QNN_OK;
}

} // namespace qnn
