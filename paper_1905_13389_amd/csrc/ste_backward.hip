// Training-side gradients (paper: sections "Multi-Branch Binary Networks Training" and "Quantized
// Networks Training").  Elementwise, streaming, HBM bound.
//
// qnn_quantize_ste_backward: the hard ladder q_k (Eq. 15) has zero derivative almost everywhere, so
// it is differentiated as the identity (straight-through) behind the range limit HTanh (Table 1):
// the gradient passes with slope 1 / clip where -1 <= x / clip <= 1 and is 0 outside.  With clip = 1
// this is also the gradient of Binarize(x) = sign(HTanh(x)) (Eq. 14).
//
// qnn_encoder_backward: plane m of an M-bit encoder (m = 1 lowest) is the sign of a sine,
// +sin(pi K t / 2^M) for m = M and -sin(pi K t / 2^m) below (K = 2^M - 1; Eq. 11 for M = 2); its
// derivative is taken as the sine's inside [-1, 1] and 0 outside (Eq. 12-13 for M = 2).  The cosine
// is evaluated as cospi(t K / 2^m): K / 2^m is exact in fp32 and cospi reduces its argument exactly.
#include "qnn_host.h"

namespace qnn {

struct SteParams {
    const float *x, *g;
    float *gx;
    int64_t count;
    float inv_clip;
    float zmul[8];  // K / 2^m
    float slope[8]; // +- pi K / 2^m
};

template <int V> struct FloatVec;
template <> struct FloatVec<1> { using type = float; };
template <> struct FloatVec<4> { using type = float4; };

template <int V> __global__ __launch_bounds__(256) void quantize_ste_backward_kernel(SteParams p)
{
    using F = typename FloatVec<V>::type;
    const int64_t n = p.count / V, stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const F xv = reinterpret_cast<const F *>(p.x)[i], gv = reinterpret_cast<const F *>(p.g)[i];
        F ov;
#pragma unroll
        for (int e = 0; e < V; ++e) {
            const float t = reinterpret_cast<const float *>(&xv)[e] * p.inv_clip;
            const bool inside = t >= -1.0f && t <= 1.0f;
            reinterpret_cast<float *>(&ov)[e] = inside ? reinterpret_cast<const float *>(&gv)[e] * p.inv_clip : 0.0f;
        }
        reinterpret_cast<F *>(p.gx)[i] = ov;
    }
}

template <int BITS, int V> __global__ __launch_bounds__(256) void encoder_backward_kernel(SteParams p)
{
    using F = typename FloatVec<V>::type;
    const int64_t n = p.count / V, stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const F xv = reinterpret_cast<const F *>(p.x)[i];
        F gv[BITS];
#pragma unroll
        for (int m = 0; m < BITS; ++m) gv[m] = reinterpret_cast<const F *>(p.g + (int64_t)m * p.count)[i];
        F ov;
#pragma unroll
        for (int e = 0; e < V; ++e) {
            const float t = reinterpret_cast<const float *>(&xv)[e] * p.inv_clip;
            const bool inside = t >= -1.0f && t <= 1.0f;
            float total = 0.0f;
#pragma unroll
            for (int m = 0; m < BITS; ++m)
                total += reinterpret_cast<const float *>(&gv[m])[e] * (p.slope[m] * cospif(t * p.zmul[m]));
            reinterpret_cast<float *>(&ov)[e] = inside ? total * p.inv_clip : 0.0f;
        }
        reinterpret_cast<F *>(p.gx)[i] = ov;
    }
}

static int ste_common(const char *who, const void *x, const void *g, const void *gx, int64_t count, float clip)
{
    if (count < 0) return fail(QNN_ERR_INVALID_ARG, "%s: negative size", who);
    if (!(clip > 0.0f && clip <= 3.0e38f)) return fail(QNN_ERR_INVALID_ARG, "%s: clip must be positive and finite", who);
    if (count == 0) return QNN_OK;
    if (!x || !g || !gx) return fail(QNN_ERR_INVALID_ARG, "%s: NULL pointer", who);
    if (!aligned16(x) || !aligned16(g) || !aligned16(gx))
        return fail(QNN_ERR_ALIGNMENT, "%s: pointers must be 16-byte aligned", who);
    return QNN_OK;
}

static dim3 ste_grid(int64_t work)
{
    const int64_t blocks = ceil_div(work, 256);
    return dim3((unsigned)(blocks < 256 * 32 ? blocks : 256 * 32));
}

template <int BITS> static void launch_encoder_backward(const SteParams &p, hipStream_t st)
{
    if (p.count % 4 == 0) hipLaunchKernelGGL((encoder_backward_kernel<BITS, 4>), ste_grid(p.count / 4), dim3(256), 0, st, p);
    else hipLaunchKernelGGL((encoder_backward_kernel<BITS, 1>), ste_grid(p.count), dim3(256), 0, st, p);
}

} // namespace qnn

using namespace qnn;

extern "C" int qnn_quantize_ste_backward(const float *x, const float *grad_q, int64_t count, float clip, float *grad_x,
                                         void *stream)
{
    const int rc = ste_common("qnn_quantize_ste_backward", x, grad_q, grad_x, count, clip);
    if (rc != QNN_OK || count == 0) return rc;
    SteParams p = {};
    p.x = x, p.g = grad_q, p.gx = grad_x, p.count = count, p.inv_clip = 1.0f / clip;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (count % 4 == 0) hipLaunchKernelGGL(quantize_ste_backward_kernel<4>, ste_grid(count / 4), dim3(256), 0, st, p);
    else hipLaunchKernelGGL(quantize_ste_backward_kernel<1>, ste_grid(count), dim3(256), 0, st, p);
    return check_launch("qnn_quantize_ste_backward");
}

extern "C" int qnn_encoder_backward(const float *x, const float *grad_planes, int64_t count, float clip, int bits,
                                    float *grad_x, void *stream)
{
    if (bits < 1 || bits > 8) return fail(QNN_ERR_INVALID_ARG, "qnn_encoder_backward: bits=%d outside [1,8]", bits);
    const int rc = ste_common("qnn_encoder_backward", x, grad_planes, grad_x, count, clip);
    if (rc != QNN_OK || count == 0) return rc;
    if (count > INT64_MAX / (8 * 4)) return fail(QNN_ERR_RANGE, "qnn_encoder_backward: size too large");
    SteParams p = {};
    p.x = x, p.g = grad_planes, p.gx = grad_x, p.count = count, p.inv_clip = 1.0f / clip;
    const double K = (double)((1 << bits) - 1);
    for (int m = 1; m <= bits; ++m) {
        p.zmul[m - 1] = (float)(K / (double)(1 << m));
        p.slope[m - 1] = (float)((m == bits ? 1.0 : -1.0) * 3.14159265358979323846 * K / (double)(1 << m));
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    switch (bits) {
    case 1: launch_encoder_backward<1>(p, st); break;
    case 2: launch_encoder_backward<2>(p, st); break;
    case 3: launch_encoder_backward<3>(p, st); break;
    case 4: launch_encoder_backward<4>(p, st); break;
    case 5: launch_encoder_backward<5>(p, st); break;
    case 6: launch_encoder_backward<6>(p, st); break;
    case 7: launch_encoder_backward<7>(p, st); break;
    default: launch_encoder_backward<8>(p, st); break;
    }
    return check_launch("qnn_encoder_backward");
}
