// qnn_dequant_scale: the decoder's scale factor (paper: section "M-bit Encoding Functions", the
// 1/alpha^2 factor shown as 1/9 in Fig. 1; Eq. 18), one fp32 factor per output channel.
// Pure streaming: 4 bytes read and 4 bytes written per output, 16-byte accesses where the row
// length allows.
#include "qnn_host.h"

namespace qnn {

__global__ __launch_bounds__(256) void dequant_scale_vec4_kernel(const int4 *__restrict__ acc,
                                                                 const float4 *__restrict__ scale,
                                                                 int64_t total4, int64_t cols4,
                                                                 float4 *__restrict__ out)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total4; i += stride) {
        const int4 a = acc[i];
        const float4 s = scale[i % cols4];
        float4 o;
        o.x = (float)a.x * s.x;
        o.y = (float)a.y * s.y;
        o.z = (float)a.z * s.z;
        o.w = (float)a.w * s.w;
        out[i] = o;
    }
}

__global__ __launch_bounds__(256) void dequant_scale_kernel(const int32_t *__restrict__ acc,
                                                            const float *__restrict__ scale,
                                                            int64_t total, int64_t cols,
                                                            float *__restrict__ out)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride)
        out[i] = (float)acc[i] * scale[i % cols];
}

} // namespace qnn

using namespace qnn;

extern "C" int qnn_dequant_scale(const int32_t *acc, const float *scale, int64_t rows, int64_t cols,
                                 float *out, void *stream)
{
    if (rows < 0 || cols < 0) return fail(QNN_ERR_INVALID_ARG, "qnn_dequant_scale: negative size");
    if (rows == 0 || cols == 0) return QNN_OK;
    if (!acc || !scale || !out) return fail(QNN_ERR_INVALID_ARG, "qnn_dequant_scale: NULL pointer");
    if (!aligned16(acc) || !aligned16(out))
        return fail(QNN_ERR_ALIGNMENT, "qnn_dequant_scale: acc and out must be 16-byte aligned");
    if (rows > INT64_MAX / cols) return fail(QNN_ERR_RANGE, "qnn_dequant_scale: rows*cols too large");
    const int64_t total = rows * cols;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t max_blocks = 256 * 16;
    if (cols % 4 == 0 && aligned16(scale)) {
        const int64_t total4 = total / 4;
        const int64_t blocks = ceil_div(total4, 256);
        hipLaunchKernelGGL(dequant_scale_vec4_kernel, dim3((unsigned)(blocks < max_blocks ? blocks : max_blocks)),
                           dim3(256), 0, st, reinterpret_cast<const int4 *>(acc),
                           reinterpret_cast<const float4 *>(scale), total4, cols / 4,
                           reinterpret_cast<float4 *>(out));
    } else {
        const int64_t blocks = ceil_div(total, 256);
        hipLaunchKernelGGL(dequant_scale_kernel, dim3((unsigned)(blocks < max_blocks ? blocks : max_blocks)),
                           dim3(256), 0, st, acc, scale, total, cols, out);
    }
    return check_launch("qnn_dequant_scale");
}
