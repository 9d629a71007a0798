// qnn_fc_fused: a small quantized fully connected layer in one launch -- the encoders (Table 1, Eq. 15,
// Eq. 10), the M x K xor + bitcount branches and their recombination (Eq. 9) and the scale -- for layers
// with far too little work to fill the chip (the 64 x 512 -> 256 layer of the smallest configuration is
// 0.04 us of VALU work), where the time of qnn_encode_pack + qnn_binary_gemm is the device's latency
// from one dependent kernel to the next.  The activation planes never leave LDS.
//
// A workgroup owns kFcRows activation rows and 256 output columns.  Phase 1: wave i encodes row i, 64
// elements per pass; a ballot of bit j of the codes is two words of plane j.  Phase 2: thread t owns
// column t and streams that column's weight words once, for all kFcRows rows:
// S[i] += bitcount(w xor a_i) << (jw + ja), acc = n top_w top_a - 2 S.
#include "qnn_host.h"
#include "quantize.h"

namespace qnn {

constexpr int kFcRows = 4;         // activation rows per workgroup (one per wave)
constexpr int kFcPlaneWords = 4096; // LDS words for [a_bits][kFcRows][nw]

struct FcParams {
    const void *src;
    int64_t rows, n, row_stride, nw, cols;
    float inv_clip, half_top;
    int top, a_bits, w_bits;
    const uint32_t *w; // [w_bits][cols][nw]
    const float *scale;
    int32_t *acc;
    float *out;
    uint32_t n_times_top;
};

__device__ __forceinline__ int fc_code(float v, const FcParams &p) { return quantize_code(v, p.inv_clip, p.half_top, p.top); }
__device__ __forceinline__ int fc_code(uint16_t v, const FcParams &p)
{
    return quantize_code(__uint_as_float((uint32_t)v << 16), p.inv_clip, p.half_top, p.top);
}
__device__ __forceinline__ int fc_code(int8_t v, const FcParams &p) { return ((int)v + p.top) >> 1; } // levels: u = (v + top) / 2

template <typename T> __global__ __launch_bounds__(64 * kFcRows) void fc_fused_kernel(FcParams p)
{
    __shared__ uint32_t planes[kFcPlaneWords];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nw = (int)p.nw;
    const int64_t row0 = (int64_t)blockIdx.x * kFcRows;

    // phase 1: this wave's row -> planes[(j * kFcRows + wave) * nw + k]; words past the row's end and rows past
    // the last one are 0 (pad bits are 0 in both operands, so they add nothing to the xor)
    const int64_t r = row0 + wave;
    const T *rp = static_cast<const T *>(p.src) + (r < p.rows ? r : 0) * p.row_stride;
    for (int k0 = 0; k0 < nw; k0 += 2) {
        const int64_t idx = (int64_t)k0 * 32 + lane;
        const int u = r < p.rows && idx < p.n ? fc_code(rp[idx], p) : 0;
        for (int j = 0; j < p.a_bits; ++j) {
            const unsigned long long m = __ballot((u >> j) & 1);
            uint32_t *dst = planes + (j * kFcRows + wave) * nw + k0;
            if (lane == 0) dst[0] = (uint32_t)m;
            if (lane == 1 && k0 + 1 < nw) dst[1] = (uint32_t)(m >> 32);
        }
    }
    __syncthreads();

    // phase 2
    const int64_t c = (int64_t)blockIdx.y * blockDim.x + tid;
    if (c >= p.cols) return;
    uint32_t S[kFcRows];
#pragma unroll
    for (int i = 0; i < kFcRows; ++i) S[i] = 0u;
    for (int jw = 0; jw < p.w_bits; ++jw) {
        const uint32_t *wrow = p.w + ((int64_t)jw * p.cols + c) * nw;
        for (int k = 0; k < nw; ++k) {
            const uint32_t wv = wrow[k];
            for (int ja = 0; ja < p.a_bits; ++ja) {
#pragma unroll
                for (int i = 0; i < kFcRows; ++i)
                    S[i] += (uint32_t)__builtin_popcount(wv ^ planes[(ja * kFcRows + i) * nw + k]) << (jw + ja);
            }
        }
    }
    const float sc = p.out ? p.scale[c] : 0.0f;
#pragma unroll
    for (int i = 0; i < kFcRows; ++i) {
        if (row0 + i >= p.rows) break;
        const int32_t v = (int32_t)(p.n_times_top - 2u * S[i]);
        const int64_t o = (row0 + i) * p.cols + c;
        if (p.acc) p.acc[o] = v;
        if (p.out) p.out[o] = (float)v * sc;
    }
}

} // namespace qnn

using namespace qnn;

extern "C" int qnn_fc_fused(const void *src, int dtype, int64_t rows, int64_t n, int64_t row_stride_elems, float clip,
                            int a_bits, const uint32_t *w_planes, int w_bits, int64_t cols, const float *scale,
                            int32_t *acc, float *out, void *stream)
{
    if (dtype != QNN_DTYPE_F32 && dtype != QNN_DTYPE_BF16 && dtype != QNN_DTYPE_I8)
        return fail(QNN_ERR_UNSUPPORTED, "qnn_fc_fused: unknown dtype %d", dtype);
    if (a_bits < 1 || a_bits > 8 || w_bits < 1 || w_bits > 8)
        return fail(QNN_ERR_INVALID_ARG, "qnn_fc_fused: bits must be in [1,8] (a_bits=%d, w_bits=%d)", a_bits, w_bits);
    if (dtype == QNN_DTYPE_I8 && a_bits > 7) return fail(QNN_ERR_UNSUPPORTED, "qnn_fc_fused: int8 levels hold at most 7 bits");
    if (rows < 0 || cols < 0 || n < 0 || row_stride_elems < n)
        return fail(QNN_ERR_INVALID_ARG, "qnn_fc_fused: negative size or row stride below n");
    if (dtype != QNN_DTYPE_I8 && !(clip > 0.0f && clip <= 3.0e38f))
        return fail(QNN_ERR_INVALID_ARG, "qnn_fc_fused: clip must be finite and > 0");
    if (!acc && !out) return fail(QNN_ERR_INVALID_ARG, "qnn_fc_fused: acc and out are both NULL");
    if (out && !scale) return fail(QNN_ERR_INVALID_ARG, "qnn_fc_fused: out given without scale");
    if (rows == 0 || cols == 0) return QNN_OK;
    if (n > 0 && (!src || !w_planes)) return fail(QNN_ERR_INVALID_ARG, "qnn_fc_fused: NULL input pointer");
    if (!aligned16(w_planes) || !aligned16(acc) || !aligned16(out))
        return fail(QNN_ERR_ALIGNMENT, "qnn_fc_fused: plane and output pointers must be 16-byte aligned");
    if (!acc_fits_int32(n, w_bits, a_bits))
        return fail(QNN_ERR_RANGE, "qnn_fc_fused: n=%lld with %dx%d bits overflows int32", (long long)n, w_bits, a_bits);
    const int64_t nw = ceil_div(n, 32);
    if ((int64_t)a_bits * kFcRows * nw > kFcPlaneWords)
        return fail(QNN_ERR_UNSUPPORTED, "qnn_fc_fused: a_bits * n above %d: use qnn_encode_pack + qnn_binary_gemm",
                    kFcPlaneWords / kFcRows * 32);
    if (ceil_div(rows, kFcRows) > 0x7fffffffLL || ceil_div(cols, 64 * kFcRows) > 65535 || rows > (INT64_MAX >> 8) / cols)
        return fail(QNN_ERR_RANGE, "qnn_fc_fused: too many rows or columns");
    FcParams p;
    p.src = src, p.rows = rows, p.n = n, p.row_stride = row_stride_elems, p.nw = nw, p.cols = cols;
    p.top = (1 << a_bits) - 1;
    p.inv_clip = dtype == QNN_DTYPE_I8 ? 1.0f : 1.0f / clip;
    p.half_top = 0.5f * (float)p.top;
    p.a_bits = a_bits, p.w_bits = w_bits, p.w = w_planes, p.scale = scale, p.acc = acc, p.out = out;
    p.n_times_top = (uint32_t)(n * ((1 << w_bits) - 1) * ((1 << a_bits) - 1));
    const dim3 grid((unsigned)ceil_div(rows, kFcRows), (unsigned)ceil_div(cols, 64 * kFcRows)), block(64 * kFcRows);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == QNN_DTYPE_F32) hipLaunchKernelGGL(fc_fused_kernel<float>, grid, block, 0, st, p);
    else if (dtype == QNN_DTYPE_BF16) hipLaunchKernelGGL(fc_fused_kernel<uint16_t>, grid, block, 0, st, p);
    else hipLaunchKernelGGL(fc_fused_kernel<int8_t>, grid, block, 0, st, p);
    return check_launch("qnn_fc_fused");
}
