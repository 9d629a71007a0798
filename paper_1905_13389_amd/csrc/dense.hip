// The unquantized ends of a network around the quantized trunk (the ResNet-18 workload keeps its first
// convolution and its classifier in full precision): a dense fp32 convolution whose epilogue can hand the
// next -- first quantized -- layer its bit planes, global average pooling, and a dense fp32 fully
// connected layer.  fp32 products and sums on the matrix cores (v_mfma_f32_32x32x2_f32); not part of the
// xor + bitcount path.
//
// dense_conv_kernel: implicit GEMM, rows = output pixels, columns = output channels, reduction axis
// k = (ky, kx, ci).  A workgroup of 4 waves owns 64 pixels x 64 channels, one 32 x 32 MFMA tile per wave.
// The reduction runs in chunks of up to kChunk values: the 64 pixel rows and the 64 weight rows of a chunk
// are staged in LDS with an odd row stride, so that the 32 rows a half-wave reads for one MFMA operand
// fall into 32 different banks; two workgroups fit a CU and cover each other's staging phases.
#include "qnn_host.h"
#include "quantize.h"
#include "fastdiv.h"

namespace qnn {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kDenseThreads = 256;
constexpr int kDenseTile = 64;             // pixels and channels per workgroup
constexpr int kChunk = 152;                // reduction values per LDS stage (even)
constexpr int kChunkStride = kChunk + 1;   // odd: conflict-free operand reads
static_assert(kChunk % 2 == 0 && 2 * kDenseTile * kChunkStride * 4 <= 80 * 1024, "two workgroups per CU");

struct DenseConvParams {
    const float *x, *w, *scale, *shift;
    float *out;
    uint32_t *next;
    int H, W, Cin, Cout, kh, kw, stride, pad, Ho, Wo;
    int64_t M; // output pixels
    int K;     // kh kw Cin
    int relu, next_bits, next_top, cwo;
    float next_inv_clip, next_half_top;
    FastDiv div_howo, div_wo;
};

__global__ __launch_bounds__(kDenseThreads) void dense_conv_kernel(DenseConvParams p)
{
    __shared__ float As[kDenseTile * kChunkStride];
    __shared__ float Ws[kDenseTile * kChunkStride];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row0 = (int64_t)blockIdx.x * kDenseTile;
    const int col0 = (int)blockIdx.y * kDenseTile;

    // staging: thread -> row tid / 4 of the tile (a pixel for A, a channel for W), every 4th reduction value
    const int srow = tid >> 2, sub = tid & 3;
    const int64_t m = row0 + srow;
    const bool pix_ok = m < p.M;
    int hi0 = 0, wi0 = 0;
    const float *xb = p.x;
    if (pix_ok) {
        const uint32_t mm = (uint32_t)m;
        const uint32_t b = fdiv(mm, p.div_howo), rem = mm - b * p.div_howo.d;
        const uint32_t ho = fdiv(rem, p.div_wo), wo = rem - ho * p.div_wo.d;
        hi0 = (int)ho * p.stride - p.pad, wi0 = (int)wo * p.stride - p.pad;
        xb = p.x + (int64_t)b * p.H * p.W * p.Cin;
    }
    const bool ch_ok = col0 + srow < p.Cout;
    const float *wb = p.w + (int64_t)(ch_ok ? col0 + srow : 0) * p.K;

    // (ky, kx, ci) of this thread's next reduction value, advanced by 4 per step
    int ci = sub, kx = 0, ky = 0;
    auto normalize = [&]() {
        while (ci >= p.Cin) {
            ci -= p.Cin;
            if (++kx == p.kw) kx = 0, ++ky;
        }
    };
    normalize();

    v16f acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
    const int arow = 32 * (wave & 1) + (lane & 31), brow = 32 * (wave >> 1) + (lane & 31), khalf = lane >> 5;

    for (int k0 = 0; k0 < p.K; k0 += kChunk) {
        const int kc = p.K - k0 < kChunk ? p.K - k0 : kChunk;
        const int kc2 = (kc + 1) & ~1; // MFMA steps take two values; an odd tail reads one staged zero
        for (int kk = sub; kk < kc2; kk += 4) {
            float xv = 0.0f, wv = 0.0f;
            if (kk < kc) {
                const int y = hi0 + ky, xx = wi0 + kx;
                if (pix_ok && (unsigned)y < (unsigned)p.H && (unsigned)xx < (unsigned)p.W)
                    xv = xb[((int64_t)y * p.W + xx) * p.Cin + ci];
                if (ch_ok) wv = wb[k0 + kk];
                ci += 4;
                normalize();
            }
            As[srow * kChunkStride + kk] = xv;
            Ws[srow * kChunkStride + kk] = wv;
        }
        __syncthreads();
        const float *ap = As + arow * kChunkStride + khalf, *bp = Ws + brow * kChunkStride + khalf;
#pragma unroll 8
        for (int s = 0; s < kc2; s += 2) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(ap[s], bp[s], acc, 0, 0, 0);
        __syncthreads();
    }

    // D layout of the 32 x 32 tile: this lane holds channel lane % 32 of the pixels 8 (r / 4) + 4 (lane / 32) + r % 4
    const int c = col0 + 32 * (wave >> 1) + (lane & 31);
    const bool c_ok = c < p.Cout;
    const float sc = p.scale && c_ok ? p.scale[c] : 1.0f, sh = p.shift && c_ok ? p.shift[c] : 0.0f;
    const int wword = (col0 >> 5) + (wave >> 1);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int64_t pix = row0 + 32 * (wave & 1) + 8 * (r >> 2) + 4 * khalf + (r & 3);
        const bool ok = pix < p.M && c_ok;
        float y = acc[r];
        if (p.scale) y = y * sc;
        if (p.shift) y = y + sh;
        if (p.relu) y = fmaxf(y, 0.0f);
        if (p.out && ok) p.out[pix * p.Cout + c] = y;
        if (p.next) {
            const int code = ok ? quantize_code(y, p.next_inv_clip, p.next_half_top, p.next_top) : 0;
            for (int j = 0; j < p.next_bits; ++j) {
                // the 32 lanes of a half-wave hold the 32 channels of one plane word
                const unsigned long long bits = __ballot((code >> j) & 1);
                if ((lane & 31) == 0 && pix < p.M && wword < p.cwo)
                    p.next[((int64_t)j * p.M + pix) * p.cwo + wword] = (uint32_t)(bits >> (32 * khalf));
            }
        }
    }
}

// out[b][c] = (sum over the hw positions of x[b][.][c]) / hw, summed in position order; one lane per (b, c)
__global__ __launch_bounds__(256) void global_avgpool_kernel(const float *__restrict__ x, int64_t B, int64_t hw, int64_t C,
                                                             float inv_hw, float *__restrict__ out)
{
    const int64_t total = B * C, stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride) {
        const int64_t b = idx / C, c = idx % C;
        const float *src = x + b * hw * C + c;
        float s = 0.0f;
        for (int64_t i = 0; i < hw; ++i) s = s + src[i * C];
        out[idx] = s * inv_hw;
    }
}

static int dense_conv_run(const char *who, const qnn_dense_conv_desc *d, const float *x, const float *w, const float *scale,
                          const float *shift, int relu, float *out, uint32_t *next_planes, float next_clip, int next_bits,
                          void *stream)
{
    if (!d) return fail(QNN_ERR_INVALID_ARG, "%s: NULL descriptor", who);
    if (d->B < 0 || d->H <= 0 || d->W <= 0 || d->Cin <= 0 || d->Cout <= 0 || d->kh <= 0 || d->kw <= 0 || d->stride <= 0 ||
        d->pad < 0)
        return fail(QNN_ERR_INVALID_ARG, "%s: sizes must be positive (pad >= 0)", who);
    if (d->H + 2 * (int64_t)d->pad < d->kh || d->W + 2 * (int64_t)d->pad < d->kw)
        return fail(QNN_ERR_INVALID_ARG, "%s: kernel larger than the padded image", who);
    if (d->B == 0) return QNN_OK; // nothing to compute: the (empty) buffers may be NULL
    if (!out && !next_planes) return fail(QNN_ERR_INVALID_ARG, "%s: out and next_planes are both NULL", who);
    if (next_planes && (next_bits < 1 || next_bits > 8 || !(next_clip > 0.0f) || next_clip > 3.0e38f))
        return fail(QNN_ERR_INVALID_ARG, "%s: next_bits in [1,8] and a finite next_clip > 0 are required with next_planes", who);
    if (!x || !w) return fail(QNN_ERR_INVALID_ARG, "%s: NULL input pointer", who);
    if (!aligned16(x) || !aligned16(w) || !aligned16(out) || !aligned16(next_planes))
        return fail(QNN_ERR_ALIGNMENT, "%s: pointers must be 16-byte aligned", who);
    const int64_t Ho = (d->H + 2 * d->pad - d->kh) / d->stride + 1, Wo = (d->W + 2 * d->pad - d->kw) / d->stride + 1;
    const int64_t M = d->B * Ho * Wo, K = (int64_t)d->kh * d->kw * d->Cin;
    if (M >= (1LL << 31) || K >= (1LL << 24) || d->Cout >= (1LL << 24) || d->H >= (1LL << 24) || d->W >= (1LL << 24) ||
        ceil_div(d->Cout, kDenseTile) > 65535)
        return fail(QNN_ERR_RANGE, "%s: tensor too large", who);
    DenseConvParams p;
    p.x = x, p.w = w, p.scale = scale, p.shift = shift, p.out = out, p.next = next_planes;
    p.H = (int)d->H, p.W = (int)d->W, p.Cin = (int)d->Cin, p.Cout = (int)d->Cout;
    p.kh = d->kh, p.kw = d->kw, p.stride = d->stride, p.pad = d->pad, p.Ho = (int)Ho, p.Wo = (int)Wo;
    p.M = M, p.K = (int)K, p.relu = relu ? 1 : 0;
    p.next_bits = next_planes ? next_bits : 0;
    p.next_top = (1 << p.next_bits) - 1;
    p.cwo = (int)ceil_div(d->Cout, 32);
    p.next_inv_clip = next_planes ? 1.0f / next_clip : 0.0f;
    p.next_half_top = 0.5f * (float)p.next_top;
    p.div_howo = make_fastdiv((uint32_t)(Ho * Wo)), p.div_wo = make_fastdiv((uint32_t)Wo);
    const dim3 grid((unsigned)ceil_div(M, kDenseTile), (unsigned)ceil_div(d->Cout, kDenseTile));
    hipLaunchKernelGGL(dense_conv_kernel, grid, dim3(kDenseThreads), 0, static_cast<hipStream_t>(stream), p);
    return check_launch(who);
}

} // namespace qnn

using namespace qnn;

extern "C" int qnn_dense_conv2d_f32(const qnn_dense_conv_desc *d, const float *x, const float *w, const float *scale,
                                    const float *shift, int relu, float *out, uint32_t *next_planes, float next_clip,
                                    int next_bits, void *stream)
{
    return dense_conv_run("qnn_dense_conv2d_f32", d, x, w, scale, shift, relu, out, next_planes, next_clip, next_bits, stream);
}

extern "C" int qnn_dense_fc_f32(const float *x, const float *w, const float *bias, int64_t rows, int64_t cols, int64_t n,
                                float *out, void *stream)
{
    if (rows < 0 || cols <= 0 || n <= 0) return fail(QNN_ERR_INVALID_ARG, "qnn_dense_fc_f32: rows >= 0, cols > 0, n > 0");
    if (!out) return fail(QNN_ERR_INVALID_ARG, "qnn_dense_fc_f32: NULL output");
    // a 1 x 1 convolution over 1 x 1 images: pixels = rows, channels = n -> cols
    const qnn_dense_conv_desc d = {rows, 1, 1, n, cols, 1, 1, 1, 0};
    return dense_conv_run("qnn_dense_fc_f32", &d, x, w, nullptr, bias, 0, out, nullptr, 0.0f, 0, stream);
}

extern "C" int qnn_global_avgpool_f32(const float *x, int64_t B, int64_t hw, int64_t C, float *out, void *stream)
{
    if (B < 0 || hw <= 0 || C <= 0) return fail(QNN_ERR_INVALID_ARG, "qnn_global_avgpool_f32: B >= 0, hw > 0, C > 0");
    if (B == 0) return QNN_OK;
    if (!x || !out) return fail(QNN_ERR_INVALID_ARG, "qnn_global_avgpool_f32: NULL pointer");
    if (B > (INT64_MAX >> 8) / C / hw) return fail(QNN_ERR_RANGE, "qnn_global_avgpool_f32: tensor too large");
    const int64_t blocks = ceil_div(B * C, 256);
    const dim3 grid((unsigned)(blocks < 65536 ? blocks : 65536));
    hipLaunchKernelGGL(global_avgpool_kernel, grid, dim3(256), 0, static_cast<hipStream_t>(stream), x, B, hw, C,
                       1.0f / (float)hw, out);
    return check_launch("qnn_global_avgpool_f32");
}
