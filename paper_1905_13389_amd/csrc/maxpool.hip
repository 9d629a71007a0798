// Max-pooling of quantized activations between layers, on the packed bit-planes (and on int8 levels
// for the matrix-core route).  The linear quantizer (paper: Table 1 range limit, Eq. 15) is monotone
// non-decreasing, so the maximum of the quantized values over a window is the quantized maximum:
// pooling the codes is exact and the activations never have to be decoded.
//
// Planes: the maximum of two codes held bit-sliced in `bits` words (32 channels at once) is a
// comparison from the top plane down: the first plane where the two differ decides, for that bit
// position, which operand is taken in every plane.  Pure streaming work: every input word is read
// about once (window = stride), bits / 8 bytes per element in and out.
#include "qnn_host.h"

namespace qnn {

struct PoolParams {
    const void *in;
    void *out;
    int64_t in_plane_stride, out_plane_stride; // words per plane (planes) or unused (levels)
    int64_t total;                             // lane work items
    int H, W, cw, Ho, Wo, k, stride, pad;      // cw: words (planes) or 16-byte groups (levels) per pixel
};

// out-of-image window elements (padding, ceil-mode overhang) are ignored
__device__ __forceinline__ bool in_image(int y, int x, const PoolParams &p)
{
    return (unsigned)y < (unsigned)p.H && (unsigned)x < (unsigned)p.W;
}

template <int BITS> __global__ __launch_bounds__(256) void maxpool_planes_kernel(PoolParams p)
{
    const uint32_t *in = static_cast<const uint32_t *>(p.in);
    uint32_t *out = static_cast<uint32_t *>(p.out);
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < p.total; idx += stride) {
        const int c = (int)(idx % p.cw);
        const int64_t pix = idx / p.cw;
        const int ox = (int)(pix % p.Wo);
        const int64_t t = pix / p.Wo;
        const int oy = (int)(t % p.Ho);
        const int64_t b = t / p.Ho;
        uint32_t best[BITS];
        bool have = false;
        for (int ky = 0; ky < p.k; ++ky)
            for (int kx = 0; kx < p.k; ++kx) {
                const int y = oy * p.stride - p.pad + ky, x = ox * p.stride - p.pad + kx;
                if (!in_image(y, x, p)) continue;
                const uint32_t *src = in + ((b * p.H + y) * p.W + x) * p.cw + c;
                uint32_t cur[BITS];
#pragma unroll
                for (int j = 0; j < BITS; ++j) cur[j] = src[j * p.in_plane_stride];
                if (!have) {
#pragma unroll
                    for (int j = 0; j < BITS; ++j) best[j] = cur[j];
                    have = true;
                    continue;
                }
                // take: bit positions where cur > best; undecided: all higher planes equal so far
                uint32_t take = 0u, undecided = ~0u;
#pragma unroll
                for (int j = BITS - 1; j >= 0; --j) {
                    const uint32_t differ = cur[j] ^ best[j];
                    take |= undecided & differ & cur[j];
                    undecided &= ~differ;
                }
#pragma unroll
                for (int j = 0; j < BITS; ++j) best[j] = (best[j] & ~take) | (cur[j] & take);
            }
#pragma unroll
        for (int j = 0; j < BITS; ++j) out[j * p.out_plane_stride + idx] = have ? best[j] : 0u;
    }
}

// signed maximum of the four int8 lanes of two words
__device__ __forceinline__ uint32_t max_i8x4(uint32_t a, uint32_t b)
{
    uint32_t r = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int x = (int)(int8_t)(a >> (8 * i)), y = (int)(int8_t)(b >> (8 * i));
        r |= (uint32_t)((x > y ? x : y) & 0xff) << (8 * i);
    }
    return r;
}

// VEC: 16 channels per lane (C a multiple of 16), else one channel per lane
template <bool VEC> __global__ __launch_bounds__(256) void maxpool_levels_kernel(PoolParams p)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < p.total; idx += stride) {
        const int c = (int)(idx % p.cw);
        const int64_t pix = idx / p.cw;
        const int ox = (int)(pix % p.Wo);
        const int64_t t = pix / p.Wo;
        const int oy = (int)(t % p.Ho);
        const int64_t b = t / p.Ho;
        uint4 best = make_uint4(0x80808080u, 0x80808080u, 0x80808080u, 0x80808080u); // -128 everywhere
        int best1 = -128;
        for (int ky = 0; ky < p.k; ++ky)
            for (int kx = 0; kx < p.k; ++kx) {
                const int y = oy * p.stride - p.pad + ky, x = ox * p.stride - p.pad + kx;
                if (!in_image(y, x, p)) continue;
                const int64_t at = ((b * p.H + y) * p.W + x) * p.cw + c;
                if (VEC) {
                    const uint4 v = static_cast<const uint4 *>(p.in)[at];
                    best.x = max_i8x4(best.x, v.x), best.y = max_i8x4(best.y, v.y);
                    best.z = max_i8x4(best.z, v.z), best.w = max_i8x4(best.w, v.w);
                } else {
                    const int v = static_cast<const int8_t *>(p.in)[at];
                    best1 = v > best1 ? v : best1;
                }
            }
        if (VEC) static_cast<uint4 *>(p.out)[idx] = best;
        else static_cast<int8_t *>(p.out)[idx] = (int8_t)best1;
    }
}

// fp4 levels (two channels per byte; nibble = sign << 3 | magnitude code, 1 = 0b0010, 3 = 0b0101), eight
// nibbles of a word at once.  Bit 0 of a nibble tells 3 from 1 and bit 3 is the sign, so the order
// -3 < -1 < +1 < +3 is the 2-bit key (hi = not sign, lo = bit 0 xor sign), held here as two words with
// one bit per nibble.
constexpr uint32_t kNib = 0x11111111u;

struct Fp4Keys {
    uint32_t hi, lo;
};

__device__ __forceinline__ Fp4Keys fp4_keys(uint32_t w)
{
    const uint32_t s = (w >> 3) & kNib, b = w & kNib;
    return {~s & kNib, (b ^ s) & kNib};
}

__device__ __forceinline__ Fp4Keys fp4_key_max(Fp4Keys a, Fp4Keys b)
{
    const uint32_t gt = (a.hi & ~b.hi) | (~(a.hi ^ b.hi) & a.lo & ~b.lo); // a > b, per nibble
    return {(a.hi & gt) | (b.hi & ~gt), (a.lo & gt) | (b.lo & ~gt)};
}

__device__ __forceinline__ uint32_t fp4_from_keys(Fp4Keys k)
{
    const uint32_t s = ~k.hi & kNib, b = (k.lo ^ s) & kNib;
    return (s << 3) | (b << 2) | ((~b & kNib) << 1) | b;
}

// VEC: 32 channels (16 bytes) per lane (C a multiple of 32), else one byte = 2 channels per lane
template <bool VEC> __global__ __launch_bounds__(256) void maxpool_fp4_kernel(PoolParams p)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < p.total; idx += stride) {
        const int c = (int)(idx % p.cw);
        const int64_t pix = idx / p.cw;
        const int ox = (int)(pix % p.Wo);
        const int64_t t = pix / p.Wo;
        const int oy = (int)(t % p.Ho);
        const int64_t b = t / p.Ho;
        Fp4Keys best[4] = {{0u, 0u}, {0u, 0u}, {0u, 0u}, {0u, 0u}}; // the lowest key: level -3
        for (int ky = 0; ky < p.k; ++ky)
            for (int kx = 0; kx < p.k; ++kx) {
                const int y = oy * p.stride - p.pad + ky, x = ox * p.stride - p.pad + kx;
                if (!in_image(y, x, p)) continue;
                const int64_t at = ((b * p.H + y) * p.W + x) * p.cw + c;
                if (VEC) {
                    const uint4 v = static_cast<const uint4 *>(p.in)[at];
                    best[0] = fp4_key_max(best[0], fp4_keys(v.x)), best[1] = fp4_key_max(best[1], fp4_keys(v.y));
                    best[2] = fp4_key_max(best[2], fp4_keys(v.z)), best[3] = fp4_key_max(best[3], fp4_keys(v.w));
                } else {
                    best[0] = fp4_key_max(best[0], fp4_keys(static_cast<const uint8_t *>(p.in)[at]));
                }
            }
        if (VEC)
            static_cast<uint4 *>(p.out)[idx] = make_uint4(fp4_from_keys(best[0]), fp4_from_keys(best[1]),
                                                          fp4_from_keys(best[2]), fp4_from_keys(best[3]));
        else static_cast<uint8_t *>(p.out)[idx] = (uint8_t)fp4_from_keys(best[0]);
    }
}

static int64_t pool_out(int64_t size, int k, int stride, int pad, int ceil_mode)
{
    const int64_t span = size + 2 * (int64_t)pad - k;
    if (size <= 0 || k < 1 || stride < 1 || pad < 0 || 2 * pad > k || span < 0) return -1;
    if (!ceil_mode) return span / stride + 1;
    int64_t out = ceil_div(span, stride) + 1;
    if ((out - 1) * stride >= size + pad) --out; // the last window must start inside the image or its left padding
    return out;
}

static int pool_common(const char *who, const void *in, const void *out, int64_t B, int64_t H, int64_t W, int64_t C,
                       int k, int stride, int pad, int ceil_mode, int64_t &Ho, int64_t &Wo)
{
    if (B < 0 || H <= 0 || W <= 0 || C <= 0) return fail(QNN_ERR_INVALID_ARG, "%s: bad tensor size", who);
    if (k < 1 || stride < 1 || pad < 0) return fail(QNN_ERR_INVALID_ARG, "%s: bad window geometry", who);
    if (2 * pad > k) return fail(QNN_ERR_INVALID_ARG, "%s: pad must be at most half the window", who);
    if (k > 7) return fail(QNN_ERR_UNSUPPORTED, "%s: window larger than 7x7", who);
    Ho = pool_out(H, k, stride, pad, ceil_mode), Wo = pool_out(W, k, stride, pad, ceil_mode);
    if (Ho < 1 || Wo < 1) return fail(QNN_ERR_INVALID_ARG, "%s: window larger than the padded image", who);
    if (H > (1 << 20) || W > (1 << 20) || C > (1 << 24) || B > (1LL << 40) / (H * W))
        return fail(QNN_ERR_RANGE, "%s: dimension too large", who);
    if (B == 0) return QNN_OK;
    if (!in || !out) return fail(QNN_ERR_INVALID_ARG, "%s: NULL pointer", who);
    if (!aligned16(in) || !aligned16(out)) return fail(QNN_ERR_ALIGNMENT, "%s: pointers must be 16-byte aligned", who);
    return QNN_OK;
}

} // namespace qnn

using namespace qnn;

extern "C" int64_t qnn_pool_out_size(int64_t size, int k, int stride, int pad, int ceil_mode)
{
    return pool_out(size, k, stride, pad, ceil_mode);
}

extern "C" int qnn_maxpool_planes(const uint32_t *planes, int bits, int64_t B, int64_t H, int64_t W, int64_t C, int k,
                                  int stride, int pad, int ceil_mode, uint32_t *out_planes, void *stream)
{
    if (bits < 1 || bits > 8) return fail(QNN_ERR_INVALID_ARG, "qnn_maxpool_planes: bits=%d outside [1,8]", bits);
    int64_t Ho = 0, Wo = 0;
    const int rc = pool_common("qnn_maxpool_planes", planes, out_planes, B, H, W, C, k, stride, pad, ceil_mode, Ho, Wo);
    if (rc != QNN_OK || B == 0) return rc;
    PoolParams p;
    p.in = planes, p.out = out_planes;
    p.H = (int)H, p.W = (int)W, p.cw = (int)ceil_div(C, 32), p.Ho = (int)Ho, p.Wo = (int)Wo;
    p.k = k, p.stride = stride, p.pad = pad;
    p.in_plane_stride = B * H * W * p.cw, p.out_plane_stride = B * Ho * Wo * p.cw;
    p.total = p.out_plane_stride;
    const int64_t blocks = ceil_div(p.total, 256);
    const dim3 grid((unsigned)(blocks < 256 * 64 ? blocks : 256 * 64)), block(256);
    hipStream_t st = static_cast<hipStream_t>(stream);
    switch (bits) {
    case 1: hipLaunchKernelGGL(maxpool_planes_kernel<1>, grid, block, 0, st, p); break;
    case 2: hipLaunchKernelGGL(maxpool_planes_kernel<2>, grid, block, 0, st, p); break;
    case 3: hipLaunchKernelGGL(maxpool_planes_kernel<3>, grid, block, 0, st, p); break;
    case 4: hipLaunchKernelGGL(maxpool_planes_kernel<4>, grid, block, 0, st, p); break;
    case 5: hipLaunchKernelGGL(maxpool_planes_kernel<5>, grid, block, 0, st, p); break;
    case 6: hipLaunchKernelGGL(maxpool_planes_kernel<6>, grid, block, 0, st, p); break;
    case 7: hipLaunchKernelGGL(maxpool_planes_kernel<7>, grid, block, 0, st, p); break;
    default: hipLaunchKernelGGL(maxpool_planes_kernel<8>, grid, block, 0, st, p); break;
    }
    return check_launch("qnn_maxpool_planes");
}

extern "C" int qnn_maxpool_levels_i8(const int8_t *levels, int64_t B, int64_t H, int64_t W, int64_t C, int k, int stride,
                                     int pad, int ceil_mode, int8_t *out_levels, void *stream)
{
    int64_t Ho = 0, Wo = 0;
    const int rc = pool_common("qnn_maxpool_levels_i8", levels, out_levels, B, H, W, C, k, stride, pad, ceil_mode, Ho, Wo);
    if (rc != QNN_OK || B == 0) return rc;
    const bool vec = C % 16 == 0;
    PoolParams p;
    p.in = levels, p.out = out_levels;
    p.H = (int)H, p.W = (int)W, p.cw = (int)(vec ? C / 16 : C), p.Ho = (int)Ho, p.Wo = (int)Wo;
    p.k = k, p.stride = stride, p.pad = pad;
    p.in_plane_stride = p.out_plane_stride = 0;
    p.total = B * Ho * Wo * p.cw;
    const int64_t blocks = ceil_div(p.total, 256);
    const dim3 grid((unsigned)(blocks < 256 * 64 ? blocks : 256 * 64)), block(256);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (vec) hipLaunchKernelGGL(maxpool_levels_kernel<true>, grid, block, 0, st, p);
    else hipLaunchKernelGGL(maxpool_levels_kernel<false>, grid, block, 0, st, p);
    return check_launch("qnn_maxpool_levels_i8");
}

extern "C" int qnn_maxpool_levels_fp4(const uint8_t *levels, int64_t B, int64_t H, int64_t W, int64_t C, int k, int stride,
                                      int pad, int ceil_mode, uint8_t *out_levels, void *stream)
{
    int64_t Ho = 0, Wo = 0;
    const int rc = pool_common("qnn_maxpool_levels_fp4", levels, out_levels, B, H, W, C, k, stride, pad, ceil_mode, Ho, Wo);
    if (rc != QNN_OK) return rc;
    if (C % 2 != 0) return fail(QNN_ERR_UNSUPPORTED, "qnn_maxpool_levels_fp4: odd channel count");
    if (B == 0) return QNN_OK;
    const bool vec = C % 32 == 0;
    PoolParams p;
    p.in = levels, p.out = out_levels;
    p.H = (int)H, p.W = (int)W, p.cw = (int)(vec ? C / 32 : C / 2), p.Ho = (int)Ho, p.Wo = (int)Wo;
    p.k = k, p.stride = stride, p.pad = pad;
    p.in_plane_stride = p.out_plane_stride = 0;
    p.total = B * Ho * Wo * p.cw;
    const int64_t blocks = ceil_div(p.total, 256);
    const dim3 grid((unsigned)(blocks < 256 * 64 ? blocks : 256 * 64)), block(256);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (vec) hipLaunchKernelGGL(maxpool_fp4_kernel<true>, grid, block, 0, st, p);
    else hipLaunchKernelGGL(maxpool_fp4_kernel<false>, grid, block, 0, st, p);
    return check_launch("qnn_maxpool_levels_fp4");
}
