// qnn_encode_pack: range limit + linear quantizer + plane split + bit-vector packing
// (paper: Table 1 HTanh, Eq. 15, Eq. 10, Table 2; "stored by bit vectors", Introduction).
//
// One wave64 turns 256 consecutive reduction elements into 8 words per plane.  In pass e (0..3)
// lane l reads element 64 e + l (a fully coalesced 256-byte row of fp32), computes its code u,
// and for every plane j a wave ballot of bit j of u yields the two words 2e and 2e+1 of that
// plane directly: bit t of a word is element 32 k + t, the layout the GEMM reads.  Lanes 0..7
// then store the 8 words of each plane as one 32-byte row.
#include "qnn_host.h"
#include "quantize.h"

namespace qnn {

struct EncodeParams {
    const void *src;
    int64_t rows, n, row_stride, nw;
    float inv_clip, half_top; // 1/clip and (2^bits - 1)/2
    int top;                  // 2^bits - 1
    uint32_t *planes;         // [bits][rows][nw]
    int64_t chunks_per_row;   // ceil(nw / 8)
};

__device__ __forceinline__ float widen(float v) { return v; }
__device__ __forceinline__ float widen(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

template <typename T> __device__ __forceinline__ int code_of(T v, const EncodeParams &p)
{
    return quantize_code(widen(v), p.inv_clip, p.half_top, p.top);
}
// int8 levels: u = (v + top) / 2, no floating point
template <> __device__ __forceinline__ int code_of<int8_t>(int8_t v, const EncodeParams &p)
{
    return ((int)v + p.top) >> 1;
}

template <typename T, int BITS>
__global__ __launch_bounds__(256) void encode_pack_kernel(EncodeParams p)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    const int64_t total = p.rows * p.chunks_per_row;
    const T *src = static_cast<const T *>(p.src);

    for (int64_t chunk = wave; chunk < total; chunk += nwaves) {
        const int64_t row = chunk / p.chunks_per_row;
        const int64_t c = chunk % p.chunks_per_row;
        const int64_t e0 = c * 256;
        const T *rp = src + row * p.row_stride;

        int u[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int64_t idx = e0 + 64 * e + lane;
            u[e] = idx < p.n ? code_of<T>(rp[idx], p) : 0; // pad bits are 0 in every plane
        }
        uint32_t word[BITS];
#pragma unroll
        for (int j = 0; j < BITS; ++j) word[j] = 0u;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
#pragma unroll
            for (int j = 0; j < BITS; ++j) {
                const uint64_t m = __ballot((u[e] >> j) & 1);
                if (lane == 2 * e) word[j] = (uint32_t)m;
                if (lane == 2 * e + 1) word[j] = (uint32_t)(m >> 32);
            }
        }
        const int64_t k = c * 8 + lane;
        if (lane < 8 && k < p.nw) {
#pragma unroll
            for (int j = 0; j < BITS; ++j) p.planes[((int64_t)j * p.rows + row) * p.nw + k] = word[j];
        }
    }
}

// Streaming variant for one long contiguous bit-vector (n a multiple of 32, 16-byte aligned
// source): lane l of a wave loads elements 4l..4l+3 of a 256-element chunk with one vector load,
// UNROLL chunks in flight per lane.  The 4 plane bits of a lane form a nibble; the 8 lanes that
// share a 32-element word OR their shifted nibbles together with three DPP steps and lane 8k
// stores word k.  The codes are the same quantize_code / level arithmetic as above.
__device__ __forceinline__ uint32_t or_reduce8_lanes(uint32_t v)
{
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true);  // quad_perm [1,0,3,2]
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true);  // quad_perm [2,3,0,1]
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, true); // row_half_mirror
    return v;
}

template <typename T> struct Vec4;
template <> struct Vec4<float> { using type = float4; };
template <> struct Vec4<uint16_t> { using type = ushort4; };
template <> struct Vec4<int8_t> { using type = char4; };

template <typename T, int BITS, int UNROLL>
__global__ __launch_bounds__(256) void encode_pack_stream_kernel(EncodeParams p)
{
    using V = typename Vec4<T>::type;
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    const int64_t chunks = p.chunks_per_row; // 256-element chunks of the single row
    const V *src = static_cast<const V *>(p.src);
    const int shift = 4 * (lane & 7);

    for (int64_t c0 = wave * UNROLL; c0 < chunks; c0 += nwaves * UNROLL) {
        V v[UNROLL];
        bool ok[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int64_t e = (c0 + u) * 256 + 4 * lane;
            ok[u] = c0 + u < chunks && e < p.n;
            if (ok[u]) v[u] = src[(c0 + u) * 64 + lane];
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            uint32_t cw4 = 0; // four byte codes; elements past the end give 0 bits
            if (ok[u]) {
                cw4 = (uint32_t)code_of<T>(v[u].x, p) | ((uint32_t)code_of<T>(v[u].y, p) << 8) |
                      ((uint32_t)code_of<T>(v[u].z, p) << 16) | ((uint32_t)code_of<T>(v[u].w, p) << 24);
            }
            const int64_t k = (c0 + u) * 8 + (lane >> 3);
#pragma unroll
            for (int j = 0; j < BITS; ++j) {
                const uint32_t x = (cw4 >> j) & 0x01010101u;
                const uint32_t word = or_reduce8_lanes((((x * 0x00204081u) >> 21) & 15u) << shift);
                if ((lane & 7) == 0 && c0 + u < chunks && k < p.nw) p.planes[(int64_t)j * p.nw + k] = word;
            }
        }
    }
}

template <typename T, int BITS> static void launch_stream(const EncodeParams &p, hipStream_t st)
{
    constexpr int UNROLL = 4;
    const int64_t waves = ceil_div(p.chunks_per_row, UNROLL);
    const int64_t blocks = ceil_div(waves, 4);
    const unsigned grid = (unsigned)(blocks < 256 * 16 ? blocks : 256 * 16);
    hipLaunchKernelGGL((encode_pack_stream_kernel<T, BITS, UNROLL>), dim3(grid), dim3(256), 0, st, p);
}

template <typename T> static void launch_stream_bits(const EncodeParams &p, int bits, hipStream_t st)
{
    switch (bits) {
    case 1: launch_stream<T, 1>(p, st); break;
    case 2: launch_stream<T, 2>(p, st); break;
    case 3: launch_stream<T, 3>(p, st); break;
    case 4: launch_stream<T, 4>(p, st); break;
    case 5: launch_stream<T, 5>(p, st); break;
    case 6: launch_stream<T, 6>(p, st); break;
    case 7: launch_stream<T, 7>(p, st); break;
    default: launch_stream<T, 8>(p, st); break;
    }
}

template <typename T> static void launch_bits(const EncodeParams &p, int bits, unsigned grid, hipStream_t st)
{
    switch (bits) {
    case 1: hipLaunchKernelGGL((encode_pack_kernel<T, 1>), dim3(grid), dim3(256), 0, st, p); break;
    case 2: hipLaunchKernelGGL((encode_pack_kernel<T, 2>), dim3(grid), dim3(256), 0, st, p); break;
    case 3: hipLaunchKernelGGL((encode_pack_kernel<T, 3>), dim3(grid), dim3(256), 0, st, p); break;
    case 4: hipLaunchKernelGGL((encode_pack_kernel<T, 4>), dim3(grid), dim3(256), 0, st, p); break;
    case 5: hipLaunchKernelGGL((encode_pack_kernel<T, 5>), dim3(grid), dim3(256), 0, st, p); break;
    case 6: hipLaunchKernelGGL((encode_pack_kernel<T, 6>), dim3(grid), dim3(256), 0, st, p); break;
    case 7: hipLaunchKernelGGL((encode_pack_kernel<T, 7>), dim3(grid), dim3(256), 0, st, p); break;
    default: hipLaunchKernelGGL((encode_pack_kernel<T, 8>), dim3(grid), dim3(256), 0, st, p); break;
    }
}

} // namespace qnn

using namespace qnn;

extern "C" int qnn_encode_pack(const void *src, int dtype, int64_t rows, int64_t n,
                               int64_t row_stride_elems, float clip, int bits, uint32_t *planes,
                               void *stream)
{
    if (dtype != QNN_DTYPE_F32 && dtype != QNN_DTYPE_BF16 && dtype != QNN_DTYPE_I8)
        return fail(QNN_ERR_UNSUPPORTED, "qnn_encode_pack: unknown dtype %d", dtype);
    if (bits < 1 || bits > 8) return fail(QNN_ERR_INVALID_ARG, "qnn_encode_pack: bits=%d outside [1,8]", bits);
    if (dtype == QNN_DTYPE_I8 && bits > 7)
        return fail(QNN_ERR_UNSUPPORTED, "qnn_encode_pack: int8 levels hold at most 7 bits");
    if (rows < 0 || n < 0) return fail(QNN_ERR_INVALID_ARG, "qnn_encode_pack: negative size");
    if (rows > 1 && row_stride_elems < n)
        return fail(QNN_ERR_INVALID_ARG, "qnn_encode_pack: row_stride_elems=%lld < n=%lld",
                    (long long)row_stride_elems, (long long)n);
    if (dtype != QNN_DTYPE_I8 && !(clip > 0.0f && clip <= 3.0e38f))
        return fail(QNN_ERR_INVALID_ARG, "qnn_encode_pack: clip must be positive and finite");
    if (rows == 0 || n == 0) return QNN_OK;
    if (!src || !planes) return fail(QNN_ERR_INVALID_ARG, "qnn_encode_pack: NULL pointer");
    if (!aligned16(planes)) return fail(QNN_ERR_ALIGNMENT, "qnn_encode_pack: planes must be 16-byte aligned");

    EncodeParams p;
    p.src = src;
    p.rows = rows;
    p.n = n;
    p.row_stride = row_stride_elems;
    // rows that are whole words long and contiguous form one long bit-vector per plane: treat
    // the tensor as a single row so that short rows (a pixel's channels) still fill whole waves
    bool single_row = false;
    if (n % 32 == 0 && (rows == 1 || row_stride_elems == n)) {
        p.rows = 1;
        p.n = rows * n;
        p.row_stride = p.n;
        single_row = true;
    }
    p.nw = ceil_div(p.n, 32);
    p.top = (1 << bits) - 1;
    p.half_top = (float)p.top * 0.5f;
    p.inv_clip = dtype == QNN_DTYPE_I8 ? 1.0f : 1.0f / clip;
    p.planes = planes;
    p.chunks_per_row = ceil_div(p.nw, 8);

    const int64_t chunks = p.rows * p.chunks_per_row;
    const int64_t blocks = ceil_div(chunks, 4); // 4 waves per workgroup
    const unsigned grid = (unsigned)(blocks < 256 * 32 ? blocks : 256 * 32);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (single_row && aligned16(src)) { // vector loads of 4 elements are whole and aligned
        switch (dtype) {
        case QNN_DTYPE_F32: launch_stream_bits<float>(p, bits, st); break;
        case QNN_DTYPE_BF16: launch_stream_bits<uint16_t>(p, bits, st); break;
        default: launch_stream_bits<int8_t>(p, bits, st); break;
        }
        return check_launch("qnn_encode_pack");
    }
    switch (dtype) {
    case QNN_DTYPE_F32: launch_bits<float>(p, bits, grid, st); break;
    case QNN_DTYPE_BF16: launch_bits<uint16_t>(p, bits, grid, st); break;
    default: launch_bits<int8_t>(p, bits, grid, st); break;
    }
    return check_launch("qnn_encode_pack");
}
