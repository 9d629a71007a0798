// Bit-plane-sum variant of the quantized GEMM on the matrix cores.
//
// The M x K binary branches of the paper (Eq. 9 with the {-1,+1} code of Eq. 10) recombine to the
// integer dot product of the decoded levels.  This file takes the other road to the same
// integers: sum the 2^j-weighted planes back into int8 levels (qnn_plane_sum_i8) and contract
// them with v_mfma_i32_32x32x32_i8 (qnn_level_gemm_i8).  It is NOT the graded xor + bitcount
// path (binary_gemm.hip); it exists to be compared with it, same inputs, same int32 outputs.
#include "qnn_host.h"

namespace qnn {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// ---------------------------------------------------------------------------------------------
// planes [bits][rows][nw] -> int8 levels [rows][nk], nk a multiple of 64 bytes, zero padded.
// One lane makes 16 levels (one 16-byte store) from 16 bits of every plane: a nibble of plane j
// is spread to four 0/1 bytes with one multiply, shifted to bit j of the byte codes u, and
// level = 2u - (2^bits - 1) is taken per byte as a carry-free byte-wise add of the negated top.
// ---------------------------------------------------------------------------------------------
template <int BITS>
__global__ __launch_bounds__(256) void plane_sum_kernel(const uint32_t *__restrict__ planes, int64_t rows,
                                                        int64_t n, int64_t nw, int64_t nk, int8_t *__restrict__ out)
{
    const int64_t groups_per_row = nk / 16;
    const int64_t total = rows * groups_per_row;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    constexpr uint32_t neg_top4 = 0x01010101u * ((256u - ((1u << BITS) - 1u)) & 0xffu); // -(2^BITS - 1) in every byte
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride) {
        const int64_t r = idx / groups_per_row, g = idx % groups_per_row;
        const int64_t word = g >> 1;
        uint32_t half[BITS];
#pragma unroll
        for (int j = 0; j < BITS; ++j)
            half[j] = word < nw ? (planes[((int64_t)j * rows + r) * nw + word] >> (16 * (g & 1))) & 0xffffu : 0u;
        uint32_t o[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            uint32_t u = 0;
#pragma unroll
            for (int j = 0; j < BITS; ++j) {
                const uint32_t nib = (half[j] >> (4 * d)) & 15u;
                u |= ((nib * 0x00204081u) & 0x01010101u) << j;
            }
            const uint32_t u2 = u << 1; // 2u <= 254 stays inside its byte
            uint32_t lv = ((u2 & 0x7f7f7f7fu) + (neg_top4 & 0x7f7f7f7fu)) ^ ((u2 ^ neg_top4) & 0x80808080u);
            // elements past n are 0 (not the level of code 0)
            const int64_t e0 = g * 16 + 4 * d;
            if (e0 + 4 > n) {
                uint32_t keep = 0;
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    if (e0 + b < n) keep |= 0xffu << (8 * b);
                lv &= keep;
            }
            o[d] = lv;
        }
        *reinterpret_cast<uint4 *>(out + r * nk + g * 16) = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

// ---------------------------------------------------------------------------------------------
// int8 GEMM acc[r][c] = sum_k a[r][k] w[c][k] on v_mfma_i32_32x32x32_i8.
// Workgroup: 256 lanes (4 waves as 2 x 2), block tile 256 x 256, each wave 128 x 128 = 4 x 4 MFMA
// tiles (256 accumulator registers), reduction staged 64 bytes per row through LDS (row stride 80
// bytes: conflict-free 16-byte reads), double buffered, one barrier per stage.
// The k order inside an MFMA operand does not matter for a dot product as long as both operands
// use the same assignment, which they do by the symmetry of the instruction.
// ---------------------------------------------------------------------------------------------
constexpr int kMB = 256, kNB = 256, kKB = 64, kRowBytes = 80;

struct LevelGemmParams {
    const int8_t *a, *w; // [rows][nk], [cols][nk]
    int64_t rows, cols, nk;
    int32_t *acc;
    const float *scale;
    float *out;
    int64_t tiles_n, tiles_m;
};

__global__ __launch_bounds__(256) void level_gemm_mfma_kernel(LevelGemmParams p)
{
    __shared__ __attribute__((aligned(16))) uint8_t smem[2][(kMB + kNB) * kRowBytes];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t row0 = ((int64_t)blockIdx.x / p.tiles_n) * kMB;
    const int64_t col0 = ((int64_t)blockIdx.x % p.tiles_n) * kNB;

    v16i acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // stage units: 16 bytes; a stage has (256 + 256) rows x 4 units = 2048 units, 8 per lane
    uint4 ra[4], rb[4];
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = tid + u * 256;
            const int r = idx >> 2, q = idx & 3;
            const int64_t gr = row0 + r, gc = col0 + r;
            ra[u] = gr < p.rows ? *reinterpret_cast<const uint4 *>(p.a + gr * p.nk + k0 + 16 * q)
                                : make_uint4(0u, 0u, 0u, 0u);
            rb[u] = gc < p.cols ? *reinterpret_cast<const uint4 *>(p.w + gc * p.nk + k0 + 16 * q)
                                : make_uint4(0u, 0u, 0u, 0u);
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = tid + u * 256;
            const int r = idx >> 2, q = idx & 3;
            *reinterpret_cast<uint4 *>(&smem[buf][r * kRowBytes + 16 * q]) = ra[u];
            *reinterpret_cast<uint4 *>(&smem[buf][(kMB + r) * kRowBytes + 16 * q]) = rb[u];
        }
    };

    const int64_t nstages = p.nk / kKB;
    if (nstages > 0) {
        fetch(0);
        stash(0);
    }
    __syncthreads();
    for (int64_t s = 0; s < nstages; ++s) {
        const int buf = (int)(s & 1);
        const bool more = s + 1 < nstages;
        if (more) fetch((s + 1) * kKB);
        const uint8_t *As = smem[buf] + (wm * 128 + (lane & 31)) * kRowBytes + (lane >> 5) * 16;
        const uint8_t *Bs = smem[buf] + (kMB + wn * 128 + (lane & 31)) * kRowBytes + (lane >> 5) * 16;
        // Both 32-byte halves of the stage are read into separate registers, the second half while
        // the first half's MFMAs run; the scheduling barriers keep the compiler from sinking the
        // reads next to their uses (which would put an LDS round trip in front of every 4 MFMAs).
        v4i af[2][4], bf[2][4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            af[0][t] = *reinterpret_cast<const v4i *>(As + t * 32 * kRowBytes);
            bf[0][t] = *reinterpret_cast<const v4i *>(Bs + t * 32 * kRowBytes);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            af[1][t] = *reinterpret_cast<const v4i *>(As + t * 32 * kRowBytes + 32);
            bf[1][t] = *reinterpret_cast<const v4i *>(Bs + t * 32 * kRowBytes + 32);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[ks][i], bf[ks][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (more) stash(buf ^ 1);
        __syncthreads();
    }

    // D layout of the 32x32 MFMA: lane holds column lane % 32 and rows 8 (r / 4) + 4 (lane / 32) + r % 4
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t c = col0 + wn * 128 + j * 32 + (lane & 31);
            if (c >= p.cols) continue;
            const float sc = p.out ? p.scale[c] : 0.0f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = row0 + wm * 128 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (row >= p.rows) continue;
                const int32_t v = acc[i][j][r];
                if (p.acc) p.acc[row * p.cols + c] = v;
                if (p.out) p.out[row * p.cols + c] = (float)v * sc;
            }
        }
}

} // namespace qnn

using namespace qnn;

extern "C" int64_t qnn_level_row_bytes(int64_t n) { return n < 0 ? -1 : ceil_div(n, kKB) * kKB; }

extern "C" int qnn_plane_sum_i8(const uint32_t *planes, int bits, int64_t rows, int64_t n, int8_t *levels,
                                void *stream)
{
    if (bits < 1 || bits > 7) return fail(QNN_ERR_UNSUPPORTED, "qnn_plane_sum_i8: int8 levels hold 1..7 bits (got %d)", bits);
    if (rows < 0 || n < 0) return fail(QNN_ERR_INVALID_ARG, "qnn_plane_sum_i8: negative size");
    if (rows == 0 || n == 0) return QNN_OK;
    if (!planes || !levels) return fail(QNN_ERR_INVALID_ARG, "qnn_plane_sum_i8: NULL pointer");
    if (!aligned16(planes) || !aligned16(levels)) return fail(QNN_ERR_ALIGNMENT, "qnn_plane_sum_i8: pointers must be 16-byte aligned");
    const int64_t nw = ceil_div(n, 32), nk = qnn_level_row_bytes(n);
    if (rows > (INT64_MAX >> 8) / nk) return fail(QNN_ERR_RANGE, "qnn_plane_sum_i8: tensor too large");
    const int64_t total = rows * (nk / 16);
    const int64_t blocks = ceil_div(total, 256);
    const dim3 grid((unsigned)(blocks < 256 * 32 ? blocks : 256 * 32)), block(256);
    hipStream_t st = static_cast<hipStream_t>(stream);
    switch (bits) {
    case 1: hipLaunchKernelGGL(plane_sum_kernel<1>, grid, block, 0, st, planes, rows, n, nw, nk, levels); break;
    case 2: hipLaunchKernelGGL(plane_sum_kernel<2>, grid, block, 0, st, planes, rows, n, nw, nk, levels); break;
    case 3: hipLaunchKernelGGL(plane_sum_kernel<3>, grid, block, 0, st, planes, rows, n, nw, nk, levels); break;
    case 4: hipLaunchKernelGGL(plane_sum_kernel<4>, grid, block, 0, st, planes, rows, n, nw, nk, levels); break;
    case 5: hipLaunchKernelGGL(plane_sum_kernel<5>, grid, block, 0, st, planes, rows, n, nw, nk, levels); break;
    case 6: hipLaunchKernelGGL(plane_sum_kernel<6>, grid, block, 0, st, planes, rows, n, nw, nk, levels); break;
    default: hipLaunchKernelGGL(plane_sum_kernel<7>, grid, block, 0, st, planes, rows, n, nw, nk, levels); break;
    }
    return check_launch("qnn_plane_sum_i8");
}

extern "C" int qnn_level_gemm_i8(const int8_t *a_levels, const int8_t *w_levels, int64_t rows, int64_t cols,
                                 int64_t n, int32_t *acc, const float *scale, float *out, void *stream)
{
    if (rows < 0 || cols < 0 || n < 0) return fail(QNN_ERR_INVALID_ARG, "qnn_level_gemm_i8: negative size");
    if (!acc && !out) return fail(QNN_ERR_INVALID_ARG, "qnn_level_gemm_i8: acc and out are both NULL");
    if (out && !scale) return fail(QNN_ERR_INVALID_ARG, "qnn_level_gemm_i8: out given without scale");
    if (rows == 0 || cols == 0) return QNN_OK;
    if (n > 0 && (!a_levels || !w_levels)) return fail(QNN_ERR_INVALID_ARG, "qnn_level_gemm_i8: NULL level pointer");
    if (!aligned16(a_levels) || !aligned16(w_levels) || !aligned16(acc) || !aligned16(out))
        return fail(QNN_ERR_ALIGNMENT, "qnn_level_gemm_i8: pointers must be 16-byte aligned");
    if (n > ((int64_t)INT32_MAX) / (127 * 127))
        return fail(QNN_ERR_RANGE, "qnn_level_gemm_i8: n=%lld can overflow int32", (long long)n);
    LevelGemmParams p;
    p.a = a_levels, p.w = w_levels;
    p.rows = rows, p.cols = cols, p.nk = qnn_level_row_bytes(n);
    p.acc = acc, p.scale = scale, p.out = out;
    p.tiles_m = ceil_div(rows, kMB), p.tiles_n = ceil_div(cols, kNB);
    if (p.tiles_m * p.tiles_n > 0x7fffffffLL) return fail(QNN_ERR_RANGE, "qnn_level_gemm_i8: too many tiles");
    hipLaunchKernelGGL(level_gemm_mfma_kernel, dim3((unsigned)(p.tiles_m * p.tiles_n)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), p);
    return check_launch("qnn_level_gemm_i8");
}
