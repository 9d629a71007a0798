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
// planes [bits][rows][nw] -> int8 levels [rows][nk], nk a multiple of 128 bytes, zero padded.
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
// tiles (256 accumulator registers).  The reduction is staged 128 bytes per row (whole cache
// lines) through two 64 KiB LDS stages filled by direct global -> LDS loads (no staging
// registers): the loads of stage S+1 are issued right after the barrier that opens stage S and
// have the 64 MFMAs of stage S to arrive.  Inside a stage the operands of the next 32-byte k step
// are read from LDS while the MFMAs of the current step run.
// LDS rows are 128 bytes apart with no padding; the 16-byte unit q of row r sits at position
// q ^ (r & 7), so the operand reads of 8 consecutive rows hit all 32 banks.
// The k order inside an MFMA operand does not matter for a dot product as long as both operands
// use the same assignment, which they do by the symmetry of the instruction.  Rows / columns past
// the end are clamped to the last one (their outputs are never stored); bytes past n are 0.
// ---------------------------------------------------------------------------------------------
constexpr int kMB = 256, kNB = 256, kKB = 128;
constexpr int kRing = 2, kStageBytes = (kMB + kNB) * kKB;
constexpr int kLoadsPerStage = kStageBytes / (256 * 16); // direct loads per lane and stage

struct LevelGemmParams {
    const int8_t *a, *w; // [rows][nk], [cols][nk]
    int64_t rows, cols, nk;
    int32_t *acc;
    const float *scale;
    float *out;
    int64_t tiles_n, tiles_m;
};

// s_waitcnt on the vector-memory counter only (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
#define QNN_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8))

__global__ __launch_bounds__(256) void level_gemm_mfma_kernel(LevelGemmParams p)
{
    __shared__ __attribute__((aligned(1024))) uint8_t smem[kRing][kStageBytes];
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

    // Direct load j of this wave fills the 1 KiB LDS chunk wave * 16 + j = stage rows chunk*8 .. +7
    // (stage rows 0..255 are A, 256..511 are W); lane l delivers row l / 8, position l % 8.
    const int8_t *src[kLoadsPerStage];
#pragma unroll
    for (int j = 0; j < kLoadsPerStage; ++j) {
        const int row = (wave * kLoadsPerStage + j) * 8 + (lane >> 3);
        const int q = (lane & 7) ^ (row & 7);
        if (row < kMB) {
            const int64_t g = row0 + row < p.rows ? row0 + row : p.rows - 1;
            src[j] = p.a + g * p.nk + 16 * q;
        } else {
            const int64_t g = col0 + row - kMB < p.cols ? col0 + row - kMB : p.cols - 1;
            src[j] = p.w + g * p.nk + 16 * q;
        }
    }
    auto issue = [&](int64_t stage) {
        uint8_t *dst = smem[stage % kRing] + wave * (kLoadsPerStage * 1024);
#pragma unroll
        for (int j = 0; j < kLoadsPerStage; ++j)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void *)(src[j] + stage * kKB),
                (__attribute__((address_space(3))) void *)(dst + j * 1024), 16, 0, 0);
    };

    // operand reads at k step ks: row = tile row + lane % 32, unit 2 ks + lane / 32, swizzled
    const int a_off = (wm * 128 + (lane & 31)) * kKB, b_off = (kMB + wn * 128 + (lane & 31)) * kKB;
    const int hi = lane >> 5, swz = lane & 7;
    auto read_step = [&](const uint8_t *st, int ks, v4i (&af)[4], v4i (&bf)[4]) {
        const int u = 16 * ((2 * ks + hi) ^ swz);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            af[t] = *reinterpret_cast<const v4i *>(st + a_off + t * 32 * kKB + u);
            bf[t] = *reinterpret_cast<const v4i *>(st + b_off + t * 32 * kKB + u);
        }
    };

    // Pipeline.  Stage s is multiplied in four 32-byte k steps; the operands of step ks+1 are read
    // while the MFMAs of step ks run.  The barrier that opens stage s+1 sits before the MFMAs of the
    // last step of stage s: by then this wave has read all of stage s (its buffer may be refilled
    // with stage s+2) and the first operands of stage s+1 are fetched under those last 16 MFMAs.
    const int64_t nstages = p.nk / kKB;
    v4i af[2][4], bf[2][4];
    // One k step: 16 MFMAs on operand set b.  The LDS reads of the following step (into the other
    // operand set) are issued right after the first MFMA: the wait the compiler puts in front of
    // that first MFMA then covers only this step's operands, and the reads fly under the other 15.
    auto mfma_step = [&](int b, const uint8_t *next_stage, int next_ks) {
        __builtin_amdgcn_sched_barrier(0);
        acc[0][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[b][0], bf[b][0], acc[0][0], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        read_step(next_stage, next_ks, af[b ^ 1], bf[b ^ 1]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (i == 0 && j == 0) continue;
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[b][i], bf[b][j], acc[i][j], 0, 0, 0);
            }
        __builtin_amdgcn_sched_barrier(0);
    };
    if (nstages > 0) {
        issue(0);
        if (nstages > 1) issue(1);
        if (nstages > 1) QNN_WAIT_VMCNT(kLoadsPerStage);
        else QNN_WAIT_VMCNT(0);
        __builtin_amdgcn_s_barrier();
        read_step(smem[0], 0, af[0], bf[0]);
    }
    for (int64_t s = 0; s < nstages; ++s) {
        const uint8_t *st = smem[s % kRing];
        mfma_step(0, st, 1);
        mfma_step(1, st, 2);
        mfma_step(0, st, 3);
        // All of this lane's LDS reads of stage s have been issued and are waited for here; its loads
        // of stage s+1 are complete.  After the barrier stage s's buffer may be refilled (stage s+2)
        // and stage s+1 is visible.  After the last stage the same sequence runs once more on stale
        // data that is never used, which keeps the loop free of branches around the LDS reads.
        QNN_WAIT_VMCNT(0);
        __builtin_amdgcn_s_waitcnt(0xC07F); // lgkmcnt(0)
        __builtin_amdgcn_s_barrier();
        if (s + 2 < nstages) issue(s + 2);
        mfma_step(1, smem[(s + 1) % kRing], 0);
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
