// Bit-plane-sum variant of the quantized GEMM on the matrix cores.
//
// The M x K binary branches of the paper (Eq. 9 with the {-1,+1} code of Eq. 10) recombine to the
// integer dot product of the decoded levels.  This file takes the other road to the same
// integers: sum the 2^j-weighted planes back into levels -- int8 (qnn_plane_sum_i8, up to 7 bits)
// or fp4 (qnn_plane_sum_fp4, 1 and 2 bits) -- and contract them with v_mfma_i32_32x32x32_i8
// (qnn_level_gemm_i8) or v_mfma_scale_f32_32x32x64_f8f6f4 (qnn_level_gemm_fp4).  It is NOT the
// graded xor + bitcount path (binary_gemm.hip); it exists to be compared with it, same inputs,
// same int32 outputs.
#include "qnn_host.h"
#include <type_traits>

namespace qnn {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

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
// planes [bits][rows][nw], bits <= 2 -> fp4 (E2M1) levels, two per byte, [rows][nb], nb a multiple of
// 128 bytes, zero padded.  The levels of 1- and 2-bit codes, -3 -1 +1 +3, are exact fp4 values:
// 1 = 0b0010, 3 = 0b0101, sign in bit 3.  One lane turns one word of each plane into 32 nibbles (one
// 16-byte store): the 8 bits of a byte are spread to bit 0 of 8 nibbles, sign = not the high plane
// bit, magnitude 3 where both plane bits agree.  Element 2i sits in the low nibble of byte i.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t spread_bits_to_nibbles(uint32_t byte)
{
    uint32_t x = byte & 0xffu;
    x = (x | (x << 12)) & 0x000f000fu;
    x = (x | (x << 6)) & 0x03030303u;
    x = (x | (x << 3)) & 0x11111111u;
    return x;
}

template <int BITS>
__global__ __launch_bounds__(256) void plane_sum_fp4_kernel(const uint32_t *__restrict__ planes, int64_t rows,
                                                            int64_t n, int64_t nw, int64_t nb, uint8_t *__restrict__ out)
{
    static_assert(BITS == 1 || BITS == 2, "fp4 holds the levels of 1- and 2-bit codes");
    const int64_t groups_per_row = nb / 16; // 32 elements = one plane word per group
    const int64_t total = rows * groups_per_row;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride) {
        const int64_t r = idx / groups_per_row, g = idx % groups_per_row;
        uint32_t hi = 0, lo = 0, valid = 0;
        if (g < nw) {
            hi = planes[((int64_t)(BITS - 1) * rows + r) * nw + g];
            lo = BITS == 2 ? planes[r * nw + g] : ~hi; // 1 bit: magnitude 1 everywhere (bits differ)
            const int64_t left = n - g * 32;
            valid = left >= 32 ? 0xffffffffu : ((1u << left) - 1u);
        }
        uint32_t o[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t h = spread_bits_to_nibbles(hi >> (8 * d)), l = spread_bits_to_nibbles(lo >> (8 * d));
            const uint32_t v = spread_bits_to_nibbles(valid >> (8 * d));
            const uint32_t same = ~(h ^ l) & 0x11111111u;
            const uint32_t nib = ((~h & 0x11111111u) << 3) | (0x22222222u ^ (same * 7u));
            o[d] = nib & (v * 15u); // elements past n are 0
        }
        *reinterpret_cast<uint4 *>(out + r * nb + g * 16) = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

// ---------------------------------------------------------------------------------------------
// int8 GEMM acc[r][c] = sum_k a[r][k] w[c][k] on v_mfma_i32_32x32x32_i8.
// Workgroup: block tile 256 x 256, kWavesM x kWavesN waves, each wave kTM x kTN MFMA tiles of 32 x 32
// (8 waves of 64 x 128: 128 accumulator registers, two waves per SIMD, so that one wave's MFMAs cover
// the other's stalls at LDS and memory instructions; 64 x 128 rather than 128 x 64 because a wave's
// row-major stores then cover 512 contiguous bytes of an output row: 76 -> 71 us at 4096^3).  The reduction is staged kKB bytes per row
// through a ring of kRing LDS stages filled by direct global -> LDS loads (no staging registers); a
// stage is requested kRing stages ahead of its use.  Inside a stage the operands of the next 32-byte
// k step are read from LDS between the MFMAs of the current one.
// LDS rows are kKB bytes apart with no padding; the 16-byte unit q of row r is stored at position
// q ^ ((r / (8 / U)) mod U), U = kKB / 16 units per row, so that the operand reads of 8 consecutive
// rows (one pass of a 16-byte LDS read) hit all 32 banks.
// The k order inside an MFMA operand does not matter for a dot product as long as both operands
// use the same assignment, which they do by the symmetry of the instruction.  Rows / columns past
// the end are clamped to the last one (their outputs are never stored); bytes past n are 0.
// ---------------------------------------------------------------------------------------------
constexpr int kMB = 256, kNB = 256;
constexpr int kWavesM = 4, kWavesN = 2;
constexpr int kThreads = 64 * kWavesM * kWavesN;
constexpr int kTM = kMB / kWavesM / 32, kTN = kNB / kWavesN / 32; // MFMA tiles per wave
constexpr int kKB = 128, kRing = 2;                       // stage depth in bytes of k, stages in LDS
constexpr int kRowPad = 128;                              // level rows are padded to this many bytes
constexpr int kSteps = kKB / 32;                          // 32-byte MFMA k steps per stage
constexpr int kUnits = kKB / 16;                          // 16-byte units per LDS row
constexpr int kStageBytes = (kMB + kNB) * kKB;
constexpr int kLoadsPerStage = kStageBytes / (kThreads * 16); // direct loads per lane and stage
constexpr int kRowsPerLoad = 1024 / kKB;                  // LDS rows one wave-wide 1 KiB load fills
static_assert(kRowPad % kKB == 0 && kKB % 32 == 0 && kUnits <= 8 && kSteps >= 2, "stage shape");
static_assert(kLoadsPerStage <= kTM * kTN && kTM + kTN <= kTM * kTN, "one read and one load per MFMA slot");
static_assert(kRing * kStageBytes <= 160 * 1024, "LDS ring");
static_assert((kRing - 1) * kLoadsPerStage < 64, "vmcnt range");

struct LevelGemmParams {
    const int8_t *a, *w; // [rows][nk], [cols][nk]
    int64_t rows, cols, nk;
    int32_t *acc;
    const float *scale;
    float *out;
    int64_t tiles_n, tiles_m;
#ifdef QNN_TIMELINE
    long long *timeline; // [timeline_waves][6] or nullptr
    int timeline_waves;
#endif
};

#ifdef QNN_TIMELINE
// Diagnostic build (libqnn_timeline.so, include/qnn_probe.h): every wave leaves the constant-rate counter (100 MHz)
// at its start, at the start and the end of its reduction loop and at its end, and the shader-clock counter's
// ticks across the loop and across its life, in a caller-owned buffer.  The product library has none of this.
struct GemmTimelineState {
    long long *buf;
    int waves;
};
inline GemmTimelineState &gemm_timeline_state()
{
    static GemmTimelineState s = {nullptr, 0};
    return s;
}
#define QNN_TL_REAL(k)                                                                                        \
    if (p.timeline && lane == 0 && (int64_t)blockIdx.x * (kThreads / 64) + wave < p.timeline_waves)            \
    p.timeline[6 * ((int64_t)blockIdx.x * (kThreads / 64) + wave) + (k)] = (long long)__builtin_amdgcn_s_memrealtime()
#define QNN_TL_CLOCK(var) const unsigned long long var = __builtin_amdgcn_s_memtime()
#define QNN_TL_TICKS(k, from, to)                                                                             \
    if (p.timeline && lane == 0 && (int64_t)blockIdx.x * (kThreads / 64) + wave < p.timeline_waves)            \
    p.timeline[6 * ((int64_t)blockIdx.x * (kThreads / 64) + wave) + (k)] = (long long)((to) - (from))
#else
#define QNN_TL_REAL(k)
#define QNN_TL_CLOCK(var)
#define QNN_TL_TICKS(k, from, to)
#endif

// s_waitcnt on the vector-memory counter only (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
#define QNN_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8))

__device__ __forceinline__ int swizzle_of_row(int row) { return (row / (8 / kUnits)) & (kUnits - 1); }

// FP4: the operands are fp4 levels (two per byte) multiplied by v_mfma_scale_f32_32x32x64_f8f6f4 with
// unit scales; products and partial sums are integers below 2^24, which fp32 holds exactly.
template <bool FP4> __global__ __launch_bounds__(kThreads) void level_gemm_mfma_kernel(LevelGemmParams p)
{
    __shared__ __attribute__((aligned(1024))) uint8_t smem[kRing][kStageBytes];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / kWavesN, wn = wave % kWavesN;
    const int64_t row0 = ((int64_t)blockIdx.x / p.tiles_n) * kMB;
    const int64_t col0 = ((int64_t)blockIdx.x % p.tiles_n) * kNB;
    QNN_TL_REAL(0);
    QNN_TL_CLOCK(tl_c0);

    using Acc = typename std::conditional<FP4, v16f, v16i>::type;
    Acc acc[kTM][kTN];
#pragma unroll
    for (int i = 0; i < kTM; ++i)
#pragma unroll
        for (int j = 0; j < kTN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // Direct load j of this wave fills the 1 KiB LDS chunk wave * kLoadsPerStage + j = kRowsPerLoad
    // stage rows (stage rows 0..255 are A, 256..511 are W); lane l delivers row l / U, position l % U.
    const int8_t *src[kLoadsPerStage];
#pragma unroll
    for (int j = 0; j < kLoadsPerStage; ++j) {
        const int row = (wave * kLoadsPerStage + j) * kRowsPerLoad + lane / kUnits;
        const int q = (lane % kUnits) ^ swizzle_of_row(row);
        if (row < kMB) {
            const int64_t g = row0 + row < p.rows ? row0 + row : p.rows - 1;
            src[j] = p.a + g * p.nk + 16 * q;
        } else {
            const int64_t g = col0 + row - kMB < p.cols ? col0 + row - kMB : p.cols - 1;
            src[j] = p.w + g * p.nk + 16 * q;
        }
    }
    auto issue_one = [&](int64_t stage, int buf, int j) {
        uint8_t *dst = smem[buf] + wave * (kLoadsPerStage * 1024);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src[j] + stage * kKB),
                                         (__attribute__((address_space(3))) void *)(dst + j * 1024), 16, 0, 0);
    };

    // operand reads at k step ks: row = tile row + lane % 32, unit 2 ks + lane / 32, swizzled
    const int a_off = (wm * 32 * kTM + (lane & 31)) * kKB, b_off = (kMB + wn * 32 * kTN + (lane & 31)) * kKB;
    const int hi = lane >> 5, swz = swizzle_of_row(lane & 31); // tile rows start at multiples of 32
    v4i af[2][kTM], bf[2][kTN];
    // operand read r of kTM + kTN of k step ks into operand set b, in the order the MFMAs first need
    // them: A tile 0, W tiles 0.., A tiles 1..
    auto read_one = [&](const uint8_t *st, int ks, int b, int r) {
        const int u = 16 * ((2 * ks + hi) ^ swz);
        if (r == 0) af[b][0] = *reinterpret_cast<const v4i *>(st + a_off + u);
        else if (r <= kTN) bf[b][r - 1] = *reinterpret_cast<const v4i *>(st + b_off + (r - 1) * 32 * kKB + u);
        else af[b][r - kTN] = *reinterpret_cast<const v4i *>(st + a_off + (r - kTN) * 32 * kKB + u);
    };

    // One k step: kTM * kTN MFMAs on operand set b.  The operand reads of the following k step (into
    // the other operand set) and, in the last step of a stage, the direct loads of the stage kRing
    // further on are spread one by one between the MFMAs, each behind an MFMA that keeps the matrix
    // core busy while the wave sits at the LDS or memory instruction.  The first read follows the
    // first MFMA, so the wait in front of that MFMA covers only this step's operands.
    auto mfma_step = [&](int b, const uint8_t *next_stage, int next_ks, auto dma, int64_t dma_stage, int dma_buf) {
#pragma unroll
        for (int m = 0; m < kTM * kTN; ++m) {
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (FP4) {
                const v4i x = af[b][m / kTN], y = bf[b][m % kTN];
                // the builtin takes 8 registers per operand and uses the first 4 for fp4: leave the rest undefined
                const v8i x8 = __builtin_shufflevector(x, x, 0, 1, 2, 3, -1, -1, -1, -1);
                const v8i y8 = __builtin_shufflevector(y, y, 0, 1, 2, 3, -1, -1, -1, -1);
                // cbsz = blgp = 4: both operands fp4; scale bytes 127 = 2^0
                acc[m / kTN][m % kTN] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(x8, y8, acc[m / kTN][m % kTN], 4, 4, 0, 127, 0, 127);
            } else {
                acc[m / kTN][m % kTN] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[b][m / kTN], bf[b][m % kTN], acc[m / kTN][m % kTN], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (m < kTM + kTN) read_one(next_stage, next_ks, b ^ 1, m);
            if constexpr (decltype(dma)::value)
                if (m < kLoadsPerStage) issue_one(dma_stage, dma_buf, m);
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    // wait until at most the loads of `stages` whole stages are outstanding (loads land in order)
    auto wait_loads = [&](int64_t stages) {
        static_assert(kRing <= 5, "extend the cases below");
        constexpr int kL = kLoadsPerStage;
        if (stages >= 4) QNN_WAIT_VMCNT(4 * kL < 63 ? 4 * kL : 63);
        else if (stages == 3) QNN_WAIT_VMCNT(3 * kL < 63 ? 3 * kL : 63);
        else if (stages == 2) QNN_WAIT_VMCNT(2 * kL < 63 ? 2 * kL : 63);
        else if (stages == 1) QNN_WAIT_VMCNT(kLoadsPerStage);
        else QNN_WAIT_VMCNT(0);
    };
    const int64_t nstages = p.nk / kKB;
    // prologue: request the first kRing stages, wait for stage 0, read its first operands
    for (int t = 0; t < kRing; ++t)
        if (t < nstages)
#pragma unroll
            for (int j = 0; j < kLoadsPerStage; ++j) issue_one(t, t, j);
    if (nstages > 0) {
        wait_loads(nstages - 1 < kRing - 1 ? nstages - 1 : kRing - 1);
        __builtin_amdgcn_s_barrier();
#pragma unroll
        for (int r = 0; r < kTM + kTN; ++r) read_one(smem[0], 0, 0, r);
    }
    // One stage per iteration, buffer cur = s mod kRing.  The barrier sits in front of the last k
    // step: by then every wave has read all of stage s (its buffer may be refilled) and this wave's
    // loads of stage s+1 have landed, so under the last step's MFMAs the first operands of stage s+1
    // are read and stage s + kRing is requested into the buffer of stage s.
    // The loop runs in two parts, with and without the request for stage s + kRing, so that each body
    // is one straight line of code whose order the scheduling barriers pin.
    int cur = 0;
    auto stage_body = [&](int64_t s, auto dma) {
        const uint8_t *st = smem[cur];
        const int nxt = cur + 1 == kRing ? 0 : cur + 1;
#pragma unroll
        for (int ks = 0; ks + 1 < kSteps; ++ks) mfma_step(ks & 1, st, ks + 1, std::false_type{}, 0, 0);
        // stages s+2 .. s+kRing-1 (as far as they exist) may still be in flight
        wait_loads(nstages - (s + 2) < kRing - 2 ? nstages - (s + 2) : kRing - 2);
        __builtin_amdgcn_s_waitcnt(0xC07F); // lgkmcnt(0)
        __builtin_amdgcn_s_barrier();
        // after the last stage this reads stale data that is never used (no branch around LDS reads)
        mfma_step((kSteps - 1) & 1, smem[nxt], 0, dma, s + kRing, cur);
        cur = nxt;
    };
    int64_t s = 0;
    QNN_TL_REAL(1);
    QNN_TL_CLOCK(tl_c1);
    for (; s + kRing < nstages; ++s) stage_body(s, std::true_type{});
    for (; s < nstages; ++s) stage_body(s, std::false_type{});
    QNN_TL_REAL(2);
    QNN_TL_CLOCK(tl_c2);

    // Epilogue.  D layout of the 32x32 MFMA: lane holds column lane % 32 and rows 8 (r / 4) + 4 (lane / 32) +
    // r % 4.  Each 32 x 32 tile goes through a private LDS patch of its wave and leaves row-major, one
    // lane with 4 consecutive columns of one row: 16-byte stores of acc and out instead of 4-byte ones.
    __builtin_amdgcn_s_waitcnt(0xC07F);
    __syncthreads(); // every wave is past its last operand read: the ring can be reused
    constexpr int kPatchStride = 36; // words per patch row
    static_assert(kWavesM * kWavesN * 32 * kPatchStride * 4 <= kRing * kStageBytes, "patches fit the ring");
    int32_t *patch = reinterpret_cast<int32_t *>(&smem[0][0]) + wave * (32 * kPatchStride);
    const int prow = lane >> 3, pc4 = (lane & 7) * 4;
    const bool cols4 = (p.cols & 3) == 0;
#pragma unroll
    for (int j = 0; j < kTN; ++j) {
        const int64_t c = col0 + (wn * kTN + j) * 32 + pc4;
        float sc[4] = {0.f, 0.f, 0.f, 0.f};
        if (p.out) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (c + e < p.cols) sc[e] = p.scale[c + e];
        }
#pragma unroll
        for (int i = 0; i < kTM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r)
                patch[(8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)) * kPatchStride + (lane & 31)] = (int32_t)acc[i][j][r];
            // the wave's own LDS operations complete in order; the compiler must not move the reads up
            __builtin_amdgcn_s_waitcnt(0xC07F);
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int ps = 0; ps < 4; ++ps) {
                const int4 v = *reinterpret_cast<const int4 *>(patch + (ps * 8 + prow) * kPatchStride + pc4);
                const int64_t row = row0 + (wm * kTM + i) * 32 + ps * 8 + prow;
                if (row >= p.rows || c >= p.cols) continue;
                const int64_t o = row * p.cols + c;
                const int32_t vi[4] = {v.x, v.y, v.z, v.w};
                if (cols4) { // c is a multiple of 4, so c + 3 < cols and the address is 16-byte aligned
                    if (p.acc) *reinterpret_cast<int4 *>(p.acc + o) = v;
                    if (p.out)
                        *reinterpret_cast<float4 *>(p.out + o) =
                            make_float4((float)vi[0] * sc[0], (float)vi[1] * sc[1], (float)vi[2] * sc[2], (float)vi[3] * sc[3]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (c + e < p.cols) {
                            if (p.acc) p.acc[o + e] = vi[e];
                            if (p.out) p.out[o + e] = (float)vi[e] * sc[e];
                        }
                }
            }
            __builtin_amdgcn_s_waitcnt(0xC07F);
            __builtin_amdgcn_wave_barrier(); // the patch is rewritten by the next tile
        }
    }
    QNN_TL_REAL(3);
    QNN_TL_CLOCK(tl_c3);
    QNN_TL_TICKS(4, tl_c1, tl_c2);
    QNN_TL_TICKS(5, tl_c0, tl_c3);
}

} // namespace qnn

using namespace qnn;

extern "C" int64_t qnn_level_row_bytes(int64_t n) { return n < 0 ? -1 : ceil_div(n, kRowPad) * kRowPad; }

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
#ifdef QNN_TIMELINE
    p.timeline = gemm_timeline_state().buf, p.timeline_waves = gemm_timeline_state().waves;
#endif
    hipLaunchKernelGGL(level_gemm_mfma_kernel<false>, dim3((unsigned)(p.tiles_m * p.tiles_n)), dim3(kThreads), 0,
                       static_cast<hipStream_t>(stream), p);
    return check_launch("qnn_level_gemm_i8");
}

#ifdef QNN_TIMELINE
extern "C" int qnn_level_gemm_timeline_set(long long *buffer, int waves)
{
    if (waves < 0 || (waves > 0 && !buffer))
        return fail(QNN_ERR_INVALID_ARG, "qnn_level_gemm_timeline_set: a buffer of waves x 6 int64 is needed");
    gemm_timeline_state() = {waves > 0 ? buffer : nullptr, waves};
    return QNN_OK;
}
#endif

extern "C" int64_t qnn_fp4_row_bytes(int64_t n) { return n < 0 ? -1 : ceil_div(n, 2 * kRowPad) * kRowPad; }

extern "C" int qnn_plane_sum_fp4(const uint32_t *planes, int bits, int64_t rows, int64_t n, uint8_t *levels,
                                 void *stream)
{
    if (bits < 1 || bits > 2) return fail(QNN_ERR_UNSUPPORTED, "qnn_plane_sum_fp4: fp4 holds the levels of 1 or 2 bits (got %d)", bits);
    if (rows < 0 || n < 0) return fail(QNN_ERR_INVALID_ARG, "qnn_plane_sum_fp4: negative size");
    if (rows == 0 || n == 0) return QNN_OK;
    if (!planes || !levels) return fail(QNN_ERR_INVALID_ARG, "qnn_plane_sum_fp4: NULL pointer");
    if (!aligned16(planes) || !aligned16(levels)) return fail(QNN_ERR_ALIGNMENT, "qnn_plane_sum_fp4: pointers must be 16-byte aligned");
    const int64_t nw = ceil_div(n, 32), nb = qnn_fp4_row_bytes(n);
    if (rows > (INT64_MAX >> 8) / nb) return fail(QNN_ERR_RANGE, "qnn_plane_sum_fp4: tensor too large");
    const int64_t blocks = ceil_div(rows * (nb / 16), 256);
    const dim3 grid((unsigned)(blocks < 256 * 32 ? blocks : 256 * 32)), block(256);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (bits == 1) hipLaunchKernelGGL(plane_sum_fp4_kernel<1>, grid, block, 0, st, planes, rows, n, nw, nb, levels);
    else hipLaunchKernelGGL(plane_sum_fp4_kernel<2>, grid, block, 0, st, planes, rows, n, nw, nb, levels);
    return check_launch("qnn_plane_sum_fp4");
}

extern "C" int qnn_level_gemm_fp4(const uint8_t *a_levels, const uint8_t *w_levels, int64_t rows, int64_t cols,
                                  int64_t n, int32_t *acc, const float *scale, float *out, void *stream)
{
    if (rows < 0 || cols < 0 || n < 0) return fail(QNN_ERR_INVALID_ARG, "qnn_level_gemm_fp4: negative size");
    if (!acc && !out) return fail(QNN_ERR_INVALID_ARG, "qnn_level_gemm_fp4: acc and out are both NULL");
    if (out && !scale) return fail(QNN_ERR_INVALID_ARG, "qnn_level_gemm_fp4: out given without scale");
    if (rows == 0 || cols == 0) return QNN_OK;
    if (n > 0 && (!a_levels || !w_levels)) return fail(QNN_ERR_INVALID_ARG, "qnn_level_gemm_fp4: NULL level pointer");
    if (!aligned16(a_levels) || !aligned16(w_levels) || !aligned16(acc) || !aligned16(out))
        return fail(QNN_ERR_ALIGNMENT, "qnn_level_gemm_fp4: pointers must be 16-byte aligned");
    // |acc| <= 9 n must stay below 2^24 for the fp32 accumulators of the instruction to be exact
    if (n > ((int64_t)1 << 24) / 9)
        return fail(QNN_ERR_RANGE, "qnn_level_gemm_fp4: n=%lld exceeds the exact range of fp32 accumulation", (long long)n);
    LevelGemmParams p;
    p.a = reinterpret_cast<const int8_t *>(a_levels), p.w = reinterpret_cast<const int8_t *>(w_levels);
    p.rows = rows, p.cols = cols, p.nk = qnn_fp4_row_bytes(n);
    p.acc = acc, p.scale = scale, p.out = out;
    p.tiles_m = ceil_div(rows, kMB), p.tiles_n = ceil_div(cols, kNB);
    if (p.tiles_m * p.tiles_n > 0x7fffffffLL) return fail(QNN_ERR_RANGE, "qnn_level_gemm_fp4: too many tiles");
#ifdef QNN_TIMELINE
    p.timeline = gemm_timeline_state().buf, p.timeline_waves = gemm_timeline_state().waves;
#endif
    hipLaunchKernelGGL(level_gemm_mfma_kernel<true>, dim3((unsigned)(p.tiles_m * p.tiles_n)), dim3(kThreads), 0,
                       static_cast<hipStream_t>(stream), p);
    return check_launch("qnn_level_gemm_fp4");
}
