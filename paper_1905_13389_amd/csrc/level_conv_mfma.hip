// Decoded-level convolution on the matrix cores, and the level encoder that feeds it.
//
// The M x K binary branches of the paper (Eq. 9 with the {-1,+1} code of Eq. 10) recombine to the
// integer dot product of the decoded levels; section "Model Decomposition" reduces a convolution to
// the same product.  Here the levels stay decoded (int8, NHWC) from layer to layer and the
// convolution is an implicit GEMM on v_mfma_i32_32x32x32_i8: same int32 accumulators as qnn_conv2d,
// a different machine route.  It is NOT the graded xor + bitcount path (conv2d.hip); it exists to
// be compared with it.
#include "qnn_host.h"
#include "quantize.h"
#include "fastdiv.h"
#include "block_terms.h"
#include <type_traits>

namespace qnn {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));

// A level of a 1- or 2-bit code (-3, -1, +1, +3) as an fp4 (E2M1) nibble: sign << 3 | magnitude code
// (1 = 0b0010, 3 = 0b0101); these values are exact in fp4.
__device__ __forceinline__ uint32_t fp4_nibble(int level)
{
    const int mag = level < 0 ? -level : level;
    return (level < 0 ? 8u : 0u) | (mag == 3 ? 5u : 2u);
}

// ---------------------------------------------------------------------------------------------
// fp32 / bf16 values -> int8 levels, elementwise: level = 2u - (2^bits - 1) with the code u of the
// linear quantizer (Table 1 HTanh, Eq. 15, Eq. 10); the same quantize_code as qnn_encode_pack.
// One lane turns 16 consecutive elements into one 16-byte store.
// ---------------------------------------------------------------------------------------------
struct EncodeLevelParams {
    const void *src;
    int64_t count;
    float inv_clip, half_top;
    int top;
    int8_t *levels; // int8 per element, or (FP4) one nibble per element, element 2i in the low nibble of byte i
};

__device__ __forceinline__ float widen_bf16(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

template <bool BF16, bool FP4> __global__ __launch_bounds__(256) void encode_levels_kernel(EncodeLevelParams p)
{
    const int64_t groups = (p.count + 15) / 16;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < groups; g += stride) {
        const int64_t e0 = g * 16;
        float x[16];
        if (e0 + 16 <= p.count) {
            if (BF16) {
                const uint4 *s = reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(p.src) + e0);
                const uint4 v0 = s[0], v1 = s[1];
                const uint32_t w[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    x[2 * i] = widen_bf16((uint16_t)(w[i] & 0xffffu));
                    x[2 * i + 1] = widen_bf16((uint16_t)(w[i] >> 16));
                }
            } else {
                const float4 *s = reinterpret_cast<const float4 *>(static_cast<const float *>(p.src) + e0);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float4 v = s[i];
                    x[4 * i] = v.x, x[4 * i + 1] = v.y, x[4 * i + 2] = v.z, x[4 * i + 3] = v.w;
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                x[i] = 0.0f;
                if (e0 + i < p.count)
                    x[i] = BF16 ? widen_bf16(static_cast<const uint16_t *>(p.src)[e0 + i])
                                : static_cast<const float *>(p.src)[e0 + i];
            }
        }
        uint32_t o[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int lv = 2 * quantize_code(x[i], p.inv_clip, p.half_top, p.top) - p.top;
            if (FP4) o[i >> 3] |= fp4_nibble(lv) << (4 * (i & 7));
            else o[i >> 2] |= ((uint32_t)lv & 0xffu) << (8 * (i & 3));
        }
        if constexpr (FP4) {
            // count is even (checked on the host): whole bytes
            uint8_t *dst = reinterpret_cast<uint8_t *>(p.levels) + e0 / 2;
            if (e0 + 16 <= p.count) {
                *reinterpret_cast<uint2 *>(dst) = make_uint2(o[0], o[1]);
            } else {
                for (int i = 0; i < 8 && e0 + 2 * i < p.count; ++i) dst[i] = (uint8_t)(o[i >> 2] >> (8 * (i & 3)));
            }
        } else if (e0 + 16 <= p.count) {
            *reinterpret_cast<uint4 *>(p.levels + e0) = make_uint4(o[0], o[1], o[2], o[3]);
        } else {
            for (int i = 0; i < 16 && e0 + i < p.count; ++i) p.levels[e0 + i] = (int8_t)(o[i >> 2] >> (8 * (i & 3)));
        }
    }
}

// int8 levels of 1- or 2-bit codes -> fp4 nibbles, 16 elements per lane (weights, once per layer)
__global__ __launch_bounds__(256) void levels_to_fp4_kernel(const int8_t *__restrict__ src, int64_t count,
                                                            uint8_t *__restrict__ dst)
{
    const int64_t groups = (count + 15) / 16, stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < groups; g += stride) {
        const int64_t e0 = g * 16;
        if (e0 + 16 <= count) {
            const uint4 v = *reinterpret_cast<const uint4 *>(src + e0);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
            uint32_t o[2] = {0u, 0u};
#pragma unroll
            for (int i = 0; i < 16; ++i)
                o[i >> 3] |= fp4_nibble((int)(int8_t)(w[i >> 2] >> (8 * (i & 3)))) << (4 * (i & 7));
            *reinterpret_cast<uint2 *>(dst + e0 / 2) = make_uint2(o[0], o[1]);
        } else {
            for (int64_t e = e0; e < count; e += 2) // count is even
                dst[e / 2] = (uint8_t)(fp4_nibble(src[e]) | (fp4_nibble(src[e + 1]) << 4));
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Implicit-GEMM convolution.  Rows = output pixels (b, oy, ox flattened, NHWC), columns = output
// channels, reduction axis = (ky, kx, ci) in bytes, nk = kh kw Cin, cut into stages of 128 (or 64)
// bytes.  A workgroup (WM x WN waves) owns an MB x NB block; stages go through a
// ring of two LDS buffers filled by direct global -> LDS loads of 16 bytes per lane.  A lane's 16
// bytes never straddle a tap because Cin is a multiple of 16: the lane looks up (tap, byte offset
// relative to the pixel's first tap) of its unit in a table built once per workgroup, tests the tap
// against the pixel's bit mask of taps that fall outside the image, and loads either the 16 levels
// or 16 zero bytes: a level of 0 contributes exactly 0, which is the zero padding of the decoded
// integers.  Units past the end of the reduction axis are zero the same way, in both operands.
// LDS rows are one stage length apart (U = 8 or 4 units of 16 bytes), the unit q of row r is stored
// at position q ^ ((r / (8 / U)) mod U), so the operand reads of 8 consecutive rows hit all 32
// banks.  The k order inside an MFMA operand is the same for both operands, which is all a dot
// product needs.
// Epilogue: int32 acc and / or fp32 acc * scale[c] stored from the MFMA layout; the next layer's
// levels (scale, quantize, 2u - top) are transposed through LDS and stored 16 channels per lane.
// ---------------------------------------------------------------------------------------------
constexpr int kRing = 2;
constexpr int kMaxUnits = 1024; // table entries: reduction axis up to 16 KiB (e.g. 3 x 3 x 1024, 5 x 5 x 512)
constexpr int kMaxMfmaTaps = 31; // tap 31 marks units past the end of the reduction axis

__device__ __attribute__((aligned(256))) uint8_t g_zero_units[256]; // zero-initialised, read only

struct LevelConvParams {
    const int8_t *a, *w; // [B][H][W][Cin], [Cout][kh][kw][Cin]
    const float *scale;
    int32_t *acc;
    float *out;
    int8_t *next;
    int H, W, Cin, Cout, Ho, Wo, kh, kw, stride, pad;
    int dil;     // distance between neighbouring taps in pixels
    int pixels;  // B Ho Wo
    int nk;      // kh kw Cin
    int units;   // nk / 16
    int nstages; // ceil(nk / stage length)
    int tiles_n;
    FastDiv div_howo, div_wo, div_cin, div_kw; // pixel -> (b, oy, ox); byte of the reduction axis -> (tap, c) -> (ky, kx)
    uint32_t row_taps, col_taps;               // bit masks of the taps of kernel row 0 / kernel column 0
    float next_inv_clip, next_half_top;
    int next_top;
    BlockTerms blk; // res_q: int8 levels [pixels][Cout]
};

#define QNN_CONV_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8))

// KB: stage length in bytes of the reduction axis, 128 or 64 (short reductions: more, smaller
// workgroups per CU, no half-empty last stage at kh kw Cin = 576)
// The 256 x 64 block runs three workgroups per CU (one wave each per SIMD): its register budget is
// held to a third of the file.
// FP4: both operands hold fp4 levels, two per byte (1- and 2-bit codes); the byte-level addressing is
// the same with Cin / 2 bytes per pixel, the product is v_mfma_scale_f32_32x32x64_f8f6f4 with unit
// scales (64 values per 32-byte k step), accumulated in fp32 -- exact, the host bounds the sums by
// 2^24 -- and the next layer's levels leave as nibbles.
// BLK: the residual-block terms (shift, shortcut) are part of the epilogue; the plain kernels carry
// none of their registers.
template <int MB, int NB, int WM, int WN, int KB, bool FP4, bool BLK>
__global__ __launch_bounds__(64 * WM * WN) __attribute__((amdgpu_waves_per_eu(MB == 256 && NB == 64 && (BLK || FP4) ? 3 : 1))) void
level_conv_mfma_kernel(LevelConvParams p)
{
    constexpr int kKB = KB, kSteps = KB / 32, kUnits = KB / 16; // k steps of 32 bytes, 16-byte units per row
    constexpr int kRowsPerLoad = 1024 / KB;                      // LDS rows one wave-wide 1 KiB load fills
    static_assert(KB == 128 || KB == 64, "stage length");
    constexpr int kWaves = WM * WN, kConvThreads = 64 * kWaves;
    constexpr int TM = MB / WM / 32, TN = NB / WN / 32;  // MFMA tiles per wave
    constexpr int NM = TM * TN, NR = TM + TN;             // MFMAs and operand reads per k step
    constexpr int LA = MB / (kRowsPerLoad * kWaves), LW = NB / (kRowsPerLoad * kWaves), L = LA + LW; // direct loads per lane and stage
    constexpr int kStageBytes = (MB + NB) * kKB;
    static_assert(MB % (kRowsPerLoad * kWaves) == 0 && NB % (kRowsPerLoad * kWaves) == 0 && TM >= 1 && TN >= 1, "tile shape");
    static_assert(kRing * kStageBytes + kMaxUnits * 4 <= 160 * 1024, "LDS");
    static_assert(MB * NB <= kRing * kStageBytes, "level transpose fits the ring");

    __shared__ __attribute__((aligned(1024))) uint8_t smem[kRing][kStageBytes];
    __shared__ uint32_t tap_table[kMaxUnits];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int row0 = ((int)blockIdx.x / p.tiles_n) * MB;
    const int col0 = ((int)blockIdx.x % p.tiles_n) * NB;

    // unit -> (tap << 24) | byte offset of the unit relative to the pixel's tap (0, 0)
    for (int u = tid; u < p.nstages * kUnits; u += kConvThreads) {
        uint32_t e = (uint32_t)kMaxMfmaTaps << 24;
        if (u < p.units) {
            const int kb = 16 * u, tap = (int)fdiv((uint32_t)kb, p.div_cin), c = kb - tap * p.Cin;
            const int ky = (int)fdiv((uint32_t)tap, p.div_kw), kx = tap - ky * p.kw;
            e = ((uint32_t)tap << 24) | (uint32_t)((ky * p.dil * p.W + kx * p.dil) * p.Cin + c);
        }
        tap_table[u] = e;
    }

    using Acc = typename std::conditional<FP4, v16f, v16i>::type;
    Acc acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // Direct load j of this wave fills the 1 KiB LDS chunk j * kWaves + wave = kRowsPerLoad stage rows
    // (stage rows 0..MB-1 are pixels, MB.. are output channels): loads j < LA gather activations, the
    // others read weights.  Lane l delivers row l / U, position l % U (U = kUnits), i.e. the unit
    // q = (l % U) ^ swizzle(row) of the stage; chunks start at multiples of 8 rows, so the swizzle and
    // with it q are the same for every load of the lane.
    const int lrow = lane / kUnits;                                  // row inside the chunk
    const int q = (lane % kUnits) ^ ((lrow / (8 / kUnits)) & (kUnits - 1));
    int a_off[LA];      // byte offset of the pixel's tap (0, 0) in the activation tensor (may be < 0)
    uint32_t a_mask[LA]; // bit t: tap t falls outside the image for this pixel; bit 31 always
    int w_off[LW];      // byte offset of the output channel's weights
#pragma unroll
    for (int j = 0; j < LA; ++j) {
        const int row = (j * kWaves + wave) * kRowsPerLoad + lrow;
        const int m = row0 + row < p.pixels ? row0 + row : p.pixels - 1;
        const int b = (int)fdiv((uint32_t)m, p.div_howo), rem = m - b * (int)p.div_howo.d;
        const int oy = (int)fdiv((uint32_t)rem, p.div_wo), ox = rem - oy * p.Wo;
        const int iy0 = oy * p.stride - p.pad, ix0 = ox * p.stride - p.pad;
        a_off[j] = ((b * p.H + iy0) * p.W + ix0) * p.Cin;
        // whole kernel rows / columns that fall outside the image
        uint32_t mask = 1u << kMaxMfmaTaps;
        for (int ky = 0; ky < p.kh; ++ky)
            if ((unsigned)(iy0 + ky * p.dil) >= (unsigned)p.H) mask |= p.row_taps << (ky * p.kw);
        for (int kx = 0; kx < p.kw; ++kx)
            if ((unsigned)(ix0 + kx * p.dil) >= (unsigned)p.W) mask |= p.col_taps << kx;
        a_mask[j] = mask;
    }
#pragma unroll
    for (int j = 0; j < LW; ++j) {
        const int col = ((LA + j) * kWaves + wave) * kRowsPerLoad + lrow - MB;
        w_off[j] = (col0 + col < p.Cout ? col0 + col : p.Cout - 1) * p.nk;
    }
    const uint8_t *zero = g_zero_units + 16 * (lane % kUnits);

    // load j of stage `stage` into ring buffer `buf`; `entry` = tap_table[8 stage + q]
    auto issue_one = [&](int stage, int buf, int j, uint32_t entry) {
        const uint8_t *src;
        if (j < LA) {
            const bool padded = (a_mask[j < LA ? j : 0] >> (entry >> 24)) & 1u;
            src = padded ? zero : reinterpret_cast<const uint8_t *>(p.a) + (a_off[j < LA ? j : 0] + (int)(entry & 0xffffffu));
        } else {
            const int u = stage * kUnits + q;
            src = u < p.units ? reinterpret_cast<const uint8_t *>(p.w) + (w_off[j >= LA ? j - LA : 0] + 16 * u) : zero;
        }
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                         (__attribute__((address_space(3))) void *)(smem[buf] + (j * kWaves + wave) * 1024), 16,
                                         0, 0);
    };

    // operand reads at k step ks: row = tile row + lane % 32, unit 2 ks + lane / 32, swizzled
    const int a_rd = (wm * 32 * TM + (lane & 31)) * kKB, b_rd = (MB + wn * 32 * TN + (lane & 31)) * kKB;
    const int hi = lane >> 5, swz = ((lane & 31) / (8 / kUnits)) & (kUnits - 1); // tile rows start at multiples of 32
    v4i af[2][TM], bf[2][TN];
    // operand read r of NR of k step ks into operand set b, in the order the MFMAs first need them
    auto read_one = [&](const uint8_t *st, int ks, int b, int r) {
        const int u = 16 * ((2 * ks + hi) ^ swz);
        if (r == 0) af[b][0] = *reinterpret_cast<const v4i *>(st + a_rd + u);
        else if (r <= TN) bf[b][r - 1] = *reinterpret_cast<const v4i *>(st + b_rd + (r - 1) * 32 * kKB + u);
        else af[b][r - TN] = *reinterpret_cast<const v4i *>(st + a_rd + (r - TN) * 32 * kKB + u);
    };
    // One k step: NM MFMAs on operand set b; the operand reads of the following step and (dma) the
    // direct loads of a later stage are issued one by one between them.
    auto mfma_step = [&](int b, const uint8_t *next_stage, int next_ks, auto dma, int dma_stage, int dma_buf, uint32_t entry) {
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (FP4) {
                // the builtin takes 8 registers per operand and uses the first 4 for fp4: the rest stay undefined;
                // cbsz = blgp = 4: both operands fp4; scale bytes 127 = 2^0
                const v4i x = af[b][m / TN], y = bf[b][m % TN];
                const v8i x8 = __builtin_shufflevector(x, x, 0, 1, 2, 3, -1, -1, -1, -1);
                const v8i y8 = __builtin_shufflevector(y, y, 0, 1, 2, 3, -1, -1, -1, -1);
                acc[m / TN][m % TN] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(x8, y8, acc[m / TN][m % TN], 4, 4, 0, 127, 0, 127);
            } else {
                acc[m / TN][m % TN] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[b][m / TN], bf[b][m % TN], acc[m / TN][m % TN], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int r = m; r < NR; r += NM) read_one(next_stage, next_ks, b ^ 1, r);
            if constexpr (decltype(dma)::value) {
#pragma unroll
                for (int j = m; j < L; j += NM) issue_one(dma_stage, dma_buf, j, entry);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    __syncthreads(); // tap table complete
    // prologue: request the first kRing stages, wait for stage 0, read its first operands
    for (int t = 0; t < kRing; ++t)
        if (t < p.nstages) {
            const uint32_t entry = tap_table[t * kUnits + q];
#pragma unroll
            for (int j = 0; j < L; ++j) issue_one(t, t, j, entry);
        }
    if (p.nstages > 1) QNN_CONV_WAIT_VMCNT(L);
    else QNN_CONV_WAIT_VMCNT(0);
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int r = 0; r < NR; ++r) read_one(smem[0], 0, 0, r);

    // One stage per iteration, buffer cur = s mod 2.  The barrier sits in front of the last k step:
    // by then every wave has read all of stage s (its buffer may be refilled) and this wave's loads
    // of stage s+1 have landed, so under the last step's MFMAs the first operands of stage s+1 are
    // read and stage s+2 is requested into the buffer of stage s.
    static_assert(kRing == 2, "the waits below assume two buffers");
    // The loop runs in two parts, with and without the request for stage s+2, so that each body is
    // one straight line of code whose order the scheduling barriers pin.
    int cur = 0;
    auto stage_body = [&](int s, auto dma) {
        const uint8_t *st = smem[cur];
#pragma unroll
        for (int ks = 0; ks + 1 < kSteps; ++ks) mfma_step(ks & 1, st, ks + 1, std::false_type{}, 0, 0, 0u);
        uint32_t entry = 0u;
        if constexpr (decltype(dma)::value) entry = tap_table[(s + kRing) * kUnits + q];
        QNN_CONV_WAIT_VMCNT(0);
        __builtin_amdgcn_s_waitcnt(0xC07F); // lgkmcnt(0)
        __builtin_amdgcn_s_barrier();
        // after the last stage this reads stale data that is never used (no branch around LDS reads)
        mfma_step((kSteps - 1) & 1, smem[cur ^ 1], 0, dma, s + kRing, cur, entry);
        cur ^= 1;
    };
    int s = 0;
    for (; s + kRing < p.nstages; ++s) stage_body(s, std::true_type{});
    for (; s < p.nstages; ++s) stage_body(s, std::false_type{});

    // ---- epilogue ----
    // The quantized shortcut tile (int8 [MB][NB]) is fetched into LDS with 16-byte loads and read back
    // bytewise; a lane later writes its level to the very byte it read, so the same region serves as
    // the level tile that leaves with 16-byte stores.
    const int8_t *resq = BLK ? static_cast<const int8_t *>(p.blk.res_q) : nullptr;
    uint8_t *lv = &smem[0][0]; // [MB][NB] bytes
    constexpr int kVecPerRow = NB / 16;
    if (resq || p.next) {
        // every wave is past its last LDS read (the loop's final reads are waited for here)
        __builtin_amdgcn_s_waitcnt(0xC07F);
        __syncthreads();
    }
    if (resq) {
        for (int v = tid; v < MB * kVecPerRow; v += kConvThreads) {
            const int rl = v / kVecPerRow, cv = (v % kVecPerRow) * 16;
            const int row = row0 + rl, c = col0 + cv;
            if (row >= p.pixels || c >= p.Cout) continue;
            if constexpr (FP4) {
                // the shortcut holds nibbles: expand them to int8 levels on the way into LDS (Cout is even)
                const uint8_t *src = reinterpret_cast<const uint8_t *>(resq) + ((int64_t)row * p.Cout + c) / 2;
                uint32_t nib[2] = {0u, 0u};
                if (c + 16 <= p.Cout && (p.Cout & 15) == 0) {
                    const uint2 t = *reinterpret_cast<const uint2 *>(src);
                    nib[0] = t.x, nib[1] = t.y;
                } else {
                    for (int e = 0; e < 8 && c + 2 * e < p.Cout; ++e) nib[e >> 2] |= (uint32_t)src[e] << (8 * (e & 3));
                }
                uint32_t o[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const uint32_t n = (nib[e >> 3] >> (4 * (e & 7))) & 15u;
                    const int level = ((n & 1u) ? 3 : 1) * ((n & 8u) ? -1 : 1);
                    o[e >> 2] |= ((uint32_t)level & 0xffu) << (8 * (e & 3));
                }
                *reinterpret_cast<uint4 *>(lv + rl * NB + cv) = make_uint4(o[0], o[1], o[2], o[3]);
                continue;
            }
            const int8_t *src = resq + (int64_t)row * p.Cout + c;
            if (c + 16 <= p.Cout && (p.Cout & 15) == 0) {
                *reinterpret_cast<uint4 *>(lv + rl * NB + cv) = *reinterpret_cast<const uint4 *>(src);
            } else {
                for (int e = 0; e < 16 && c + e < p.Cout; ++e) lv[rl * NB + cv + e] = (uint8_t)src[e];
            }
        }
        __syncthreads();
    }
    // scale, then the residual-block terms in their documented order (one fp32 rounding each);
    // `at`: this output's byte in the LDS tile, `o`: its element offset in the global tensors
    auto block_y = [&](int32_t v, float sc, float bi, int at, int row, int c) -> float {
        float y = (float)v * sc;
        if constexpr (BLK) {
            if (p.blk.bias) y = y + bi;
            if (resq) {
                const float term = (float)(int)(int8_t)lv[at] * p.blk.res_scale;
                y = y + term;
            }
            if (p.blk.res_f32) y = y + p.blk.res_f32[(int64_t)row * p.Cout + c];
            if (p.blk.relu) y = fmaxf(y, 0.0f);
        }
        return y;
    };

    // D layout of the 32x32 MFMA: lane holds column lane % 32 and rows 8 (r / 4) + 4 (lane / 32) + r % 4
    if (p.acc || p.out) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int cl = (wn * TN + j) * 32 + (lane & 31);
                const int c = col0 + cl;
                if (c >= p.Cout) continue;
                const float sc = p.out ? p.scale[c] : 0.0f;
                const float bi = BLK && p.out && p.blk.bias ? p.blk.bias[c] : 0.0f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int rl = (wm * TM + i) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    if (row0 + rl >= p.pixels) continue;
                    const int32_t v = (int32_t)acc[i][j][r]; // fp4: an integer-valued float
                    const int64_t o = (int64_t)(row0 + rl) * p.Cout + c;
                    if (p.acc) p.acc[o] = v;
                    if (p.out) p.out[o] = block_y(v, sc, bi, rl * NB + cl, row0 + rl, c);
                }
            }
    }
    if (p.next) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int cl = (wn * TN + j) * 32 + (lane & 31);
                const int c = col0 + cl < p.Cout ? col0 + cl : p.Cout - 1;
                const float sc = p.scale[c];
                const float bi = BLK && p.blk.bias ? p.blk.bias[c] : 0.0f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int rl = (wm * TM + i) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    // rows past the last pixel and columns past Cout are never stored: any in-range address does
                    const int row = row0 + rl < p.pixels ? row0 + rl : p.pixels - 1;
                    const float y = block_y((int32_t)acc[i][j][r], sc, bi, rl * NB + cl, row, c);
                    lv[rl * NB + cl] =
                        (uint8_t)(2 * quantize_code(y, p.next_inv_clip, p.next_half_top, p.next_top) - p.next_top);
                }
            }
    }
    if (p.next) {
        __syncthreads();
        for (int v = tid; v < MB * kVecPerRow; v += kConvThreads) {
            const int rl = v / kVecPerRow, cv = (v % kVecPerRow) * 16;
            const int row = row0 + rl, c = col0 + cv;
            if (row >= p.pixels || c >= p.Cout) continue;
            const uint4 val = *reinterpret_cast<const uint4 *>(lv + rl * NB + cv);
            const uint32_t w4[4] = {val.x, val.y, val.z, val.w};
            if constexpr (FP4) {
                // 16 levels -> 16 nibbles = 8 bytes; Cout is even (checked on the host)
                uint32_t o[2] = {0u, 0u};
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    o[e >> 3] |= fp4_nibble((int)(int8_t)(w4[e >> 2] >> (8 * (e & 3)))) << (4 * (e & 7));
                uint8_t *dst = reinterpret_cast<uint8_t *>(p.next) + ((int64_t)row * p.Cout + c) / 2;
                if (c + 16 <= p.Cout && (p.Cout & 15) == 0) {
                    *reinterpret_cast<uint2 *>(dst) = make_uint2(o[0], o[1]);
                } else {
                    for (int e = 0; e < 8 && c + 2 * e < p.Cout; ++e) dst[e] = (uint8_t)(o[e >> 2] >> (8 * (e & 3)));
                }
                continue;
            }
            int8_t *dst = p.next + (int64_t)row * p.Cout + c;
            if (c + 16 <= p.Cout && (p.Cout & 15) == 0) {
                *reinterpret_cast<uint4 *>(dst) = val;
            } else {
                for (int e = 0; e < 16 && c + e < p.Cout; ++e) dst[e] = (int8_t)(w4[e >> 2] >> (8 * (e & 3)));
            }
        }
    }
}

template <int MB_, int NB_, int WM_, int WN_, int KB_> struct BlockShape {
    static constexpr int MB = MB_, NB = NB_, WM = WM_, WN = WN_, KB = KB_;
};

template <int MB, int NB, int WM, int WN, int KB, bool FP4, bool BLK> int launch_level_conv_k(LevelConvParams &p, hipStream_t st)
{
    p.nstages = (int)ceil_div(p.nk, KB);
    const int64_t tiles_m = ceil_div(p.pixels, MB), tiles_n = ceil_div(p.Cout, NB);
    if (tiles_m * tiles_n > 0x7fffffffLL) return fail(QNN_ERR_RANGE, "qnn_level_conv2d_i8: too many tiles");
    p.tiles_n = (int)tiles_n;
    hipLaunchKernelGGL((level_conv_mfma_kernel<MB, NB, WM, WN, KB, FP4, BLK>), dim3((unsigned)(tiles_m * tiles_n)), dim3(64 * WM * WN),
                       0, st, p);
    return check_launch("qnn_level_conv2d_i8");
}

} // namespace qnn

using namespace qnn;

static int encode_levels_run(const char *who, bool fp4, const void *src, int dtype, int64_t count, float clip, int bits,
                             void *levels, void *stream)
{
    const int max_bits = fp4 ? 2 : 7;
    if (dtype != QNN_DTYPE_F32 && dtype != QNN_DTYPE_BF16)
        return fail(QNN_ERR_UNSUPPORTED, "%s: dtype %d (fp32 or bf16 only)", who, dtype);
    if (bits < 1 || bits > max_bits) return fail(QNN_ERR_INVALID_ARG, "%s: bits=%d outside [1,%d]", who, bits, max_bits);
    if (count < 0 || (fp4 && count % 2 != 0)) return fail(QNN_ERR_INVALID_ARG, "%s: bad size", who);
    if (!(clip > 0.0f && clip <= 3.0e38f)) return fail(QNN_ERR_INVALID_ARG, "%s: clip must be positive and finite", who);
    if (count == 0) return QNN_OK;
    if (!src || !levels) return fail(QNN_ERR_INVALID_ARG, "%s: NULL pointer", who);
    if (!aligned16(src) || !aligned16(levels)) return fail(QNN_ERR_ALIGNMENT, "%s: pointers must be 16-byte aligned", who);
    EncodeLevelParams p;
    p.src = src, p.count = count, p.levels = static_cast<int8_t *>(levels);
    p.top = (1 << bits) - 1;
    p.half_top = (float)p.top * 0.5f;
    p.inv_clip = 1.0f / clip;
    const int64_t blocks = ceil_div(ceil_div(count, 16), 256);
    const dim3 grid((unsigned)(blocks < 256 * 64 ? blocks : 256 * 64)), block(256);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool bf16 = dtype == QNN_DTYPE_BF16;
    if (fp4 && bf16) hipLaunchKernelGGL((encode_levels_kernel<true, true>), grid, block, 0, st, p);
    else if (fp4) hipLaunchKernelGGL((encode_levels_kernel<false, true>), grid, block, 0, st, p);
    else if (bf16) hipLaunchKernelGGL((encode_levels_kernel<true, false>), grid, block, 0, st, p);
    else hipLaunchKernelGGL((encode_levels_kernel<false, false>), grid, block, 0, st, p);
    return check_launch(who);
}

extern "C" int qnn_encode_levels_i8(const void *src, int dtype, int64_t count, float clip, int bits, int8_t *levels,
                                    void *stream)
{
    return encode_levels_run("qnn_encode_levels_i8", false, src, dtype, count, clip, bits, levels, stream);
}

extern "C" int qnn_encode_levels_fp4(const void *src, int dtype, int64_t count, float clip, int bits, uint8_t *levels,
                                     void *stream)
{
    return encode_levels_run("qnn_encode_levels_fp4", true, src, dtype, count, clip, bits, levels, stream);
}

// fp4: the operands and next_levels hold two levels per byte (1- and 2-bit codes); the kernel then sees
// Cin / 2 bytes per pixel
// check_only: every argument check, nothing enqueued (for entry points that enqueue work of their own before the
// convolution and must refuse a bad call as a whole).
static int level_conv_run(const char *who, bool fp4, const qnn_conv_desc *d, const int8_t *a_levels, const int8_t *w_levels,
                          const float *scale, const qnn_block_epilogue *epi, int32_t *acc, float *out,
                          int8_t *next_levels, float next_clip, int next_bits, void *stream, bool check_only = false,
                          int dilation = 1)
{
    const int max_bits = fp4 ? 2 : 7;
    if (!d) return fail(QNN_ERR_INVALID_ARG, "%s: NULL descriptor", who);
    BlockTerms blk;
    const int brc = block_terms(who, epi, scale, 7, blk);
    if (brc != QNN_OK) return brc;
    const int hard_bits = fp4 ? 8 : 7; // int8 levels hold 7 bits; wider fp4 requests are valid codes that fp4 cannot hold
    if (d->a_bits < 1 || d->a_bits > hard_bits || d->w_bits < 1 || d->w_bits > hard_bits)
        return fail(QNN_ERR_INVALID_ARG, "%s: bits must be in [1,%d]", who, hard_bits);
    if (d->a_bits > max_bits || d->w_bits > max_bits)
        return fail(QNN_ERR_UNSUPPORTED, "%s: more than %d bits (%s levels)", who, max_bits, fp4 ? "fp4" : "int8");
    if (fp4 && blk.res_q && (blk.res_bits > 2 || d->Cout % 2 != 0))
        return fail(QNN_ERR_UNSUPPORTED, "%s: an fp4 shortcut holds 1- or 2-bit codes of an even channel count", who);
    if (d->B < 0 || d->H <= 0 || d->W <= 0 || d->Cin <= 0 || d->Cout <= 0)
        return fail(QNN_ERR_INVALID_ARG, "%s: bad tensor size", who);
    if (d->kh < 1 || d->kw < 1 || d->stride < 1 || d->pad < 0)
        return fail(QNN_ERR_INVALID_ARG, "%s: bad kernel geometry", who);
    if (dilation < 1) return fail(QNN_ERR_INVALID_ARG, "%s: dilation must be at least 1", who);
    if (dilation > 64) return fail(QNN_ERR_UNSUPPORTED, "%s: dilation above 64", who);
    const int64_t eh = (int64_t)dilation * (d->kh - 1) + 1, ew = (int64_t)dilation * (d->kw - 1) + 1; // extent of the taps
    if (d->H + 2 * (int64_t)d->pad < eh || d->W + 2 * (int64_t)d->pad < ew)
        return fail(QNN_ERR_INVALID_ARG, "%s: kernel larger than the padded image", who);
    if (!acc && !out && !next_levels) return fail(QNN_ERR_INVALID_ARG, "%s: no output requested", who);
    if ((out || next_levels) && !scale)
        return fail(QNN_ERR_INVALID_ARG, "%s: out / next_levels given without scale", who);
    if (next_levels && (next_bits < 1 || next_bits > max_bits))
        return fail(QNN_ERR_INVALID_ARG, "%s: next_bits=%d outside [1,%d]", who, next_bits, max_bits);
    if (next_levels && !(next_clip > 0.0f && next_clip <= 3.0e38f))
        return fail(QNN_ERR_INVALID_ARG, "%s: next_clip must be positive and finite", who);
    if (d->Cin % (fp4 ? 32 : 16) != 0)
        return fail(QNN_ERR_UNSUPPORTED, "%s: Cin=%lld is not a multiple of %d", who, (long long)d->Cin, fp4 ? 32 : 16);
    if (fp4 && next_levels && d->Cout % 2 != 0)
        return fail(QNN_ERR_UNSUPPORTED, "%s: fp4 next_levels need an even Cout", who);
    const int64_t cinb = fp4 ? d->Cin / 2 : d->Cin; // bytes per pixel
    if ((int64_t)d->kh * d->kw > kMaxMfmaTaps)
        return fail(QNN_ERR_UNSUPPORTED, "%s: more than %d taps", who, kMaxMfmaTaps);
    const int64_t nk = (int64_t)d->kh * d->kw * cinb; // bytes of the reduction axis
    if (ceil_div(nk, 128) * 8 > kMaxUnits)
        return fail(QNN_ERR_UNSUPPORTED, "%s: reduction axis of %lld bytes (limit %d)", who, (long long)nk,
                    kMaxUnits * 16);
    const int64_t n = (int64_t)d->kh * d->kw * d->Cin;
    if (!acc_fits_int32(n, d->w_bits, d->a_bits))
        return fail(QNN_ERR_RANGE, "%s: reduction length %lld with %dx%d bits overflows int32", who, (long long)n,
                    d->w_bits, d->a_bits);
    if (fp4 && n * ((1 << d->w_bits) - 1) * ((1 << d->a_bits) - 1) >= (1LL << 24))
        return fail(QNN_ERR_RANGE, "%s: reduction length %lld exceeds the exact range of fp32 accumulation", who, (long long)n);
    const int64_t Ho = (d->H + 2 * (int64_t)d->pad - eh) / d->stride + 1;
    const int64_t Wo = (d->W + 2 * (int64_t)d->pad - ew) / d->stride + 1;
    // the kernel indexes both tensors and the output pixels with 32-bit integers
    if (d->H > (1 << 20) || d->W > (1 << 20) || d->B > (1LL << 31) / (d->H * d->W * cinb) - 1 ||
        d->B > ((1LL << 31) - 1025) / (Ho * Wo) || d->Cout > ((1LL << 31) - 1) / nk ||
        (eh * d->W + ew) * cinb >= (1LL << 24))
        return fail(QNN_ERR_RANGE, "%s: tensor too large for 32-bit indexing", who);
    if (d->B == 0) return QNN_OK;
    if (!a_levels || !w_levels) return fail(QNN_ERR_INVALID_ARG, "%s: NULL level pointer", who);
    if (!aligned16(a_levels) || !aligned16(w_levels) || !aligned16(acc) || !aligned16(out) || !aligned16(next_levels))
        return fail(QNN_ERR_ALIGNMENT, "%s: pointers must be 16-byte aligned", who);
    if (check_only) return QNN_OK;

    LevelConvParams p;
    p.a = a_levels, p.w = w_levels, p.scale = scale, p.acc = acc, p.out = out, p.next = next_levels;
    p.blk = blk;
    p.H = (int)d->H, p.W = (int)d->W, p.Cin = (int)cinb, p.Cout = (int)d->Cout, p.Ho = (int)Ho, p.Wo = (int)Wo;
    p.kh = d->kh, p.kw = d->kw, p.stride = d->stride, p.pad = d->pad, p.dil = dilation;
    p.pixels = (int)(d->B * Ho * Wo);
    p.nk = (int)nk, p.units = (int)(nk / 16), p.nstages = 0;
    p.tiles_n = 0;
    p.div_howo = make_fastdiv((uint32_t)(Ho * Wo)), p.div_wo = make_fastdiv((uint32_t)Wo);
    p.div_cin = make_fastdiv((uint32_t)cinb), p.div_kw = make_fastdiv((uint32_t)d->kw);
    p.row_taps = (1u << d->kw) - 1u;
    p.col_taps = 0;
    for (int ky = 0; ky < d->kh; ++ky) p.col_taps |= 1u << (ky * d->kw);
    p.next_top = next_levels ? (1 << next_bits) - 1 : 0;
    p.next_half_top = (float)p.next_top * 0.5f;
    p.next_inv_clip = next_levels ? 1.0f / next_clip : 0.0f;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // Block shape and stage length, measured per layer shape of the two stacks: up to 128 output
    // channels the reduction is short (576 .. 1152 bytes), so 64-byte stages with several small
    // workgroups per CU hide each other's prologue and epilogue; above that 256 x 256 with 128-byte
    // stages (one workgroup per CU) when its workgroups fill at least three quarters of the CU rounds
    // they take, otherwise 128 x 128 with four waves, two workgroups per CU.
    const bool terms = blk.any();
    auto go = [&](auto shape) {
        constexpr int MB = decltype(shape)::MB, NB = decltype(shape)::NB, WM = decltype(shape)::WM, WN = decltype(shape)::WN,
                      KB = decltype(shape)::KB;
        if (fp4 && terms) return launch_level_conv_k<MB, NB, WM, WN, KB, true, true>(p, st);
        if (fp4) return launch_level_conv_k<MB, NB, WM, WN, KB, true, false>(p, st);
        if (terms) return launch_level_conv_k<MB, NB, WM, WN, KB, false, true>(p, st);
        return launch_level_conv_k<MB, NB, WM, WN, KB, false, false>(p, st);
    };
    if (d->Cout <= 64) return go(BlockShape<256, 64, 4, 1, 64>{});
    if (d->Cout <= 128) return go(BlockShape<256, 128, 4, 2, 64>{});
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (cus < 1) cus = 256;
    const int64_t tiles = ceil_div(p.pixels, 256) * ceil_div(d->Cout, 256);
    if (4 * tiles >= 3 * ceil_div(tiles, cus) * cus) return go(BlockShape<256, 256, 2, 4, 128>{});
    return go(BlockShape<128, 128, 2, 2, 128>{});
}

extern "C" int qnn_level_conv2d_i8(const qnn_conv_desc *d, const int8_t *a_levels, const int8_t *w_levels,
                                   const float *scale, int32_t *acc, float *out, int8_t *next_levels,
                                   float next_clip, int next_bits, void *stream)
{
    return level_conv_run("qnn_level_conv2d_i8", false, d, a_levels, w_levels, scale, nullptr, acc, out, next_levels,
                          next_clip, next_bits, stream);
}

extern "C" int qnn_level_conv2d_dilated_i8(const qnn_conv_desc *d, int dilation, const int8_t *a_levels, const int8_t *w_levels,
                                           const float *scale, int32_t *acc, float *out, int8_t *next_levels,
                                           float next_clip, int next_bits, void *stream)
{
    return level_conv_run("qnn_level_conv2d_dilated_i8", false, d, a_levels, w_levels, scale, nullptr, acc, out, next_levels,
                          next_clip, next_bits, stream, false, dilation);
}

extern "C" int qnn_level_conv2d_dilated_fp4(const qnn_conv_desc *d, int dilation, const uint8_t *a_levels, const uint8_t *w_levels,
                                            const float *scale, int32_t *acc, float *out, uint8_t *next_levels,
                                            float next_clip, int next_bits, void *stream)
{
    return level_conv_run("qnn_level_conv2d_dilated_fp4", true, d, reinterpret_cast<const int8_t *>(a_levels),
                          reinterpret_cast<const int8_t *>(w_levels), scale, nullptr, acc, out,
                          reinterpret_cast<int8_t *>(next_levels), next_clip, next_bits, stream, false, dilation);
}

extern "C" int qnn_level_conv2d_block_i8(const qnn_conv_desc *d, const int8_t *a_levels, const int8_t *w_levels,
                                         const float *scale, const qnn_block_epilogue *epi, int32_t *acc, float *out,
                                         int8_t *next_levels, float next_clip, int next_bits, void *stream)
{
    return level_conv_run("qnn_level_conv2d_block_i8", false, d, a_levels, w_levels, scale, epi, acc, out, next_levels,
                          next_clip, next_bits, stream);
}

extern "C" int qnn_level_conv2d_fp4(const qnn_conv_desc *d, const uint8_t *a_levels, const uint8_t *w_levels,
                                    const float *scale, int32_t *acc, float *out, uint8_t *next_levels,
                                    float next_clip, int next_bits, void *stream)
{
    return level_conv_run("qnn_level_conv2d_fp4", true, d, reinterpret_cast<const int8_t *>(a_levels),
                          reinterpret_cast<const int8_t *>(w_levels), scale, nullptr, acc, out,
                          reinterpret_cast<int8_t *>(next_levels), next_clip, next_bits, stream);
}

extern "C" int qnn_level_conv2d_block_fp4(const qnn_conv_desc *d, const uint8_t *a_levels, const uint8_t *w_levels,
                                          const float *scale, const qnn_block_epilogue *epi, int32_t *acc, float *out,
                                          uint8_t *next_levels, float next_clip, int next_bits, void *stream)
{
    return level_conv_run("qnn_level_conv2d_block_fp4", true, d, reinterpret_cast<const int8_t *>(a_levels),
                          reinterpret_cast<const int8_t *>(w_levels), scale, epi, acc, out,
                          reinterpret_cast<int8_t *>(next_levels), next_clip, next_bits, stream);
}

extern "C" int qnn_levels_to_fp4(const int8_t *levels, int64_t count, uint8_t *fp4, void *stream)
{
    if (count < 0 || count % 2 != 0) return fail(QNN_ERR_INVALID_ARG, "qnn_levels_to_fp4: count must be even and >= 0");
    if (count == 0) return QNN_OK;
    if (!levels || !fp4) return fail(QNN_ERR_INVALID_ARG, "qnn_levels_to_fp4: NULL pointer");
    if (!aligned16(levels) || !aligned16(fp4)) return fail(QNN_ERR_ALIGNMENT, "qnn_levels_to_fp4: pointers must be 16-byte aligned");
    const int64_t blocks = ceil_div(ceil_div(count, 16), 256);
    hipLaunchKernelGGL(levels_to_fp4_kernel, dim3((unsigned)(blocks < 256 * 64 ? blocks : 256 * 64)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), levels, count, fp4);
    return check_launch("qnn_levels_to_fp4");
}

// ---- transposed convolution on decoded levels ----
// A transposed convolution with stride s and padding p is the stride-1 convolution of the input with s - 1 zeros
// inserted between neighbouring pixels, the kernel flipped in both axes, and padding k - 1 - p.  A zero byte is
// level 0 (int8) or two +0 values (fp4): it contributes exactly 0 to every sum, like the padding of the
// convolution itself, so the level convolution runs unchanged on the widened tensor.

namespace qnn {

struct ZeroInsertParams {
    const uint4 *a; // [B][H][W][units]
    uint4 *up;      // [B][Hu][Wu][units]
    uint32_t units, Wu, HuWu, W, HW, stride, total;
};

__global__ __launch_bounds__(256) void zero_insert_kernel(ZeroInsertParams p)
{
    for (uint32_t i = blockIdx.x * 256u + threadIdx.x; i < p.total; i += gridDim.x * 256u) {
        const uint32_t pix = i / p.units, u = i - pix * p.units;
        const uint32_t b = pix / p.HuWu, r = pix - b * p.HuWu;
        const uint32_t y = r / p.Wu, x = r - y * p.Wu;
        const uint32_t sy = y / p.stride, sx = x / p.stride;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (sy * p.stride == y && sx * p.stride == x) v = p.a[((size_t)b * p.HW + sy * p.W + sx) * p.units + u];
        p.up[i] = v;
    }
}

// flipped[co][ky][kx][:] = w[co][kh - 1 - ky][kw - 1 - kx][:], 16-byte units
__global__ __launch_bounds__(256) void flip_taps_kernel(const uint4 *w, uint4 *flipped, uint32_t units, uint32_t taps, uint32_t total)
{
    for (uint32_t i = blockIdx.x * 256u + threadIdx.x; i < total; i += gridDim.x * 256u) {
        const uint32_t ct = i / units, u = i - ct * units;
        const uint32_t co = ct / taps, t = ct - co * taps;
        flipped[i] = w[((size_t)co * taps + (taps - 1 - t)) * units + u];
    }
}

static int level_deconv_geometry(const char *who, bool fp4, const qnn_conv_desc *d, qnn_conv_desc &wide, int64_t &units)
{
    if (!d) return fail(QNN_ERR_INVALID_ARG, "%s: NULL descriptor", who);
    if (d->B < 0 || d->H <= 0 || d->W <= 0 || d->Cin <= 0 || d->Cout <= 0)
        return fail(QNN_ERR_INVALID_ARG, "%s: bad tensor size", who);
    if (d->kh < 1 || d->kw < 1 || d->stride < 1 || d->pad < 0)
        return fail(QNN_ERR_INVALID_ARG, "%s: bad kernel geometry", who);
    if (d->H > (1 << 20) || d->W > (1 << 20) || d->stride > (1 << 10))
        return fail(QNN_ERR_RANGE, "%s: tensor too large for 32-bit indexing", who);
    if ((d->H - 1) * d->stride - 2 * (int64_t)d->pad + d->kh < 1 || (d->W - 1) * d->stride - 2 * (int64_t)d->pad + d->kw < 1)
        return fail(QNN_ERR_INVALID_ARG, "%s: empty output", who);
    if (d->kh != d->kw || d->pad > d->kh - 1)
        return fail(QNN_ERR_UNSUPPORTED, "%s: the level route needs a square kernel and pad <= k - 1", who);
    if (d->Cin % (fp4 ? 32 : 16) != 0)
        return fail(QNN_ERR_UNSUPPORTED, "%s: Cin=%lld is not a multiple of %d", who, (long long)d->Cin, fp4 ? 32 : 16);
    wide = *d;
    wide.H = (d->H - 1) * d->stride + 1, wide.W = (d->W - 1) * d->stride + 1;
    wide.stride = 1, wide.pad = d->kh - 1 - d->pad;
    units = (fp4 ? d->Cin / 2 : d->Cin) / 16;
    if (wide.H > (1 << 20) || wide.W > (1 << 20) || (d->B > 0 && d->B > ((1LL << 31) - 1) / (wide.H * wide.W * units)))
        return fail(QNN_ERR_RANGE, "%s: tensor too large for 32-bit indexing", who);
    return QNN_OK;
}

static int level_deconv_run(const char *who, bool fp4, const qnn_conv_desc *d, const int8_t *a_levels, const int8_t *flipped_w,
                            void *workspace, const float *scale, const float *bias, int32_t *acc, float *out,
                            int8_t *next_levels, float next_clip, int next_bits, void *stream)
{
    qnn_conv_desc wide;
    int64_t units = 0;
    int rc = level_deconv_geometry(who, fp4, d, wide, units);
    if (rc != QNN_OK) return rc;
    qnn_block_epilogue epi = {};
    epi.bias = bias;
    const qnn_block_epilogue *e = bias ? &epi : nullptr;
    int8_t *up = static_cast<int8_t *>(workspace);
    // the convolution's own checks, on the widened tensor, before anything is enqueued
    rc = level_conv_run(who, fp4, &wide, d->B > 0 && up ? up : a_levels, flipped_w, scale, e, acc, out, next_levels,
                        next_clip, next_bits, stream, true);
    if (rc != QNN_OK) return rc;
    if (d->B == 0) return QNN_OK;
    if (!workspace) return fail(QNN_ERR_INVALID_ARG, "%s: NULL workspace", who);
    if (!aligned16(workspace) || !aligned16(a_levels)) return fail(QNN_ERR_ALIGNMENT, "%s: pointers must be 16-byte aligned", who);
    ZeroInsertParams z;
    z.a = reinterpret_cast<const uint4 *>(a_levels), z.up = reinterpret_cast<uint4 *>(up);
    z.units = (uint32_t)units, z.Wu = (uint32_t)wide.W, z.HuWu = (uint32_t)(wide.H * wide.W);
    z.W = (uint32_t)d->W, z.HW = (uint32_t)(d->H * d->W), z.stride = (uint32_t)d->stride;
    z.total = (uint32_t)(d->B * wide.H * wide.W * units);
    const int64_t blocks = ceil_div(z.total, 256);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(zero_insert_kernel, dim3((unsigned)(blocks < 256 * 32 ? blocks : 256 * 32)), dim3(256), 0, st, z);
    rc = check_launch(who);
    if (rc != QNN_OK) return rc;
    return level_conv_run(who, fp4, &wide, up, flipped_w, scale, e, acc, out, next_levels, next_clip, next_bits, stream);
}

} // namespace qnn

extern "C" int64_t qnn_level_deconv_workspace_bytes(const qnn_conv_desc *d, int fp4)
{
    qnn_conv_desc wide;
    int64_t units = 0;
    if (level_deconv_geometry("qnn_level_deconv_workspace_bytes", fp4 != 0, d, wide, units) != QNN_OK) return -1;
    return d->B * wide.H * wide.W * units * 16;
}

extern "C" int qnn_level_deconv_flip_weights(const void *w_levels, int64_t Cout, int kh, int kw, int64_t tap_bytes,
                                             void *flipped, void *stream)
{
    const char *who = "qnn_level_deconv_flip_weights";
    if (Cout <= 0 || kh < 1 || kw < 1 || tap_bytes <= 0) return fail(QNN_ERR_INVALID_ARG, "%s: bad geometry", who);
    if (tap_bytes % 16 != 0) return fail(QNN_ERR_UNSUPPORTED, "%s: a tap must be a multiple of 16 bytes", who);
    if (kh > (1 << 10) || kw > (1 << 10) || Cout > ((1LL << 31) - 1) / ((int64_t)kh * kw * (tap_bytes / 16)))
        return fail(QNN_ERR_RANGE, "%s: tensor too large for 32-bit indexing", who);
    if (!w_levels || !flipped) return fail(QNN_ERR_INVALID_ARG, "%s: NULL pointer", who);
    if (!aligned16(w_levels) || !aligned16(flipped)) return fail(QNN_ERR_ALIGNMENT, "%s: pointers must be 16-byte aligned", who);
    const uint32_t units = (uint32_t)(tap_bytes / 16), taps = (uint32_t)(kh * kw);
    const uint32_t total = (uint32_t)(Cout * taps * units);
    const int64_t blocks = ceil_div(total, 256);
    hipLaunchKernelGGL(flip_taps_kernel, dim3((unsigned)(blocks < 256 * 32 ? blocks : 256 * 32)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), reinterpret_cast<const uint4 *>(w_levels),
                       reinterpret_cast<uint4 *>(flipped), units, taps, total);
    return check_launch(who);
}

extern "C" int qnn_level_deconv2d_i8(const qnn_conv_desc *d, const int8_t *a_levels, const int8_t *flipped_w, void *workspace,
                                     const float *scale, const float *bias, int32_t *acc, float *out, int8_t *next_levels,
                                     float next_clip, int next_bits, void *stream)
{
    return level_deconv_run("qnn_level_deconv2d_i8", false, d, a_levels, flipped_w, workspace, scale, bias, acc, out,
                            next_levels, next_clip, next_bits, stream);
}

extern "C" int qnn_level_deconv2d_fp4(const qnn_conv_desc *d, const uint8_t *a_levels, const uint8_t *flipped_w, void *workspace,
                                      const float *scale, const float *bias, int32_t *acc, float *out, uint8_t *next_levels,
                                      float next_clip, int next_bits, void *stream)
{
    return level_deconv_run("qnn_level_deconv2d_fp4", true, d, reinterpret_cast<const int8_t *>(a_levels),
                            reinterpret_cast<const int8_t *>(flipped_w), workspace, scale, bias, acc, out,
                            reinterpret_cast<int8_t *>(next_levels), next_clip, next_bits, stream);
}
