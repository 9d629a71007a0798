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
typedef int v16i __attribute__((ext_vector_type(16)));

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
    int8_t *levels;
};

__device__ __forceinline__ float widen_bf16(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

template <bool BF16> __global__ __launch_bounds__(256) void encode_levels_kernel(EncodeLevelParams p)
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
            o[i >> 2] |= ((uint32_t)lv & 0xffu) << (8 * (i & 3));
        }
        if (e0 + 16 <= p.count) {
            *reinterpret_cast<uint4 *>(p.levels + e0) = make_uint4(o[0], o[1], o[2], o[3]);
        } else {
            for (int i = 0; i < 16 && e0 + i < p.count; ++i) p.levels[e0 + i] = (int8_t)(o[i >> 2] >> (8 * (i & 3)));
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
template <int MB, int NB, int WM, int WN, int KB>
__global__ __launch_bounds__(64 * WM * WN) __attribute__((amdgpu_waves_per_eu(MB == 256 && NB == 64 ? 3 : 1))) void
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
            e = ((uint32_t)tap << 24) | (uint32_t)((ky * p.W + kx) * p.Cin + c);
        }
        tap_table[u] = e;
    }

    v16i acc[TM][TN];
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
            if ((unsigned)(iy0 + ky) >= (unsigned)p.H) mask |= p.row_taps << (ky * p.kw);
        for (int kx = 0; kx < p.kw; ++kx)
            if ((unsigned)(ix0 + kx) >= (unsigned)p.W) mask |= p.col_taps << kx;
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
            acc[m / TN][m % TN] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[b][m / TN], bf[b][m % TN], acc[m / TN][m % TN], 0, 0, 0);
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
    const int8_t *resq = static_cast<const int8_t *>(p.blk.res_q);
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
    auto block_y = [&](int32_t v, float sc, float bi, int at, int64_t o) -> float {
        float y = (float)v * sc;
        if (p.blk.bias) y = y + bi;
        if (resq) {
            const float term = (float)(int)(int8_t)lv[at] * p.blk.res_scale;
            y = y + term;
        }
        if (p.blk.res_f32) y = y + p.blk.res_f32[o];
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
                const float bi = p.out && p.blk.bias ? p.blk.bias[c] : 0.0f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int rl = (wm * TM + i) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    if (row0 + rl >= p.pixels) continue;
                    const int32_t v = acc[i][j][r];
                    const int64_t o = (int64_t)(row0 + rl) * p.Cout + c;
                    if (p.acc) p.acc[o] = v;
                    if (p.out) p.out[o] = block_y(v, sc, bi, rl * NB + cl, o);
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
                const float bi = p.blk.bias ? p.blk.bias[c] : 0.0f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int rl = (wm * TM + i) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    // rows past the last pixel and columns past Cout are never stored: any in-range address does
                    const int row = row0 + rl < p.pixels ? row0 + rl : p.pixels - 1;
                    const float y = block_y(acc[i][j][r], sc, bi, rl * NB + cl, (int64_t)row * p.Cout + c);
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
            int8_t *dst = p.next + (int64_t)row * p.Cout + c;
            if (c + 16 <= p.Cout && (p.Cout & 15) == 0) {
                *reinterpret_cast<uint4 *>(dst) = val;
            } else {
                const uint32_t w4[4] = {val.x, val.y, val.z, val.w};
                for (int e = 0; e < 16 && c + e < p.Cout; ++e) dst[e] = (int8_t)(w4[e >> 2] >> (8 * (e & 3)));
            }
        }
    }
}

template <int MB, int NB, int WM, int WN, int KB> int launch_level_conv(LevelConvParams &p, hipStream_t st)
{
    p.nstages = (int)ceil_div(p.nk, KB);
    const int64_t tiles_m = ceil_div(p.pixels, MB), tiles_n = ceil_div(p.Cout, NB);
    if (tiles_m * tiles_n > 0x7fffffffLL) return fail(QNN_ERR_RANGE, "qnn_level_conv2d_i8: too many tiles");
    p.tiles_n = (int)tiles_n;
    hipLaunchKernelGGL((level_conv_mfma_kernel<MB, NB, WM, WN, KB>), dim3((unsigned)(tiles_m * tiles_n)), dim3(64 * WM * WN),
                       0, st, p);
    return check_launch("qnn_level_conv2d_i8");
}

} // namespace qnn

using namespace qnn;

extern "C" int qnn_encode_levels_i8(const void *src, int dtype, int64_t count, float clip, int bits, int8_t *levels,
                                    void *stream)
{
    if (dtype != QNN_DTYPE_F32 && dtype != QNN_DTYPE_BF16)
        return fail(QNN_ERR_UNSUPPORTED, "qnn_encode_levels_i8: dtype %d (fp32 or bf16 only)", dtype);
    if (bits < 1 || bits > 7) return fail(QNN_ERR_INVALID_ARG, "qnn_encode_levels_i8: bits=%d outside [1,7]", bits);
    if (count < 0) return fail(QNN_ERR_INVALID_ARG, "qnn_encode_levels_i8: negative size");
    if (!(clip > 0.0f && clip <= 3.0e38f))
        return fail(QNN_ERR_INVALID_ARG, "qnn_encode_levels_i8: clip must be positive and finite");
    if (count == 0) return QNN_OK;
    if (!src || !levels) return fail(QNN_ERR_INVALID_ARG, "qnn_encode_levels_i8: NULL pointer");
    if (!aligned16(src) || !aligned16(levels))
        return fail(QNN_ERR_ALIGNMENT, "qnn_encode_levels_i8: pointers must be 16-byte aligned");
    EncodeLevelParams p;
    p.src = src, p.count = count, p.levels = levels;
    p.top = (1 << bits) - 1;
    p.half_top = (float)p.top * 0.5f;
    p.inv_clip = 1.0f / clip;
    const int64_t blocks = ceil_div(ceil_div(count, 16), 256);
    const dim3 grid((unsigned)(blocks < 256 * 64 ? blocks : 256 * 64)), block(256);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == QNN_DTYPE_BF16) hipLaunchKernelGGL(encode_levels_kernel<true>, grid, block, 0, st, p);
    else hipLaunchKernelGGL(encode_levels_kernel<false>, grid, block, 0, st, p);
    return check_launch("qnn_encode_levels_i8");
}

extern "C" int qnn_level_conv2d_i8(const qnn_conv_desc *d, const int8_t *a_levels, const int8_t *w_levels,
                                   const float *scale, int32_t *acc, float *out, int8_t *next_levels,
                                   float next_clip, int next_bits, void *stream)
{
    return qnn_level_conv2d_block_i8(d, a_levels, w_levels, scale, nullptr, acc, out, next_levels, next_clip, next_bits,
                                     stream);
}

extern "C" int qnn_level_conv2d_block_i8(const qnn_conv_desc *d, const int8_t *a_levels, const int8_t *w_levels,
                                         const float *scale, const qnn_block_epilogue *epi, int32_t *acc, float *out,
                                         int8_t *next_levels, float next_clip, int next_bits, void *stream)
{
    if (!d) return fail(QNN_ERR_INVALID_ARG, "qnn_level_conv2d_i8: NULL descriptor");
    BlockTerms blk;
    const int brc = block_terms("qnn_level_conv2d_block_i8", epi, scale, 7, blk);
    if (brc != QNN_OK) return brc;
    if (d->a_bits < 1 || d->a_bits > 7 || d->w_bits < 1 || d->w_bits > 7)
        return fail(QNN_ERR_INVALID_ARG, "qnn_level_conv2d_i8: bits must be in [1,7] (int8 levels)");
    if (d->B < 0 || d->H <= 0 || d->W <= 0 || d->Cin <= 0 || d->Cout <= 0)
        return fail(QNN_ERR_INVALID_ARG, "qnn_level_conv2d_i8: bad tensor size");
    if (d->kh < 1 || d->kw < 1 || d->stride < 1 || d->pad < 0)
        return fail(QNN_ERR_INVALID_ARG, "qnn_level_conv2d_i8: bad kernel geometry");
    if (d->H + 2 * (int64_t)d->pad < d->kh || d->W + 2 * (int64_t)d->pad < d->kw)
        return fail(QNN_ERR_INVALID_ARG, "qnn_level_conv2d_i8: kernel larger than the padded image");
    if (!acc && !out && !next_levels) return fail(QNN_ERR_INVALID_ARG, "qnn_level_conv2d_i8: no output requested");
    if ((out || next_levels) && !scale)
        return fail(QNN_ERR_INVALID_ARG, "qnn_level_conv2d_i8: out / next_levels given without scale");
    if (next_levels && (next_bits < 1 || next_bits > 7))
        return fail(QNN_ERR_INVALID_ARG, "qnn_level_conv2d_i8: next_bits=%d outside [1,7]", next_bits);
    if (next_levels && !(next_clip > 0.0f && next_clip <= 3.0e38f))
        return fail(QNN_ERR_INVALID_ARG, "qnn_level_conv2d_i8: next_clip must be positive and finite");
    if (d->Cin % 16 != 0)
        return fail(QNN_ERR_UNSUPPORTED, "qnn_level_conv2d_i8: Cin=%lld is not a multiple of 16", (long long)d->Cin);
    if ((int64_t)d->kh * d->kw > kMaxMfmaTaps)
        return fail(QNN_ERR_UNSUPPORTED, "qnn_level_conv2d_i8: more than %d taps", kMaxMfmaTaps);
    const int64_t nk = (int64_t)d->kh * d->kw * d->Cin;
    if (ceil_div(nk, 128) * 8 > kMaxUnits)
        return fail(QNN_ERR_UNSUPPORTED, "qnn_level_conv2d_i8: reduction axis of %lld bytes (limit %d)", (long long)nk,
                    kMaxUnits * 16);
    if (!acc_fits_int32(nk, d->w_bits, d->a_bits))
        return fail(QNN_ERR_RANGE, "qnn_level_conv2d_i8: reduction length %lld with %dx%d bits overflows int32",
                    (long long)nk, d->w_bits, d->a_bits);
    const int64_t Ho = (d->H + 2 * (int64_t)d->pad - d->kh) / d->stride + 1;
    const int64_t Wo = (d->W + 2 * (int64_t)d->pad - d->kw) / d->stride + 1;
    // the kernel indexes both tensors and the output pixels with 32-bit integers
    if (d->H > (1 << 20) || d->W > (1 << 20) || d->B > (1LL << 31) / (d->H * d->W * d->Cin) - 1 ||
        d->B * Ho * Wo >= (1LL << 31) - 1024 || d->Cout * nk >= (1LL << 31) ||
        ((int64_t)d->kh * d->W + d->kw) * d->Cin >= (1LL << 24))
        return fail(QNN_ERR_RANGE, "qnn_level_conv2d_i8: tensor too large for 32-bit indexing");
    if (d->B == 0) return QNN_OK;
    if (!a_levels || !w_levels) return fail(QNN_ERR_INVALID_ARG, "qnn_level_conv2d_i8: NULL level pointer");
    if (!aligned16(a_levels) || !aligned16(w_levels) || !aligned16(acc) || !aligned16(out) || !aligned16(next_levels))
        return fail(QNN_ERR_ALIGNMENT, "qnn_level_conv2d_i8: pointers must be 16-byte aligned");

    LevelConvParams p;
    p.a = a_levels, p.w = w_levels, p.scale = scale, p.acc = acc, p.out = out, p.next = next_levels;
    p.blk = blk;
    p.H = (int)d->H, p.W = (int)d->W, p.Cin = (int)d->Cin, p.Cout = (int)d->Cout, p.Ho = (int)Ho, p.Wo = (int)Wo;
    p.kh = d->kh, p.kw = d->kw, p.stride = d->stride, p.pad = d->pad;
    p.pixels = (int)(d->B * Ho * Wo);
    p.nk = (int)nk, p.units = (int)(nk / 16), p.nstages = 0;
    p.tiles_n = 0;
    p.div_howo = make_fastdiv((uint32_t)(Ho * Wo)), p.div_wo = make_fastdiv((uint32_t)Wo);
    p.div_cin = make_fastdiv((uint32_t)d->Cin), p.div_kw = make_fastdiv((uint32_t)d->kw);
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
    if (d->Cout <= 64) return launch_level_conv<256, 64, 4, 1, 64>(p, st);
    if (d->Cout <= 128) return launch_level_conv<256, 128, 4, 2, 64>(p, st);
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (cus < 1) cus = 256;
    const int64_t tiles = ceil_div(p.pixels, 256) * ceil_div(d->Cout, 256);
    if (4 * tiles >= 3 * ceil_div(tiles, cus) * cus) return launch_level_conv<256, 256, 2, 4, 128>(p, st);
    return launch_level_conv<128, 128, 2, 2, 128>(p, st);
}
