// The register-blocked xor + bitcount convolution kernel and its launchers, shared by the two
// translation units that instantiate it: without (conv2d.hip) and with (conv2d_block.hip) the
// residual-block terms in the epilogue.  The terms are a template parameter so that the plain
// convolution's kernels carry none of their registers or kernel arguments.
#pragma once

#include <atomic>

#include "bdot_tile.h"
#include "qnn_host.h"
#include "quantize.h"
#include "fastdiv.h"
#include "block_terms.h"

namespace qnn {

constexpr int kMaxGroups = 1024; // reduction words (or word groups) addressable through the tap table
constexpr int kMaxTaps = 32;      // tap sets are 32-bit masks
constexpr int kMaxOutExtent = 2048; // Ho + Wo entries of the border-mask tables
constexpr int kConvKB = 20; // an LDS stage holds up to 20 reduction words per row and plane

// The register-blocked kernel's view: 32-bit indices (checked on the host), few fields.
struct ConvTileParams {
    const uint32_t *a, *w;
    const float *scale;
    int32_t *acc;
    float *out;
    uint32_t *next; // [next_bits][M][cwo]
    int H, W, HW, Cin, Cout, M, cw, nw, cwo, Ho, Wo;
    int kh, kw, stride, pad;
    int dil; // distance between neighbouring taps in pixels (1: an ordinary convolution)
    int a_plane_stride;
    uint32_t n_times_top; // kh kw Cin (2^WB-1)(2^AB-1)
    int top_a;
    int next_bits, next_top;
    float next_inv_clip, next_half_top;
    int wvec; // nw % 4 == 0
    FastDiv div_howo, div_wo;
    int tiles_m, tiles_n, row_tile_step; // persistent schedule: see bconv_tile_kernel
    int kb, nchunks;                     // reduction words per LDS stage (multiple of 4), stages per tile
    // pair_hint != 0: the launch puts exactly two workgroups on every CU and they balance their progress through
    // pair_progress (see there); pair_tag tells this launch's progress words from those of earlier launches
    int pair_hint;
    uint32_t pair_tag;
#ifdef QNN_TIMELINE
    long long *timeline; // [timeline_waves][5] or nullptr
    int timeline_waves;
#endif
    // Bit widths above 4 run as up to four launches over chunks of at most 4 planes per operand (the
    // double sum of Eq. 9 splits into chunk pairs); `shift` is the weight 2^shift of this pair,
    // `partial` the running int32 sum: read when bit 0 of partial_mode is set, written instead of the
    // outputs when bit 1 is set.
    int shift, partial_mode;
    int32_t *partial;
    BlockTerms blk;
    // BLK kernels only.  Window origin per axis: (ho stride - pad_y, wo stride - pad_x), pads may be
    // negative.  With scatter != 0 the output pixel (b, ho, wo) of this launch is pixel
    // (b, ho os + oy0, wo os + ox0) of a [B][HO][WO] tensor of M_out pixels: the phases of a
    // transposed convolution interleave that way.
    int pad_y, pad_x;
    int scatter, os, oy0, ox0, HO, WO, M_out;
    // nphase > 1: one launch runs all os x os phases of a transposed convolution whose phases have the
    // same shape; workgroup b belongs to phase b / wgs_per_phase = fy os + fx, whose weights start
    // phase_words further on and whose window origin and first output coordinate per axis come
    // from the tables (pad_y, pad_x, oy0, ox0 above are then unused).
    int nphase, wgs_per_phase, phase_words;
    int ph_pad_y[8], ph_pad_x[8], ph_first_y[8], ph_first_x[8];
};

// Gather 4 consecutive reduction words of one output pixel.  VW = gcd(cw, 4) words share a tap;
// the table gives each word group its tap number and its word offset from the pixel's window
// origin; `padded` has a bit set for every tap of this pixel that lies outside the image.
template <int VW>
__device__ __forceinline__ uint4 gather4(const uint32_t *__restrict__ a, const uint32_t *tap_table, int nw,
                                         uint32_t padded, int base, int kword)
{
    uint32_t v[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int g = 0; g < 4 / VW; ++g) {
        const int kw0 = kword + g * VW;
        if (kw0 < nw) {
            const uint32_t e = tap_table[kw0 / VW];
            if (!((padded >> (e >> 24)) & 1u)) {
                const uint32_t *src = a + (base + (int)(e & 0xffffffu));
                if constexpr (VW == 4) {
                    const uint4 t = *reinterpret_cast<const uint4 *>(src);
                    v[0] = t.x, v[1] = t.y, v[2] = t.z, v[3] = t.w;
                } else if constexpr (VW == 2) {
                    const uint2 t = *reinterpret_cast<const uint2 *>(src);
                    v[2 * g] = t.x, v[2 * g + 1] = t.y;
                } else {
                    v[g] = *src;
                }
            }
        }
    }
    return make_uint4(v[0], v[1], v[2], v[3]);
}

// OR of a value over each aligned group of LANES = 4 or 8 lanes (every lane of the group gets the result).
template <int LANES> __device__ __forceinline__ uint32_t or_reduce_lanes(uint32_t v)
{
    static_assert(LANES == 4 || LANES == 8, "groups of 4 or 8 lanes");
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true);  // quad_perm [1,0,3,2]
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true);  // quad_perm [2,3,0,1]
    if constexpr (LANES == 8) v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, true); // row_half_mirror
    return v;
}

// Persistent workgroups.  Workgroup b keeps one column tile (b % tiles_n) for its whole life and
// walks the row tiles b / tiles_n, + row_tile_step, ...; the reduction stages of consecutive tiles
// form one software pipeline: while the xor + bitcount block runs on one LDS stage, the next
// stage -- of this tile or the first of the next tile -- is already on its way from global memory.
// The tap table and the per-tap weight sums S are built once per workgroup.
//
// Epilogue.  The recombined accumulators go through LDS once so that the rest runs row-major:
// one lane owns 4 consecutive channels of one pixel (16-byte loads / stores of acc, scale, out),
// rolled over the rows of the tile, and the next layer's plane words are assembled from 8 lanes'
// nibbles with three DPP ORs.
// KEEPW: the reduction fits one stage (nchunks == 1) and the weight stage is written to LDS once per
// workgroup instead of once per row tile; the two stage buffers then hold activations only.  Nothing
// else is shared between the waves then, so each wave works on a slice of a tile on its own: the tile
// rows of 4 row groups (slice s: row groups 4 s .. 4 s + 3), which it gathers into its own share of a
// stage buffer, hands over through the same share, and finishes in the row-major half of the epilogue.
// The three workgroup barriers per tile become wave-local ordering points, and the waves of a workgroup
// drift apart instead of idling together (short reductions spend a large share of a tile outside the
// xor + bitcount block).  Which slice of which tile a wave does next it takes from a counter in LDS, so
// the waves that the SIMD serves first do more of the workgroup's rows and all of them end together.
// BLK: the residual-block terms (bias, shortcut) are part of the epilogue.
// NT: lanes per workgroup.  With 256 or 512 lanes two workgroups share a CU (LDS), so 256 lanes run two waves per
// SIMD with up to 256 registers per lane and 512 lanes four waves with up to 128: the same 16 RG x 16 TN tile, each
// lane holding half as many rows, and twice as many waves to issue from while others wait.  1024 lanes (one stage
// only) are one workgroup per CU: the same four waves per SIMD behind one row counter, one prologue per CU.
// Progress words of the resident workgroups, one per workgroup: (pair_tag << 32) | reduction stages done.
// Two persistent workgroups share a CU, and a SIMD issues from its older waves first: left alone, the workgroup
// that was dispatched first gets about four issue slots out of five, finishes its row tiles long before the
// other, and the other then runs the rest of the kernel (40 % of it) with half the waves per SIMD.  Workgroups
// b and b + gridDim.x / 2 are such a pair (the dispatcher fills every CU once before it starts the second
// round).  So each workgroup publishes its stage count here after every stage, reads its partner's, and raises
// its own wave priority (s_setprio) while it is behind: both advance at the same average rate, keep four waves
// on every SIMD until the end, and the kernel ends when both do.  The words are a hint and nothing else: no
// result depends on them, a stale or foreign word (another launch's tag) only means default priorities, and a
// pairing other than the assumed one costs the balance, not correctness.  One copy per translation unit.
#ifdef QNN_TIMELINE
// Diagnostic build (libqnn_timeline.so, include/qnn_probe.h): every wave of the convolution kernel leaves the
// constant-rate counter (100 MHz) at its start, after its workgroup's prologue and at its end, its hardware ids
// and the shader-clock counter's ticks across its life, in a caller-owned buffer; the pair balance can be switched off for comparison.  The product library is
// compiled without any of this.
struct TimelineState {
    long long *buf;
    int waves, pair_hint;
};
inline TimelineState &timeline_state()
{
    static TimelineState s = {nullptr, 0, 1};
    return s;
}
#endif

constexpr int kPairSlots = 1024;
static __device__ unsigned long long pair_progress[kPairSlots];
static inline uint32_t next_pair_tag()
{
    static std::atomic<uint32_t> launches{0};
    return ++launches;
}

template <int WB, int AB, int TM, int TN, int KV, int VW, bool KEEPW, bool BLK, int NT>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(NT / 128, NT / 128))) void
bconv_tile_kernel(ConvTileParams p)
{
    using T = Tile<WB, AB, TM, TN, KV, kConvKB, NT>;
    constexpr int RG = T::RG, NW = NT / 64;
    constexpr int UQ = T::UQ;
    constexpr int BN = T::BN, BM = T::BM;
    constexpr int EPI_STRIDE = BN + 16; // the 4 rows a wave writes at once land in 4 different bank groups
    constexpr int EPI_WORDS = BM * EPI_STRIDE;
    // with the weights resident elsewhere a stage buffer holds activations only
    constexpr int STAGE_NEED = KEEPW ? T::A_WORDS : T::STAGE_WORDS;
    constexpr int STAGE_ALLOC = STAGE_NEED > EPI_WORDS ? STAGE_NEED : EPI_WORDS;
    __shared__ __attribute__((aligned(16))) uint32_t smem[2][STAGE_ALLOC];
    constexpr int W_WORDS = T::STAGE_WORDS - T::A_WORDS;
    __shared__ __attribute__((aligned(16))) uint32_t w_resident[KEEPW ? W_WORDS : 4];
    __shared__ uint32_t tap_table[kMaxGroups];
    __shared__ unsigned wave_ticket; // one stage: the next piece of this workgroup's work that no wave has taken yet
    __shared__ __attribute__((aligned(16))) float bias_lds[BLK ? BN : 4]; // the column tile's shifts (0 without)
    extern __shared__ __attribute__((aligned(16))) int32_t dyn_smem[];
    int32_t *S = dyn_smem;                                                   // [taps][BN]
    uint32_t *ymask = reinterpret_cast<uint32_t *>(dyn_smem) + BN * p.kh * p.kw; // [Ho] taps whose row is outside
    uint32_t *xmask = ymask + p.Ho;                                          // [Wo] taps whose column is outside

#ifdef QNN_TIMELINE
    const long long tl_start = __builtin_amdgcn_s_memrealtime();
    const unsigned long long tl_clock = __builtin_amdgcn_s_memtime();
    long long tl_loop = 0;
#endif
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int lane = tid & 63, wave = tid >> 6;
    constexpr int WR = BM / NW;              // tile rows of one wave; tile row ty + RG i <-> its row (ty & 3) + 4 i
    constexpr int WAVE_UNITS = AB * WR * UQ; // stage units of one wave's rows
    constexpr int A_PT = KEEPW ? (WAVE_UNITS + 63) / 64 : T::A_PER_THREAD;
    constexpr int CHUNK = STAGE_ALLOC / NW;  // a wave's share of a stage buffer (its rows' stage, then its V rows)
    static_assert(STAGE_ALLOC % (4 * NW) == 0 && CHUNK >= AB * WR * T::BKP && CHUNK >= WR * EPI_STRIDE, "wave shares");
    // ordering point between a tile's phases
    auto tile_sync = [&]() {
        if constexpr (KEEPW) {
            // a wave's LDS operations execute in order; the compiler must keep them in program order
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        } else {
            __syncthreads();
        }
    };
    // stage unit u of this lane: plane and tile row it belongs to, 4-word unit inside the row, LDS word offset
    auto unit = [&](int u, int &plane, int &trow, int &q, int &lds, int slice) {
        if constexpr (KEEPW) {
            const int idx = lane + u * 64;
            const int rp = idx / UQ, slot = rp % WR; // rp = plane * WR + row of the wave
            q = idx % UQ, plane = rp / WR;
            trow = 4 * slice + (slot & 3) + RG * (slot >> 2);
            lds = wave * CHUNK + rp * T::BKP + 4 * q;
            return WAVE_UNITS % 64 == 0 || idx < WAVE_UNITS;
        } else {
            const int idx = tid + u * NT;
            const int rp = idx / UQ;
            q = idx % UQ, plane = rp / BM, trow = rp % BM;
            lds = rp * T::BKP + 4 * q;
            return T::A_UNITS % NT == 0 || idx < T::A_UNITS;
        }
    };
    int bid = (int)blockIdx.x;
    const uint32_t *wbase = p.w;
    int pad_y = BLK ? p.pad_y : p.pad, pad_x = BLK ? p.pad_x : p.pad, oy0 = 0, ox0 = 0;
    if constexpr (BLK) {
        oy0 = p.oy0, ox0 = p.ox0;
        if (p.nphase > 1) {
            const int ph = bid / p.wgs_per_phase, fy = ph / p.os, fx = ph - fy * p.os;
            bid -= ph * p.wgs_per_phase;
            wbase += (int64_t)ph * p.phase_words;
            pad_y = p.ph_pad_y[fy], pad_x = p.ph_pad_x[fx], oy0 = p.ph_first_y[fy], ox0 = p.ph_first_x[fx];
        }
    }
    const int col0 = (bid % p.tiles_n) * BN;
    const int rt_first = bid / p.tiles_n;
    const bool wvec = p.wvec != 0;
    const int taps = p.kh * p.kw;

    if constexpr (BLK) {
        for (int e = tid; e < BN; e += NT)
            bias_lds[e] = p.blk.bias && col0 + e < p.Cout ? p.blk.bias[col0 + e] : 0.0f;
    }
    if (KEEPW && tid == 0) wave_ticket = NW; // pieces 0 .. NW-1 are the waves' first ones
    // reduction word group -> tap number and word offset from the window origin
    for (int g = tid; g * VW < p.nw; g += NT) {
        const int kword = g * VW;
        const int tap = kword / p.cw, ci = kword % p.cw;
        tap_table[g] = ((uint32_t)tap << 24) | (uint32_t)(((tap / p.kw) * p.dil * p.W + (tap % p.kw) * p.dil) * p.cw + ci);
    }
    // output row / column -> set of taps that fall outside the image
    for (int o = tid; o < p.Ho + p.Wo; o += NT) {
        uint32_t m = 0;
        if (o < p.Ho) {
            const int h0 = o * p.stride - pad_y;
            for (int ky = 0; ky < p.kh; ++ky)
                if ((unsigned)(h0 + ky * p.dil) >= (unsigned)p.H) m |= ((1u << p.kw) - 1u) << (ky * p.kw);
        } else {
            const int w0 = (o - p.Ho) * p.stride - pad_x;
            for (int kx = 0; kx < p.kw; ++kx)
                if ((unsigned)(w0 + kx * p.dil) >= (unsigned)p.W)
                    for (int ky = 0; ky < p.kh; ++ky) m |= 1u << (ky * p.kw + kx);
        }
        ymask[o] = m; // xmask follows ymask
    }
    // where this lane's stage units start in the activation planes, and their padded taps
    int abase[A_PT];
    uint32_t apad[A_PT];
    auto locate = [&](int row0, int slice) {
#pragma unroll
        for (int u = 0; u < A_PT; ++u) {
            int plane, trow, q, lds;
            const bool in_stage = unit(u, plane, trow, q, lds, slice);
            const int m = row0 + trow;
            const bool ok = in_stage && m < p.M;
            const uint32_t mm = ok ? (uint32_t)m : 0u;
            const uint32_t b = fdiv(mm, p.div_howo), rem = mm - b * p.div_howo.d;
            const uint32_t ho = fdiv(rem, p.div_wo), wo = rem - ho * p.div_wo.d;
            apad[u] = ok ? (ymask[ho] | xmask[wo]) : 0xffffffffu;
            abase[u] = plane * p.a_plane_stride +
                       ((int)b * p.HW + ((int)ho * p.stride - pad_y) * p.W + (int)wo * p.stride - pad_x) * p.cw;
        }
    };

    uint4 ra[A_PT], rw[T::W_PER_THREAD];
    constexpr bool keep_w = KEEPW;
    bool w_staged = false;
    auto fetch = [&](int k0) {
#pragma unroll
        for (int u = 0; u < A_PT; ++u) {
            int plane, trow, q, lds;
            unit(u, plane, trow, q, lds, wave);
            ra[u] = gather4<VW>(p.a, tap_table, 4 * q < p.kb ? p.nw : 0, apad[u], abase[u], k0 + 4 * q);
        }
        if (w_staged) return;
#pragma unroll
        for (int u = 0; u < T::W_PER_THREAD; ++u) {
            const int idx = tid + u * NT;
            const int rp = idx / UQ, q = idx % UQ;
            rw[u] = make_uint4(0u, 0u, 0u, 0u);
            if ((T::W_UNITS % NT == 0 || idx < T::W_UNITS) && 4 * q < p.kb)
                rw[u] = load_rowmajor4(wbase, p.Cout, p.nw, rp / BN, col0 + rp % BN, k0 + 4 * q, wvec);
        }
    };
    auto stash = [&](int buf) {
        uint32_t *As = smem[buf], *Ws = keep_w ? w_resident : smem[buf] + T::A_WORDS;
#pragma unroll
        for (int u = 0; u < A_PT; ++u) {
            int plane, trow, q, lds;
            if (unit(u, plane, trow, q, lds, wave)) lds_write_unit<KV>(As + lds, ra[u]);
        }
        if (w_staged) return;
        w_staged = keep_w;
#pragma unroll
        for (int u = 0; u < T::W_PER_THREAD; ++u) {
            const int idx = tid + u * NT;
            if (T::W_UNITS % NT == 0 || idx < T::W_UNITS)
                lds_write_unit<KV>(Ws + (idx / UQ) * T::BKP + 4 * (idx % UQ), rw[u]);
        }
    };

    // this lane's EW consecutive channels of one pixel in the row-major half of the epilogue: 8 where the tile
    // has that many outputs per lane (fewer passes, and a plane word is assembled from 4 lanes' bytes with two
    // DPP steps instead of 8 lanes' nibbles with three), else 4
    constexpr int EW = (BM * BN) / NT >= 8 ? 8 : 4;
    constexpr int EQ = EW / 4;              // 16-byte pieces per lane
    constexpr int LPR = BN / EW;            // lanes per pixel row
    constexpr int RPP = NT / LPR;           // pixel rows per pass
    constexpr int LPW = 32 / EW;            // lanes per 32-channel plane word
    static_assert(LPR <= 16 && BM % RPP == 0 && BM >= RPP, "a pass row lies inside one 16-lane row group; whole passes");
    // tile row of this lane in pass `pass`: consecutive rows, or (KEEPW) rows its own wave owns
    auto pass_row = [&](int pass, int slice) {
        return KEEPW ? 4 * slice + (ty & 3) + RG * (pass * (16 / LPR) + (tid & 15) / LPR) : pass * RPP + tid / LPR;
    };
    const int c4 = (tid % LPR) * EW;
    const int cidx = col0 + c4;
    const bool cols4 = cidx + EW - 1 < p.Cout && (p.Cout & 3) == 0; // 16-byte accesses are whole and aligned
    float sc[EW];
#pragma unroll
    for (int e = 0; e < EW; ++e) sc[e] = p.scale && cidx + e < p.Cout ? p.scale[cidx + e] : 0.f;

    const unsigned pair_half = gridDim.x >> 1;
    const unsigned pair_other = blockIdx.x < pair_half ? blockIdx.x + pair_half : blockIdx.x - pair_half;
    const bool second_of_pair = blockIdx.x >= pair_half;
    unsigned pair_steps = 0;          // reduction stages this workgroup has done
    unsigned long long pair_seen = 0; // the partner's word as of one stage ago
    if (p.pair_hint && tid == 0)
        __hip_atomic_store(&pair_progress[blockIdx.x], (unsigned long long)p.pair_tag << 32, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);

    // This workgroup's work as a sequence of pieces.  Streamed reductions: piece k is row tile rt_first + k step,
    // done by all waves together.  One stage, where every wave gathers, multiplies and finishes rows of its own:
    // piece j is the rows of slice j % NW of row tile rt_first + (j / NW) step, and a wave that is through with a
    // piece takes the next one from a counter in LDS -- a SIMD serves its older waves first, so with fixed shares
    // the younger waves of a workgroup ended several microseconds after the others and ran the tail alone.
    auto piece_rt = [&](int piece) { return rt_first + (KEEPW ? piece / NW : piece) * p.row_tile_step; };
    auto piece_slice = [&](int piece) { return KEEPW ? piece % NW : wave; };
    auto next_piece = [&](int piece) {
        if constexpr (KEEPW) {
            unsigned t = 0;
            if (lane == 0) t = __hip_atomic_fetch_add(&wave_ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            return (int)__builtin_amdgcn_readfirstlane((int)t);
        } else {
            return piece + 1;
        }
    };

    uint32_t P[TM][TN][T::S];
    __syncthreads(); // tap_table, the masks and the counter are complete
    int buf = 0;
    int piece = KEEPW ? wave : 0; // row tile rt_first exists (the grid has at most one workgroup per tile)
    locate(piece_rt(piece) * BM, piece_slice(piece));
    fetch(0);
    // S[t][c] = sum over channels of the weight levels of tap t, from the planes; its loads travel with those of
    // the first stage, which are already requested
    for (int e = tid; e < BN * taps; e += NT) {
        const int t = e / BN, cl = e % BN;
        const int c = col0 + cl;
        int32_t s = 0;
        if (c < p.Cout) {
            for (int i = 0; i < WB; ++i) {
                const uint32_t *wp = wbase + ((int64_t)i * p.Cout + c) * p.nw + t * p.cw;
                int32_t cnt = 0;
                for (int k = 0; k < p.cw; ++k) cnt += __builtin_popcount(wp[k]);
                s += (2 * cnt - p.Cin) << i;
            }
        }
        S[e] = s;
    }
    stash(0);
    __syncthreads(); // S and the first stage are complete

#ifdef QNN_TIMELINE
    tl_loop = __builtin_amdgcn_s_memrealtime();
#endif
    while (piece_rt(piece) < p.tiles_m) {
        const int row0 = piece_rt(piece) * BM, slice = piece_slice(piece);
        const int piece_after = next_piece(piece);
        const bool next_tile = piece_rt(piece_after) < p.tiles_m;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int n = 0; n < TN; ++n)
#pragma unroll
                for (int s = 0; s < T::S; ++s) P[i][n][s] = 0u;

        for (int c = 0; c < p.nchunks; ++c) {
            const bool more = c + 1 < p.nchunks;
            if (more) {
                fetch((c + 1) * p.kb);
            } else if (next_tile) {
                locate(piece_rt(piece_after) * BM, piece_slice(piece_after));
                fetch(0);
            }
            const int left = p.nw - c * p.kb;
            const int words = left < p.kb ? left : p.kb;
            // up to 4 planes in all, a stage that ends 1 or 2 words into a 4-word group finishes with a 2-word
            // group (with more planes the lane has no registers left for that second copy of the block)
            constexpr bool HALF = KV == 4 && WB + AB <= 4;
            const bool half_tail = HALF && ((words & 3) == 1 || (words & 3) == 2);
            const int nkq = half_tail ? words / KV : (words + KV - 1) / KV;
            if constexpr (KEEPW)
                tile_mac<WB, AB, TM, TN, KV, kConvKB, WR, 4, HALF>(smem[buf] + wave * CHUNK, w_resident, ty & 3, tx, nkq, P,
                                                                  half_tail);
            else
                tile_mac<WB, AB, TM, TN, KV, kConvKB, BM, RG, HALF>(smem[buf], smem[buf] + T::A_WORDS, ty, tx, nkq, P,
                                                                   half_tail);
            if (more || next_tile) stash(buf ^ 1);
            tile_sync();
            buf ^= 1;
            if (p.pair_hint) {
                // behind the partner (as of its word read one stage ago): issue first; level or ahead: default.
                // A tie goes to the second workgroup of the pair, the first has its age.
                // progress: stages done, or (one stage) pieces the workgroup's waves had taken when this wave last took one
                if constexpr (KEEPW) pair_steps = (unsigned)piece_after;
                else ++pair_steps;
                const unsigned seen_tag = (unsigned)__builtin_amdgcn_readfirstlane((int)(pair_seen >> 32));
                const unsigned seen_steps = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)pair_seen);
                // (one stage: compared in whole tiles, the unit the partner reports in)
                const unsigned mine = KEEPW ? pair_steps / NW : pair_steps, theirs = KEEPW ? seen_steps / NW : seen_steps;
                if (seen_tag == p.pair_tag && (mine < theirs || (mine == theirs && second_of_pair)))
                    __builtin_amdgcn_s_setprio(1);
                else
                    __builtin_amdgcn_s_setprio(0);
                // one stage: the wave that took a tile's first piece reports
                if (KEEPW ? lane == 0 && pair_steps % NW == 0 : tid == 0) {
                    __hip_atomic_store(&pair_progress[blockIdx.x], ((unsigned long long)p.pair_tag << 32) | pair_steps,
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                pair_seen = __hip_atomic_load(&pair_progress[pair_other], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        // stage `buf` now holds the next tile's first stage (if any); stage buf^1 is free

        // ---- epilogue, first half: recombine and hand the tile over to a row-major layout ----
        int32_t *V = reinterpret_cast<int32_t *>(&smem[buf ^ 1][0]) + (KEEPW ? wave * CHUNK : 0);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int n = 0; n < TN; ++n)
                V[(KEEPW ? (ty & 3) + 4 * i : ty + RG * i) * EPI_STRIDE + tx + 16 * n] =
                    recombine<T::S>(P[i][n], p.n_times_top);
        // this lane's EW bits of the 32-channel plane word its channels belong to
        const int wword = (col0 >> 5) + (tid % LPR) / LPW;
        const int nib_shift = EW * (tid & (LPW - 1));
        // The shortcut operands of all passes are requested here, in one go, now that the partial sums
        // no longer occupy registers: one memory latency per tile, hidden behind the barrier, the
        // LDS reads and the other resident workgroup, instead of one per pass.
        constexpr int NPASS = BM / RPP;
        uint32_t rq_pre[BLK ? NPASS : 1][8];
        float4 rf_pre[BLK ? NPASS : 1][EQ];
        if constexpr (BLK) {
            const uint32_t *rq = static_cast<const uint32_t *>(p.blk.res_q);
#pragma unroll
            for (int ps = 0; ps < NPASS; ++ps) {
                const int r = row0 + pass_row(ps, slice);
                const bool rvalid = r < p.M;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    rq_pre[ps][j] = 0u;
                    if (rq && rvalid && wword < p.cwo && j < p.blk.res_bits)
                        rq_pre[ps][j] = rq[((int64_t)j * p.M + r) * p.cwo + wword];
                }
#pragma unroll
                for (int q = 0; q < EQ; ++q) {
                    rf_pre[ps][q] = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (p.blk.res_f32 && rvalid) {
                        const float *src = p.blk.res_f32 + ((int64_t)r * p.Cout + cidx + 4 * q);
                        if (cols4) {
                            rf_pre[ps][q] = *reinterpret_cast<const float4 *>(src);
                        } else {
                            if (cidx + 4 * q + 0 < p.Cout) rf_pre[ps][q].x = src[0];
                            if (cidx + 4 * q + 1 < p.Cout) rf_pre[ps][q].y = src[1];
                            if (cidx + 4 * q + 2 < p.Cout) rf_pre[ps][q].z = src[2];
                            if (cidx + 4 * q + 3 < p.Cout) rf_pre[ps][q].w = src[3];
                        }
                    }
                }
            }
        }
        tile_sync();

        // ---- second half: padding correction, stores, scale, quantize, plane split ----
        auto do_pass = [&](const int pass, const uint32_t (&rqw)[8], const float4 (&rf)[EQ]) {
            const int rl = pass_row(pass, slice);
            const int r = row0 + rl;
            const bool rvalid = r < p.M;
            int32_t v[EW];
#pragma unroll
            for (int q = 0; q < EQ; ++q) {
                const int4 vv = *reinterpret_cast<const int4 *>(V + (KEEPW ? (rl & 3) + 4 * (rl / RG) : rl) * EPI_STRIDE + c4 + 4 * q);
                v[4 * q] = vv.x, v[4 * q + 1] = vv.y, v[4 * q + 2] = vv.z, v[4 * q + 3] = vv.w;
            }
            // padded taps of this output pixel
            uint32_t padded = 0;
            int64_t ro = r, Mo = p.M; // pixel index in the output tensors, their pixel count
            if (rvalid) {
                const uint32_t b = fdiv((uint32_t)r, p.div_howo), rem = (uint32_t)r - b * p.div_howo.d;
                const uint32_t ho = fdiv(rem, p.div_wo), wo = rem - ho * p.div_wo.d;
                padded = ymask[ho] | xmask[wo];
                if constexpr (BLK) {
                    if (p.scatter) {
                        ro = ((int64_t)b * p.HO + (ho * p.os + oy0)) * p.WO + (wo * p.os + ox0);
                        Mo = p.M_out;
                    }
                }
            }
            if (padded) {
                int32_t corr[EW];
#pragma unroll
                for (int e = 0; e < EW; ++e) corr[e] = 0;
                for (uint32_t m = padded; m; m &= m - 1) {
#pragma unroll
                    for (int q = 0; q < EQ; ++q) {
                        const int4 s4 = *reinterpret_cast<const int4 *>(S + __builtin_ctz(m) * BN + c4 + 4 * q);
                        corr[4 * q] += s4.x, corr[4 * q + 1] += s4.y, corr[4 * q + 2] += s4.z, corr[4 * q + 3] += s4.w;
                    }
                }
#pragma unroll
                for (int e = 0; e < EW; ++e) v[e] += p.top_a * corr[e];
            }
            if (p.partial_mode | p.shift) {
                const int64_t off = ro * p.Cout + cidx;
#pragma unroll
                for (int e = 0; e < EW; ++e) {
                    v[e] = (int32_t)((uint32_t)v[e] << p.shift);
                    if ((p.partial_mode & 1) && rvalid && cidx + e < p.Cout) v[e] += p.partial[off + e];
                }
                if (p.partial_mode & 2) {
#pragma unroll
                    for (int e = 0; e < EW; ++e)
                        if (rvalid && cidx + e < p.Cout) p.partial[off + e] = v[e];
                    return;
                }
            }
            float o[EW];
#pragma unroll
            for (int e = 0; e < EW; ++e) o[e] = (float)v[e] * sc[e];
            // residual-block terms, in the documented order (one fp32 rounding each)
            if constexpr (BLK) {
                if (p.blk.bias) {
#pragma unroll
                    for (int q = 0; q < EQ; ++q) {
                        const float4 bi = *reinterpret_cast<const float4 *>(bias_lds + c4 + 4 * q);
                        o[4 * q] = o[4 * q] + bi.x, o[4 * q + 1] = o[4 * q + 1] + bi.y;
                        o[4 * q + 2] = o[4 * q + 2] + bi.z, o[4 * q + 3] = o[4 * q + 3] + bi.w;
                    }
                }
                if (p.blk.res_q) {
                    uint32_t code[EW];
#pragma unroll
                    for (int e = 0; e < EW; ++e) code[e] = 0u;
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        if (j < p.blk.res_bits) {
                            const uint32_t nib = rqw[j] >> nib_shift;
#pragma unroll
                            for (int e = 0; e < EW; ++e) code[e] |= ((nib >> e) & 1u) << j;
                        }
                    }
#pragma unroll
                    for (int e = 0; e < EW; ++e) {
                        const float term = (float)(2 * (int)code[e] - p.blk.res_top) * p.blk.res_scale;
                        o[e] = o[e] + term;
                    }
                }
                if (p.blk.res_f32) {
#pragma unroll
                    for (int q = 0; q < EQ; ++q) {
                        o[4 * q] = o[4 * q] + rf[q].x, o[4 * q + 1] = o[4 * q + 1] + rf[q].y;
                        o[4 * q + 2] = o[4 * q + 2] + rf[q].z, o[4 * q + 3] = o[4 * q + 3] + rf[q].w;
                    }
                }
                if (p.blk.relu) {
#pragma unroll
                    for (int e = 0; e < EW; ++e) o[e] = fmaxf(o[e], 0.0f);
                }
            }
            if (rvalid) {
                const int64_t off = ro * p.Cout + cidx;
                if (cols4) {
#pragma unroll
                    for (int q = 0; q < EQ; ++q) {
                        if (p.acc) *reinterpret_cast<int4 *>(p.acc + off + 4 * q) = make_int4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
                        if (p.out) *reinterpret_cast<float4 *>(p.out + off + 4 * q) = make_float4(o[4 * q], o[4 * q + 1], o[4 * q + 2], o[4 * q + 3]);
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < EW; ++e)
                        if (cidx + e < p.Cout) {
                            if (p.acc) p.acc[off + e] = v[e];
                            if (p.out) p.out[off + e] = o[e];
                        }
                }
            }
            if (p.next) {
                // byte codes, four to a register; channels past Cout give 0 bits (pad bits are 0)
                uint32_t cw4[EQ];
#pragma unroll
                for (int q = 0; q < EQ; ++q) {
                    cw4[q] = 0;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const uint32_t code = cols4 || cidx + 4 * q + e < p.Cout
                                                  ? (uint32_t)quantize_code(o[4 * q + e], p.next_inv_clip, p.next_half_top, p.next_top)
                                                  : 0u;
                        cw4[q] |= code << (8 * e);
                    }
                }
                for (int j = 0; j < p.next_bits; ++j) {
                    // bit j of the lane's codes -> EW bits -> this lane's place in the 32-channel word
                    uint32_t piece = 0;
#pragma unroll
                    for (int q = 0; q < EQ; ++q) {
                        const uint32_t x = (cw4[q] >> j) & 0x01010101u;
                        piece |= (((x * 0x00204081u) >> 21) & 15u) << (4 * q);
                    }
                    const uint32_t word = or_reduce_lanes<LPW>(piece << nib_shift);
                    if ((tid & (LPW - 1)) == 0 && rvalid && wword < p.cwo)
                        p.next[((int64_t)j * Mo + ro) * p.cwo + wword] = word;
                }
            }
        };
        if constexpr (BLK) {
#pragma unroll
            for (int pass = 0; pass < NPASS; ++pass) do_pass(pass, rq_pre[pass], rf_pre[pass]);
        } else {
#pragma unroll 1
            for (int pass = 0; pass < NPASS; ++pass) do_pass(pass, rq_pre[0], rf_pre[0]);
        }
        tile_sync(); // V's stage is about to be refilled by the next tile's pipeline
        piece = piece_after;
    }
#ifdef QNN_TIMELINE
    {
        const long long tl_end = __builtin_amdgcn_s_memrealtime();
        const int w = (int)blockIdx.x * NW + wave;
        if (p.timeline && lane == 0 && w < p.timeline_waves) {
            unsigned xcc = 0, hwid = 0;
            asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
            asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hwid));
            long long *t = p.timeline + 5 * (int64_t)w;
            t[0] = tl_start, t[1] = tl_loop, t[2] = tl_end, t[3] = ((long long)xcc << 32) | hwid;
            t[4] = (long long)(__builtin_amdgcn_s_memtime() - tl_clock);
        }
    }
#endif
}

// Workgroups resident on the whole chip for one kernel (occupancy x CU count); two host-side queries
// per launch, negligible against the launch itself.
template <typename K> static int resident_workgroups(K kernel, int threads, size_t dyn_smem, int *cu_count = nullptr)
{
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, dyn_smem) != hipSuccess)
        return 0;
    if (cu_count) *cu_count = cus;
    return cus * per_cu;
}

// Lane tile, LDS read width and workgroup size of the convolution kernel, by the number of planes WB + AB and by
// whether the reduction is one LDS stage (at most kConvKB words: the 64-channel 3x3 layers) or streamed in several.
// Measured per layer shape of the benchmark stacks against the other candidates (tiles of 1..4 x 1..4 outputs per
// lane, 8- and 16-byte LDS reads, 256 and 512 lanes).  512 lanes put four waves on a SIMD: a wave issues at most
// one instruction every four to five cycles, so two resident waves leave the SIMD idle whenever one of them
// waits, and the streamed reductions gain 5 .. 24 % from the two extra waves; the lane tiles shrink to stay
// inside 128 registers.  The column tile stays a multiple of 32 channels because the fused epilogue packs whole
// plane words.
// One-stage picks, measured again with the pair balance in place (which took away most of what 512 lanes lost to
// the 256-lane tiles): 2 or 3 planes in all 2 x 4 outputs per lane (-19 .. -25 % against 1 x 4 at 64 -> 64 @56x56,
// batch 256); 4 planes 1 x 4, or 2 x 4 when every resident workgroup has about ten or more 64-row tiles (-3 % at 2x2
// bit, -10 % at 1x3 bit for batch 256; +5 .. +20 % with fewer tiles than that: kOneStageTallTiles); 5 planes 2 x 4
// with 8-byte LDS reads (-7 .. -13 % against 4 x 4 at 256 lanes); 6 planes stay at 4 x 4 on 256 lanes (2 x 4 at 512
// lanes: +1 % at 3x3 bit, +6 % at 2x4 bit); 7 and 8 planes 1 x 4 (2 x 4: +10 %).
// With the waves of a workgroup taking their pieces from a counter (see the kernel), one workgroup of 1024 lanes per
// CU -- sixteen waves behind one counter, the prologue once per CU -- became worth its while for 2 and for 6 planes
// (at the sustained clock, 64 -> 64 @56x56, batch 256: 1x1 bit 103 -> 93 us, 3x3 bit 480 -> 444 us with 2 x 4 outputs
// per lane in place of 4 x 4 at 256 lanes); 3, 4, 5 and 8 planes are as fast or faster at 512 lanes (config 3: 70 us
// against 78 .. 94).
template <int WB, int AB> struct ConvPickOneStage { // (TM, TN, KV, NT)
    static constexpr int S = WB + AB;
    static constexpr int TM = S <= 3 ? 2 : S == 4 ? 1 : S <= 6 ? 2 : 1;
    static constexpr int TN = 4;
    static constexpr int KV = S <= 4 ? 4 : 2;
    static constexpr int NT = S == 2 || S == 6 ? 1024 : 512;
};
// 4 planes in all and many row tiles per workgroup
template <int WB, int AB> struct ConvPickOneStageTall {
    static constexpr int TM = 2, TN = 4, KV = 4, NT = 512;
};
constexpr int64_t kOneStageTallTiles = 10; // 64-row tiles per resident workgroup from which the taller tile pays
// Streamed picks.  7 and 8 planes in all: 2 x 2 outputs per lane and 8-byte LDS reads, the shape the GEMM uses at 4x4 bit;
// its two stage buffers take 60 KB, so two workgroups share a CU (four waves per SIMD, balanced as a pair), where the
// 2 x 4 tile's 80 KB left room for one: -2 .. -6 % on the 4x4-bit layers of the detection stack, -16 % at 4x3 bit.
template <int WB, int AB> struct ConvPickStreamed {
    static constexpr int S = WB + AB;
    static constexpr int TM = 2;
    static constexpr int TN = S <= 4 ? 4 : 2;
    static constexpr int KV = S <= 4 ? 2 : S <= 6 ? 4 : 2;
    static constexpr int NT = 512;
};

template <int WB, int AB, int VW, bool BLK, class G, bool ONE_STAGE>
static int launch_conv_vw(ConvTileParams p, hipStream_t st)
{
    constexpr int TN = G::TN;
    static_assert(TN % 2 == 0, "column tile must be a multiple of 32");
    constexpr int NT = G::NT;
    using T = Tile<WB, AB, G::TM, TN, G::KV, kConvKB, NT>;
    static_assert(T::BM * (T::BN / 4) >= NT, "the row-major half of the epilogue needs at least one pass");
    const size_t dyn = ((size_t)T::BN * p.kh * p.kw + p.Ho + p.Wo) * sizeof(int32_t);
    p.tiles_m = (int)ceil_div(p.M, T::BM);
    p.tiles_n = (int)ceil_div(p.Cout, T::BN);
    // stage length: of the multiples of 4 up to the stage capacity, the one whose last stage is
    // longest (the last stage of a tile hides the first fetch of the next tile); ties -> fewer stages
    int best_kb = 4, best_last = 0;
    for (int kb = 4; kb <= kConvKB; kb += 4) {
        const int nch = (int)ceil_div(p.nw, kb);
        const int last = p.nw - (nch - 1) * kb;
        if (last >= best_last) best_last = last, best_kb = kb;
    }
    p.kb = best_kb;
    p.nchunks = (int)ceil_div(p.nw, best_kb);
    if (ONE_STAGE != (p.nchunks == 1)) return fail(QNN_ERR_LAUNCH, "qnn_conv2d: stage plan does not match the kernel");
    auto kernel = bconv_tile_kernel<WB, AB, G::TM, TN, G::KV, VW, ONE_STAGE, BLK, NT>;
    int cus = 0;
    int slots = resident_workgroups(kernel, NT, dyn, &cus);
    if (slots <= 0) return fail(QNN_ERR_LAUNCH, "qnn_conv2d: occupancy query failed");
    // every workgroup owns one column tile; the row tiles are dealt round-robin to the
    // slots / tiles_n workgroups of that column
    const int phases = BLK && p.nphase > 1 ? p.nphase : 1; // phases of one launch share the slots
    int groups = slots / (p.tiles_n * phases);
    if (groups < 1) groups = 1;
    if (groups > p.tiles_m) groups = p.tiles_m;
    p.row_tile_step = groups;
    p.wgs_per_phase = groups * p.tiles_n;
    const int grid = groups * p.tiles_n * phases;
    p.pair_hint = grid == 2 * cus && grid <= kPairSlots;
    p.pair_tag = next_pair_tag();
#ifdef QNN_TIMELINE
    p.timeline = timeline_state().buf, p.timeline_waves = timeline_state().waves;
    p.pair_hint = p.pair_hint && timeline_state().pair_hint;
#endif
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(NT), dyn, st, p);
    return (int)QNN_OK;
}

template <int WB, int AB, bool BLK, class G, bool ONE_STAGE>
static int launch_conv_tile(const ConvTileParams &p, hipStream_t st)
{
    if (p.cw % 4 == 0) return launch_conv_vw<WB, AB, 4, BLK, G, ONE_STAGE>(p, st);
    if (p.cw % 2 == 0) return launch_conv_vw<WB, AB, 2, BLK, G, ONE_STAGE>(p, st);
    return launch_conv_vw<WB, AB, 1, BLK, G, ONE_STAGE>(p, st);
}

template <int WB, int AB, bool BLK> static int launch_conv(const ConvTileParams &p, hipStream_t st)
{
    // a reduction of at most kConvKB words is one stage (the stage length chosen above is then kConvKB)
    if (p.nw <= kConvKB) {
        if constexpr (WB + AB == 4) {
            int dev = 0, cus = 0;
            if (hipGetDevice(&dev) == hipSuccess &&
                hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0 &&
                ceil_div(p.M, 64) * ceil_div(p.Cout, 64) >= kOneStageTallTiles * 2 * cus)
                return launch_conv_tile<WB, AB, BLK, ConvPickOneStageTall<WB, AB>, true>(p, st);
        }
        return launch_conv_tile<WB, AB, BLK, ConvPickOneStage<WB, AB>, true>(p, st);
    }
    return launch_conv_tile<WB, AB, BLK, ConvPickStreamed<WB, AB>, false>(p, st);
}

template <int WB, bool BLK> static int conv_dispatch_a(int a_bits, const ConvTileParams &p, hipStream_t st)
{
    switch (a_bits) {
    case 1: return launch_conv<WB, 1, BLK>(p, st);
    case 2: return launch_conv<WB, 2, BLK>(p, st);
    case 3: return launch_conv<WB, 3, BLK>(p, st);
    default: return launch_conv<WB, 4, BLK>(p, st);
    }
}

// wb, ab in 1..4
template <bool BLK> static int conv_dispatch(int wb, int ab, const ConvTileParams &p, hipStream_t st)
{
    switch (wb) {
    case 1: return conv_dispatch_a<1, BLK>(ab, p, st);
    case 2: return conv_dispatch_a<2, BLK>(ab, p, st);
    case 3: return conv_dispatch_a<3, BLK>(ab, p, st);
    default: return conv_dispatch_a<4, BLK>(ab, p, st);
    }
}

// conv_dispatch<true>, compiled in its own translation unit
int conv_tiles_block(int wb, int ab, const ConvTileParams &p, hipStream_t st);

} // namespace qnn
