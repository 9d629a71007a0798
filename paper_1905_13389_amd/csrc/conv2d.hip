// qnn_conv2d: the multi-branch binary product with the reduction axis (ky, kx, ci) gathered
// implicitly from an NHWC bit-plane tensor (paper: section "Model Decomposition", convolution
// reduces to the same vector product; Eq. 9 with Eq. 10), plus the fused epilogue
// scale -> quantize -> plane split that hands the next layer its planes (Eq. 18, Eq. 15).
//
// Zero padding.  0 is not a level of the {-1,+1} code, so a padded tap cannot be stored as bits.
// The kernel reads padded taps as all-zero words, i.e. as the lowest level -(2^AB - 1), runs the
// uniform xor + bitcount loop over the full reduction length, and then removes what those
// pretend values added:  acc += (2^AB - 1) * sum over padded taps t of S[c][t],
// S[c][t] = sum_ci w[c][t][ci] (from the weight planes: sum_i 2^i (2 bitcount(W_i) - Cin)).
// Only workgroups that own border pixels compute S.
#include "bdot_tile.h"
#include "qnn_host.h"
#include "quantize.h"
#include "fastdiv.h"

namespace qnn {

constexpr int kMaxGroups = 1024; // reduction words (or word groups) addressable through the tap table
constexpr int kMaxTaps = 32;      // tap sets are 32-bit masks
constexpr int kMaxOutExtent = 2048; // Ho + Wo entries of the border-mask tables
constexpr int kConvKB = 20; // an LDS stage holds up to 20 reduction words per row and plane

// Everything the plain kernel needs (64-bit sizes).
struct ConvParams {
    const uint32_t *a; // [AB][B][H][W][cw]
    const uint32_t *w; // [WB][Cout][kh][kw][cw]
    int64_t B, H, W, Cin, Cout, Ho, Wo;
    int kh, kw, stride, pad;
    int64_t cw, nw, M; // words per pixel, reduction words, output pixels
    int64_t a_plane_stride;
    const float *scale;
    int32_t *acc;
    float *out;
};

// The register-blocked kernel's view: 32-bit indices (checked on the host), few fields.
struct ConvTileParams {
    const uint32_t *a, *w;
    const float *scale;
    int32_t *acc;
    float *out;
    uint32_t *next; // [next_bits][M][cwo]
    int H, W, HW, Cin, Cout, M, cw, nw, cwo, Ho, Wo;
    int kh, kw, stride, pad;
    int a_plane_stride;
    uint32_t n_times_top; // kh kw Cin (2^WB-1)(2^AB-1)
    int top_a;
    int next_bits, next_top;
    float next_inv_clip, next_half_top;
    int wvec; // nw % 4 == 0
    FastDiv div_howo, div_wo;
    int tiles_m, tiles_n, row_tile_step; // persistent schedule: see bconv_tile_kernel
    int kb, nchunks;                     // reduction words per LDS stage (multiple of 4), stages per tile
    // Bit widths above 4 run as up to four launches over chunks of at most 4 planes per operand (the
    // double sum of Eq. 9 splits into chunk pairs); `shift` is the weight 2^shift of this pair,
    // `partial` the running int32 sum: read when bit 0 of partial_mode is set, written instead of the
    // outputs when bit 1 is set.
    int shift, partial_mode;
    int32_t *partial;
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

// OR of a value over each aligned group of 8 lanes (every lane of the group gets the result).
__device__ __forceinline__ uint32_t or_reduce8(uint32_t v)
{
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true);  // quad_perm [1,0,3,2]
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true);  // quad_perm [2,3,0,1]
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, true); // row_half_mirror
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
// workgroup instead of once per row tile; the two stage buffers then hold activations only.
template <int WB, int AB, int TM, int TN, int KV, int VW, bool KEEPW>
__global__ __launch_bounds__(kTileThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void
bconv_tile_kernel(ConvTileParams p)
{
    using T = Tile<WB, AB, TM, TN, KV, kConvKB>;
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
    extern __shared__ __attribute__((aligned(16))) int32_t dyn_smem[];
    int32_t *S = dyn_smem;                                                   // [taps][BN]
    uint32_t *ymask = reinterpret_cast<uint32_t *>(dyn_smem) + BN * p.kh * p.kw; // [Ho] taps whose row is outside
    uint32_t *xmask = ymask + p.Ho;                                          // [Wo] taps whose column is outside

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int col0 = ((int)blockIdx.x % p.tiles_n) * BN;
    const int rt_first = (int)blockIdx.x / p.tiles_n;
    const bool wvec = p.wvec != 0;
    const int taps = p.kh * p.kw;

    // reduction word group -> tap number and word offset from the window origin
    for (int g = tid; g * VW < p.nw; g += kTileThreads) {
        const int kword = g * VW;
        const int tap = kword / p.cw, ci = kword % p.cw;
        tap_table[g] = ((uint32_t)tap << 24) | (uint32_t)(((tap / p.kw) * p.W + tap % p.kw) * p.cw + ci);
    }
    // output row / column -> set of taps that fall outside the image
    for (int o = tid; o < p.Ho + p.Wo; o += kTileThreads) {
        uint32_t m = 0;
        if (o < p.Ho) {
            const int h0 = o * p.stride - p.pad;
            for (int ky = 0; ky < p.kh; ++ky)
                if ((unsigned)(h0 + ky) >= (unsigned)p.H) m |= ((1u << p.kw) - 1u) << (ky * p.kw);
        } else {
            const int w0 = (o - p.Ho) * p.stride - p.pad;
            for (int kx = 0; kx < p.kw; ++kx)
                if ((unsigned)(w0 + kx) >= (unsigned)p.W)
                    for (int ky = 0; ky < p.kh; ++ky) m |= 1u << (ky * p.kw + kx);
        }
        ymask[o] = m; // xmask follows ymask
    }
    // S[t][c] = sum over channels of the weight levels of tap t, from the planes
    for (int e = tid; e < BN * taps; e += kTileThreads) {
        const int t = e / BN, cl = e % BN;
        const int c = col0 + cl;
        int32_t s = 0;
        if (c < p.Cout) {
            for (int i = 0; i < WB; ++i) {
                const uint32_t *wp = p.w + ((int64_t)i * p.Cout + c) * p.nw + t * p.cw;
                int32_t cnt = 0;
                for (int k = 0; k < p.cw; ++k) cnt += __builtin_popcount(wp[k]);
                s += (2 * cnt - p.Cin) << i;
            }
        }
        S[e] = s;
    }

    // where this lane's stage units start in the activation planes, and their padded taps
    int abase[T::A_PER_THREAD];
    uint32_t apad[T::A_PER_THREAD];
    auto locate = [&](int row0) {
#pragma unroll
        for (int u = 0; u < T::A_PER_THREAD; ++u) {
            const int idx = tid + u * kTileThreads;
            const int rp = idx / UQ;
            const int m = row0 + rp % BM;
            const bool ok = (T::A_UNITS % kTileThreads == 0 || idx < T::A_UNITS) && m < p.M;
            const uint32_t mm = ok ? (uint32_t)m : 0u;
            const uint32_t b = fdiv(mm, p.div_howo), rem = mm - b * p.div_howo.d;
            const uint32_t ho = fdiv(rem, p.div_wo), wo = rem - ho * p.div_wo.d;
            apad[u] = ok ? (ymask[ho] | xmask[wo]) : 0xffffffffu;
            abase[u] = (rp / BM) * p.a_plane_stride +
                       ((int)b * p.HW + ((int)ho * p.stride - p.pad) * p.W + (int)wo * p.stride - p.pad) * p.cw;
        }
    };

    uint4 ra[T::A_PER_THREAD], rw[T::W_PER_THREAD];
    constexpr bool keep_w = KEEPW;
    bool w_staged = false;
    auto fetch = [&](int k0) {
#pragma unroll
        for (int u = 0; u < T::A_PER_THREAD; ++u) {
            const int q = (tid + u * kTileThreads) % UQ;
            ra[u] = gather4<VW>(p.a, tap_table, 4 * q < p.kb ? p.nw : 0, apad[u], abase[u], k0 + 4 * q);
        }
        if (w_staged) return;
#pragma unroll
        for (int u = 0; u < T::W_PER_THREAD; ++u) {
            const int idx = tid + u * kTileThreads;
            const int rp = idx / UQ, q = idx % UQ;
            rw[u] = make_uint4(0u, 0u, 0u, 0u);
            if ((T::W_UNITS % kTileThreads == 0 || idx < T::W_UNITS) && 4 * q < p.kb)
                rw[u] = load_rowmajor4(p.w, p.Cout, p.nw, rp / BN, col0 + rp % BN, k0 + 4 * q, wvec);
        }
    };
    auto stash = [&](int buf) {
        uint32_t *As = smem[buf], *Ws = keep_w ? w_resident : smem[buf] + T::A_WORDS;
#pragma unroll
        for (int u = 0; u < T::A_PER_THREAD; ++u) {
            const int idx = tid + u * kTileThreads;
            if (T::A_UNITS % kTileThreads == 0 || idx < T::A_UNITS)
                lds_write_unit<KV>(As + (idx / UQ) * T::BKP + 4 * (idx % UQ), ra[u]);
        }
        if (w_staged) return;
        w_staged = keep_w;
#pragma unroll
        for (int u = 0; u < T::W_PER_THREAD; ++u) {
            const int idx = tid + u * kTileThreads;
            if (T::W_UNITS % kTileThreads == 0 || idx < T::W_UNITS)
                lds_write_unit<KV>(Ws + (idx / UQ) * T::BKP + 4 * (idx % UQ), rw[u]);
        }
    };

    // this lane's 4 channels in the row-major half of the epilogue
    constexpr int LPR = BN / 4;            // lanes per pixel row
    constexpr int RPP = kTileThreads / LPR; // pixel rows per pass
    const int c4 = (tid % LPR) * 4;
    const int cidx = col0 + c4;
    const bool cols4 = cidx + 3 < p.Cout && (p.Cout & 3) == 0; // 16-byte accesses are whole and aligned
    float sc[4] = {0.f, 0.f, 0.f, 0.f};
    if (p.scale) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (cidx + e < p.Cout) sc[e] = p.scale[cidx + e];
    }

    uint32_t P[TM][TN][T::S];
    __syncthreads(); // tap_table and S are complete
    int buf = 0;
    locate(rt_first * BM);
    fetch(0);
    stash(0);
    __syncthreads();

    for (int rt = rt_first; rt < p.tiles_m; rt += p.row_tile_step) {
        const int row0 = rt * BM;
        const bool next_tile = rt + p.row_tile_step < p.tiles_m;
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
                locate((rt + p.row_tile_step) * BM);
                fetch(0);
            }
            const int left = p.nw - c * p.kb;
            const int nkq = ((left < p.kb ? left : p.kb) + KV - 1) / KV;
            tile_mac<WB, AB, TM, TN, KV, kConvKB>(smem[buf], keep_w ? w_resident : smem[buf] + T::A_WORDS, ty, tx, nkq, P);
            if (more || next_tile) stash(buf ^ 1);
            __syncthreads();
            buf ^= 1;
        }
        // stage `buf` now holds the next tile's first stage (if any); stage buf^1 is free

        // ---- epilogue, first half: recombine and hand the tile over to a row-major layout ----
        int32_t *V = reinterpret_cast<int32_t *>(&smem[buf ^ 1][0]);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int n = 0; n < TN; ++n)
                V[(ty + 16 * i) * EPI_STRIDE + tx + 16 * n] = recombine<T::S>(P[i][n], p.n_times_top);
        __syncthreads();

        // ---- second half: padding correction, stores, scale, quantize, plane split ----
#pragma unroll 1
        for (int pass = 0; pass < BM / RPP; ++pass) {
            const int rl = pass * RPP + tid / LPR;
            const int r = row0 + rl;
            const bool rvalid = r < p.M;
            const int4 vv = *reinterpret_cast<const int4 *>(V + rl * EPI_STRIDE + c4);
            int32_t v[4] = {vv.x, vv.y, vv.z, vv.w};
            // padded taps of this output pixel
            uint32_t padded = 0;
            if (rvalid) {
                const uint32_t b = fdiv((uint32_t)r, p.div_howo), rem = (uint32_t)r - b * p.div_howo.d;
                const uint32_t ho = fdiv(rem, p.div_wo), wo = rem - ho * p.div_wo.d;
                padded = ymask[ho] | xmask[wo];
            }
            if (padded) {
                int32_t corr[4] = {0, 0, 0, 0};
                for (uint32_t m = padded; m; m &= m - 1) {
                    const int4 s4 = *reinterpret_cast<const int4 *>(S + __builtin_ctz(m) * BN + c4);
                    corr[0] += s4.x, corr[1] += s4.y, corr[2] += s4.z, corr[3] += s4.w;
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] += p.top_a * corr[e];
            }
            if (p.partial_mode | p.shift) {
                const int64_t off = (int64_t)r * p.Cout + cidx;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[e] = (int32_t)((uint32_t)v[e] << p.shift);
                    if ((p.partial_mode & 1) && rvalid && cidx + e < p.Cout) v[e] += p.partial[off + e];
                }
                if (p.partial_mode & 2) {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (rvalid && cidx + e < p.Cout) p.partial[off + e] = v[e];
                    continue;
                }
            }
            float o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (float)v[e] * sc[e];
            if (rvalid) {
                const int64_t off = (int64_t)r * p.Cout + cidx;
                if (cols4) {
                    if (p.acc) *reinterpret_cast<int4 *>(p.acc + off) = make_int4(v[0], v[1], v[2], v[3]);
                    if (p.out) *reinterpret_cast<float4 *>(p.out + off) = make_float4(o[0], o[1], o[2], o[3]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (cidx + e < p.Cout) {
                            if (p.acc) p.acc[off + e] = v[e];
                            if (p.out) p.out[off + e] = o[e];
                        }
                }
            }
            if (p.next) {
                // four byte codes in one register; channels past Cout give 0 bits (pad bits are 0)
                uint32_t cw4 = 0;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t code = cidx + e < p.Cout
                                              ? (uint32_t)quantize_code(o[e], p.next_inv_clip, p.next_half_top, p.next_top)
                                              : 0u;
                    cw4 |= code << (8 * e);
                }
                const int wword = (col0 >> 5) + (tid % LPR) / 8;
                const int shift = 4 * (tid & 7);
                for (int j = 0; j < p.next_bits; ++j) {
                    // bit j of the four codes -> a nibble -> this lane's place in the 32-channel word
                    const uint32_t x = (cw4 >> j) & 0x01010101u;
                    const uint32_t word = or_reduce8((((x * 0x00204081u) >> 21) & 15u) << shift);
                    if ((tid & 7) == 0 && rvalid && wword < p.cwo)
                        p.next[((int64_t)j * p.M + r) * p.cwo + wword] = word;
                }
            }
        }
        __syncthreads(); // V's stage is about to be refilled by the next tile's pipeline
    }
}

// Any bit widths 1..8 and any reduction length: one lane per output, taps / words / plane pairs
// looped at run time, padded taps skipped (they contribute 0).  Slow and plain.
__global__ __launch_bounds__(256) void bconv_plain_kernel(ConvParams p, int w_bits, int a_bits)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= p.M * p.Cout) return;
    const int64_t m = idx / p.Cout, c = idx % p.Cout;
    const int64_t b = m / (p.Ho * p.Wo), rem = m % (p.Ho * p.Wo);
    const int h0 = (int)(rem / p.Wo) * p.stride - p.pad, w0 = (int)(rem % p.Wo) * p.stride - p.pad;
    uint32_t sum = 0;
    int64_t valid_taps = 0;
    for (int ky = 0; ky < p.kh; ++ky) {
        const int hi = h0 + ky;
        if (hi < 0 || hi >= p.H) continue;
        for (int kx = 0; kx < p.kw; ++kx) {
            const int wi = w0 + kx;
            if (wi < 0 || wi >= p.W) continue;
            ++valid_taps;
            for (int i = 0; i < w_bits; ++i) {
                const uint32_t *wp = p.w + ((int64_t)i * p.Cout + c) * p.nw + (int64_t)(ky * p.kw + kx) * p.cw;
                for (int j = 0; j < a_bits; ++j) {
                    const uint32_t *ap =
                        p.a + (int64_t)j * p.a_plane_stride + ((b * p.H + hi) * p.W + wi) * p.cw;
                    uint32_t cnt = 0;
                    for (int64_t k = 0; k < p.cw; ++k) cnt += __builtin_popcount(wp[k] ^ ap[k]);
                    sum += cnt << (i + j);
                }
            }
        }
    }
    const uint32_t top = (uint32_t)(((1 << w_bits) - 1) * ((1 << a_bits) - 1));
    const int32_t v = (int32_t)((uint32_t)(valid_taps * p.Cin) * top - 2u * sum);
    if (p.acc) p.acc[idx] = v;
    if (p.out) p.out[idx] = (float)v * p.scale[c];
}

// Workgroups resident on the whole chip for one kernel (occupancy x CU count); two host-side queries
// per launch, negligible against the launch itself.
template <typename K> static int resident_workgroups(K kernel, size_t dyn_smem)
{
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, kTileThreads, dyn_smem) != hipSuccess)
        return 0;
    return cus * per_cu;
}

// Lane tile of the convolution kernel per (w_bits, a_bits).  The kernel carries more live state
// than the GEMM (pixel coordinates, the prefetched chunk across the epilogue), so its tiles are
// smaller; the column tile stays a multiple of 32 because the fused epilogue packs whole words.
template <int WB, int AB> struct ConvPick {
    static constexpr int TM = 4, TN = (WB + AB >= 7 ? 2 : 4), KV = (WB + AB >= 6 ? 2 : 4);
};

template <int WB, int AB, int VW> static int launch_conv_vw(ConvTileParams p, hipStream_t st)
{
    using G = ConvPick<WB, AB>;
    constexpr int TN = G::TN;
    static_assert(TN % 2 == 0, "column tile must be a multiple of 32");
    using T = Tile<WB, AB, G::TM, TN, G::KV, kConvKB>;
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
    auto launch = [&](auto kernel) {
        int slots = resident_workgroups(kernel, dyn);
        if (slots <= 0) return fail(QNN_ERR_LAUNCH, "qnn_conv2d: occupancy query failed");
        // every workgroup owns one column tile; the row tiles are dealt round-robin to the
        // slots / tiles_n workgroups of that column
        int groups = slots / p.tiles_n;
        if (groups < 1) groups = 1;
        if (groups > p.tiles_m) groups = p.tiles_m;
        p.row_tile_step = groups;
        hipLaunchKernelGGL(kernel, dim3((unsigned)(groups * p.tiles_n)), dim3(kTileThreads), dyn, st, p);
        return (int)QNN_OK;
    };
    if (p.nchunks == 1) return launch(bconv_tile_kernel<WB, AB, G::TM, TN, G::KV, VW, true>);
    return launch(bconv_tile_kernel<WB, AB, G::TM, TN, G::KV, VW, false>);
}

template <int WB, int AB> static int launch_conv(const ConvTileParams &p, hipStream_t st)
{
    if (p.cw % 4 == 0) return launch_conv_vw<WB, AB, 4>(p, st);
    if (p.cw % 2 == 0) return launch_conv_vw<WB, AB, 2>(p, st);
    return launch_conv_vw<WB, AB, 1>(p, st);
}

template <int WB> static int conv_dispatch_a(int a_bits, const ConvTileParams &p, hipStream_t st)
{
    switch (a_bits) {
    case 1: return launch_conv<WB, 1>(p, st);
    case 2: return launch_conv<WB, 2>(p, st);
    case 3: return launch_conv<WB, 3>(p, st);
    default: return launch_conv<WB, 4>(p, st);
    }
}

} // namespace qnn

using namespace qnn;

extern "C" int qnn_conv2d(const qnn_conv_desc *d, const uint32_t *a_planes, const uint32_t *w_planes,
                          const float *scale, int32_t *acc, float *out, uint32_t *next_planes,
                          float next_clip, int next_bits, void *stream)
{
    if (!d) return fail(QNN_ERR_INVALID_ARG, "qnn_conv2d: NULL descriptor");
    if (d->a_bits < 1 || d->a_bits > 8 || d->w_bits < 1 || d->w_bits > 8)
        return fail(QNN_ERR_INVALID_ARG, "qnn_conv2d: bits must be in [1,8]");
    if (d->B < 0 || d->H <= 0 || d->W <= 0 || d->Cin <= 0 || d->Cout <= 0)
        return fail(QNN_ERR_INVALID_ARG, "qnn_conv2d: bad tensor size");
    if (d->kh < 1 || d->kw < 1 || d->stride < 1 || d->pad < 0)
        return fail(QNN_ERR_INVALID_ARG, "qnn_conv2d: bad kernel geometry");
    if (d->kh > 7 || d->kw > 7) return fail(QNN_ERR_UNSUPPORTED, "qnn_conv2d: kernel larger than 7x7");
    if (d->H + 2 * (int64_t)d->pad < d->kh || d->W + 2 * (int64_t)d->pad < d->kw)
        return fail(QNN_ERR_INVALID_ARG, "qnn_conv2d: kernel larger than the padded image");
    if (!acc && !out && !next_planes) return fail(QNN_ERR_INVALID_ARG, "qnn_conv2d: no output requested");
    if ((out || next_planes) && !scale)
        return fail(QNN_ERR_INVALID_ARG, "qnn_conv2d: out / next_planes given without scale");
    if (next_planes && (next_bits < 1 || next_bits > 8))
        return fail(QNN_ERR_INVALID_ARG, "qnn_conv2d: next_bits=%d outside [1,8]", next_bits);
    if (next_planes && !(next_clip > 0.0f && next_clip <= 3.0e38f))
        return fail(QNN_ERR_INVALID_ARG, "qnn_conv2d: next_clip must be positive and finite");
    if (d->H > (1 << 20) || d->W > (1 << 20) || d->Cin > (1 << 20) || d->Cout > (1 << 24))
        return fail(QNN_ERR_RANGE, "qnn_conv2d: dimension too large");
    if (d->B == 0) return QNN_OK;
    if (!a_planes || !w_planes) return fail(QNN_ERR_INVALID_ARG, "qnn_conv2d: NULL plane pointer");
    if (!aligned16(a_planes) || !aligned16(w_planes) || !aligned16(acc) || !aligned16(out) ||
        !aligned16(next_planes))
        return fail(QNN_ERR_ALIGNMENT, "qnn_conv2d: pointers must be 16-byte aligned");
    const int64_t n = (int64_t)d->kh * d->kw * d->Cin;
    if (!acc_fits_int32(n, d->w_bits, d->a_bits))
        return fail(QNN_ERR_RANGE, "qnn_conv2d: reduction length %lld with %dx%d bits overflows int32",
                    (long long)n, d->w_bits, d->a_bits);

    ConvParams p;
    p.a = a_planes;
    p.w = w_planes;
    p.B = d->B, p.H = d->H, p.W = d->W, p.Cin = d->Cin, p.Cout = d->Cout;
    p.kh = d->kh, p.kw = d->kw, p.stride = d->stride, p.pad = d->pad;
    p.Ho = (d->H + 2 * (int64_t)d->pad - d->kh) / d->stride + 1;
    p.Wo = (d->W + 2 * (int64_t)d->pad - d->kw) / d->stride + 1;
    p.cw = ceil_div(d->Cin, 32);
    p.nw = (int64_t)d->kh * d->kw * p.cw;
    if (d->B > (INT64_MAX >> 24) / (p.Ho * p.Wo)) return fail(QNN_ERR_RANGE, "qnn_conv2d: too many output pixels");
    p.M = d->B * p.Ho * p.Wo;
    p.a_plane_stride = d->B * d->H * d->W * p.cw;
    p.scale = scale;
    p.acc = acc;
    p.out = out;
    const int64_t cwo = ceil_div(d->Cout, 32);
    hipStream_t st = static_cast<hipStream_t>(stream);

    // the register-blocked kernel indexes pixels and plane words with 32-bit integers
    const bool small_index = p.M < (1LL << 29) && p.a_plane_stride * d->a_bits < (1LL << 31) &&
                             p.M * cwo < (1LL << 31) && p.Ho + p.Wo <= kMaxOutExtent &&
                             ((int64_t)d->kh * d->W + d->kw) * p.cw < (1LL << 24);
    bool done = false;
    const bool wide = d->w_bits > 4 || d->a_bits > 4;
    if (p.nw <= kMaxGroups && d->kh * d->kw <= kMaxTaps && small_index && (!wide || acc || out)) {
        ConvTileParams t;
        t.a = a_planes, t.w = w_planes, t.scale = scale, t.acc = acc, t.out = out, t.next = next_planes;
        t.H = (int)d->H, t.W = (int)d->W, t.HW = (int)(d->H * d->W), t.Cin = (int)d->Cin, t.Cout = (int)d->Cout;
        t.M = (int)p.M, t.cw = (int)p.cw, t.nw = (int)p.nw, t.cwo = (int)cwo, t.Ho = (int)p.Ho, t.Wo = (int)p.Wo;
        t.kh = d->kh, t.kw = d->kw, t.stride = d->stride, t.pad = d->pad;
        t.a_plane_stride = (int)p.a_plane_stride;
        t.top_a = t.shift = t.partial_mode = 0;
        t.n_times_top = 0;
        t.next_bits = next_planes ? next_bits : 0;
        t.next_top = next_planes ? (1 << next_bits) - 1 : 0;
        t.next_inv_clip = next_planes ? 1.0f / next_clip : 0.0f;
        t.next_half_top = (float)t.next_top * 0.5f;
        t.wvec = (p.nw % 4 == 0) ? 1 : 0;
        t.div_howo = make_fastdiv((uint32_t)(p.Ho * p.Wo));
        t.div_wo = make_fastdiv((uint32_t)p.Wo);
        t.tiles_m = t.tiles_n = t.row_tile_step = t.kb = t.nchunks = 0;
        // chunk pairs of at most 4 x 4 planes; the running sum lives in acc, or (bit for bit) in the
        // memory of out; only the last launch writes the outputs and the next layer's planes
        t.partial = acc ? acc : reinterpret_cast<int32_t *>(out);
        const int w_chunks = (d->w_bits + 3) / 4, a_chunks = (d->a_bits + 3) / 4;
        const int64_t w_plane_words = (int64_t)d->Cout * p.nw;
        int launch = 0;
        for (int cw = 0; cw < w_chunks; ++cw)
            for (int ca = 0; ca < a_chunks; ++ca, ++launch) {
                const int wb = d->w_bits - 4 * cw < 4 ? d->w_bits - 4 * cw : 4;
                const int ab = d->a_bits - 4 * ca < 4 ? d->a_bits - 4 * ca : 4;
                ConvTileParams q = t;
                q.w = w_planes + 4 * cw * w_plane_words;
                q.a = a_planes + 4 * ca * p.a_plane_stride;
                q.top_a = (1 << ab) - 1;
                q.n_times_top = (uint32_t)(n * ((1 << wb) - 1) * q.top_a);
                q.shift = 4 * (cw + ca);
                q.partial_mode = (launch > 0 ? 1 : 0) | (launch + 1 < w_chunks * a_chunks ? 2 : 0);
                int rc = QNN_OK;
                switch (wb) {
                case 1: rc = conv_dispatch_a<1>(ab, q, st); break;
                case 2: rc = conv_dispatch_a<2>(ab, q, st); break;
                case 3: rc = conv_dispatch_a<3>(ab, q, st); break;
                default: rc = conv_dispatch_a<4>(ab, q, st); break;
                }
                if (rc != QNN_OK) return rc;
                rc = check_launch("qnn_conv2d");
                if (rc != QNN_OK) return rc;
            }
        done = true;
    }
    if (!done) {
        if (next_planes)
            return fail(QNN_ERR_UNSUPPORTED,
                        "qnn_conv2d: the fused next-layer epilogue needs <= %d reduction words and <= %d taps, and "
                        "above 4 bits an acc or out buffer for the running sum",
                        kMaxGroups, kMaxTaps);
        const int64_t total = p.M * p.Cout;
        if (ceil_div(total, 256) > 0x7fffffffLL) return fail(QNN_ERR_UNSUPPORTED, "qnn_conv2d: output too large");
        hipLaunchKernelGGL(bconv_plain_kernel, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, st, p,
                           d->w_bits, d->a_bits);
    }
    return check_launch("qnn_conv2d");
}
