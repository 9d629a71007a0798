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

namespace qnn {

constexpr int kMaxGroups = 1024; // reduction words (or word groups) addressable through the tap table
constexpr int kMaxTaps = 49;

struct ConvParams {
    const uint32_t *a; // [AB][B][H][W][cw]
    const uint32_t *w; // [WB][Cout][kh][kw][cw]
    int64_t B, H, W, Cin, Cout, Ho, Wo;
    int kh, kw, stride, pad;
    int64_t cw, nw, M; // words per pixel, reduction words, output pixels
    int64_t a_plane_stride;
    uint32_t n_times_top; // kh kw Cin (2^WB-1)(2^AB-1)
    int top_a;
    const float *scale;
    int32_t *acc;
    float *out;
    uint32_t *next; // [next_bits][M][cwo]
    int next_bits, next_top;
    float next_inv_clip, next_half_top;
    int64_t cwo;
    int wvec; // nw % 4 == 0
    int64_t tiles_n, nblocks;
};

// gather 4 consecutive reduction words of one output pixel; VW = gcd(cw, 4) words share a tap
template <int VW>
__device__ __forceinline__ uint4 gather4(const ConvParams &p, const uint32_t *__restrict__ plane,
                                         const uint32_t *tap_table, bool row_ok, int64_t pix_base,
                                         int hi0, int wi0, int64_t kword)
{
    uint32_t v[4] = {0u, 0u, 0u, 0u};
    if (row_ok) {
#pragma unroll
        for (int g = 0; g < 4 / VW; ++g) {
            const int64_t kw0 = kword + g * VW;
            if (kw0 < p.nw) {
                const uint32_t e = tap_table[kw0 / VW];
                const int ky = (int)(e >> 24), kx = (int)((e >> 16) & 255), ci = (int)(e & 0xffff);
                const int hi = hi0 + ky, wi = wi0 + kx;
                if (hi >= 0 && hi < p.H && wi >= 0 && wi < p.W) {
                    const uint32_t *src = plane + (pix_base + (int64_t)hi * p.W + wi) * p.cw + ci;
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
    }
    return make_uint4(v[0], v[1], v[2], v[3]);
}

template <int WB, int AB, int TM, int TN, int KV, int VW>
__global__ __launch_bounds__(kTileThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void
bconv_tile_kernel(ConvParams p)
{
    using T = Tile<WB, AB, TM, TN, KV>;
    __shared__ __attribute__((aligned(16))) uint32_t smem[2][T::STAGE_WORDS];
    __shared__ uint32_t tap_table[kMaxGroups];

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int64_t tile = xcd_band_remap(blockIdx.x, p.nblocks);
    const int64_t row0 = (tile / p.tiles_n) * T::BM;
    const int64_t col0 = (tile % p.tiles_n) * T::BN;
    const bool wvec = p.wvec != 0;
    const int taps = p.kh * p.kw;

    // reduction word group -> (ky, kx, first channel word)
    for (int64_t g = tid; g * VW < p.nw; g += kTileThreads) {
        const int64_t kword = g * VW;
        const int tap = (int)(kword / p.cw), ci = (int)(kword % p.cw);
        tap_table[g] = ((uint32_t)(tap / p.kw) << 24) | ((uint32_t)(tap % p.kw) << 16) | (uint32_t)ci;
    }

    // the output pixels this lane fetches for the workgroup (fixed for the whole reduction)
    int hi0[T::A_PER_THREAD], wi0[T::A_PER_THREAD];
    int64_t pbase[T::A_PER_THREAD];
    bool rok[T::A_PER_THREAD];
#pragma unroll
    for (int u = 0; u < T::A_PER_THREAD; ++u) {
        const int idx = tid + u * kTileThreads;
        const int64_t m = row0 + (idx >> 2) % T::BM;
        rok[u] = (T::A_UNITS % kTileThreads == 0 || idx < T::A_UNITS) && m < p.M;
        const int64_t mm = rok[u] ? m : 0;
        const int64_t b = mm / (p.Ho * p.Wo), rem = mm % (p.Ho * p.Wo);
        hi0[u] = (int)(rem / p.Wo) * p.stride - p.pad;
        wi0[u] = (int)(rem % p.Wo) * p.stride - p.pad;
        pbase[u] = b * p.H * p.W;
    }

    uint32_t P[TM][TN][T::S];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int n = 0; n < TN; ++n)
#pragma unroll
            for (int s = 0; s < T::S; ++s) P[i][n][s] = 0u;

    uint4 ra[T::A_PER_THREAD], rw[T::W_PER_THREAD];
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int u = 0; u < T::A_PER_THREAD; ++u) {
            const int idx = tid + u * kTileThreads;
            const int plane = (idx >> 2) / T::BM;
            ra[u] = gather4<VW>(p, p.a + (int64_t)plane * p.a_plane_stride, tap_table, rok[u], pbase[u],
                                hi0[u], wi0[u], k0 + 4 * (idx & 3));
        }
#pragma unroll
        for (int u = 0; u < T::W_PER_THREAD; ++u) {
            const int idx = tid + u * kTileThreads;
            const int rp = idx >> 2;
            rw[u] = make_uint4(0u, 0u, 0u, 0u);
            if (T::W_UNITS % kTileThreads == 0 || idx < T::W_UNITS)
                rw[u] = load_rowmajor4(p.w, p.Cout, p.nw, rp / T::BN, col0 + rp % T::BN,
                                       k0 + 4 * (idx & 3), wvec);
        }
    };
    auto stash = [&](int buf) {
        uint32_t *As = smem[buf], *Ws = smem[buf] + T::A_WORDS;
#pragma unroll
        for (int u = 0; u < T::A_PER_THREAD; ++u) {
            const int idx = tid + u * kTileThreads;
            if (T::A_UNITS % kTileThreads == 0 || idx < T::A_UNITS)
                *reinterpret_cast<uint4 *>(As + (idx >> 2) * kBKP + 4 * (idx & 3)) = ra[u];
        }
#pragma unroll
        for (int u = 0; u < T::W_PER_THREAD; ++u) {
            const int idx = tid + u * kTileThreads;
            if (T::W_UNITS % kTileThreads == 0 || idx < T::W_UNITS)
                *reinterpret_cast<uint4 *>(Ws + (idx >> 2) * kBKP + 4 * (idx & 3)) = rw[u];
        }
    };

    __syncthreads(); // tap_table
    const int64_t nchunks = (p.nw + kBK - 1) / kBK;
    fetch(0);
    stash(0);
    __syncthreads();
    for (int64_t c = 0; c < nchunks; ++c) {
        const int buf = (int)(c & 1);
        const bool more = c + 1 < nchunks;
        if (more) fetch((c + 1) * kBK);
        tile_mac<WB, AB, TM, TN, KV>(smem[buf], smem[buf] + T::A_WORDS, ty, tx, P);
        if (more) stash(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue.  The staging buffers are free now and are reused for S and for codes. ----
    // padded-tap mask of each of this lane's rows
    uint64_t padmask[TM];
    bool any_pad = false;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        padmask[i] = 0;
        const int64_t m = row0 + ty + 16 * i;
        if (m < p.M) {
            const int64_t rem = m % (p.Ho * p.Wo);
            const int h0 = (int)(rem / p.Wo) * p.stride - p.pad, w0 = (int)(rem % p.Wo) * p.stride - p.pad;
            for (int t = 0; t < taps; ++t) {
                const int hi = h0 + t / p.kw, wi = w0 + t % p.kw;
                if (hi < 0 || hi >= p.H || wi < 0 || wi >= p.W) padmask[i] |= (uint64_t)1 << t;
            }
            any_pad |= padmask[i] != 0;
        }
    }
    int32_t *S = reinterpret_cast<int32_t *>(&smem[0][0]); // [BN][taps]
    const bool block_pad = __syncthreads_or(any_pad ? 1 : 0) != 0;
    if (block_pad) {
        for (int e = tid; e < T::BN * taps; e += kTileThreads) {
            const int cl = e / taps, t = e % taps;
            const int64_t c = col0 + cl;
            int32_t s = 0;
            if (c < p.Cout) {
                for (int i = 0; i < WB; ++i) {
                    const uint32_t *wp = p.w + ((int64_t)i * p.Cout + c) * p.nw + (int64_t)t * p.cw;
                    int32_t cnt = 0;
                    for (int64_t k = 0; k < p.cw; ++k) cnt += __builtin_popcount(wp[k]);
                    s += (2 * cnt - (int32_t)p.Cin) << i;
                }
            }
            S[e] = s;
        }
        __syncthreads();
    }

    uint8_t *codes = reinterpret_cast<uint8_t *>(&smem[1][0]); // [BM][BN]
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int64_t r = row0 + ty + 16 * i;
#pragma unroll
        for (int n = 0; n < TN; ++n) {
            const int cl = tx + 16 * n;
            const int64_t cidx = col0 + cl;
            const bool ok = r < p.M && cidx < p.Cout;
            int32_t v = recombine<T::S>(P[i][n], p.n_times_top);
            if (ok && padmask[i]) {
                int32_t corr = 0;
                for (uint64_t mbits = padmask[i]; mbits; mbits &= mbits - 1)
                    corr += S[cl * taps + __builtin_ctzll(mbits)];
                v += p.top_a * corr;
            }
            float o = 0.0f;
            if (ok) {
                if (p.acc) p.acc[r * p.Cout + cidx] = v;
                if (p.scale) o = (float)v * p.scale[cidx];
                if (p.out) p.out[r * p.Cout + cidx] = o;
            }
            if (p.next)
                codes[(ty + 16 * i) * T::BN + cl] =
                    ok ? (uint8_t)quantize_code(o, p.next_inv_clip, p.next_half_top, p.next_top) : (uint8_t)0;
        }
    }

    if (p.next) {
        // plane split of the staged codes: one lane builds one 32-channel word of every plane
        static_assert(T::BN % 32 == 0, "the fused epilogue packs whole words");
        constexpr int WPR = T::BN / 32;
        __syncthreads();
        for (int e = tid; e < T::BM * WPR; e += kTileThreads) {
            const int rl = e / WPR, wc = e % WPR;
            const int64_t r = row0 + rl;
            const int64_t wword = col0 / 32 + wc;
            if (r >= p.M || wword >= p.cwo) continue;
            const uint32_t *src = reinterpret_cast<const uint32_t *>(codes + rl * T::BN + wc * 32);
            uint32_t d[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) d[q] = src[q];
            for (int j = 0; j < p.next_bits; ++j) {
                uint32_t word = 0;
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    // bit j of four byte codes -> four adjacent bits
                    const uint32_t x = (d[q] >> j) & 0x01010101u;
                    word |= ((x * 0x00204081u >> 21) & 15u) << (4 * q);
                }
                p.next[((int64_t)j * p.M + r) * p.cwo + wword] = word;
            }
        }
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

template <int WB, int AB> static void launch_conv(ConvParams p, hipStream_t st)
{
    using G = TilePick<WB, AB>;
    // the fused epilogue packs whole 32-channel words, so the column tile is a multiple of 32
    constexpr int TN = G::TN % 2 == 0 ? G::TN : G::TN + 1;
    using T = Tile<WB, AB, G::TM, TN, G::KV>;
    const int64_t tiles_m = ceil_div(p.M, T::BM);
    p.tiles_n = ceil_div(p.Cout, T::BN);
    p.nblocks = tiles_m * p.tiles_n;
    const dim3 grid((unsigned)p.nblocks), block(kTileThreads);
    if (p.cw % 4 == 0)
        hipLaunchKernelGGL((bconv_tile_kernel<WB, AB, G::TM, TN, G::KV, 4>), grid, block, 0, st, p);
    else if (p.cw % 2 == 0)
        hipLaunchKernelGGL((bconv_tile_kernel<WB, AB, G::TM, TN, G::KV, 2>), grid, block, 0, st, p);
    else
        hipLaunchKernelGGL((bconv_tile_kernel<WB, AB, G::TM, TN, G::KV, 1>), grid, block, 0, st, p);
}

template <int WB> static bool conv_dispatch_a(int a_bits, const ConvParams &p, hipStream_t st)
{
    switch (a_bits) {
    case 1: launch_conv<WB, 1>(p, st); return true;
    case 2: launch_conv<WB, 2>(p, st); return true;
    case 3: launch_conv<WB, 3>(p, st); return true;
    case 4: launch_conv<WB, 4>(p, st); return true;
    default: return false;
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
    const int top_w = (1 << d->w_bits) - 1;
    p.top_a = (1 << d->a_bits) - 1;
    p.n_times_top = (uint32_t)(n * top_w * p.top_a);
    p.scale = scale;
    p.acc = acc;
    p.out = out;
    p.next = next_planes;
    p.next_bits = next_planes ? next_bits : 0;
    p.next_top = next_planes ? (1 << next_bits) - 1 : 0;
    p.next_inv_clip = next_planes ? 1.0f / next_clip : 0.0f;
    p.next_half_top = (float)p.next_top * 0.5f;
    p.cwo = ceil_div(d->Cout, 32);
    p.wvec = (p.nw % 4 == 0) ? 1 : 0;
    p.tiles_n = p.nblocks = 0;
    hipStream_t st = static_cast<hipStream_t>(stream);

    bool done = false;
    if (p.nw <= kMaxGroups && d->kh * d->kw <= kMaxTaps) {
        switch (d->w_bits) {
        case 1: done = conv_dispatch_a<1>(d->a_bits, p, st); break;
        case 2: done = conv_dispatch_a<2>(d->a_bits, p, st); break;
        case 3: done = conv_dispatch_a<3>(d->a_bits, p, st); break;
        case 4: done = conv_dispatch_a<4>(d->a_bits, p, st); break;
        default: break;
        }
    }
    if (!done) {
        if (next_planes)
            return fail(QNN_ERR_UNSUPPORTED,
                        "qnn_conv2d: the fused next-layer epilogue needs bits <= 4 and <= %d reduction words",
                        kMaxGroups);
        const int64_t total = p.M * p.Cout;
        if (ceil_div(total, 256) > 0x7fffffffLL) return fail(QNN_ERR_UNSUPPORTED, "qnn_conv2d: output too large");
        hipLaunchKernelGGL(bconv_plain_kernel, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, st, p,
                           d->w_bits, d->a_bits);
    }
    return check_launch("qnn_conv2d");
}
