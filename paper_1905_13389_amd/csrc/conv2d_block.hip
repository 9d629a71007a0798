// The convolution kernels of conv2d_tile.h with the extended epilogue compiled in: the residual-block
// terms (bias, shortcut) that qnn_conv2d_block launches when it is given any, and the scattered
// output with per-axis signed window origins that the phases of a transposed convolution need.
//
// qnn_deconv2d.  Transposed convolution (paper: section "Model Decomposition", deconvolution layers
// reduce to the same vector products): out[y][x] = sum over (i, ky), (j, kx) with
// i s + ky - p = y, j s + kx - p = x of a[i][j] . w[ky][kx].  For a fixed y only the taps
// ky = fy + t s (fy = (y + p) mod s) take part, and with q = (y + p - fy) / s the sum runs over
// a[q - t] w[fy + t s]: a stride-1 convolution of the input with the sub-kernel of phase fy, flipped.
// So the s x s phases are ordinary runs of the tile kernel, each on its own sub-kernel (gathered once
// by qnn_deconv_pack_weights), each writing every s-th output pixel per axis: one launch with the
// resident workgroups divided among the phases when all phases have one shape, else one launch each.
#include "conv2d_tile.h"

namespace qnn {

int conv_tiles_block(int wb, int ab, const ConvTileParams &p, hipStream_t st) { return conv_dispatch<true>(wb, ab, p, st); }

// Words of one phase's sub-kernel planes [w_bits][Cout][ty][tx][cw], rounded up to a multiple of 4 so
// that every phase starts 16-byte aligned.
__host__ __device__ inline int64_t phase_words(int w_bits, int64_t Cout, int ty, int tx, int cw)
{
    return ((int64_t)w_bits * Cout * ty * tx * cw + 3) / 4 * 4;
}

__host__ __device__ inline int phase_taps(int f, int k, int s) { return f < k ? (k - f + s - 1) / s : 0; }

// One axis of one phase: taps, first output coordinate, outputs, window origin.
struct PhaseAxis {
    int taps, first, count, pad;
};

static PhaseAxis phase_axis(int f, int k, int s, int p, int64_t out_extent)
{
    PhaseAxis a;
    a.taps = phase_taps(f, k, s);
    a.first = ((f - p) % s + s) % s;                                   // smallest y >= 0 with (y + p) mod s == f
    a.count = a.first < out_extent ? (int)((out_extent - a.first + s - 1) / s) : 0;
    const int q_min = (a.first + p - f) / s;                           // exact, >= 0
    a.pad = (a.taps - 1) - q_min;                                      // window of output q' starts at q' - pad
    return a;
}

struct DeconvPackParams {
    const uint32_t *w;
    uint32_t *out;
    int64_t Cout, total; // total = words per plane
    int w_bits, kh, kw, cw, s;
};

// One lane per (plane, output channel, tap, word) of the source; its word goes to the tap's place
// in the (flipped) sub-kernel of the tap's phase.
__global__ __launch_bounds__(256) void deconv_pack_weights_kernel(DeconvPackParams p)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x, all = p.total * p.w_bits;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < all; idx += stride) {
        const int c = (int)(idx % p.cw);
        int64_t t = idx / p.cw;
        const int kx = (int)(t % p.kw);
        t /= p.kw;
        const int ky = (int)(t % p.kh);
        t /= p.kh;
        const int64_t co = t % p.Cout;
        const int i = (int)(t / p.Cout);
        const int fy = ky % p.s, fx = kx % p.s;
        const int Ty = phase_taps(fy, p.kh, p.s), Tx = phase_taps(fx, p.kw, p.s);
        // words of all phases before (fy, fx): phases are stored one after another in (fy, fx) order,
        // each as [w_bits][Cout][Ty][Tx][cw]
        int64_t before = 0;
        for (int gy = 0; gy < p.s; ++gy)
            for (int gx = 0; gx < p.s; ++gx) {
                if (gy * p.s + gx >= fy * p.s + fx) break;
                before += phase_words(p.w_bits, p.Cout, phase_taps(gy, p.kh, p.s), phase_taps(gx, p.kw, p.s), p.cw);
            }
        const int u = Ty - 1 - (ky - fy) / p.s, v = Tx - 1 - (kx - fx) / p.s; // flipped position
        p.out[before + ((((int64_t)i * p.Cout + co) * Ty + u) * Tx + v) * p.cw + c] = p.w[idx];
    }
}

} // namespace qnn

using namespace qnn;

extern "C" int64_t qnn_deconv_phase_words(int w_bits, int64_t Cout, int kh, int kw, int64_t Cin, int stride)
{
    if (w_bits < 1 || w_bits > 8 || Cout <= 0 || Cin <= 0 || kh < 1 || kw < 1 || stride < 1 || kh > 16 || kw > 16 ||
        stride > 8 || Cin > (1 << 20) || Cout > (1 << 24))
        return -1;
    int64_t words = 0;
    for (int fy = 0; fy < stride; ++fy)
        for (int fx = 0; fx < stride; ++fx)
            words += phase_words(w_bits, Cout, phase_taps(fy, kh, stride), phase_taps(fx, kw, stride), (int)ceil_div(Cin, 32));
    return words;
}

extern "C" int qnn_deconv_pack_weights(const uint32_t *w_planes, int w_bits, int64_t Cout, int kh, int kw, int64_t Cin,
                                       int stride, uint32_t *phase_planes, void *stream)
{
    if (w_bits < 1 || w_bits > 8) return fail(QNN_ERR_INVALID_ARG, "qnn_deconv_pack_weights: bits=%d outside [1,8]", w_bits);
    if (Cout <= 0 || Cin <= 0 || kh < 1 || kw < 1 || stride < 1)
        return fail(QNN_ERR_INVALID_ARG, "qnn_deconv_pack_weights: bad size");
    if (kh > 16 || kw > 16 || stride > 8 || Cin > (1 << 20) || Cout > (1 << 24))
        return fail(QNN_ERR_UNSUPPORTED, "qnn_deconv_pack_weights: kernel, stride or channel count too large");
    if (!w_planes || !phase_planes) return fail(QNN_ERR_INVALID_ARG, "qnn_deconv_pack_weights: NULL pointer");
    if (!aligned16(w_planes) || !aligned16(phase_planes))
        return fail(QNN_ERR_ALIGNMENT, "qnn_deconv_pack_weights: pointers must be 16-byte aligned");
    DeconvPackParams p;
    p.w = w_planes, p.out = phase_planes, p.Cout = Cout, p.w_bits = w_bits, p.kh = kh, p.kw = kw, p.s = stride;
    p.cw = (int)ceil_div(Cin, 32);
    p.total = Cout * kh * kw * p.cw;
    const int64_t blocks = ceil_div(p.total * w_bits, 256);
    hipLaunchKernelGGL(deconv_pack_weights_kernel, dim3((unsigned)(blocks < 65536 ? blocks : 65536)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), p);
    return check_launch("qnn_deconv_pack_weights");
}

extern "C" int qnn_deconv2d(const qnn_conv_desc *d, const uint32_t *a_planes, const uint32_t *phase_planes,
                            const float *scale, const float *bias, int32_t *acc, float *out, uint32_t *next_planes,
                            float next_clip, int next_bits, void *stream)
{
    if (!d) return fail(QNN_ERR_INVALID_ARG, "qnn_deconv2d: NULL descriptor");
    if (d->a_bits < 1 || d->a_bits > 8 || d->w_bits < 1 || d->w_bits > 8)
        return fail(QNN_ERR_INVALID_ARG, "qnn_deconv2d: bits must be in [1,8]");
    if ((d->a_bits > 4 || d->w_bits > 4) && !acc && !out)
        return fail(QNN_ERR_UNSUPPORTED, "qnn_deconv2d: above 4 bits an acc or out buffer is needed for the running sum of the plane chunks");
    if (d->B < 0 || d->H <= 0 || d->W <= 0 || d->Cin <= 0 || d->Cout <= 0)
        return fail(QNN_ERR_INVALID_ARG, "qnn_deconv2d: bad tensor size");
    if (d->kh < 1 || d->kw < 1 || d->stride < 1 || d->pad < 0) return fail(QNN_ERR_INVALID_ARG, "qnn_deconv2d: bad kernel geometry");
    const int s = d->stride;
    if (d->kh < s || d->kw < s)
        return fail(QNN_ERR_UNSUPPORTED, "qnn_deconv2d: kernel smaller than the stride (output pixels no tap reaches)");
    if (d->kh > 16 || d->kw > 16 || s > 8) return fail(QNN_ERR_UNSUPPORTED, "qnn_deconv2d: kernel or stride too large");
    const int64_t HO = (d->H - 1) * s - 2 * (int64_t)d->pad + d->kh, WO = (d->W - 1) * s - 2 * (int64_t)d->pad + d->kw;
    if (HO < 1 || WO < 1) return fail(QNN_ERR_INVALID_ARG, "qnn_deconv2d: pad leaves no output");
    if (!acc && !out && !next_planes) return fail(QNN_ERR_INVALID_ARG, "qnn_deconv2d: no output requested");
    if ((out || next_planes || bias) && !scale) return fail(QNN_ERR_INVALID_ARG, "qnn_deconv2d: out / next_planes / bias given without scale");
    if (next_planes && (next_bits < 1 || next_bits > 8))
        return fail(QNN_ERR_INVALID_ARG, "qnn_deconv2d: next_bits=%d outside [1,8]", next_bits);
    if (next_planes && !(next_clip > 0.0f && next_clip <= 3.0e38f))
        return fail(QNN_ERR_INVALID_ARG, "qnn_deconv2d: next_clip must be positive and finite");
    if (d->H > (1 << 20) || d->W > (1 << 20) || d->Cin > (1 << 20) || d->Cout > (1 << 24))
        return fail(QNN_ERR_RANGE, "qnn_deconv2d: dimension too large");
    const int64_t cw = ceil_div(d->Cin, 32), cwo = ceil_div(d->Cout, 32);
    const int Tmax_y = (d->kh + s - 1) / s, Tmax_x = (d->kw + s - 1) / s;
    if (!acc_fits_int32((int64_t)Tmax_y * Tmax_x * d->Cin, d->w_bits, d->a_bits))
        return fail(QNN_ERR_RANGE, "qnn_deconv2d: reduction length overflows int32");
    if (d->B == 0) return QNN_OK;
    if (!a_planes || !phase_planes) return fail(QNN_ERR_INVALID_ARG, "qnn_deconv2d: NULL plane pointer");
    if (!aligned16(a_planes) || !aligned16(phase_planes) || !aligned16(acc) || !aligned16(out) || !aligned16(next_planes) ||
        !aligned16(bias))
        return fail(QNN_ERR_ALIGNMENT, "qnn_deconv2d: pointers must be 16-byte aligned");
    if (d->B > (1LL << 29) / (HO * WO) || d->B * d->H * d->W * cw * d->a_bits >= (1LL << 31) ||
        d->B * HO * WO * cwo >= (1LL << 31) || HO + WO > kMaxOutExtent || ((int64_t)Tmax_y * d->W + Tmax_x) * cw >= (1LL << 24) ||
        (int64_t)Tmax_y * Tmax_x * cw > kMaxGroups || Tmax_y * Tmax_x > kMaxTaps)
        return fail(QNN_ERR_UNSUPPORTED, "qnn_deconv2d: tensor or sub-kernel too large for the tiled kernel");

    hipStream_t st = static_cast<hipStream_t>(stream);
    ConvTileParams t = {};
    t.dil = 1;
    t.a = a_planes, t.scale = scale, t.acc = acc, t.out = out, t.next = next_planes;
    t.H = (int)d->H, t.W = (int)d->W, t.HW = (int)(d->H * d->W), t.Cin = (int)d->Cin, t.Cout = (int)d->Cout;
    t.cw = (int)cw, t.cwo = (int)cwo;
    t.stride = 1, t.pad = 0;
    t.a_plane_stride = (int)(d->B * d->H * d->W * cw);
    t.next_bits = next_planes ? next_bits : 0;
    t.next_top = next_planes ? (1 << next_bits) - 1 : 0;
    t.next_inv_clip = next_planes ? 1.0f / next_clip : 0.0f;
    t.next_half_top = (float)t.next_top * 0.5f;
    t.blk.bias = bias;
    t.scatter = 1, t.os = s, t.HO = (int)HO, t.WO = (int)WO, t.M_out = (int)(d->B * HO * WO);
    t.nphase = 1;
    // All phases for one chunk pair of planes (w_bits, a_bits <= 4: the only pair): wb x ab planes starting at
    // weight plane w0 and activation plane a0, entering the running sum with weight 2^shift.
    auto run_phases = [&](int wb, int ab, int w0, int a0, int shift, int partial_mode) -> int {
        ConvTileParams base = t;
        base.a = a_planes + (int64_t)a0 * t.a_plane_stride;
        base.top_a = (1 << ab) - 1;
        base.shift = shift, base.partial_mode = partial_mode;
        base.partial = acc ? acc : reinterpret_cast<int32_t *>(out);
        const int64_t top = (int64_t)((1 << wb) - 1) * base.top_a;
        // Phases of one shape (kernel extents and output extents multiples of the stride: the usual
        // upsampling layers) run as one launch, the resident workgroups divided among them.
        if (s > 1 && d->kh % s == 0 && d->kw % s == 0 && HO % s == 0 && WO % s == 0) {
            const PhaseAxis ay0 = phase_axis(0, d->kh, s, d->pad, HO), ax0 = phase_axis(0, d->kw, s, d->pad, WO);
            const int64_t words = phase_words(d->w_bits, d->Cout, ay0.taps, ax0.taps, (int)cw);
            if (words * s * s < (1LL << 31)) {
                ConvTileParams q = base;
                q.nphase = s * s, q.phase_words = (int)words;
                for (int f = 0; f < s; ++f) {
                    const PhaseAxis ay = phase_axis(f, d->kh, s, d->pad, HO), ax = phase_axis(f, d->kw, s, d->pad, WO);
                    q.ph_pad_y[f] = ay.pad, q.ph_first_y[f] = ay.first, q.ph_pad_x[f] = ax.pad, q.ph_first_x[f] = ax.first;
                }
                q.kh = ay0.taps, q.kw = ax0.taps;
                q.nw = (int)(ay0.taps * ax0.taps * cw);
                q.w = phase_planes + (int64_t)w0 * d->Cout * q.nw; // plane w0 of every phase (phases are phase_words apart)
                q.wvec = q.nw % 4 == 0 ? 1 : 0;
                q.Ho = ay0.count, q.Wo = ax0.count, q.M = (int)(d->B * ay0.count * ax0.count);
                q.n_times_top = (uint32_t)((int64_t)ay0.taps * ax0.taps * d->Cin * top);
                q.div_howo = make_fastdiv((uint32_t)(ay0.count * ax0.count));
                q.div_wo = make_fastdiv((uint32_t)ax0.count);
                const int rc = conv_dispatch<true>(wb, ab, q, st);
                return rc != QNN_OK ? rc : check_launch("qnn_deconv2d");
            }
        }
        int64_t w_off = 0;
        for (int fy = 0; fy < s; ++fy)
            for (int fx = 0; fx < s; ++fx) {
                const PhaseAxis ay = phase_axis(fy, d->kh, s, d->pad, HO), ax = phase_axis(fx, d->kw, s, d->pad, WO);
                const int64_t words = phase_words(d->w_bits, d->Cout, ay.taps, ax.taps, (int)cw);
                if (ay.count > 0 && ax.count > 0) {
                    ConvTileParams q = base;
                    q.kh = ay.taps, q.kw = ax.taps;
                    q.nw = (int)(ay.taps * ax.taps * cw);
                    q.w = phase_planes + w_off + (int64_t)w0 * d->Cout * q.nw;
                    q.wvec = q.nw % 4 == 0 ? 1 : 0;
                    q.Ho = ay.count, q.Wo = ax.count, q.M = (int)(d->B * ay.count * ax.count);
                    q.pad_y = ay.pad, q.pad_x = ax.pad, q.oy0 = ay.first, q.ox0 = ax.first;
                    q.n_times_top = (uint32_t)((int64_t)ay.taps * ax.taps * d->Cin * top);
                    q.div_howo = make_fastdiv((uint32_t)(ay.count * ax.count));
                    q.div_wo = make_fastdiv((uint32_t)ax.count);
                    int rc = conv_dispatch<true>(wb, ab, q, st);
                    if (rc != QNN_OK) return rc;
                    rc = check_launch("qnn_deconv2d");
                    if (rc != QNN_OK) return rc;
                }
                w_off += words;
            }
        return QNN_OK;
    };
    // Bit widths above 4: chunk pairs of at most 4 x 4 planes as in qnn_conv2d; every output pixel belongs to
    // exactly one phase, so the running sum (in acc, or in the memory of out) is read and written by the same
    // phase of consecutive chunk pairs; only the last pair writes the outputs and the next layer's planes.
    const int w_chunks = (d->w_bits + 3) / 4, a_chunks = (d->a_bits + 3) / 4;
    int launch = 0;
    for (int cwi = 0; cwi < w_chunks; ++cwi)
        for (int cai = 0; cai < a_chunks; ++cai, ++launch) {
            const int wb = d->w_bits - 4 * cwi < 4 ? d->w_bits - 4 * cwi : 4;
            const int ab = d->a_bits - 4 * cai < 4 ? d->a_bits - 4 * cai : 4;
            const int mode = (launch > 0 ? 1 : 0) | (launch + 1 < w_chunks * a_chunks ? 2 : 0);
            const int rc = run_phases(wb, ab, 4 * cwi, 4 * cai, 4 * (cwi + cai), mode);
            if (rc != QNN_OK) return rc;
        }
    return QNN_OK;
}
