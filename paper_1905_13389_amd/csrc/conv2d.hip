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
#include "conv2d_tile.h"

namespace qnn {

// Everything the plain kernel needs (64-bit sizes).
struct ConvParams {
    const uint32_t *a; // [AB][B][H][W][cw]
    const uint32_t *w; // [WB][Cout][kh][kw][cw]
    int64_t B, H, W, Cin, Cout, Ho, Wo;
    int kh, kw, stride, pad, dil;
    int64_t cw, nw, M; // words per pixel, reduction words, output pixels
    int64_t a_plane_stride;
    const float *scale;
    int32_t *acc;
    float *out;
    BlockTerms blk;
    int64_t cwo; // words per output pixel of the shortcut planes
};

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
        const int hi = h0 + ky * p.dil;
        if (hi < 0 || hi >= p.H) continue;
        for (int kx = 0; kx < p.kw; ++kx) {
            const int wi = w0 + kx * p.dil;
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
    if (p.out) {
        float o = (float)v * p.scale[c];
        if (p.blk.bias) o = o + p.blk.bias[c];
        if (p.blk.res_q) {
            const uint32_t *rq = static_cast<const uint32_t *>(p.blk.res_q);
            int code = 0;
            for (int j = 0; j < p.blk.res_bits; ++j)
                code |= (int)((rq[((int64_t)j * p.M + m) * p.cwo + (c >> 5)] >> (c & 31)) & 1u) << j;
            const float term = (float)(2 * code - p.blk.res_top) * p.blk.res_scale;
            o = o + term;
        }
        if (p.blk.res_f32) o = o + p.blk.res_f32[idx];
        if (p.blk.relu) o = fmaxf(o, 0.0f);
        p.out[idx] = o;
    }
}

} // namespace qnn

using namespace qnn;

extern "C" int qnn_conv2d(const qnn_conv_desc *d, const uint32_t *a_planes, const uint32_t *w_planes,
                          const float *scale, int32_t *acc, float *out, uint32_t *next_planes,
                          float next_clip, int next_bits, void *stream)
{
    return qnn_conv2d_block(d, a_planes, w_planes, scale, nullptr, acc, out, next_planes, next_clip, next_bits, stream);
}

static int conv_run(const qnn_conv_desc *d, int dilation, const uint32_t *a_planes, const uint32_t *w_planes,
                    const float *scale, const qnn_block_epilogue *epi, int32_t *acc, float *out,
                    uint32_t *next_planes, float next_clip, int next_bits, void *stream);

extern "C" int qnn_conv2d_block(const qnn_conv_desc *d, const uint32_t *a_planes, const uint32_t *w_planes,
                                const float *scale, const qnn_block_epilogue *epi, int32_t *acc, float *out,
                                uint32_t *next_planes, float next_clip, int next_bits, void *stream)
{
    return conv_run(d, 1, a_planes, w_planes, scale, epi, acc, out, next_planes, next_clip, next_bits, stream);
}

extern "C" int qnn_conv2d_dilated(const qnn_conv_desc *d, int dilation, const uint32_t *a_planes, const uint32_t *w_planes,
                                  const float *scale, int32_t *acc, float *out, uint32_t *next_planes, float next_clip,
                                  int next_bits, void *stream)
{
    return conv_run(d, dilation, a_planes, w_planes, scale, nullptr, acc, out, next_planes, next_clip, next_bits, stream);
}

// dilation: distance between neighbouring taps in pixels
static int conv_run(const qnn_conv_desc *d, int dilation, const uint32_t *a_planes, const uint32_t *w_planes,
                    const float *scale, const qnn_block_epilogue *epi, int32_t *acc, float *out,
                    uint32_t *next_planes, float next_clip, int next_bits, void *stream)
{
    if (!d) return fail(QNN_ERR_INVALID_ARG, "qnn_conv2d: NULL descriptor");
    BlockTerms blk;
    const int brc = block_terms("qnn_conv2d_block", epi, scale, 8, blk);
    if (brc != QNN_OK) return brc;
    if (d->a_bits < 1 || d->a_bits > 8 || d->w_bits < 1 || d->w_bits > 8)
        return fail(QNN_ERR_INVALID_ARG, "qnn_conv2d: bits must be in [1,8]");
    if (d->B < 0 || d->H <= 0 || d->W <= 0 || d->Cin <= 0 || d->Cout <= 0)
        return fail(QNN_ERR_INVALID_ARG, "qnn_conv2d: bad tensor size");
    if (d->kh < 1 || d->kw < 1 || d->stride < 1 || d->pad < 0)
        return fail(QNN_ERR_INVALID_ARG, "qnn_conv2d: bad kernel geometry");
    if (d->kh > 7 || d->kw > 7) return fail(QNN_ERR_UNSUPPORTED, "qnn_conv2d: kernel larger than 7x7");
    if (dilation < 1) return fail(QNN_ERR_INVALID_ARG, "qnn_conv2d: dilation must be at least 1");
    if (dilation > 64) return fail(QNN_ERR_UNSUPPORTED, "qnn_conv2d: dilation above 64");
    const int64_t eh = (int64_t)dilation * (d->kh - 1) + 1, ew = (int64_t)dilation * (d->kw - 1) + 1; // extent of the taps
    if (d->H + 2 * (int64_t)d->pad < eh || d->W + 2 * (int64_t)d->pad < ew)
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
    p.kh = d->kh, p.kw = d->kw, p.stride = d->stride, p.pad = d->pad, p.dil = dilation;
    p.Ho = (d->H + 2 * (int64_t)d->pad - eh) / d->stride + 1;
    p.Wo = (d->W + 2 * (int64_t)d->pad - ew) / d->stride + 1;
    p.cw = ceil_div(d->Cin, 32);
    p.nw = (int64_t)d->kh * d->kw * p.cw;
    if (d->B > (INT64_MAX >> 24) / (p.Ho * p.Wo)) return fail(QNN_ERR_RANGE, "qnn_conv2d: too many output pixels");
    p.M = d->B * p.Ho * p.Wo;
    p.a_plane_stride = d->B * d->H * d->W * p.cw;
    p.scale = scale;
    p.acc = acc;
    p.out = out;
    p.blk = blk;
    const int64_t cwo = ceil_div(d->Cout, 32);
    p.cwo = cwo;
    hipStream_t st = static_cast<hipStream_t>(stream);

    // the register-blocked kernel indexes pixels and plane words with 32-bit integers
    const bool small_index = p.M < (1LL << 29) && p.a_plane_stride * d->a_bits < (1LL << 31) &&
                             p.M * cwo < (1LL << 31) && p.Ho + p.Wo <= kMaxOutExtent &&
                             (eh * d->W + ew) * p.cw < (1LL << 24);
    bool done = false;
    const bool wide = d->w_bits > 4 || d->a_bits > 4;
    if (p.nw <= kMaxGroups && d->kh * d->kw <= kMaxTaps && small_index && (!wide || acc || out)) {
        ConvTileParams t = {};
        t.a = a_planes, t.w = w_planes, t.scale = scale, t.acc = acc, t.out = out, t.next = next_planes;
        t.H = (int)d->H, t.W = (int)d->W, t.HW = (int)(d->H * d->W), t.Cin = (int)d->Cin, t.Cout = (int)d->Cout;
        t.M = (int)p.M, t.cw = (int)p.cw, t.nw = (int)p.nw, t.cwo = (int)cwo, t.Ho = (int)p.Ho, t.Wo = (int)p.Wo;
        t.kh = d->kh, t.kw = d->kw, t.stride = d->stride, t.pad = d->pad, t.dil = dilation;
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
        t.blk = blk;
        t.pad_y = t.pad_x = d->pad;
        t.nphase = 1, t.wgs_per_phase = 0, t.phase_words = 0;
        t.scatter = 0, t.os = 1, t.oy0 = t.ox0 = 0, t.HO = (int)p.Ho, t.WO = (int)p.Wo, t.M_out = (int)p.M;
        const bool has_terms = blk.any();
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
                int rc = has_terms ? conv_tiles_block(wb, ab, q, st) : conv_dispatch<false>(wb, ab, q, st);
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

#ifdef QNN_TIMELINE
extern "C" int qnn_timeline_set(long long *buffer, int waves, int pair_hint)
{
    if (waves < 0 || (waves > 0 && !buffer)) return fail(QNN_ERR_INVALID_ARG, "qnn_timeline_set: a buffer of waves x 5 int64 is needed");
    timeline_state() = {waves > 0 ? buffer : nullptr, waves, pair_hint ? 1 : 0};
    return QNN_OK;
}
#endif
