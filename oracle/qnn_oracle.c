/*
 * CPU oracle for the encoding-decomposition QNN hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what the
 * GPU library must compute.  Only the test-suite, the smoke check and the
 * cpu_baseline leg of the benchmark may load it; the product library never does,
 * and the two share no code.
 *
 * The method is an exact re-association of an integer dot product (paper, Section
 * "Model Decomposition", Eq. 7-9 with the {-1,+1} code of Eq. 10), so the oracle
 * for GEMM / convolution is the plain definition on decoded integer levels: no
 * bit-packing, no popcount, no blocking.  The pieces of the decomposition itself
 * (planes, xnor+bitcount, M x K branches) are written out separately, literally,
 * so the tests can check the paper's identities on small inputs.
 *
 * Conventions (same letters as the public header of the GPU library, but nothing
 * is shared): a level is an odd integer v = 2u - (2^b - 1), u in [0, 2^b - 1] its
 * code; plane j holds bit j of u; bit 1 <=> +1, bit 0 <=> -1 (Eq. 10, Table 2).
 *
 * Parity pins: every function below is pinned by tests/test_oracle_*.py against
 * values printed in the paper (Table 2, the 1/9 of Fig. 1), closed forms, brute
 * force on tiny inputs, numpy int64 matmul and torch float64 conv2d.
 * "Tables 3-4" of the paper (trained-network accuracies) are out of scope and are
 * parity unpinned.
 *
 * Build: gcc -O3 -fopenmp -ffp-contract=off -shared -fPIC (see oracle/build.py).
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Range limit + linear quantizer (Table 1 HTanh; Eq. 15; Eq. 10).            */
/*                                                                           */
/* t = HTanh(x / clip) in [-1, 1]; code u = <(2^b - 1)(t + 1)/2>, rounding    */
/* half up; level v = 2u - (2^b - 1), which is (2^b - 1) * q_b(t) of Eq. 15.  */
/* The decision is taken in fp32 with this exact operation sequence (each op  */
/* a single correctly rounded IEEE operation; the fma is explicit):           */
/*   inv = 1.0f / clip; t = x * inv; t = min(max(t, -1), 1);                  */
/*   h = (2^b - 1) / 2 (exact in fp32); r = fma(t, h, h) + 0.5f; u = floor(r) */
/* NaN input is outside the contract.                                        */
/* ------------------------------------------------------------------------- */
/* Levels are int16 so that 8-bit codes (levels up to +-255) fit. */
int oracle_quantize16(const float *x, int64_t count, float clip, int bits,
                      int16_t *level, uint8_t *code)
{
    if (!x || count < 0 || bits < 1 || bits > 8 || !(clip > 0.0f) || isinf(clip))
        return -1;
    const int top = (1 << bits) - 1;
    const float inv = 1.0f / clip;
    const float h = (float)top * 0.5f;
    for (int64_t i = 0; i < count; ++i) {
        float t = x[i] * inv;
        t = fmaxf(t, -1.0f);
        t = fminf(t, 1.0f);
        float r = fmaf(t, h, h);
        r = r + 0.5f;
        int u = (int)floorf(r);
        if (u < 0) u = 0;
        if (u > top) u = top;
        if (code) code[i] = (uint8_t)u;
        if (level) level[i] = (int16_t)(2 * u - top);
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Plane split + bit-vector storage (Eq. 4-6 plane matrix, Eq. 10, Table 2;   */
/* "stored by bit vectors", Introduction).                                    */
/* level: [rows][n] int16 odd levels.  planes: [bits][rows][nw] uint32,        */
/* nw = ceil(n/32); bit t of word j is element 32j+t; pad bits are 0.          */
/* Returns -2 if a level is even or out of range for `bits`.                   */
/* ------------------------------------------------------------------------- */
int oracle_pack_planes(const int16_t *level, int64_t rows, int64_t n, int bits,
                       uint32_t *planes)
{
    if (!level || !planes || rows < 0 || n < 0 || bits < 1 || bits > 8) return -1;
    const int top = (1 << bits) - 1;
    const int64_t nw = (n + 31) / 32;
    memset(planes, 0, (size_t)bits * (size_t)rows * (size_t)nw * sizeof(uint32_t));
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t t = 0; t < n; ++t) {
            int v = level[r * n + t];
            if (v < -top || v > top || ((v + top) & 1)) return -2;
            int u = (v + top) / 2;
            for (int j = 0; j < bits; ++j) {
                if ((u >> j) & 1)
                    planes[((int64_t)j * rows + r) * nw + t / 32] |= (uint32_t)1 << (t % 32);
            }
        }
    }
    return 0;
}

/* Decode (Eq. 10): v = sum_j 2^j * c_j with c_j = +1 if bit j set else -1. */
int oracle_unpack_planes(const uint32_t *planes, int64_t rows, int64_t n, int bits,
                         int16_t *level)
{
    if (!level || !planes || rows < 0 || n < 0 || bits < 1 || bits > 8) return -1;
    const int64_t nw = (n + 31) / 32;
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t t = 0; t < n; ++t) {
            int v = 0;
            for (int j = 0; j < bits; ++j) {
                uint32_t word = planes[((int64_t)j * rows + r) * nw + t / 32];
                int c = ((word >> (t % 32)) & 1u) ? 1 : -1;
                v += (1 << j) * c;
            }
            level[r * n + t] = (int16_t)v;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* GEMM on decoded levels: the plain definition (Eq. 1-2).                    */
/* a: [rows][n], w: [cols][n] (both reduction-contiguous), acc: [rows][cols]. */
/* ------------------------------------------------------------------------- */
int oracle_gemm(const int16_t *a, const int16_t *w, int64_t rows, int64_t cols,
                int64_t n, int32_t *acc)
{
    if (!a || !w || !acc || rows < 0 || cols < 0 || n < 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t c = 0; c < cols; ++c) {
            int32_t s = 0;
            for (int64_t t = 0; t < n; ++t)
                s += (int32_t)a[r * n + t] * (int32_t)w[c * n + t];
            acc[r * cols + c] = s;
        }
    }
    return 0;
}

/* int8 twin of oracle_gemm (levels of up to 7 bits), same loops. */
int oracle_gemm8(const int8_t *a, const int8_t *w, int64_t rows, int64_t cols,
                 int64_t n, int32_t *acc)
{
    if (!a || !w || !acc || rows < 0 || cols < 0 || n < 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t c = 0; c < cols; ++c) {
            int32_t s = 0;
            for (int64_t t = 0; t < n; ++t)
                s += (int32_t)a[r * n + t] * (int32_t)w[c * n + t];
            acc[r * cols + c] = s;
        }
    }
    return 0;
}

/* One output of the GEMM, for sampled checks at sizes the full loop is slow on. */
int32_t oracle_gemm8_one(const int8_t *a_row, const int8_t *w_row, int64_t n)
{
    int32_t s = 0;
    for (int64_t t = 0; t < n; ++t) s += (int32_t)a_row[t] * (int32_t)w_row[t];
    return s;
}

/* ------------------------------------------------------------------------- */
/* Convolution on decoded levels (Section "Model Decomposition": convolution  */
/* reduces to the same vector product).  NHWC activations, weights            */
/* [Cout][kh][kw][Cin], output [B][Ho][Wo][Cout]; taps that fall outside the   */
/* image contribute exactly 0 (zero padding in the decoded-integer domain).   */
/* Ho = (H + 2p - kh)/s + 1, floor.                                           */
/* ------------------------------------------------------------------------- */
int oracle_conv2d8(const int8_t *a, const int8_t *w, int64_t B, int64_t H, int64_t W,
                   int64_t Cin, int64_t Cout, int kh, int kw, int stride, int pad,
                   int32_t *acc)
{
    if (!a || !w || !acc || B < 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 ||
        kh <= 0 || kw <= 0 || stride <= 0 || pad < 0)
        return -1;
    const int64_t Ho = (H + 2 * pad - kh) / stride + 1;
    const int64_t Wo = (W + 2 * pad - kw) / stride + 1;
    if (Ho <= 0 || Wo <= 0) return -1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t ho = 0; ho < Ho; ++ho) {
            for (int64_t wo = 0; wo < Wo; ++wo) {
                for (int64_t co = 0; co < Cout; ++co) {
                    int32_t s = 0;
                    for (int y = 0; y < kh; ++y) {
                        int64_t hi = ho * stride + y - pad;
                        if (hi < 0 || hi >= H) continue;
                        for (int x = 0; x < kw; ++x) {
                            int64_t wi = wo * stride + x - pad;
                            if (wi < 0 || wi >= W) continue;
                            const int8_t *ap = a + ((b * H + hi) * W + wi) * Cin;
                            const int8_t *wp = w + ((co * kh + y) * kw + x) * Cin;
                            for (int64_t ci = 0; ci < Cin; ++ci)
                                s += (int32_t)ap[ci] * (int32_t)wp[ci];
                        }
                    }
                    acc[((b * Ho + ho) * Wo + wo) * Cout + co] = s;
                }
            }
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* The same sum with the taps `dilation` pixels apart (the detection network   */
/* of the experiments section, SSD on a backbone, has one such layer):         */
/* tap (y, x) reads input pixel (ho s + y d - p, wo s + x d - p);              */
/* Ho = (H + 2p - d (kh - 1) - 1)/s + 1, floor.  dilation = 1 is the           */
/* convolution above.                                                          */
/* ------------------------------------------------------------------------- */
int oracle_conv2d8_dilated(const int8_t *a, const int8_t *w, int64_t B, int64_t H, int64_t W,
                           int64_t Cin, int64_t Cout, int kh, int kw, int stride, int pad,
                           int dilation, int32_t *acc)
{
    if (!a || !w || !acc || B < 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 ||
        kh <= 0 || kw <= 0 || stride <= 0 || pad < 0 || dilation <= 0)
        return -1;
    const int64_t eh = (int64_t)dilation * (kh - 1) + 1, ew = (int64_t)dilation * (kw - 1) + 1;
    if (H + 2 * pad < eh || W + 2 * pad < ew) return -1;
    const int64_t Ho = (H + 2 * pad - eh) / stride + 1;
    const int64_t Wo = (W + 2 * pad - ew) / stride + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t ho = 0; ho < Ho; ++ho) {
            for (int64_t wo = 0; wo < Wo; ++wo) {
                for (int64_t co = 0; co < Cout; ++co) {
                    int32_t s = 0;
                    for (int y = 0; y < kh; ++y) {
                        int64_t hi = ho * stride + (int64_t)y * dilation - pad;
                        if (hi < 0 || hi >= H) continue;
                        for (int x = 0; x < kw; ++x) {
                            int64_t wi = wo * stride + (int64_t)x * dilation - pad;
                            if (wi < 0 || wi >= W) continue;
                            const int8_t *ap = a + ((b * H + hi) * W + wi) * Cin;
                            const int8_t *wp = w + ((co * kh + y) * kw + x) * Cin;
                            for (int64_t ci = 0; ci < Cin; ++ci)
                                s += (int32_t)ap[ci] * (int32_t)wp[ci];
                        }
                    }
                    acc[((b * Ho + ho) * Wo + wo) * Cout + co] = s;
                }
            }
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Decoder scale (Section "M-bit Encoding Functions": the 1/alpha^2 factor,   */
/* 1/9 in Fig. 1; Eq. 18), generalised to one fp32 factor per output channel. */
/* One int->fp32 conversion and one IEEE fp32 multiply.                       */
/* ------------------------------------------------------------------------- */
int oracle_scale(const int32_t *acc, const float *scale, int64_t rows, int64_t cols,
                 float *out)
{
    if (!acc || !scale || !out || rows < 0 || cols < 0) return -1;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c)
            out[r * cols + c] = (float)acc[r * cols + c] * scale[c];
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Self-test helpers: the decomposition written out literally.  The GPU path  */
/* shares none of these; they exist so the tests can check the identities.    */
/* ------------------------------------------------------------------------- */

/* Binary dot of two {-1,+1}^n vectors stored as bits (Abstract / Section     */
/* "Model Decomposition": xnor and bitcount): 2 * popcount(xnor) - n over the */
/* n valid bits, counted one bit at a time.                                   */
int32_t oracle_xnor_bitcount_dot(const uint32_t *a, const uint32_t *b, int64_t n)
{
    int32_t same = 0;
    for (int64_t t = 0; t < n; ++t) {
        uint32_t abit = (a[t / 32] >> (t % 32)) & 1u;
        uint32_t bbit = (b[t / 32] >> (t % 32)) & 1u;
        uint32_t xnor = (~(abit ^ bbit)) & 1u;
        same += (int32_t)xnor;
    }
    return 2 * same - (int32_t)n;
}

/* M x K multi-branch product (Eq. 9 with the {-1,+1} code of Eq. 10; Fig. 1): */
/* y_ij = w_i . a_j over {-1,+1} planes via xnor+bitcount, recombined with     */
/* 2^(i+j).  Planes as produced by oracle_pack_planes.  branch_out (optional)  */
/* receives the w_bits*a_bits branch results [rows][cols][w_bits][a_bits].     */
int oracle_multibranch_gemm(const uint32_t *a_planes, int a_bits, const uint32_t *w_planes,
                            int w_bits, int64_t rows, int64_t cols, int64_t n,
                            int32_t *acc, int32_t *branch_out)
{
    if (!a_planes || !w_planes || !acc || rows < 0 || cols < 0 || n < 0 || a_bits < 1 ||
        a_bits > 8 || w_bits < 1 || w_bits > 8)
        return -1;
    const int64_t nw = (n + 31) / 32;
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t c = 0; c < cols; ++c) {
            int64_t s = 0;
            for (int i = 0; i < w_bits; ++i) {
                for (int j = 0; j < a_bits; ++j) {
                    const uint32_t *wp = w_planes + ((int64_t)i * cols + c) * nw;
                    const uint32_t *ap = a_planes + ((int64_t)j * rows + r) * nw;
                    int32_t y = oracle_xnor_bitcount_dot(wp, ap, n);
                    if (branch_out)
                        branch_out[((r * cols + c) * w_bits + i) * a_bits + j] = y;
                    s += ((int64_t)1 << (i + j)) * (int64_t)y;
                }
            }
            acc[r * cols + c] = (int32_t)s;
        }
    }
    return 0;
}

/* Number of OpenMP threads the row-parallel loops above use (for benchmark reports). */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif
