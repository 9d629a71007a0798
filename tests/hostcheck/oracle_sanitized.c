/*
 * Sanitizer run of the CPU oracle (compiled together with oracle/qnn_oracle.c under
 * -fsanitize=address,undefined by tests/test_sanitized_host.py).  Every oracle function runs on small,
 * odd-shaped inputs held in exactly-sized heap blocks, so an access one element past a tensor, a signed
 * overflow or a bad shift is reported.  A few values fixed by the paper are asserted on the way
 * (Table 2's states; the hand-worked 2-bit example acc = 6 with branches 2, 0, 0, -2 of Eq. 9).
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_quantize16(const float *, int64_t, float, int, int16_t *, uint8_t *);
int oracle_pack_planes(const int16_t *, int64_t, int64_t, int, uint32_t *);
int oracle_unpack_planes(const uint32_t *, int64_t, int64_t, int, int16_t *);
int oracle_gemm(const int16_t *, const int16_t *, int64_t, int64_t, int64_t, int32_t *);
int oracle_gemm8(const int8_t *, const int8_t *, int64_t, int64_t, int64_t, int32_t *);
int32_t oracle_gemm8_one(const int8_t *, const int8_t *, int64_t);
int oracle_conv2d8(const int8_t *, const int8_t *, int64_t, int64_t, int64_t, int64_t, int64_t, int, int, int, int,
                   int32_t *);
int oracle_conv2d8_dilated(const int8_t *, const int8_t *, int64_t, int64_t, int64_t, int64_t, int64_t, int, int, int, int,
                           int, int32_t *);
int oracle_scale(const int32_t *, const float *, int64_t, int64_t, float *);
int32_t oracle_xnor_bitcount_dot(const uint32_t *, const uint32_t *, int64_t);
int oracle_multibranch_gemm(const uint32_t *, int, const uint32_t *, int, int64_t, int64_t, int64_t, int32_t *,
                            int32_t *);

#define CHECK(cond)                                                                                                 \
    do {                                                                                                            \
        if (!(cond)) {                                                                                              \
            fprintf(stderr, "oracle_sanitized: check failed at line %d: %s\n", __LINE__, #cond);                    \
            exit(1);                                                                                                \
        }                                                                                                           \
    } while (0)

static uint32_t lcg(uint32_t *s) { return *s = *s * 1664525u + 1013904223u; }

static void levels_fill(int16_t *v, int64_t count, int bits, uint32_t *seed)
{
    const int top = (1 << bits) - 1;
    for (int64_t i = 0; i < count; ++i) v[i] = (int16_t)(2 * (int)((lcg(seed) >> 8) % (uint32_t)(top + 1)) - top);
}

int main(void)
{
    uint32_t seed = 7;

    /* Table 2: -1, -1/3, 1/3, 1 -> {high, low} states {-1,-1}, {-1,+1}, {+1,-1}, {+1,+1}, i.e. codes 0..3 */
    {
        float *x = malloc(4 * sizeof *x);
        int16_t *lv = malloc(4 * sizeof *lv);
        uint8_t *code = malloc(4);
        x[0] = -1.0f, x[1] = -1.0f / 3, x[2] = 1.0f / 3, x[3] = 1.0f;
        CHECK(oracle_quantize16(x, 4, 1.0f, 2, lv, code) == 0);
        for (int i = 0; i < 4; ++i) CHECK(code[i] == i && lv[i] == 2 * i - 3);
        CHECK(oracle_quantize16(x, 4, 1.0f, 9, lv, code) != 0 && oracle_quantize16(x, 4, 0.0f, 2, lv, code) != 0);
        CHECK(oracle_quantize16(x, 0, 1.0f, 8, lv, code) == 0);
        free(x), free(lv), free(code);
    }

    /* pack / unpack round trip on ragged rows for every bit width */
    for (int bits = 1; bits <= 8; ++bits) {
        const int64_t shapes[][2] = {{1, 1}, {3, 31}, {2, 32}, {5, 33}, {2, 100}};
        for (unsigned s = 0; s < sizeof shapes / sizeof shapes[0]; ++s) {
            const int64_t rows = shapes[s][0], n = shapes[s][1], nw = (n + 31) / 32;
            int16_t *lv = malloc((size_t)(rows * n) * sizeof *lv), *back = malloc((size_t)(rows * n) * sizeof *back);
            uint32_t *planes = malloc((size_t)(bits * rows * nw) * sizeof *planes);
            levels_fill(lv, rows * n, bits, &seed);
            CHECK(oracle_pack_planes(lv, rows, n, bits, planes) == 0);
            CHECK(oracle_unpack_planes(planes, rows, n, bits, back) == 0);
            for (int64_t i = 0; i < rows * n; ++i) CHECK(lv[i] == back[i]);
            if (n % 32) /* pad bits are 0 */
                for (int64_t r = 0; r < bits * rows; ++r) CHECK((planes[r * nw + nw - 1] >> (n % 32)) == 0);
            lv[0] = 0; /* an even level is refused */
            CHECK(oracle_pack_planes(lv, rows, n, bits, planes) == -2);
            free(lv), free(back), free(planes);
        }
    }

    /* the hand-worked example: a = [3, -1], w = [1, -3] at 2 x 2 bit: branches [[-2, 0], [0, 2]], acc = 6 */
    {
        int16_t *a = malloc(2 * sizeof *a), *w = malloc(2 * sizeof *w);
        uint32_t *ap = malloc(2 * sizeof *ap), *wp = malloc(2 * sizeof *wp);
        int32_t *acc = malloc(sizeof *acc), *br = malloc(4 * sizeof *br), *plain = malloc(sizeof *plain);
        a[0] = 3, a[1] = -1, w[0] = 1, w[1] = -3;
        CHECK(oracle_pack_planes(a, 1, 2, 2, ap) == 0 && oracle_pack_planes(w, 1, 2, 2, wp) == 0);
        CHECK(oracle_multibranch_gemm(ap, 2, wp, 2, 1, 1, 2, acc, br) == 0);
        CHECK(acc[0] == 6 && br[0] == -2 && br[1] == 0 && br[2] == 0 && br[3] == 2);
        CHECK(oracle_gemm(a, w, 1, 1, 2, plain) == 0 && plain[0] == 6);
        free(a), free(w), free(ap), free(wp), free(acc), free(br), free(plain);
    }

    /* all-maximum 8 x 8 bit operands at the longest reduction int32 holds: n 255 255 < 2^31 */
    {
        const int64_t n = 33025;
        int16_t *a = malloc((size_t)n * sizeof *a), *w = malloc((size_t)n * sizeof *w);
        int32_t *acc = malloc(sizeof *acc);
        for (int64_t i = 0; i < n; ++i) a[i] = 255, w[i] = -255;
        CHECK(oracle_gemm(a, w, 1, 1, n, acc) == 0 && acc[0] == -(int32_t)(n * 255 * 255));
        free(a), free(w), free(acc);
    }

    /* GEMM, the int8 twin, the single-output form and the branch sum agree on ragged shapes */
    for (int bits = 1; bits <= 7; bits += 2) {
        const int64_t rows = 3, cols = 5, n = 45, nw = 2;
        int16_t *a = malloc((size_t)(rows * n) * sizeof *a), *w = malloc((size_t)(cols * n) * sizeof *w);
        int8_t *a8 = malloc((size_t)(rows * n)), *w8 = malloc((size_t)(cols * n));
        int32_t *acc = malloc((size_t)(rows * cols) * sizeof *acc), *acc8 = malloc((size_t)(rows * cols) * sizeof *acc8);
        int32_t *accb = malloc((size_t)(rows * cols) * sizeof *accb);
        uint32_t *ap = malloc((size_t)(bits * rows * nw) * sizeof *ap), *wp = malloc((size_t)(bits * cols * nw) * sizeof *wp);
        levels_fill(a, rows * n, bits, &seed), levels_fill(w, cols * n, bits, &seed);
        for (int64_t i = 0; i < rows * n; ++i) a8[i] = (int8_t)a[i];
        for (int64_t i = 0; i < cols * n; ++i) w8[i] = (int8_t)w[i];
        CHECK(oracle_gemm(a, w, rows, cols, n, acc) == 0 && oracle_gemm8(a8, w8, rows, cols, n, acc8) == 0);
        CHECK(oracle_pack_planes(a, rows, n, bits, ap) == 0 && oracle_pack_planes(w, cols, n, bits, wp) == 0);
        CHECK(oracle_multibranch_gemm(ap, bits, wp, bits, rows, cols, n, accb, NULL) == 0);
        for (int64_t r = 0; r < rows; ++r)
            for (int64_t c = 0; c < cols; ++c) {
                CHECK(acc[r * cols + c] == acc8[r * cols + c] && acc[r * cols + c] == accb[r * cols + c]);
                CHECK(acc[r * cols + c] == oracle_gemm8_one(a8 + r * n, w8 + c * n, n));
            }
        CHECK(oracle_xnor_bitcount_dot(ap, ap, n) == (int32_t)n);
        free(a), free(w), free(a8), free(w8), free(acc), free(acc8), free(accb), free(ap), free(wp);
    }

    /* convolution: windows that lie mostly in the padding, strides, a rectangular kernel; 1x1 == GEMM */
    {
        const int geoms[][9] = {{2, 4, 5, 3, 4, 3, 3, 1, 2}, {1, 7, 6, 5, 2, 5, 3, 2, 1}, {1, 3, 3, 2, 3, 1, 1, 1, 0},
                                {2, 5, 5, 1, 1, 3, 3, 3, 0}};
        for (unsigned g = 0; g < sizeof geoms / sizeof geoms[0]; ++g) {
            const int64_t B = geoms[g][0], H = geoms[g][1], W = geoms[g][2], Cin = geoms[g][3], Cout = geoms[g][4];
            const int kh = geoms[g][5], kw = geoms[g][6], st = geoms[g][7], pad = geoms[g][8];
            const int64_t Ho = (H + 2 * pad - kh) / st + 1, Wo = (W + 2 * pad - kw) / st + 1;
            int8_t *a = malloc((size_t)(B * H * W * Cin)), *w = malloc((size_t)(Cout * kh * kw * Cin));
            int32_t *acc = malloc((size_t)(B * Ho * Wo * Cout) * sizeof *acc);
            for (int64_t i = 0; i < B * H * W * Cin; ++i) a[i] = (int8_t)(2 * (int)((lcg(&seed) >> 9) % 8) - 7);
            for (int64_t i = 0; i < Cout * kh * kw * Cin; ++i) w[i] = (int8_t)(2 * (int)((lcg(&seed) >> 9) % 8) - 7);
            CHECK(oracle_conv2d8(a, w, B, H, W, Cin, Cout, kh, kw, st, pad, acc) == 0);
            if (kh == 1 && kw == 1 && st == 1 && pad == 0) {
                int32_t *ref = malloc((size_t)(B * H * W * Cout) * sizeof *ref);
                CHECK(oracle_gemm8(a, w, B * H * W, Cout, Cin, ref) == 0);
                for (int64_t i = 0; i < B * H * W * Cout; ++i) CHECK(ref[i] == acc[i]);
                free(ref);
            }
            /* dilation 1 is the same sum; dilation 2 with enough padding keeps the extent */
            {
                int32_t *again = malloc((size_t)(B * Ho * Wo * Cout) * sizeof *again);
                CHECK(oracle_conv2d8_dilated(a, w, B, H, W, Cin, Cout, kh, kw, st, pad, 1, again) == 0);
                for (int64_t i = 0; i < B * Ho * Wo * Cout; ++i) CHECK(again[i] == acc[i]);
                free(again);
                const int64_t H2 = (H + 2 * (pad + kh) - 2 * (kh - 1) - 1) / st + 1, W2 = (W + 2 * (pad + kh) - 2 * (kw - 1) - 1) / st + 1;
                int32_t *wide = malloc((size_t)(B * H2 * W2 * Cout) * sizeof *wide);
                CHECK(oracle_conv2d8_dilated(a, w, B, H, W, Cin, Cout, kh, kw, st, pad + kh, 2, wide) == 0);
                free(wide);
            }
            free(a), free(w), free(acc);
        }
        int32_t dummy;
        int8_t one = 1;
        CHECK(oracle_conv2d8(&one, &one, 1, 1, 1, 1, 1, 3, 3, 1, 0, &dummy) != 0); /* kernel larger than the image */
        CHECK(oracle_conv2d8_dilated(&one, &one, 1, 1, 1, 1, 1, 3, 3, 1, 1, 2, &dummy) != 0);
        CHECK(oracle_conv2d8_dilated(&one, &one, 1, 1, 1, 1, 1, 1, 1, 1, 0, 0, &dummy) != 0);
    }

    /* scale: Fig. 1's 1/9 on the worked example's accumulator */
    {
        int32_t *acc = malloc(3 * sizeof *acc);
        float *s = malloc(3 * sizeof *s), *out = malloc(3 * sizeof *out);
        acc[0] = 6, acc[1] = -9, acc[2] = 0;
        s[0] = s[1] = s[2] = 1.0f / 9.0f;
        CHECK(oracle_scale(acc, s, 1, 3, out) == 0);
        CHECK(out[0] > 0.66666f && out[0] < 0.66667f && out[1] == -1.0f && out[2] == 0.0f);
        free(acc), free(s), free(out);
    }
    puts("oracle_sanitized: ok");
    return 0;
}
