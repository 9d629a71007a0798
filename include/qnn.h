/*
 * qnn.h -- C ABI of the MI355X (gfx950) library for the hot path of encoding-decomposition
 * quantized networks ("Multi-Precision Quantized Neural Networks via Encoding Decomposition
 * of {-1,+1}").
 *
 * An M-bit weight and a K-bit activation are each a sum of 2^i-weighted {-1,+1} planes
 * (paper, Eq. 10), so a quantized GEMM / convolution is M x K binary products done with
 * xor + bitcount on packed bit-vectors and recombined with 2^(i+j) (Eq. 9, Fig. 1), then
 * multiplied by a scale factor (the 1/alpha^2 of the section "M-bit Encoding Functions",
 * Eq. 18).
 *
 * Naming.  The paper calls the bit widths M and K (and swaps which is which between
 * sections); here they are always `w_bits` (weights) and `a_bits` (activations).
 *
 * Data conventions (all entry points)
 *   level  odd integer v = 2u - (2^b - 1), u in [0, 2^b - 1] its code (Eq. 10; remark after
 *          Eq. 20: odd, |v| <= 2^b - 1).
 *   planes uint32 bit-vectors along the reduction axis: plane j holds bit j of u (j = 0 is
 *          the low bit, weight 2^0); bit 1 <=> +1, bit 0 <=> -1 (Table 2, x = x1 + 2 x2).
 *          nw = ceil(n/32) words per row; bit t of word k is element 32k + t; PAD BITS ARE 0
 *          in every plane of both operands.
 *          activations: [a_bits][rows][nw];  weights: [w_bits][cols][nw].
 *
 * Pointers.  Every pointer marked DEVICE is device memory owned by the caller; the library
 * never allocates, frees or keeps it.  `stream` is a hipStream_t passed as void* (NULL = the
 * null stream).  Every call only enqueues work on `stream` and returns; outputs are valid
 * after that stream has been synchronised.  Plane / accumulator / output pointers must be
 * 16-byte aligned.
 *
 * Errors.  Return value 0 = QNN_OK, otherwise a negative QNN_ERR_* code; argument errors are
 * found on the host before any HIP call is made (nothing is enqueued then).
 * qnn_last_error() returns a thread-local message for the last failing call on this thread.
 */
#ifndef QNN_H_
#define QNN_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define QNN_OK 0
#define QNN_ERR_INVALID_ARG (-1) /* null pointer, size < 0, bits outside [1,8], bad clip   */
#define QNN_ERR_UNSUPPORTED (-2) /* dtype / kernel size / combination that is not built     */
#define QNN_ERR_ALIGNMENT (-3)   /* pointer not 16-byte aligned                             */
#define QNN_ERR_RANGE (-4)       /* n (2^w_bits - 1)(2^a_bits - 1) >= 2^31: int32 overflow  */
#define QNN_ERR_LAUNCH (-5)      /* the HIP runtime refused the launch                      */

#define QNN_DTYPE_F32 0  /* IEEE fp32 values                                   */
#define QNN_DTYPE_BF16 1 /* bfloat16 values (widened exactly to fp32 first)    */
#define QNN_DTYPE_I8 2   /* int8 levels (already quantized odd integers)       */

/*
 * qnn_encode_pack -- range limit, linear quantizer, plane split and bit-vector packing
 * (Table 1 HTanh; Eq. 15; Eq. 10; Table 2; "stored by bit vectors", Introduction).
 *
 * For fp inputs, in fp32, one correctly rounded operation per step:
 *   t = x * (1.0f / clip);  t = min(max(t, -1), 1);  h = (2^bits - 1) / 2;
 *   u = floor(fma(t, h, h) + 0.5f), clamped to [0, 2^bits - 1]      (round half up)
 * so x = 0 maps to level +1 and |x| >= clip saturates.  NaN inputs give an unspecified code.
 * For QNN_DTYPE_I8 the input already holds levels: u = (v + 2^bits - 1) / 2; even or
 * out-of-range levels are the caller's error and give unspecified planes. `clip` is ignored.
 *
 *   src     DEVICE, [rows] rows of n elements, consecutive rows `row_stride_elems` apart
 *   planes  DEVICE out, [bits][rows][ceil(n/32)] uint32, pad bits written as 0
 * rows == 0 or n == 0 is a successful no-op.
 */
int qnn_encode_pack(const void *src, int dtype, int64_t rows, int64_t n,
                    int64_t row_stride_elems, float clip, int bits, uint32_t *planes,
                    void *stream);

/*
 * qnn_binary_gemm -- the M x K multi-branch binary product and its recombination
 * (Eq. 7-9 with Eq. 10; Fig. 1):
 *   P_ij[r][c] = bitcount(W_i[c][:] xor A_j[r][:])           (binary dot y_ij = n - 2 P_ij)
 *   acc[r][c]  = sum_ij 2^(i+j) y_ij = n (2^w_bits-1)(2^a_bits-1) - 2 sum_ij 2^(i+j) P_ij
 * which equals the integer dot product of the decoded levels of row r of A and row c of W.
 * Optionally fused with the scale of qnn_dequant_scale: out[r][c] = (float)acc[r][c]*scale[c].
 *
 *   a_planes DEVICE [a_bits][rows][nw], w_planes DEVICE [w_bits][cols][nw], nw = ceil(n/32)
 *   acc      DEVICE out int32 [rows][cols], or NULL
 *   scale    DEVICE fp32 [cols]; required iff out != NULL
 *   out      DEVICE out fp32 [rows][cols], or NULL         (acc and out not both NULL)
 * Bit widths above 4 run as up to four launches over chunks of at most 4 planes per operand (the
 * double sum of Eq. 9 splits into chunk pairs); the running int32 sum is kept in acc, or in the
 * memory of out when acc is NULL, until the last launch writes the results.
 */
int qnn_binary_gemm(const uint32_t *a_planes, int a_bits, const uint32_t *w_planes, int w_bits,
                    int64_t rows, int64_t cols, int64_t n, int32_t *acc, const float *scale,
                    float *out, void *stream);

/*
 * qnn_dequant_scale -- the decoder's scale factor (section "M-bit Encoding Functions": the
 * product of two encoded vectors is alpha^2 times too large, 1/9 in Fig. 1; Eq. 18), one
 * fp32 factor per output channel: out[r][c] = (float)acc[r][c] * scale[c], one int->fp32
 * conversion and one fp32 multiply.
 *   acc DEVICE int32 [rows][cols]; scale DEVICE fp32 [cols]; out DEVICE fp32 [rows][cols]
 */
int qnn_dequant_scale(const int32_t *acc, const float *scale, int64_t rows, int64_t cols,
                      float *out, void *stream);

/*
 * qnn_conv2d -- the same multi-branch product with the reduction axis gathered implicitly
 * from an NHWC bit-plane tensor (section "Model Decomposition": convolution layers reduce to
 * the same vector product).  Reduction axis = (ky, kx, ci); channels are the packed axis,
 * cw = ceil(Cin/32) words per pixel.  Taps outside the image contribute exactly 0 to acc
 * (zero padding of the decoded integers; 0 is not itself a level).
 *   Ho = (H + 2 pad - kh)/stride + 1, Wo likewise (floor).
 *
 *   a_planes DEVICE [a_bits][B][H][W][cw]
 *   w_planes DEVICE [w_bits][Cout][kh][kw][cw]
 *   scale    DEVICE fp32 [Cout]; required iff out or next_planes is given
 *   acc      DEVICE out int32 [B][Ho][Wo][Cout], or NULL
 *   out      DEVICE out fp32  [B][Ho][Wo][Cout], or NULL
 *   next_planes DEVICE out [next_bits][B][Ho][Wo][ceil(Cout/32)], or NULL: the fused epilogue
 *            out -> qnn_encode_pack(out, clip = next_clip, bits = next_bits), so the next
 *            layer's planes are produced without the accumulator leaving the chip.
 * At least one of acc / out / next_planes must be given.  kh, kw in [1,7].  Bit widths above 4 run as
 * plane chunks like qnn_binary_gemm and need acc or out for the running sum (QNN_ERR_UNSUPPORTED with
 * next_planes alone).
 */
typedef struct qnn_conv_desc {
    int64_t B, H, W, Cin, Cout;
    int32_t kh, kw, stride, pad;
    int32_t a_bits, w_bits;
} qnn_conv_desc;

int qnn_conv2d(const qnn_conv_desc *desc, const uint32_t *a_planes, const uint32_t *w_planes,
               const float *scale, int32_t *acc, float *out, uint32_t *next_planes,
               float next_clip, int next_bits, void *stream);

/*
 * qnn_conv2d_dilated -- qnn_conv2d with the taps `dilation` pixels apart: tap (ky, kx) of output pixel (ho, wo) reads
 * input pixel (ho stride + ky dilation - pad, wo stride + kx dilation - pad); Ho = (H + 2 pad - dilation (kh - 1) - 1)
 * / stride + 1.  The detection network of the experiments section (SSD on a backbone) has one such layer.  Everything
 * else -- operands, outputs, the fused next-layer epilogue, padding, bit widths, errors -- as qnn_conv2d;
 * dilation = 1 is qnn_conv2d.  QNN_ERR_INVALID_ARG for dilation < 1, QNN_ERR_UNSUPPORTED above 64.
 * qnn_level_conv2d_dilated_i8 / _fp4: the same for qnn_level_conv2d_i8 / qnn_level_conv2d_fp4 (matrix-core route).
 */
int qnn_conv2d_dilated(const qnn_conv_desc *desc, int dilation, const uint32_t *a_planes, const uint32_t *w_planes,
                       const float *scale, int32_t *acc, float *out, uint32_t *next_planes, float next_clip,
                       int next_bits, void *stream);
int qnn_level_conv2d_dilated_i8(const qnn_conv_desc *desc, int dilation, const int8_t *a_levels, const int8_t *w_levels,
                                const float *scale, int32_t *acc, float *out, int8_t *next_levels, float next_clip,
                                int next_bits, void *stream);
int qnn_level_conv2d_dilated_fp4(const qnn_conv_desc *desc, int dilation, const uint8_t *a_levels, const uint8_t *w_levels,
                                 const float *scale, int32_t *acc, float *out, uint8_t *next_levels, float next_clip,
                                 int next_bits, void *stream);

/*
 * qnn_conv2d_chain_static -- qnn_conv2d in its layer-to-layer form (planes in, the next layer's planes out, no acc
 * and no out) for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Above 4 bits qnn_conv2d needs an acc or out buffer for the running int32 sum of
 * its plane-chunk launches; such callers have none to lend, so here that sum lives in a device array that is part
 * of the library image: qnn_conv2d_chain_static_max_outputs() = 2^23 int32 (32 MiB on every GPU the library
 * runs on, held until the process ends).  The call allocates and frees nothing and gives the same next_planes,
 * bit for bit, as qnn_conv2d with a caller-owned acc.  Up to 4 bits it is qnn_conv2d(acc = out = NULL).
 *   arguments as qnn_conv2d; scale and next_planes are required.
 *   QNN_ERR_RANGE when B Ho Wo Cout exceeds qnn_conv2d_chain_static_max_outputs() (nothing is enqueued): use
 *   qnn_conv2d with a buffer of your own.  Other errors as qnn_conv2d.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams, or
 * different host threads without ordering between their streams) race on it.  Calls on one stream are ordered.  The first plane-chunk launch of
 * a call overwrites the array, so no state carries over from one call to the next.
 */
int64_t qnn_conv2d_chain_static_max_outputs(void);
int qnn_conv2d_chain_static(const qnn_conv_desc *desc, const uint32_t *a_planes, const uint32_t *w_planes,
                            const float *scale, uint32_t *next_planes, float next_clip, int next_bits, void *stream);

/*
 * qnn_conv2d_block -- qnn_conv2d with the terms a residual block puts between the scale factor and
 * the next quantizer (the experiments section's ResNet-18 has shortcuts and batch normalisation; the
 * derivation itself leaves the bias out).  With epi == NULL it is qnn_conv2d.  Otherwise, per output
 * element, in fp32 with one rounding per step and in this order:
 *     y = (float)acc * scale[c]
 *     y = y + bias[c]                               if bias     (a folded batch-norm shift)
 *     y = y + ((float)res_level * res_scale)        if res_q    (shortcut held as quantized codes)
 *     y = y + res_f32[...]                          if res_f32  (shortcut held in fp32)
 *     y = max(y, 0)                                 if relu     (HReLU's lower limit, Table 1)
 * `out` receives y and next_planes its codes; `acc` stays the integer product.
 *   bias     DEVICE fp32 [Cout], or NULL
 *   res_q    DEVICE bit-planes [res_bits][B][Ho][Wo][ceil(Cout/32)] (as qnn_encode_pack or a fused
 *            epilogue writes them for a tensor of the output's shape), or NULL; level = 2 u - (2^res_bits - 1)
 *            (Eq. 10); res_bits in [1,8]; res_scale finite: the real value of one level step, e.g.
 *            clip / (2^res_bits - 1) for codes made with that clip
 *   res_f32  DEVICE fp32 [B][Ho][Wo][Cout], or NULL
 * All three 16-byte aligned; scale is required when epi is given.
 */
typedef struct qnn_block_epilogue {
    const float *bias;
    const void *res_q;
    int32_t res_bits;
    float res_scale;
    const float *res_f32;
    int32_t relu; /* nonzero: y = max(y, 0) after the other terms -- the lower limit of HReLU (Table 1); the upper
                     one is the next quantizer's clip, so the encoder sees clamp(y / clip, 0, 1) */
} qnn_block_epilogue;

int qnn_conv2d_block(const qnn_conv_desc *desc, const uint32_t *a_planes, const uint32_t *w_planes,
                     const float *scale, const qnn_block_epilogue *epi, int32_t *acc, float *out,
                     uint32_t *next_planes, float next_clip, int next_bits, void *stream);

/*
 * qnn_deconv2d -- transposed convolution ("deconvolution"; section "Model Decomposition": deconvolution
 * layers reduce to the same vector products) on bit-planes:
 *     acc[b][y][x][co] = sum over (i, ky), (j, kx) with i stride + ky - pad = y, j stride + kx - pad = x
 *                        of a[b][i][j][:] . w[co][ky][kx][:],    Ho = (H - 1) stride - 2 pad + kh, Wo likewise.
 * For one output row only every stride-th kernel row takes part, so the stride x stride phases of the
 * output are ordinary stride-1 convolutions with the (flipped) sub-kernels, run as that many launches of
 * qnn_conv2d's kernel, each writing every stride-th output pixel per axis.
 *
 * qnn_deconv_phase_words: uint32 words of the phase-ordered weight planes (-1 for a bad geometry).
 * qnn_deconv_pack_weights: w_planes DEVICE [w_bits][Cout][kh][kw][ceil(Cin/32)] (as for qnn_conv2d) ->
 *     phase_planes DEVICE, qnn_deconv_phase_words(...) words: for fy, fx in 0..stride-1 (fy outer), the
 *     planes [w_bits][Cout][Ty][Tx][ceil(Cin/32)] of the taps ky = fy + t stride, kx = fx + t' stride in
 *     flipped order, each phase starting at a multiple of 4 words.  Done once per layer.
 * qnn_deconv2d: desc->H, W, Cin describe the input, Cout / kh / kw / stride / pad the transposed
 *     convolution; a_planes DEVICE [a_bits][B][H][W][ceil(Cin/32)]; scale, acc, out, next_planes,
 *     next_clip, next_bits as in qnn_conv2d on the [B][Ho][Wo][Cout] output; bias DEVICE fp32 [Cout] or
 *     NULL, added after the scale as in qnn_conv2d_block.  Bit widths above 4 run as plane chunks like qnn_conv2d and
 *     need acc or out for the running sum.  QNN_ERR_UNSUPPORTED for kh or kw below stride (output pixels that no
 *     tap reaches) or above 16, stride above 8.
 */
int64_t qnn_deconv_phase_words(int w_bits, int64_t Cout, int kh, int kw, int64_t Cin, int stride);
int qnn_deconv_pack_weights(const uint32_t *w_planes, int w_bits, int64_t Cout, int kh, int kw, int64_t Cin,
                            int stride, uint32_t *phase_planes, void *stream);
int qnn_deconv2d(const qnn_conv_desc *desc, const uint32_t *a_planes, const uint32_t *phase_planes,
                 const float *scale, const float *bias, int32_t *acc, float *out, uint32_t *next_planes,
                 float next_clip, int next_bits, void *stream);

/*
 * qnn_maxpool_planes / qnn_maxpool_levels_i8 -- max-pooling between quantized layers, taken on the
 * codes.  The linear quantizer (Table 1 range limit, Eq. 15) is monotone non-decreasing, so the
 * maximum of quantized values over a window equals the quantized maximum: pooling planes is exact.
 * Window k x k (k <= 7), `stride`, `pad` (2 pad <= k); window elements outside the image are ignored.
 *   Ho = qnn_pool_out_size(H, k, stride, pad, ceil_mode): floor((H + 2 pad - k) / stride) + 1, or with
 *   ceil_mode != 0 the ceiling of the quotient, less one if the last window would start past H + pad;
 *   -1 for an invalid geometry.
 *   planes     DEVICE [bits][B][H][W][ceil(C/32)]  ->  out_planes DEVICE [bits][B][Ho][Wo][ceil(C/32)]
 *   levels     DEVICE int8 [B][H][W][C]            ->  out_levels DEVICE int8 [B][Ho][Wo][C]
 */
int64_t qnn_pool_out_size(int64_t size, int k, int stride, int pad, int ceil_mode);
int qnn_maxpool_planes(const uint32_t *planes, int bits, int64_t B, int64_t H, int64_t W, int64_t C, int k,
                       int stride, int pad, int ceil_mode, uint32_t *out_planes, void *stream);
int qnn_maxpool_levels_i8(const int8_t *levels, int64_t B, int64_t H, int64_t W, int64_t C, int k, int stride,
                          int pad, int ceil_mode, int8_t *out_levels, void *stream);

/*
 * Training-side gradients (sections "Multi-Branch Binary Networks Training" and "Quantized Networks
 * Training"), elementwise; x, the gradients and grad_x are DEVICE fp32, 16-byte aligned, count elements.
 *
 * qnn_quantize_ste_backward: the straight-through gradient of the hard ladder q_k (Eq. 15) behind the
 *     range limit HTanh (Table 1): with t = x * (1 / clip) in fp32,
 *         grad_x = grad_q * (1 / clip)  where -1 <= t <= 1,  0 elsewhere.
 *     grad_q is the gradient w.r.t. q_k(HTanh(x / clip)) in [-1, 1] (= level / (2^k - 1)).  With clip = 1
 *     it is also the gradient of Binarize(x) = sign(HTanh(x)) (Eq. 14), whose forward is
 *     qnn_encode_pack with bits = 1.
 * qnn_encoder_backward: the surrogate gradient of the M-bit encoder (Eq. 12-13 for M = 2).  Plane m
 *     (m = 1 lowest; grad_planes DEVICE fp32 [bits][count], index m - 1) is the sign of +sin(pi K t / 2^M)
 *     for m = M and of -sin(pi K t / 2^m) below, K = 2^M - 1; its derivative is the sine's on [-1, 1]:
 *         grad_x = (1 / clip) * sum_m grad_planes[m] * (+-)(pi K / 2^m) cos(pi K t / 2^m),  0 outside.
 *     fp32 arithmetic; the cosine's argument t K / 2^m carries one rounding and is reduced exactly
 *     (cospi), so with s_m = pi K / 2^m the result is within
 *     (1 / clip) sum_m |grad_planes[m]| s_m (s_m + 4) 2^-24 of the value in real arithmetic.
 */
int qnn_quantize_ste_backward(const float *x, const float *grad_q, int64_t count, float clip, float *grad_x,
                              void *stream);
int qnn_encoder_backward(const float *x, const float *grad_planes, int64_t count, float clip, int bits,
                         float *grad_x, void *stream);

/*
 * Bit-plane-sum variant on the matrix cores (for comparison with qnn_binary_gemm; same integers).
 * The M x K branch sum of Eq. 9 equals the integer dot product of the decoded levels (Eq. 7-10),
 * so one can also sum the 2^j-weighted planes back into int8 levels and contract those with int8
 * MFMA instructions.  Bit widths 1..7 (levels must fit int8).
 *
 * qnn_level_row_bytes(n): bytes per row of a level tensor = n rounded up to a multiple of 128.
 * qnn_plane_sum_i8: planes DEVICE [bits][rows][ceil(n/32)] -> levels DEVICE int8
 *     [rows][qnn_level_row_bytes(n)], level = sum_j 2^j (2 b_j - 1), bytes past n written as 0.
 * qnn_level_gemm_i8: acc[r][c] = sum_k a[r][k] w[c][k] (int32, exact), optional
 *     out[r][c] = (float)acc[r][c] * scale[c]; a_levels / w_levels as written by qnn_plane_sum_i8.
 *     acc / out / scale as in qnn_binary_gemm.
 */
int64_t qnn_level_row_bytes(int64_t n);
int qnn_plane_sum_i8(const uint32_t *planes, int bits, int64_t rows, int64_t n, int8_t *levels,
                     void *stream);
int qnn_level_gemm_i8(const int8_t *a_levels, const int8_t *w_levels, int64_t rows, int64_t cols,
                      int64_t n, int32_t *acc, const float *scale, float *out, void *stream);

/*
 * The same variant for 1- and 2-bit codes on the fp4 matrix-core path: the levels -3, -1, +1, +3 are
 * exact fp4 (E2M1) values, products and partial sums are integers that fp32 accumulates exactly
 * while 9 n < 2^24 (QNN_ERR_RANGE beyond), and the instruction runs twice as many multiply-adds per
 * clock as the int8 one on half the bytes.
 *
 * qnn_fp4_row_bytes(n): bytes per row of an fp4 level tensor = n / 2 rounded up to a multiple of 128.
 * qnn_plane_sum_fp4: planes DEVICE [bits][rows][ceil(n/32)], bits 1 or 2 -> levels DEVICE uint8
 *     [rows][qnn_fp4_row_bytes(n)], element 2i in the low nibble of byte i, nibble = sign << 3 | E2M1
 *     magnitude (1 = 0b0010, 3 = 0b0101), nibbles past n written as 0.
 * qnn_level_gemm_fp4: as qnn_level_gemm_i8 on such tensors; acc is the exact int32 value.
 */
int64_t qnn_fp4_row_bytes(int64_t n);
int qnn_plane_sum_fp4(const uint32_t *planes, int bits, int64_t rows, int64_t n, uint8_t *levels,
                      void *stream);
int qnn_level_gemm_fp4(const uint8_t *a_levels, const uint8_t *w_levels, int64_t rows, int64_t cols,
                       int64_t n, int32_t *acc, const float *scale, float *out, void *stream);

/*
 * Decoded-level convolution on the matrix cores (for comparison with qnn_conv2d; same integers).
 * Section "Model Decomposition" reduces a convolution to the vector product of Eq. 7-10; here the
 * levels stay decoded as int8 from layer to layer and the product is an implicit GEMM on int8 MFMA.
 *
 * qnn_encode_levels_i8: the quantizer of qnn_encode_pack (same fp32 steps, Table 1 HTanh, Eq. 15)
 *     followed by level = 2u - (2^bits - 1) (Eq. 10), elementwise.
 *     src DEVICE fp32 / bf16 [count] (QNN_DTYPE_F32 / QNN_DTYPE_BF16), levels DEVICE out int8 [count];
 *     both 16-byte aligned; bits 1..7.
 * qnn_level_conv2d_i8: as qnn_conv2d with int8 levels in place of planes.
 *     a_levels DEVICE int8 [B][H][W][Cin], w_levels DEVICE int8 [Cout][kh][kw][Cin];
 *     acc / out / scale as in qnn_conv2d; next_levels DEVICE out int8 [B][Ho][Wo][Cout], or NULL: the
 *     fused epilogue out -> qnn_encode_levels_i8(out, clip = next_clip, bits = next_bits).
 *     Taps outside the image contribute exactly 0.  desc->a_bits / w_bits (1..7) bound the levels for
 *     the int32 range check only.  QNN_ERR_UNSUPPORTED unless Cin is a multiple of 16, kh * kw <= 31
 *     and kh * kw * Cin <= 16384; QNN_ERR_RANGE when a tensor needs more than 32-bit byte offsets.
 */
int qnn_encode_levels_i8(const void *src, int dtype, int64_t count, float clip, int bits, int8_t *levels,
                         void *stream);
int qnn_level_conv2d_i8(const qnn_conv_desc *desc, const int8_t *a_levels, const int8_t *w_levels,
                        const float *scale, int32_t *acc, float *out, int8_t *next_levels,
                        float next_clip, int next_bits, void *stream);

/*
 * Transposed convolution on decoded levels (matrix-core route of qnn_deconv2d; section "Model Decomposition":
 * deconvolution layers reduce to the same products).  With stride s and padding p it equals the stride-1
 * convolution, padding k - 1 - p, of the input with s - 1 zeros inserted between neighbouring pixels and the
 * kernel flipped in both axes; a zero byte is level 0 (int8) or a pair of +0 (fp4) and contributes exactly 0,
 * like the convolution's own padding, so the level convolution runs on the widened tensor as it is.
 *   qnn_level_deconv_workspace_bytes(desc, fp4): bytes of the widened tensor, B ((H-1) s + 1) ((W-1) s + 1) Cin
 *     (Cin / 2 for fp4); -1 on bad geometry.
 *   qnn_level_deconv_flip_weights: w_levels DEVICE [Cout][kh][kw][tap_bytes] -> flipped DEVICE, same shape, tap
 *     (ky, kx) taken from (kh-1-ky, kw-1-kx); tap_bytes = Cin (int8) or Cin / 2 (fp4), a multiple of 16.  Once per layer.
 *   qnn_level_deconv2d_i8 / _fp4: desc as for qnn_deconv2d (H, W, Cin of the input; Cout, kh, kw, stride, pad of the
 *     transposed convolution); a_levels DEVICE [B][H][W][Cin (/2)]; flipped_w from qnn_level_deconv_flip_weights;
 *     workspace DEVICE, qnn_level_deconv_workspace_bytes bytes, 16-byte aligned, owned by the caller and
 *     overwritten by every call; scale, acc, out, next_levels, next_clip, next_bits as in qnn_level_conv2d_i8 / _fp4
 *     on the [B][Ho][Wo][Cout] output, Ho = (H-1) s - 2 p + kh; bias DEVICE fp32 [Cout] or NULL, added after the scale.
 *   QNN_ERR_UNSUPPORTED unless kh == kw and pad <= kh - 1; other limits and errors as qnn_level_conv2d_i8 / _fp4
 *   (the reduction-length checks count all kh kw taps).  Every check precedes the first launch.
 */
int64_t qnn_level_deconv_workspace_bytes(const qnn_conv_desc *desc, int fp4);
int qnn_level_deconv_flip_weights(const void *w_levels, int64_t Cout, int kh, int kw, int64_t tap_bytes, void *flipped,
                                  void *stream);
int qnn_level_deconv2d_i8(const qnn_conv_desc *desc, const int8_t *a_levels, const int8_t *flipped_w, void *workspace,
                          const float *scale, const float *bias, int32_t *acc, float *out, int8_t *next_levels,
                          float next_clip, int next_bits, void *stream);
int qnn_level_deconv2d_fp4(const qnn_conv_desc *desc, const uint8_t *a_levels, const uint8_t *flipped_w, void *workspace,
                           const float *scale, const float *bias, int32_t *acc, float *out, uint8_t *next_levels,
                           float next_clip, int next_bits, void *stream);

/*
 * qnn_level_conv2d_block_i8 -- qnn_level_conv2d_i8 with the residual-block terms of qnn_conv2d_block
 * (same steps, same order); here epi->res_q is DEVICE int8 levels [B][Ho][Wo][Cout] and res_bits only
 * bounds them (1..7).
 */
int qnn_level_conv2d_block_i8(const qnn_conv_desc *desc, const int8_t *a_levels, const int8_t *w_levels,
                              const float *scale, const qnn_block_epilogue *epi, int32_t *acc, float *out,
                              int8_t *next_levels, float next_clip, int next_bits, void *stream);

/*
 * The decoded-level convolution for 1- and 2-bit codes on the fp4 matrix-core path (as
 * qnn_level_gemm_fp4: the levels -3, -1, +1, +3 are exact fp4 values, fp32 accumulates their products
 * exactly while 9 kh kw Cin < 2^24).  Level tensors hold two channels per byte, channel 2i in the low
 * nibble of byte i, nibble = sign << 3 | E2M1 magnitude (1 = 0b0010, 3 = 0b0101).
 *
 * qnn_encode_levels_fp4: as qnn_encode_levels_i8 (bits 1 or 2, count even) -> DEVICE uint8 [count / 2].
 * qnn_levels_to_fp4: int8 levels (odd, |level| <= 3) DEVICE [count], count even -> DEVICE uint8 [count / 2]
 *     (weights, once per layer).
 * qnn_level_conv2d_fp4: as qnn_level_conv2d_i8 with a_levels DEVICE uint8 [B][H][W][Cin / 2], w_levels
 *     DEVICE uint8 [Cout][kh][kw][Cin / 2], next_levels DEVICE out uint8 [B][Ho][Wo][Cout / 2]; acc is the
 *     exact int32 value.  QNN_ERR_UNSUPPORTED unless a_bits, w_bits <= 2, Cin is a multiple of 32 and (with
 *     next_levels) Cout is even; QNN_ERR_RANGE beyond the exact range of fp32 accumulation.
 */
int qnn_encode_levels_fp4(const void *src, int dtype, int64_t count, float clip, int bits, uint8_t *levels,
                          void *stream);
int qnn_levels_to_fp4(const int8_t *levels, int64_t count, uint8_t *fp4, void *stream);
int qnn_level_conv2d_fp4(const qnn_conv_desc *desc, const uint8_t *a_levels, const uint8_t *w_levels,
                         const float *scale, int32_t *acc, float *out, uint8_t *next_levels,
                         float next_clip, int next_bits, void *stream);
/* qnn_level_conv2d_block_fp4: qnn_level_conv2d_fp4 with the residual-block terms of qnn_conv2d_block; epi->res_q is
 * DEVICE uint8 fp4 levels [B][Ho][Wo][Cout / 2] of a 1- or 2-bit code (Cout even). */
int qnn_level_conv2d_block_fp4(const qnn_conv_desc *desc, const uint8_t *a_levels, const uint8_t *w_levels,
                               const float *scale, const qnn_block_epilogue *epi, int32_t *acc, float *out,
                               uint8_t *next_levels, float next_clip, int next_bits, void *stream);
/* qnn_maxpool_levels_fp4: qnn_maxpool_levels_i8 on fp4 levels, DEVICE uint8 [B][H][W][C / 2] -> [B][Ho][Wo][C / 2], C even. */
int qnn_maxpool_levels_fp4(const uint8_t *levels, int64_t B, int64_t H, int64_t W, int64_t C, int k, int stride,
                           int pad, int ceil_mode, uint8_t *out_levels, void *stream);

/*
 * qnn_fc_fused -- qnn_encode_pack followed by qnn_binary_gemm (Fig. 1: encoders, M x K binary branches, decoder
 * with its scale) in ONE launch, for layers too small to fill the chip, where the two-launch form costs the
 * device's latency from one dependent kernel to the next.  Same results, bit for bit; the activation planes
 * never reach memory.
 *   src  DEVICE in, [rows][row_stride_elems] of dtype (QNN_DTYPE_F32 / BF16 values quantized with clip and
 *        a_bits as qnn_encode_pack does, or QNN_DTYPE_I8 odd levels), n elements used per row
 *   w_planes  DEVICE in uint32 [w_bits][cols][ceil(n/32)];  scale  DEVICE in fp32 [cols] (required with out)
 *   acc  DEVICE out int32 [rows][cols] or NULL;  out  DEVICE out fp32 [rows][cols] or NULL (at least one)
 * QNN_ERR_UNSUPPORTED when a_bits * ceil(n/32) exceeds 1024 words (the planes of 4 rows must fit 16 KiB of LDS:
 * use the two-launch form); otherwise the argument errors of the two calls it replaces.
 */
int qnn_fc_fused(const void *src, int dtype, int64_t rows, int64_t n, int64_t row_stride_elems, float clip, int a_bits,
                 const uint32_t *w_planes, int w_bits, int64_t cols, const float *scale, int32_t *acc, float *out,
                 void *stream);

/*
 * The unquantized ends of a network (the ResNet-18 workload of the ImageNet experiment keeps its first
 * convolution and its classifier in full precision; nothing of Eq. 9 is involved).  fp32 throughout,
 * products and sums on the matrix cores in fp32: a result differs from the real-number value by at most
 * a small multiple of 2^-24 sum |x| |w| (the summation order is the kernel's own).
 *
 * qnn_dense_conv2d_f32: y[b][ho][wo][c] = sum over (ky, kx, ci) of x[b][ho stride + ky - pad][wo stride + kx - pad][ci]
 *     w[c][ky][kx][ci] (taps outside the image contribute 0), then y * scale[c] (if scale), + shift[c] (if shift),
 *     max(y, 0) (if relu), one fp32 operation each.
 *   x  DEVICE in fp32 [B][H][W][Cin];  w  DEVICE in fp32 [Cout][kh][kw][Cin];  scale, shift  DEVICE in fp32 [Cout] or NULL
 *   out  DEVICE out fp32 [B][Ho][Wo][Cout] or NULL, Ho = (H + 2 pad - kh) / stride + 1
 *   next_planes  DEVICE out uint32 [next_bits][B Ho Wo][ceil(Cout / 32)] or NULL: the planes qnn_encode_pack would
 *     make of y with (next_clip, next_bits) -- the first quantized layer's input without y going through memory
 *   At least one output; all pointers 16-byte aligned; the caller owns every buffer.  QNN_ERR_INVALID_ARG,
 *   QNN_ERR_ALIGNMENT, QNN_ERR_RANGE (2^31 output pixels, 2^24 reduction values or more) before any launch.
 * qnn_global_avgpool_f32: out[b][c] = (sum over the hw positions of x[b][.][c]) / hw; x DEVICE fp32 [B][hw][C],
 *     out DEVICE fp32 [B][C].
 * qnn_dense_fc_f32: out[r][o] = sum_i x[r][i] w[o][i] + bias[o] (Eq. 1 on unquantized values); x DEVICE fp32
 *     [rows][n], w DEVICE fp32 [cols][n], bias DEVICE fp32 [cols] or NULL, out DEVICE fp32 [rows][cols].
 */
typedef struct {
    int64_t B, H, W, Cin, Cout;
    int kh, kw, stride, pad;
} qnn_dense_conv_desc;
int qnn_dense_conv2d_f32(const qnn_dense_conv_desc *desc, const float *x, const float *w, const float *scale,
                         const float *shift, int relu, float *out, uint32_t *next_planes, float next_clip,
                         int next_bits, void *stream);
/* qnn_dense_conv2d_f32_levels: the same layer with the quantized output as int8 levels 2 u - (2^next_bits - 1), DEVICE out
 * int8 [B][Ho][Wo][Cout] or NULL (next_bits <= 7): the input of qnn_level_conv2d_i8 / qnn_maxpool_levels_i8. */
int qnn_dense_conv2d_f32_levels(const qnn_dense_conv_desc *desc, const float *x, const float *w, const float *scale,
                                const float *shift, int relu, float *out, int8_t *next_levels, float next_clip,
                                int next_bits, void *stream);
int qnn_global_avgpool_f32(const float *x, int64_t B, int64_t hw, int64_t C, float *out, void *stream);
int qnn_dense_fc_f32(const float *x, const float *w, const float *bias, int64_t rows, int64_t cols, int64_t n,
                     float *out, void *stream);

/* Message for the last error returned on the calling thread ("" if none). Never NULL. */
const char *qnn_last_error(void);

/* Library version: major * 10000 + minor * 100 + patch. */
int qnn_version(void);

/* Hex digest of the source files this library was compiled from (the build script passes it in; "" when built by
 * hand).  The Python binding compares it with the sources beside it and rebuilds a library that is out of date. */
const char *qnn_build_id(void);

#ifdef __cplusplus
}
#endif
#endif /* QNN_H_ */
