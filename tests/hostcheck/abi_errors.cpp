// Sanitizer run of the host side of libqnn (tests/test_sanitized_host.py builds the library's sources host-only
// under -fsanitize=address,undefined and links them with hip_runtime_stub.cpp instead of the HIP runtime).
// Every entry point of include/qnn.h is called with arguments it must refuse; the checks must (1) return a
// negative QNN_ERR_* code, (2) leave a message, (3) make no HIP call at all -- argument errors are found on the
// host before anything is enqueued -- and (4) do so without the sanitizers finding a bad access, overflow or
// shift in the checking code itself (descriptors are read, sizes multiplied, messages formatted).
#include <initializer_list>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/qnn.h"

extern "C" int hipstub_device_calls(void);

static int g_failures = 0, g_calls = 0;

static void expect(int rc, int want, const char *what, int line)
{
    ++g_calls;
    const bool code_ok = want == 0 ? rc == QNN_OK : (want == 1 ? rc < 0 : rc == want);
    if (!code_ok) {
        fprintf(stderr, "abi_errors line %d: %s returned %d, expected %s%d\n", line, what, rc, want == 1 ? "any error, not " : "", want);
        ++g_failures;
    }
    if (rc < 0 && strlen(qnn_last_error()) == 0) {
        fprintf(stderr, "abi_errors line %d: %s failed without a message\n", line, what);
        ++g_failures;
    }
    if (hipstub_device_calls() != 0) {
        fprintf(stderr, "abi_errors line %d: %s made a HIP call before rejecting its arguments\n", line, what);
        exit(1);
    }
}
#define EXPECT(call, want) expect((call), (want), #call, __LINE__)
#define ANY_ERROR 1

int main()
{
    uint32_t *FAKE = reinterpret_cast<uint32_t *>(0x1000); // 16-byte aligned, never dereferenced
    uint32_t *ODD = reinterpret_cast<uint32_t *>(0x1004);
    float *FF = reinterpret_cast<float *>(0x2000);
    int32_t *FI = reinterpret_cast<int32_t *>(0x3000);
    int8_t *F8 = reinterpret_cast<int8_t *>(0x4000);
    uint8_t *FU = reinterpret_cast<uint8_t *>(0x5000);
    const float nanv = nanf(""), inf = INFINITY;
    const int64_t big = INT64_MAX / 2;

    // qnn_encode_pack
    EXPECT(qnn_encode_pack(FAKE, 7, 4, 64, 64, 1.0f, 2, FAKE, nullptr), QNN_ERR_UNSUPPORTED);
    for (int bits : {0, -1, 9, 1 << 30}) EXPECT(qnn_encode_pack(FAKE, 0, 4, 64, 64, 1.0f, bits, FAKE, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_encode_pack(FAKE, 0, -1, 64, 64, 1.0f, 2, FAKE, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_encode_pack(FAKE, 0, 4, 64, 32, 1.0f, 2, FAKE, nullptr), QNN_ERR_INVALID_ARG);
    for (float clip : {0.0f, -1.0f, nanv, inf}) EXPECT(qnn_encode_pack(FAKE, 0, 4, 64, 64, clip, 2, FAKE, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_encode_pack(nullptr, 0, 4, 64, 64, 1.0f, 2, FAKE, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_encode_pack(FAKE, 0, 4, 64, 64, 1.0f, 2, ODD, nullptr), QNN_ERR_ALIGNMENT);
    EXPECT(qnn_encode_pack(FAKE, 2, 4, 64, 64, 1.0f, 8, FAKE, nullptr), QNN_ERR_UNSUPPORTED);
    EXPECT(qnn_encode_pack(nullptr, 0, 0, 64, 64, 1.0f, 2, nullptr, nullptr), 0);

    // qnn_binary_gemm
    EXPECT(qnn_binary_gemm(FAKE, 0, FAKE, 2, 4, 4, 64, FI, nullptr, nullptr, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_binary_gemm(FAKE, 2, FAKE, 9, 4, 4, 64, FI, nullptr, nullptr, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_binary_gemm(FAKE, 2, FAKE, 2, -4, 4, 64, FI, nullptr, nullptr, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_binary_gemm(FAKE, 2, FAKE, 2, 4, 4, 64, nullptr, nullptr, nullptr, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_binary_gemm(FAKE, 2, FAKE, 2, 4, 4, 64, nullptr, nullptr, FF, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_binary_gemm(ODD, 2, FAKE, 2, 4, 4, 64, FI, nullptr, nullptr, nullptr), QNN_ERR_ALIGNMENT);
    EXPECT(qnn_binary_gemm(FAKE, 8, FAKE, 8, 4, 4, 33026, FI, nullptr, nullptr, nullptr), QNN_ERR_RANGE);
    EXPECT(qnn_binary_gemm(FAKE, 8, FAKE, 8, big, big, big, FI, nullptr, nullptr, nullptr), ANY_ERROR);

    // qnn_dequant_scale
    EXPECT(qnn_dequant_scale(nullptr, FF, 4, 4, FF, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_dequant_scale(FI, FF, -1, 4, FF, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_dequant_scale(FI, FF, 4, 4, reinterpret_cast<float *>(ODD), nullptr), QNN_ERR_ALIGNMENT);

    // qnn_conv2d / qnn_conv2d_block / qnn_conv2d_chain_static / qnn_deconv2d: descriptors
    const qnn_conv_desc ok = {1, 8, 8, 64, 64, 3, 3, 1, 1, 2, 2};
    auto with = [&](auto edit) { qnn_conv_desc d = ok; edit(d); return d; };
    const qnn_conv_desc bad[] = {
        with([](qnn_conv_desc &d) { d.a_bits = 0; }),    with([](qnn_conv_desc &d) { d.w_bits = 9; }),
        with([](qnn_conv_desc &d) { d.H = 0; }),         with([](qnn_conv_desc &d) { d.Cin = -5; }),
        with([](qnn_conv_desc &d) { d.stride = 0; }),    with([](qnn_conv_desc &d) { d.pad = -1; }),
        with([](qnn_conv_desc &d) { d.kh = d.kw = 9; }), with([](qnn_conv_desc &d) { d.H = d.W = 2, d.kh = d.kw = 8, d.pad = 0; }),
        with([](qnn_conv_desc &d) { d.B = big, d.H = d.W = 1 << 20; }), with([](qnn_conv_desc &d) { d.Cin = 4096, d.a_bits = d.w_bits = 8; }),
        with([](qnn_conv_desc &d) { d.Cout = big; }),    with([](qnn_conv_desc &d) { d.kh = INT32_MAX, d.kw = INT32_MAX; }),
    };
    for (const qnn_conv_desc &d : bad) {
        EXPECT(qnn_conv2d(&d, FAKE, FAKE, FF, FI, nullptr, nullptr, 0.0f, 0, nullptr), ANY_ERROR);
        EXPECT(qnn_conv2d_block(&d, FAKE, FAKE, FF, nullptr, FI, FF, FAKE, 1.0f, 2, nullptr), ANY_ERROR);
        // a transposed convolution accepts kernels up to 16 x 16 and kernels larger than its input
        if (d.kh <= 7 || d.kh > 16)
            EXPECT(qnn_deconv2d(&d, FAKE, FAKE, FF, nullptr, FI, nullptr, nullptr, 0.0f, 0, nullptr), ANY_ERROR);
        EXPECT(qnn_level_conv2d_i8(&d, F8, F8, FF, FI, nullptr, nullptr, 0.0f, 0, nullptr), ANY_ERROR);
        EXPECT(qnn_level_conv2d_fp4(&d, FU, FU, FF, FI, nullptr, nullptr, 0.0f, 0, nullptr), ANY_ERROR);
        EXPECT(qnn_conv2d_dilated(&d, 2, FAKE, FAKE, FF, FI, nullptr, nullptr, 0.0f, 0, nullptr), ANY_ERROR);
        EXPECT(qnn_level_conv2d_dilated_i8(&d, 2, F8, F8, FF, FI, nullptr, nullptr, 0.0f, 0, nullptr), ANY_ERROR);
    }
    EXPECT(qnn_conv2d_dilated(&ok, 0, FAKE, FAKE, FF, FI, nullptr, nullptr, 0.0f, 0, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_conv2d_dilated(&ok, INT32_MAX, FAKE, FAKE, FF, FI, nullptr, nullptr, 0.0f, 0, nullptr), QNN_ERR_UNSUPPORTED);
    EXPECT(qnn_level_conv2d_dilated_i8(&ok, INT32_MAX, F8, F8, FF, FI, nullptr, nullptr, 0.0f, 0, nullptr), QNN_ERR_UNSUPPORTED);
    EXPECT(qnn_conv2d_dilated(&ok, 5, FAKE, FAKE, FF, FI, nullptr, nullptr, 0.0f, 0, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_conv2d(nullptr, FAKE, FAKE, FF, FI, nullptr, nullptr, 0.0f, 0, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_conv2d(&ok, FAKE, FAKE, nullptr, nullptr, nullptr, nullptr, 0.0f, 0, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_conv2d(&ok, FAKE, FAKE, nullptr, nullptr, FF, nullptr, 0.0f, 0, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_conv2d(&ok, FAKE, FAKE, FF, nullptr, nullptr, FAKE, 1.0f, 0, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_conv2d(&ok, FAKE, FAKE, FF, nullptr, nullptr, FAKE, nanv, 2, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_conv2d(&ok, nullptr, FAKE, FF, FI, nullptr, nullptr, 0.0f, 0, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_conv2d(&ok, FAKE, ODD, FF, FI, nullptr, nullptr, 0.0f, 0, nullptr), QNN_ERR_ALIGNMENT);
    const qnn_conv_desc wide = with([](qnn_conv_desc &d) { d.a_bits = d.w_bits = 5; });
    EXPECT(qnn_conv2d(&wide, FAKE, FAKE, FF, nullptr, nullptr, FAKE, 1.0f, 2, nullptr), QNN_ERR_UNSUPPORTED);

    qnn_block_epilogue epi = {FF, FAKE, 0, 1.0f, nullptr, 0};
    EXPECT(qnn_conv2d_block(&ok, FAKE, FAKE, FF, &epi, FI, nullptr, nullptr, 0.0f, 0, nullptr), ANY_ERROR); // res_bits = 0
    epi.res_bits = 2, epi.res_scale = nanv;
    EXPECT(qnn_conv2d_block(&ok, FAKE, FAKE, FF, &epi, FI, nullptr, nullptr, 0.0f, 0, nullptr), ANY_ERROR);
    epi.res_scale = 1.0f, epi.res_f32 = reinterpret_cast<float *>(ODD);
    EXPECT(qnn_conv2d_block(&ok, FAKE, FAKE, FF, &epi, FI, nullptr, nullptr, 0.0f, 0, nullptr), ANY_ERROR);
    epi.res_f32 = nullptr;
    EXPECT(qnn_conv2d_block(&ok, FAKE, FAKE, nullptr, &epi, FI, nullptr, nullptr, 0.0f, 0, nullptr), ANY_ERROR); // no scale
    EXPECT(qnn_level_conv2d_block_i8(&ok, F8, F8, nullptr, &epi, FI, nullptr, nullptr, 0.0f, 0, nullptr), ANY_ERROR);
    EXPECT(qnn_level_conv2d_block_fp4(&ok, FU, FU, nullptr, &epi, FI, nullptr, nullptr, 0.0f, 0, nullptr), ANY_ERROR);

    // the static-accumulator form: too many outputs for its array, and the usual argument errors
    const qnn_conv_desc huge = with([](qnn_conv_desc &d) { d.B = 64, d.H = d.W = 64, d.Cout = 256, d.a_bits = d.w_bits = 5; });
    EXPECT(qnn_conv2d_chain_static(&huge, FAKE, FAKE, FF, FAKE, 1.0f, 2, nullptr), QNN_ERR_RANGE);
    EXPECT(qnn_conv2d_chain_static(&wide, FAKE, FAKE, FF, nullptr, 1.0f, 2, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_conv2d_chain_static(&wide, FAKE, FAKE, nullptr, FAKE, 1.0f, 2, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_conv2d_chain_static(&wide, FAKE, ODD, FF, FAKE, 1.0f, 2, nullptr), QNN_ERR_ALIGNMENT);
    EXPECT(qnn_conv2d_chain_static(&wide, FAKE, FAKE, FF, FAKE, 0.0f, 2, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_conv2d_chain_static(nullptr, FAKE, FAKE, FF, FAKE, 1.0f, 2, nullptr), QNN_ERR_INVALID_ARG);
    if (qnn_conv2d_chain_static_max_outputs() != (int64_t(1) << 23)) ++g_failures;

    // transposed convolution
    EXPECT((int)(qnn_deconv_phase_words(2, 64, 4, 4, 64, 0) >= 0 ? 0 : -1), ANY_ERROR);
    EXPECT((int)(qnn_deconv_phase_words(9, 64, 4, 4, 64, 2) >= 0 ? 0 : -1), ANY_ERROR);
    EXPECT(qnn_deconv_pack_weights(nullptr, 2, 64, 4, 4, 64, 2, FAKE, nullptr), ANY_ERROR);
    EXPECT(qnn_deconv_pack_weights(FAKE, 2, 64, 4, 4, 64, 2, ODD, nullptr), ANY_ERROR);
    const qnn_conv_desc dc = {1, 4, 4, 64, 32, 4, 4, 2, 1, 5, 2};   // above 4 bits the running sum needs acc or out
    EXPECT(qnn_deconv2d(&dc, FAKE, FAKE, FF, nullptr, nullptr, nullptr, FAKE, 1.0f, 2, nullptr), QNN_ERR_UNSUPPORTED);
    // ... on decoded levels: nothing may be enqueued (the widening kernel included) before an error return
    for (const qnn_conv_desc &d : bad) {
        if (d.kh > 7 && d.kh <= 16) continue; // kernels larger than the input are valid transposed convolutions
        EXPECT(qnn_level_deconv2d_i8(&d, F8, F8, FAKE, FF, nullptr, FI, nullptr, nullptr, 0.0f, 0, nullptr), ANY_ERROR);
        EXPECT(qnn_level_deconv2d_fp4(&d, FU, FU, FAKE, FF, nullptr, FI, nullptr, nullptr, 0.0f, 0, nullptr), ANY_ERROR);
    }
    if (qnn_level_deconv_workspace_bytes(nullptr, 0) != -1) ++g_failures;
    const qnn_conv_desc dl = {1, 4, 4, 64, 32, 4, 4, 2, 1, 2, 2};
    EXPECT(qnn_level_deconv2d_i8(&dl, F8, F8, nullptr, FF, nullptr, FI, nullptr, nullptr, 0.0f, 0, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_level_deconv2d_i8(&dl, F8, F8, ODD, FF, nullptr, FI, nullptr, nullptr, 0.0f, 0, nullptr), QNN_ERR_ALIGNMENT);
    EXPECT(qnn_level_deconv2d_i8(&dl, F8, F8, FAKE, nullptr, FF, FI, nullptr, nullptr, 0.0f, 0, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_level_deconv2d_i8(&dl, F8, F8, FAKE, FF, nullptr, nullptr, nullptr, nullptr, 0.0f, 0, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_level_deconv_flip_weights(nullptr, 32, 4, 4, 64, FAKE, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_level_deconv_flip_weights(FAKE, 32, 4, 4, 24, FAKE, nullptr), QNN_ERR_UNSUPPORTED);
    EXPECT(qnn_level_deconv_flip_weights(FAKE, big, 1024, 1024, 64, FAKE, nullptr), QNN_ERR_RANGE);

    // pooling
    if (qnn_pool_out_size(8, 0, 2, 0, 0) != -1 || qnn_pool_out_size(8, 2, 0, 0, 0) != -1 || qnn_pool_out_size(8, 2, 2, 3, 0) != -1) ++g_failures;
    EXPECT(qnn_maxpool_planes(FAKE, 0, 1, 8, 8, 64, 2, 2, 0, 0, FAKE, nullptr), ANY_ERROR);
    EXPECT(qnn_maxpool_planes(FAKE, 2, 1, 8, 8, 64, 9, 2, 0, 0, FAKE, nullptr), ANY_ERROR);
    EXPECT(qnn_maxpool_planes(nullptr, 2, 1, 8, 8, 64, 2, 2, 0, 0, FAKE, nullptr), ANY_ERROR);
    EXPECT(qnn_maxpool_levels_i8(F8, 1, 8, 8, 64, 2, 0, 0, 0, F8, nullptr), ANY_ERROR);
    EXPECT(qnn_maxpool_levels_fp4(FU, 1, 8, 8, 63, 2, 2, 0, 0, FU, nullptr), ANY_ERROR);

    // gradients
    EXPECT(qnn_quantize_ste_backward(nullptr, FF, 16, 1.0f, FF, nullptr), ANY_ERROR);
    EXPECT(qnn_quantize_ste_backward(FF, FF, -1, 1.0f, FF, nullptr), ANY_ERROR);
    EXPECT(qnn_quantize_ste_backward(FF, FF, 16, nanv, FF, nullptr), ANY_ERROR);
    EXPECT(qnn_encoder_backward(FF, FF, 16, 1.0f, 0, FF, nullptr), ANY_ERROR);
    EXPECT(qnn_encoder_backward(FF, FF, 16, 1.0f, 9, FF, nullptr), ANY_ERROR);

    // matrix-core variants
    if (qnn_level_row_bytes(1) != 128 || qnn_fp4_row_bytes(1) != 128) ++g_failures;
    EXPECT(qnn_plane_sum_i8(FAKE, 8, 4, 64, F8, nullptr), ANY_ERROR);
    EXPECT(qnn_plane_sum_i8(nullptr, 2, 4, 64, F8, nullptr), ANY_ERROR);
    EXPECT(qnn_plane_sum_fp4(FAKE, 3, 4, 64, FU, nullptr), ANY_ERROR);
    EXPECT(qnn_level_gemm_i8(F8, F8, 4, 4, 64, nullptr, nullptr, nullptr, nullptr), ANY_ERROR);
    EXPECT(qnn_level_gemm_i8(F8, F8, 4, 4, big, FI, nullptr, nullptr, nullptr), ANY_ERROR);
    EXPECT(qnn_level_gemm_fp4(FU, FU, 4, 4, (1 << 24) / 9 + 1, FI, nullptr, nullptr, nullptr), QNN_ERR_RANGE);
    EXPECT(qnn_encode_levels_i8(FF, 2, 16, 1.0f, 2, F8, nullptr), ANY_ERROR);
    EXPECT(qnn_encode_levels_i8(FF, 0, 16, 1.0f, 8, F8, nullptr), ANY_ERROR);
    EXPECT(qnn_encode_levels_fp4(FF, 0, 15, 1.0f, 2, FU, nullptr), ANY_ERROR);
    EXPECT(qnn_encode_levels_fp4(FF, 0, 16, 1.0f, 3, FU, nullptr), ANY_ERROR);
    EXPECT(qnn_levels_to_fp4(nullptr, 16, FU, nullptr), ANY_ERROR);
    const qnn_conv_desc odd_c = with([](qnn_conv_desc &d) { d.Cin = 24; });
    EXPECT(qnn_level_conv2d_i8(&odd_c, F8, F8, FF, FI, nullptr, nullptr, 0.0f, 0, nullptr), QNN_ERR_UNSUPPORTED);
    EXPECT(qnn_level_conv2d_fp4(&odd_c, FU, FU, FF, FI, nullptr, nullptr, 0.0f, 0, nullptr), QNN_ERR_UNSUPPORTED);

    // one-launch small layer
    EXPECT(qnn_fc_fused(FF, 0, 4, 64, 32, 1.0f, 2, FAKE, 2, 8, FF, FI, FF, nullptr), QNN_ERR_INVALID_ARG);
    EXPECT(qnn_fc_fused(FF, 0, 4, 40000, 40000, 1.0f, 2, FAKE, 2, 8, FF, FI, FF, nullptr), QNN_ERR_UNSUPPORTED);
    EXPECT(qnn_fc_fused(FF, 0, 4, 64, 64, 1.0f, 2, FAKE, 2, 8, nullptr, nullptr, FF, nullptr), QNN_ERR_INVALID_ARG);

    // unquantized ends
    const qnn_dense_conv_desc dd = {1, 8, 8, 3, 64, 7, 7, 2, 3};
    qnn_dense_conv_desc dbad = dd;
    dbad.kh = 0;
    EXPECT(qnn_dense_conv2d_f32(&dbad, FF, FF, nullptr, nullptr, 0, FF, nullptr, 0.0f, 0, nullptr), ANY_ERROR);
    EXPECT(qnn_dense_conv2d_f32(&dd, FF, FF, nullptr, nullptr, 0, nullptr, nullptr, 0.0f, 0, nullptr), ANY_ERROR);
    EXPECT(qnn_dense_conv2d_f32(&dd, FF, FF, nullptr, nullptr, 0, nullptr, FAKE, 1.0f, 9, nullptr), ANY_ERROR);
    EXPECT(qnn_dense_conv2d_f32_levels(&dd, FF, FF, nullptr, nullptr, 0, nullptr, F8, 1.0f, 8, nullptr), ANY_ERROR);
    dbad = dd, dbad.B = big, dbad.H = dbad.W = 1 << 20;
    EXPECT(qnn_dense_conv2d_f32(&dbad, FF, FF, nullptr, nullptr, 0, FF, nullptr, 0.0f, 0, nullptr), ANY_ERROR);
    EXPECT(qnn_global_avgpool_f32(nullptr, 2, 49, 512, FF, nullptr), ANY_ERROR);
    EXPECT(qnn_global_avgpool_f32(FF, 2, -1, 512, FF, nullptr), ANY_ERROR);
    EXPECT(qnn_dense_fc_f32(FF, nullptr, nullptr, 4, 4, 4, FF, nullptr), ANY_ERROR);
    EXPECT(qnn_dense_fc_f32(FF, FF, nullptr, 4, -4, 4, FF, nullptr), ANY_ERROR);

    if (qnn_version() < 100 || !qnn_build_id() || !qnn_last_error()) ++g_failures;
    printf("abi_errors: %d calls, %d failures\n", g_calls, g_failures);
    return g_failures ? 1 : 0;
}
