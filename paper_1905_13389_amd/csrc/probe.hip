// qnn_probe_valu: register-only issue-rate loops for the two instructions of the binary dot
// product.  A measurement aid (the benchmark derives the VALU roofline of qnn_binary_gemm from
// it), not part of the hot path.  Every loop iteration issues 64 VALU instructions per wave.
#include "qnn_host.h"
#include <type_traits>

namespace qnn {

#define QNN_PR_X(t, a, b) "v_xor_b32 " t ", " a ", " b "\n\t"
#define QNN_PR_B(t, p) "v_bcnt_u32_b32 " p ", " t ", " p "\n\t"
#define QNN_PR_PAIR(a, b, p) QNN_PR_X("%0", a, b) QNN_PR_B("%0", p) "s_nop 0\n\t"
#define QNN_PR_REP4(x) x x x x
#define QNN_PR_REP8(x) QNN_PR_REP4(x) QNN_PR_REP4(x)
#define QNN_PR_REP16(x) QNN_PR_REP8(x) QNN_PR_REP8(x)

// MODE 0: v_xor_b32 only; 1: v_bcnt_u32_b32 only (8 independent chains); 2: xor + count pairs with
// one s_nop after each pair (the order the GEMM kernels use)
template <int MODE> __global__ __launch_bounds__(256) void probe_kernel(uint32_t *out, int iters, uint32_t seed)
{
    uint32_t a0 = seed + threadIdx.x, a1 = a0 * 3u, a2 = a0 * 5u, a3 = a0 * 7u;
    uint32_t b0 = seed ^ 0x55u, b1 = b0 * 3u, b2 = b0 * 5u, b3 = b0 * 7u;
    uint32_t p0 = 0, p1 = 0, p2 = 0, p3 = 0, p4 = 0, p5 = 0, p6 = 0, p7 = 0;
    uint32_t t0 = 0, t1 = 0, t2 = 0, t3 = 0;
    for (int it = 0; it < iters; ++it) {
        if constexpr (MODE == 0) {
            asm volatile(QNN_PR_REP16(QNN_PR_X("%0", "%12", "%16") QNN_PR_X("%1", "%13", "%17")
                                          QNN_PR_X("%2", "%14", "%18") QNN_PR_X("%3", "%15", "%19"))
                         : "+v"(t0), "+v"(t1), "+v"(t2), "+v"(t3), "+v"(p0), "+v"(p1), "+v"(p2), "+v"(p3), "+v"(p4),
                           "+v"(p5), "+v"(p6), "+v"(p7)
                         : "v"(a0), "v"(a1), "v"(a2), "v"(a3), "v"(b0), "v"(b1), "v"(b2), "v"(b3));
        } else if constexpr (MODE == 1) {
            asm volatile(QNN_PR_REP8(QNN_PR_B("%12", "%4") QNN_PR_B("%13", "%5") QNN_PR_B("%14", "%6")
                                         QNN_PR_B("%15", "%7") QNN_PR_B("%16", "%8") QNN_PR_B("%17", "%9")
                                             QNN_PR_B("%18", "%10") QNN_PR_B("%19", "%11"))
                         : "+v"(t0), "+v"(t1), "+v"(t2), "+v"(t3), "+v"(p0), "+v"(p1), "+v"(p2), "+v"(p3), "+v"(p4),
                           "+v"(p5), "+v"(p6), "+v"(p7)
                         : "v"(a0), "v"(a1), "v"(a2), "v"(a3), "v"(b0), "v"(b1), "v"(b2), "v"(b3));
        } else {
            asm volatile(QNN_PR_REP4(QNN_PR_PAIR("%12", "%16", "%4") QNN_PR_PAIR("%13", "%17", "%5")
                                         QNN_PR_PAIR("%14", "%18", "%6") QNN_PR_PAIR("%15", "%19", "%7")
                                             QNN_PR_PAIR("%12", "%17", "%8") QNN_PR_PAIR("%13", "%18", "%9")
                                                 QNN_PR_PAIR("%14", "%19", "%10") QNN_PR_PAIR("%15", "%16", "%11"))
                         : "+v"(t0), "+v"(t1), "+v"(t2), "+v"(t3), "+v"(p0), "+v"(p1), "+v"(p2), "+v"(p3), "+v"(p4),
                           "+v"(p5), "+v"(p6), "+v"(p7)
                         : "v"(a0), "v"(a1), "v"(a2), "v"(a3), "v"(b0), "v"(b1), "v"(b2), "v"(b3));
        }
    }
    out[blockIdx.x * blockDim.x + threadIdx.x] = p0 + p1 + p2 + p3 + p4 + p5 + p6 + p7 + t0 + t1 + t2 + t3;
}

typedef int pv4i __attribute__((ext_vector_type(4)));
typedef int pv8i __attribute__((ext_vector_type(8)));
typedef int pv16i __attribute__((ext_vector_type(16)));
typedef float pv16f __attribute__((ext_vector_type(16)));

// Register-only matrix-core loops: 16 MFMAs per wave and iteration on four independent accumulators.
// MODE 0: v_mfma_i32_32x32x32_i8; 1: v_mfma_scale_f32_32x32x64_f8f6f4 on fp4 operands, unit scales.
template <int MODE> __global__ __launch_bounds__(256) void mfma_probe_kernel(uint32_t *out, int iters)
{
    // int8: small values; fp4: +1 against alternating +1 / -1, so the sums stay at 0
    const pv4i a = MODE == 0 ? pv4i{0x01010101, 0x01010101, 0x01010101, 0x01010101}
                             : pv4i{0x22222222, 0x22222222, 0x22222222, 0x22222222};
    const pv4i b = MODE == 0 ? pv4i{0x01ff01ff, 0x01ff01ff, 0x01ff01ff, 0x01ff01ff}
                             : pv4i{0x2a2a2a2a, 0x2a2a2a2a, 0x2a2a2a2a, 0x2a2a2a2a};
    using Acc = typename std::conditional<MODE == 0, pv16i, pv16f>::type;
    Acc acc[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[k][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                if constexpr (MODE == 0) {
                    acc[k] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[k], 0, 0, 0);
                } else {
                    const pv8i a8 = __builtin_shufflevector(a, a, 0, 1, 2, 3, -1, -1, -1, -1);
                    const pv8i b8 = __builtin_shufflevector(b, b, 0, 1, 2, 3, -1, -1, -1, -1);
                    acc[k] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, acc[k], 4, 4, 0, 127, 0, 127);
                }
            }
    }
    uint32_t sum = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += (uint32_t)(int)acc[k][r];
    out[blockIdx.x * blockDim.x + threadIdx.x] = sum;
}

} // namespace qnn

using namespace qnn;

extern "C" int qnn_probe_mfma(int mode, int workgroups, int iters, uint32_t *out, void *stream)
{
    if (mode < 0 || mode > 1) return fail(QNN_ERR_INVALID_ARG, "qnn_probe_mfma: mode must be 0 or 1");
    if (workgroups < 1 || workgroups > 65536 || iters < 0 || iters > (1 << 24))
        return fail(QNN_ERR_INVALID_ARG, "qnn_probe_mfma: workgroups in [1,65536], iters in [0,2^24]");
    if (!out) return fail(QNN_ERR_INVALID_ARG, "qnn_probe_mfma: NULL output buffer");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)workgroups), block(256);
    if (mode == 0) hipLaunchKernelGGL(mfma_probe_kernel<0>, grid, block, 0, st, out, iters);
    else hipLaunchKernelGGL(mfma_probe_kernel<1>, grid, block, 0, st, out, iters);
    return check_launch("qnn_probe_mfma");
}

extern "C" int qnn_probe_valu(int mode, int workgroups, int iters, uint32_t *out, void *stream)
{
    if (mode < 0 || mode > 2) return fail(QNN_ERR_INVALID_ARG, "qnn_probe_valu: mode must be 0, 1 or 2");
    if (workgroups < 1 || workgroups > 65536 || iters < 0 || iters > (1 << 24))
        return fail(QNN_ERR_INVALID_ARG, "qnn_probe_valu: workgroups in [1,65536], iters in [0,2^24]");
    if (!out) return fail(QNN_ERR_INVALID_ARG, "qnn_probe_valu: NULL output buffer");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)workgroups), block(256);
    if (mode == 0) hipLaunchKernelGGL(probe_kernel<0>, grid, block, 0, st, out, iters, 1u);
    else if (mode == 1) hipLaunchKernelGGL(probe_kernel<1>, grid, block, 0, st, out, iters, 1u);
    else hipLaunchKernelGGL(probe_kernel<2>, grid, block, 0, st, out, iters, 1u);
    return check_launch("qnn_probe_valu");
}
