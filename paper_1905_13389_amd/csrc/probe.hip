// libqnn_probe.so: register-only issue-rate loops (include/qnn_probe.h).  Measurement aids: the benchmark
// derives the VALU roofline of the binary dot product from them -- the sustained rate of its two
// instructions, and the clock the chip holds while it runs them.  Not part of the product library.
// Every VALU loop iteration issues 64 VALU instructions per wave.
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>
#include <type_traits>

#include "../../include/qnn_probe.h"

namespace {

char *probe_error_buffer()
{
    static thread_local char buf[256] = {0};
    return buf;
}

int probe_fail(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(probe_error_buffer(), 256, fmt, ap);
    va_end(ap);
    return -1;
}

#define QNN_PR_X(t, a, b) "v_xor_b32 " t ", " a ", " b "\n\t"
#define QNN_PR_B(t, p) "v_bcnt_u32_b32 " p ", " t ", " p "\n\t"
#define QNN_PR_NOP "s_nop 0\n\t"
#define QNN_PR_PAIR(a, b, p) QNN_PR_X("%0", a, b) QNN_PR_B("%0", p)
#define QNN_PR_PAIRN(a, b, p) QNN_PR_PAIR(a, b, p) QNN_PR_NOP
#define QNN_PR_REP2(x) x x
#define QNN_PR_REP4(x) x x x x
#define QNN_PR_REP8(x) QNN_PR_REP4(x) QNN_PR_REP4(x)
#define QNN_PR_REP16(x) QNN_PR_REP8(x) QNN_PR_REP8(x)

// operands: %0..%3 temporaries t0..t3, %4..%11 counts p0..p7, %12..%15 a0..a3, %16..%19 b0..b3
#define QNN_PR_OPERANDS                                                                                            \
    : "+v"(t0), "+v"(t1), "+v"(t2), "+v"(t3), "+v"(p0), "+v"(p1), "+v"(p2), "+v"(p3), "+v"(p4), "+v"(p5),          \
      "+v"(p6), "+v"(p7)                                                                                           \
    : "v"(a0), "v"(a1), "v"(a2), "v"(a3), "v"(b0), "v"(b1), "v"(b2), "v"(b3)

// Eight pairs, two deep through the rotating temporaries t0..t3: the count of pair k is issued after the xor of
// pair k + 1, so no instruction reads the result of the one before it.  NOP = text put after every second
// instruction.
#define QNN_PR_PIPE8(NOP)                                                                                          \
    QNN_PR_X("%0", "%12", "%16") QNN_PR_X("%1", "%13", "%17") NOP                                                  \
    QNN_PR_B("%0", "%4") QNN_PR_X("%2", "%14", "%18") NOP                                                          \
    QNN_PR_B("%1", "%5") QNN_PR_X("%3", "%15", "%19") NOP                                                          \
    QNN_PR_B("%2", "%6") QNN_PR_X("%0", "%12", "%17") NOP                                                          \
    QNN_PR_B("%3", "%7") QNN_PR_X("%1", "%13", "%18") NOP                                                          \
    QNN_PR_B("%0", "%8") QNN_PR_X("%2", "%14", "%19") NOP                                                          \
    QNN_PR_B("%1", "%9") QNN_PR_X("%3", "%15", "%16") NOP                                                          \
    QNN_PR_B("%2", "%10") QNN_PR_B("%3", "%11") NOP

// Four xors into the four temporaries, then their four counts.
#define QNN_PR_GROUP4(a0_, a1_, a2_, a3_, b0_, b1_, b2_, b3_, p0_, p1_, p2_, p3_)                                   \
    QNN_PR_X("%0", a0_, b0_) QNN_PR_X("%1", a1_, b1_) QNN_PR_X("%2", a2_, b2_) QNN_PR_X("%3", a3_, b3_)             \
    QNN_PR_B("%0", p0_) QNN_PR_B("%1", p1_) QNN_PR_B("%2", p2_) QNN_PR_B("%3", p3_)

template <int MODE>
__global__ __launch_bounds__(256) void probe_kernel(uint32_t *out, int64_t *clocks, int iters, uint32_t seed)
{
    uint32_t a0 = seed + threadIdx.x, a1 = a0 * 3u, a2 = a0 * 5u, a3 = a0 * 7u;
    uint32_t b0 = seed ^ 0x55u, b1 = b0 * 3u, b2 = b0 * 5u, b3 = b0 * 7u;
    uint32_t p0 = 0, p1 = 0, p2 = 0, p3 = 0, p4 = 0, p5 = 0, p6 = 0, p7 = 0;
    uint32_t t0 = 0, t1 = 0, t2 = 0, t3 = 0;
    const uint64_t c_begin = __builtin_amdgcn_s_memtime();
    const uint64_t r_begin = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
        if constexpr (MODE == 0) {
            asm volatile(QNN_PR_REP16(QNN_PR_X("%0", "%12", "%16") QNN_PR_X("%1", "%13", "%17")
                                          QNN_PR_X("%2", "%14", "%18") QNN_PR_X("%3", "%15", "%19")) QNN_PR_OPERANDS);
        } else if constexpr (MODE == 1) {
            asm volatile(QNN_PR_REP8(QNN_PR_B("%12", "%4") QNN_PR_B("%13", "%5") QNN_PR_B("%14", "%6")
                                         QNN_PR_B("%15", "%7") QNN_PR_B("%16", "%8") QNN_PR_B("%17", "%9")
                                             QNN_PR_B("%18", "%10") QNN_PR_B("%19", "%11")) QNN_PR_OPERANDS);
        } else if constexpr (MODE == 2) {
            asm volatile(QNN_PR_REP4(QNN_PR_PAIRN("%12", "%16", "%4") QNN_PR_PAIRN("%13", "%17", "%5")
                                         QNN_PR_PAIRN("%14", "%18", "%6") QNN_PR_PAIRN("%15", "%19", "%7")
                                             QNN_PR_PAIRN("%12", "%17", "%8") QNN_PR_PAIRN("%13", "%18", "%9")
                                                 QNN_PR_PAIRN("%14", "%19", "%10") QNN_PR_PAIRN("%15", "%16", "%11"))
                             QNN_PR_OPERANDS);
        } else if constexpr (MODE == 3) {
            asm volatile(QNN_PR_REP4(QNN_PR_PAIR("%12", "%16", "%4") QNN_PR_PAIR("%13", "%17", "%5")
                                         QNN_PR_PAIR("%14", "%18", "%6") QNN_PR_PAIR("%15", "%19", "%7")
                                             QNN_PR_PAIR("%12", "%17", "%8") QNN_PR_PAIR("%13", "%18", "%9")
                                                 QNN_PR_PAIR("%14", "%19", "%10") QNN_PR_PAIR("%15", "%16", "%11"))
                             QNN_PR_OPERANDS);
        } else if constexpr (MODE == 4) {
            asm volatile(QNN_PR_REP4(QNN_PR_PIPE8("")) QNN_PR_OPERANDS);
        } else if constexpr (MODE == 5) {
            asm volatile(QNN_PR_REP4(QNN_PR_GROUP4("%12", "%13", "%14", "%15", "%16", "%17", "%18", "%19", "%4", "%5", "%6", "%7")
                                         QNN_PR_GROUP4("%12", "%13", "%14", "%15", "%17", "%18", "%19", "%16", "%8", "%9", "%10", "%11"))
                             QNN_PR_OPERANDS);
        } else if constexpr (MODE == 6) {
            asm volatile(QNN_PR_REP4(QNN_PR_PIPE8(QNN_PR_NOP)) QNN_PR_OPERANDS);
        } else if constexpr (MODE == 7) { // counts only, an s_nop after each
            asm volatile(QNN_PR_REP8(QNN_PR_B("%12", "%4") QNN_PR_NOP QNN_PR_B("%13", "%5") QNN_PR_NOP QNN_PR_B("%14", "%6") QNN_PR_NOP
                                         QNN_PR_B("%15", "%7") QNN_PR_NOP QNN_PR_B("%16", "%8") QNN_PR_NOP QNN_PR_B("%17", "%9") QNN_PR_NOP
                                             QNN_PR_B("%18", "%10") QNN_PR_NOP QNN_PR_B("%19", "%11") QNN_PR_NOP) QNN_PR_OPERANDS);
        } else if constexpr (MODE == 8) { // xors only, an s_nop after every second
            asm volatile(QNN_PR_REP16(QNN_PR_X("%0", "%12", "%16") QNN_PR_X("%1", "%13", "%17") QNN_PR_NOP
                                          QNN_PR_X("%2", "%14", "%18") QNN_PR_X("%3", "%15", "%19") QNN_PR_NOP) QNN_PR_OPERANDS);
        } else if constexpr (MODE == 9) { // xor xor count count, then an s_nop
            asm volatile(QNN_PR_REP8(QNN_PR_X("%0", "%12", "%16") QNN_PR_X("%1", "%13", "%17") QNN_PR_B("%0", "%4") QNN_PR_B("%1", "%5") QNN_PR_NOP
                                         QNN_PR_X("%2", "%14", "%18") QNN_PR_X("%3", "%15", "%19") QNN_PR_B("%2", "%6") QNN_PR_B("%3", "%7") QNN_PR_NOP)
                             QNN_PR_OPERANDS);
        } else if constexpr (MODE == 10) { // two pairs, then an s_nop
            asm volatile(QNN_PR_REP8(QNN_PR_X("%0", "%12", "%16") QNN_PR_B("%0", "%4") QNN_PR_X("%1", "%13", "%17") QNN_PR_B("%1", "%5") QNN_PR_NOP
                                         QNN_PR_X("%2", "%14", "%18") QNN_PR_B("%2", "%6") QNN_PR_X("%3", "%15", "%19") QNN_PR_B("%3", "%7") QNN_PR_NOP)
                             QNN_PR_OPERANDS);
        } else if constexpr (MODE == 11) { // pairs with the s_nop between the xor and its count
            asm volatile(QNN_PR_REP16(QNN_PR_X("%0", "%12", "%16") QNN_PR_NOP QNN_PR_B("%0", "%4") QNN_PR_X("%1", "%13", "%17") QNN_PR_NOP QNN_PR_B("%1", "%5"))
                             QNN_PR_OPERANDS);
        } else { // count of the previous pair's xor next to the new xor: count, xor, s_nop
            asm volatile(QNN_PR_REP16(QNN_PR_B("%0", "%4") QNN_PR_X("%1", "%13", "%17") QNN_PR_NOP QNN_PR_B("%1", "%5") QNN_PR_X("%0", "%12", "%16") QNN_PR_NOP)
                             QNN_PR_OPERANDS);
        }
    }
    const uint64_t c_end = __builtin_amdgcn_s_memtime();
    const uint64_t r_end = __builtin_amdgcn_s_memrealtime();
    out[blockIdx.x * blockDim.x + threadIdx.x] = p0 + p1 + p2 + p3 + p4 + p5 + p6 + p7 + t0 + t1 + t2 + t3;
    if (clocks && (threadIdx.x & 63) == 0) {
        const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
        clocks[2 * wave] = (int64_t)(c_end - c_begin);
        clocks[2 * wave + 1] = (int64_t)(r_end - r_begin);
    }
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

// The same loop with operands that the caller supplies: lane t of every workgroup takes the 8 x 16 bytes at
// operands + 128 t (4 A and 4 B operands); acc[k] += A[u] B[k] for u, k = 0..3.  What the operands hold
// decides how much the matrix cores' data paths toggle, and with that the power the loop draws and the clock
// the chip holds under it, which the two counters across the loop give per wave.
template <int MODE>
__global__ __launch_bounds__(256) void mfma_operand_probe_kernel(const pv4i *__restrict__ operands, uint32_t *out,
                                                                  int64_t *clocks, int iters)
{
    pv4i a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = operands[threadIdx.x * 8 + i];
        b[i] = operands[threadIdx.x * 8 + 4 + i];
    }
    using Acc = typename std::conditional<MODE == 0, pv16i, pv16f>::type;
    Acc acc[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[k][r] = 0;
    const uint64_t c_begin = __builtin_amdgcn_s_memtime();
    const uint64_t r_begin = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                if constexpr (MODE == 0) {
                    acc[k] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[u], b[k], acc[k], 0, 0, 0);
                } else {
                    const pv8i a8 = __builtin_shufflevector(a[u], a[u], 0, 1, 2, 3, -1, -1, -1, -1);
                    const pv8i b8 = __builtin_shufflevector(b[k], b[k], 0, 1, 2, 3, -1, -1, -1, -1);
                    acc[k] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, acc[k], 4, 4, 0, 127, 0, 127);
                }
            }
    }
    const uint64_t c_end = __builtin_amdgcn_s_memtime();
    const uint64_t r_end = __builtin_amdgcn_s_memrealtime();
    uint32_t sum = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += (uint32_t)(int)acc[k][r];
    out[blockIdx.x * blockDim.x + threadIdx.x] = sum;
    if (clocks && (threadIdx.x & 63) == 0) {
        const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
        clocks[2 * wave] = (int64_t)(c_end - c_begin);
        clocks[2 * wave + 1] = (int64_t)(r_end - r_begin);
    }
}

int check_probe_args(const char *what, int mode, int modes, int workgroups, int iters, const void *out)
{
    if (mode < 0 || mode >= modes) return probe_fail("%s: mode must be in [0,%d]", what, modes - 1);
    if (workgroups < 1 || workgroups > 65536 || iters < 0 || iters > (1 << 24))
        return probe_fail("%s: workgroups in [1,65536], iters in [0,2^24]", what);
    if (!out) return probe_fail("%s: NULL output buffer", what);
    return 0;
}

int check_probe_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return probe_fail("%s: %s", what, hipGetErrorString(e));
    return 0;
}

} // namespace

extern "C" const char *qnn_probe_last_error(void) { return probe_error_buffer(); }

extern "C" int qnn_probe_mfma(int mode, int workgroups, int iters, uint32_t *out, void *stream)
{
    if (int rc = check_probe_args("qnn_probe_mfma", mode, 2, workgroups, iters, out)) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)workgroups), block(256);
    if (mode == 0) hipLaunchKernelGGL(mfma_probe_kernel<0>, grid, block, 0, st, out, iters);
    else hipLaunchKernelGGL(mfma_probe_kernel<1>, grid, block, 0, st, out, iters);
    return check_probe_launch("qnn_probe_mfma");
}

extern "C" int qnn_probe_mfma_operands(int mode, int workgroups, int iters, const void *operands, uint32_t *out,
                                       int64_t *clocks, void *stream)
{
    if (int rc = check_probe_args("qnn_probe_mfma_operands", mode, 2, workgroups, iters, out)) return rc;
    if (!operands) return probe_fail("qnn_probe_mfma_operands: NULL operand buffer");
    if (reinterpret_cast<uintptr_t>(operands) % 16 != 0) return probe_fail("qnn_probe_mfma_operands: operands must be 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)workgroups), block(256);
    const pv4i *ops = static_cast<const pv4i *>(operands);
    if (mode == 0) hipLaunchKernelGGL(mfma_operand_probe_kernel<0>, grid, block, 0, st, ops, out, clocks, iters);
    else hipLaunchKernelGGL(mfma_operand_probe_kernel<1>, grid, block, 0, st, ops, out, clocks, iters);
    return check_probe_launch("qnn_probe_mfma_operands");
}

extern "C" int qnn_probe_valu(int mode, int workgroups, int iters, uint32_t *out, int64_t *clocks, void *stream)
{
    if (int rc = check_probe_args("qnn_probe_valu", mode, 13, workgroups, iters, out)) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)workgroups), block(256);
    switch (mode) {
    case 0: hipLaunchKernelGGL(probe_kernel<0>, grid, block, 0, st, out, clocks, iters, 1u); break;
    case 1: hipLaunchKernelGGL(probe_kernel<1>, grid, block, 0, st, out, clocks, iters, 1u); break;
    case 2: hipLaunchKernelGGL(probe_kernel<2>, grid, block, 0, st, out, clocks, iters, 1u); break;
    case 3: hipLaunchKernelGGL(probe_kernel<3>, grid, block, 0, st, out, clocks, iters, 1u); break;
    case 4: hipLaunchKernelGGL(probe_kernel<4>, grid, block, 0, st, out, clocks, iters, 1u); break;
    case 5: hipLaunchKernelGGL(probe_kernel<5>, grid, block, 0, st, out, clocks, iters, 1u); break;
    case 6: hipLaunchKernelGGL(probe_kernel<6>, grid, block, 0, st, out, clocks, iters, 1u); break;
    case 7: hipLaunchKernelGGL(probe_kernel<7>, grid, block, 0, st, out, clocks, iters, 1u); break;
    case 8: hipLaunchKernelGGL(probe_kernel<8>, grid, block, 0, st, out, clocks, iters, 1u); break;
    case 9: hipLaunchKernelGGL(probe_kernel<9>, grid, block, 0, st, out, clocks, iters, 1u); break;
    case 10: hipLaunchKernelGGL(probe_kernel<10>, grid, block, 0, st, out, clocks, iters, 1u); break;
    case 11: hipLaunchKernelGGL(probe_kernel<11>, grid, block, 0, st, out, clocks, iters, 1u); break;
    default: hipLaunchKernelGGL(probe_kernel<12>, grid, block, 0, st, out, clocks, iters, 1u); break;
    }
    return check_probe_launch("qnn_probe_valu");
}
