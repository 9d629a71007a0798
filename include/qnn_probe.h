/*
 * qnn_probe.h -- C ABI of libqnn_probe.so: measurement aids for the MI355X (gfx950) library declared in qnn.h.
 * Nothing here is a step of the hot path and the product library does not contain it.  The benchmark uses these
 * register-only loops to state, on the device at hand and at the clock it actually holds under that load, the issue
 * rate of the two instructions the binary dot product consists of (the "xnor" and "bitcount" of the paper's abstract
 * and of Eq. 9's branches) and what the matrix cores sustain for the decoded-level comparison routes.
 *
 * Pointers are DEVICE memory owned by the caller; `stream` is a hipStream_t passed as void*.  Calls only enqueue a
 * kernel.  Return 0 on success, a negative value otherwise (qnn_probe_last_error() gives the thread-local message);
 * argument errors are found on the host before any HIP call.
 */
#ifndef QNN_PROBE_H_
#define QNN_PROBE_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * qnn_probe_valu -- launches `workgroups` workgroups of 256 lanes (4 wave64) that each run `iters` iterations of a
 * register-only loop of 64 VALU instructions per wave.
 *   mode 0: v_xor_b32 only (4 independent destinations)
 *        1: v_bcnt_u32_b32 only (8 independent count chains)
 *        2: xor/count pairs through one temporary, an s_nop 0 after each pair
 *        3: the same pairs back to back (no s_nop)
 *        4: pairs through 4 rotating temporaries, two deep: each count reads the xor issued two instructions
 *           earlier, no instruction reads its predecessor's result, no s_nop
 *        5: 4 xors into 4 temporaries, then their 4 counts, no s_nop
 *        6: as 4 with an s_nop 0 after every second instruction
 *        7: counts only, an s_nop 0 after each;  8: xors only, an s_nop 0 after every second
 *        9: xor, xor, count, count, s_nop 0;  10: two pairs, then s_nop 0
 *        11: xor, s_nop 0, count (the s_nop between the two instructions of a pair)
 *        12: count of the previous pair, xor of the next, s_nop 0
 *   out     DEVICE, workgroups * 256 uint32 (receives the loops' results so that they are not removed)
 *   clocks  DEVICE, workgroups * 4 waves * 2 int64, or NULL: per wave, the ticks the loop took on the s_memtime
 *           counter and on the s_memrealtime counter (constant 100 MHz).  Where s_memtime follows the shader
 *           clock their ratio is that clock in units of 100 MHz; where it is constant-rate too the ratio is 1.
 */
int qnn_probe_valu(int mode, int workgroups, int iters, uint32_t *out, int64_t *clocks, void *stream);

/*
 * qnn_probe_mfma -- every workgroup of 256 lanes runs `iters` iterations of 16 register-only MFMA instructions per
 * wave on four independent accumulators.
 *   mode 0: v_mfma_i32_32x32x32_i8 (65536 operations each); 1: v_mfma_scale_f32_32x32x64_f8f6f4 on fp4 operands
 *   (131072 operations each)
 *   out  DEVICE, workgroups * 256 uint32
 */
int qnn_probe_mfma(int mode, int workgroups, int iters, uint32_t *out, void *stream);

/*
 * qnn_probe_mfma_operands -- the loop of qnn_probe_mfma on operands the caller supplies, with the two counters of
 * qnn_probe_valu across it: what the operands hold (zeros, constant bytes, quantization levels, random bytes) decides
 * how much power the matrix cores draw, and with that the clock the chip holds under the loop.
 *   mode      as qnn_probe_mfma
 *   operands  DEVICE, 16-byte aligned, 256 lanes * 8 * 16 bytes = 32 KiB, read by every workgroup: lane t takes 4 A
 *             operands (16 bytes each: 16 int8 values, or 32 fp4 values) at 128 t and 4 B operands at 128 t + 64
 *   out       DEVICE, workgroups * 256 uint32
 *   clocks    DEVICE, workgroups * 4 waves * 2 int64, or NULL: as in qnn_probe_valu
 */
int qnn_probe_mfma_operands(int mode, int workgroups, int iters, const void *operands, uint32_t *out, int64_t *clocks,
                            void *stream);

/* Message for the last error returned on the calling thread ("" if none). Never NULL. */
const char *qnn_probe_last_error(void);

/*
 * libqnn_timeline.so -- the convolution entry points of libqnn.so (qnn_conv2d, qnn_conv2d_block, qnn_deconv2d, same
 * arguments and results, declared in qnn.h) compiled with wave timestamps, plus:
 *
 * qnn_timeline_set -- where the convolution kernels launched after this call leave their timestamps.
 *   buffer     DEVICE, waves * 5 int64, owned by the caller, or NULL with waves = 0 (nothing is recorded).  Wave w of
 *              workgroup b of a launch with W waves per workgroup writes entry b W + w if it is below `waves`:
 *              [0] the constant 100 MHz counter (s_memrealtime) at its start, [1] after its workgroup's prologue,
 *              [2] at its end, [3] its hardware ids (XCC id << 32 | HW_ID register), [4] the ticks of the shader's
 *              cycle counter (s_memtime) across its life: [4] / ([2] - [0]) is the clock it ran at, in units of
 *              100 MHz.  Every launch overwrites.
 *   pair_hint  0: the two workgroups of a CU run with the hardware's default priorities (for comparison);
 *              otherwise they balance their progress as in libqnn.so
 *   Returns 0, or QNN_ERR_INVALID_ARG.  Host state of the process, not thread safe.
 */
int qnn_timeline_set(int64_t *buffer, int waves, int pair_hint);

/*
 * libqnn_timeline.so also holds the matrix-core GEMM of libqnn.so (qnn_level_row_bytes, qnn_plane_sum_i8,
 * qnn_level_gemm_i8, qnn_fp4_row_bytes, qnn_plane_sum_fp4, qnn_level_gemm_fp4: same arguments and results, declared
 * in qnn.h) compiled with wave timestamps, plus:
 *
 * qnn_level_gemm_timeline_set -- where the level GEMM kernels launched after this call leave their timestamps.
 *   buffer  DEVICE, waves * 6 int64, owned by the caller, or NULL with waves = 0 (nothing is recorded).  Wave w of
 *           workgroup b (8 waves per workgroup) writes entry 8 b + w if it is below `waves`: the constant 100 MHz
 *           counter (s_memrealtime) [0] at its start, [1] at the start and [2] at the end of its reduction loop,
 *           [3] at its end; the ticks of the shader's cycle counter (s_memtime) [4] across the reduction loop and
 *           [5] across its life.  [4] / ([2] - [1]) is the clock the chip held in the loop, in units of 100 MHz.
 *   Returns 0, or QNN_ERR_INVALID_ARG.  Host state of the process, not thread safe.
 */
int qnn_level_gemm_timeline_set(int64_t *buffer, int waves);

#ifdef __cplusplus
}
#endif
#endif /* QNN_PROBE_H_ */
