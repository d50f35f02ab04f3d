/*
 * fq_peak.h — measurement hooks of libfq: what the matrix pipes and the memory system of the GPU at hand
 * deliver to the simplest possible kernels, so that a benchmark can state the ceilings next to the nominal
 * peaks it prices the GEMMs and the quantizer against.  Not part of the quantized layer; nothing here is
 * called by the fq_* entry points.
 *
 * Conventions as in fq.h: device pointers, caller-owned buffers, nothing allocated, nothing synchronized,
 * kernels enqueued on `stream`; FQ_OK or an FQ_ERR_* code with fq_last_error_string().
 */
#ifndef FQ_PEAK_H
#define FQ_PEAK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    FQ_PEAK_I8 = 0,         /* v_mfma_i32_32x32x32_i8, operands = int8 bytes                                    */
    FQ_PEAK_BF16 = 1,       /* v_mfma_f32_32x32x16_bf16                                                         */
    FQ_PEAK_E3M2 = 2,       /* v_mfma_scale_f32_32x32x64_f8f6f4, both operands 6-bit E3M2 codes (24 bytes/lane) */
    FQ_PEAK_I8_NIBBLES = 3  /* the int8 MFMA on operands widened from packed nibbles as fq_gemm_i4 widens them   */
};

/* fq_peak_mfma — an MFMA-only loop: `blocks` workgroups of four waves (one per SIMD), each wave holding 16
 * accumulator blocks of 32 x 32 and two sets of 4 + 4 operand vectors in registers, loaded once; every loop
 * iteration issues the 16 independent MFMAs of one set, the sets alternating.  No memory traffic inside the loop.
 *   operands   device buffer of operand_bytes >= 65536 bytes the operand vectors are read from (e.g. a
 *              quantized tensor of the workload, so that the pipe multiplies live values), or NULL: all zeros.
 *   iters      loop iterations per wave (>= 1; rounded up to an even number: a pass issues both operand sets).
 *   ticks_out  NULL, or uint64 [2 * blocks]: for each workgroup the shader-clock ticks (s_memtime) and the
 *              constant-rate ticks (s_memrealtime) its first wave spent in the loop; their ratio times the
 *              constant rate (hipDeviceAttributeWallClockRate) is the shader clock the loop ran at.
 *   sink       float [blocks * 256], receives a value derived from the accumulators (keeps the loop alive).
 * Work done: blocks * 4 * iters * 16 MFMAs of 32 x 32 x {32, 16, 64, 32} multiply-adds. */
int fq_peak_mfma(int kind, const void* operands, size_t operand_bytes, int blocks, long long iters,
                 unsigned long long* ticks_out, float* sink, void* stream);

/* fq_peak_copy — a plain device copy, 16 bytes per lane and step: dst[i] = src[i] for `bytes` bytes (a multiple of
 * 16; both pointers 16-byte aligned).  The reference kernel for "what a copy reaches on this GPU" and for scaling
 * the profiler's FETCH_SIZE / WRITE_SIZE counters. */
int fq_peak_copy(const void* src, void* dst, size_t bytes, void* stream);

/* fq_peak_gemm_ticks — clock probe of the GEMM kernels.  While ticks_dev != NULL on the calling thread, every GEMM
 * kernel launched by that thread (fq_gemm_*, fq_bmm_*, fq_linear*) has the first wave of each workgroup add the
 * shader-clock ticks (s_memtime) and the constant-rate ticks (s_memrealtime) it spent in the kernel to
 * ticks_dev[0] and ticks_dev[1] (uint64, device, 8-byte aligned; the caller zeroes them): ticks_dev[0] / ticks_dev[1]
 * times fq_peak_wall_clock_khz() is the average shader clock the kernel ran at.  NULL switches the probe off. */
int fq_peak_gemm_ticks(unsigned long long* ticks_dev);
/* Rate of the constant-rate counter on the current device in kHz (0 if it cannot be read). */
int fq_peak_wall_clock_khz(void);

#ifdef __cplusplus
}
#endif
#endif /* FQ_PEAK_H */
