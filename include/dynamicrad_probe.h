/*
 * dynamicrad_probe.h -- measurement aids shipped beside the DynamicRad library.  They are not steps of the method
 * and not part of its product ABI (include/dynamicrad.h): bench.py uses them to report the shader clock the device
 * sustains under the attention kernel and what its matrix cores deliver on their own.
 */
#ifndef DYNAMICRAD_PROBE_H_
#define DYNAMICRAD_PROBE_H_

#include "dynamicrad.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Measurement aid (not a step of the method): average shader clock over a window.
 * Enqueues a one-wavefront kernel on `stream` that polls the constant 100 MHz counter for
 * `window_us` microseconds (1 .. 2 000 000) and then writes two uint64 to the device buffer
 * `out`: out[0] = shader-clock ticks elapsed, out[1] = 100 MHz ticks elapsed, so that
 * 100 * out[0] / out[1] is the mean shader clock in MHz over the window.  Run on a second
 * stream beside the attention kernel it reports the clock the chip sustains under that load;
 * the matrix-core peak the roofline is priced against assumes 2400 MHz.  Asynchronous; the
 * caller synchronises `stream` before reading `out`.  Errors: DR_ERR_INVALID_ARG for a NULL
 * pointer or a window out of range. */
dr_status dr_clock_probe(dr_ctx* ctx, uint64_t window_us, uint64_t* out, void* stream);

/* Measurement aid (not a step of the method): an MFMA-only loop, to price the attention kernel against what the
 * matrix cores of this device sustain rather than against the data-sheet peak alone.  Enqueues `workgroups`
 * workgroups of 4 wavefronts, each issuing iters * 8 matrix instructions (iters a multiple of 8) on register
 * operands and eight independent accumulators: shape 32 = v_mfma_f32_32x32x16_bf16 (32768 flop each), shape 16 =
 * v_mfma_f32_16x16x32_bf16 (16384 flop each).  Operands are one repeated value (random_operands = 0) or
 * pseudo-random bf16 numbers in [-1, 1) (1; the switching activity of real data).  `sink` is a device float the
 * kernel may write; *flop (host, optional) receives the flop count of the launch.  The caller times the launch
 * with events on `stream`.  Errors: DR_ERR_INVALID_ARG, also when workgroups * iters exceeds 2^26 (tens of
 * milliseconds of matrix work on a full device: the kernel cannot be pre-empted). */
dr_status dr_mfma_probe(dr_ctx* ctx, int32_t shape, int32_t workgroups, int32_t iters, int32_t random_operands,
                        float* sink, double* flop, void* stream);

/* Measurement aid (not a step of the method): the matrix instruction in the company it has inside the attention
 * loop.  Enqueues `workgroups` workgroups of 4 wavefronts, one wavefront per SIMD as in the attention kernels;
 * every wavefront runs iters * 8 slots of one v_mfma_f32_32x32x16_bf16 on pseudo-random bf16 register operands,
 * one v_exp_f32 and two v_fma_f32 (the attention loop has, per matrix instruction, 0.9 exponentials, 0.45 packs
 * to bf16, 0.65 LDS fragment reads and about one scalar instruction).  The rate it reaches is what a loop of that
 * instruction mix sustains on this device with no memory traffic at all.  `sink`, *flop (matrix flop only), timing
 * and errors as for dr_mfma_probe; workgroups * iters may not exceed 2^26. */
dr_status dr_mfma_mix_probe(dr_ctx* ctx, int32_t workgroups, int32_t iters, float* sink, double* flop, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DYNAMICRAD_PROBE_H_ */
