/*
 * libasa -- tooling for benchmarks and tests.  NOT part of the product interface (asa.h): a
 * caller of the library needs nothing from this file.  The symbols live in the same shared
 * library so that a benchmark can time the very kernels that the product calls launch.
 */
#ifndef ASA_BENCH_H_
#define ASA_BENCH_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Calibration for benchmarks: a kernel of nothing but independent 32x32x16 bf16 MFMAs
 * (`workgroups` x 8 wavefronts, 4 * iters MFMAs each), so that a report can state the rate the
 * matrix cores sustain on the device at hand next to the published peak that the roofline uses.
 * The operands are pseudo-random and differ between consecutive MFMAs (with identical operands
 * far fewer gates switch and the clock runs higher than in any real kernel).
 * idle_sleep (0..7) and vector_stream (0 / 1) vary the load to show how the device's power limit
 * answers: with idle_sleep > 0 only 4 wavefronts per workgroup (one per SIMD) issue MFMAs and
 * each pauses for `s_sleep idle_sleep` behind every 16 of them (a duty cycle below 1 when one
 * workgroup runs per compute unit); with vector_stream the other 4 wavefronts run exponentials
 * and multiply-adds beside them until the MFMA loops end.  In both cases 4 wavefronts count in *flop.
 * sink: DEVICE, workgroups * 512 floats (written).  Of every workgroup's 512, element 0 holds the
 * shader-clock cycles of its first wavefront's MFMA loop and element 1 the same interval in
 * ticks of the constant 100 MHz clock (their ratio is the shader clock under this load); the
 * rest is meaningless.  *flop (HOST, optional) receives the floating-point operations of the
 * launch.  The profiling hook below brackets it.  Returns an asa_status (asa.h).
 */
int asa_mfma_rate_probe(int32_t workgroups, int32_t iters, int32_t idle_sleep, int32_t vector_stream,
                        float *sink, double *flop, void *hip_stream);

/*
 * Calibration for benchmarks: the rate of fp32 atomic adds (atomic != 0) or of plain stores of
 * the same bytes (atomic == 0) in the access pattern that a backward pass with a single walk over
 * the tiles would need for dQ: `workgroups` workgroups each add `tiles_per_workgroup` tiles of
 * 128 x 128 fp32 to pseudo-randomly chosen blocks of buf.
 * buf: DEVICE, n_qblocks * 128 * 128 floats (read and written).  *bytes (HOST, optional) receives
 * the payload bytes of the launch.  The profiling hook below brackets the kernel.
 */
int asa_add_rate_probe(int32_t atomic, int32_t workgroups, int32_t tiles_per_workgroup, int32_t n_qblocks,
                       float *buf, double *bytes, void *hip_stream);

/*
 * Profiling hook for benchmarks.  Arms the calling thread so that the NEXT asa_attn_fwd,
 * asa_attn_bwd, asa_build_mask, asa_reorder_tokens (asa.h) or probe call (this file) records
 * `start_event` immediately before and `stop_event` immediately after its dominant kernel(s) -- the tile loop of the forward, the
 * dK/dV and dQ kernels of the backward, the probe of the mask build -- on the call's stream,
 * leaving out the small preparation kernels around them.  Both are hipEvent_t handles owned by
 * the caller.  One shot: the hook disarms itself when used; pass NULL, NULL to disarm.
 */
int asa_set_kernel_timing(void *start_event, void *stop_event);

/*
 * Test switch: which forward kernel asa_attn_fwd launches.  0 = the library's own choice (the
 * default), 1 = the lock-step kernel only, 2 = the ping-pong kernel only (global tokens always
 * take the ping-pong kernel).  Process-wide; lets the tests put every edge case through both
 * kernels at every tile shape.  Returns an asa_status.
 */
int asa_test_force_fwd_kernel(int which);

#ifdef __cplusplus
}
#endif
#endif /* ASA_BENCH_H_ */
