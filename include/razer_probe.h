/*
 * razer_probe.h -- measurement utilities exported by the gfx950 RaZeR library next to razer.h.
 * Nothing here is part of the method of arxiv 2501.04052: these calls exist so that a benchmark can
 * time, in the same process and on the same GPU as the kernels it reports,
 *   - the duration of single kernel dispatches of the library (what a kernel trace shows per dispatch),
 *   - a pure streaming read of a buffer (the bandwidth a kernel that only loads can reach), and
 *   - a register-resident bf16 matrix-instruction loop (the rate the matrix cores reach with no memory
 *     traffic at all),
 * i.e. the measured ceilings that roofline fractions are read against.  All pointers except `flops`
 * are DEVICE pointers; the calls enqueue on the given HIP stream and return; 0 = ok, 1 = null
 * pointer, 2 = bad argument, 6 = launch failure.
 */
#ifndef RAZER_PROBE_H
#define RAZER_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Per host thread: while start_event / stop_event (hipEvent_t cast to void*, created with timing
 * enabled) are set, every kernel the library launches from this thread records the begin and end
 * time stamps of its own dispatch into them (a later launch overwrites an earlier one: bracket calls
 * that launch ONE kernel); hipEventElapsedTime(start, stop) after synchronizing on stop is then that
 * dispatch's duration.  Pass NULL, NULL to switch the recording off again (the default). */
void razer_probe_dispatch_events(void *start_event, void *stop_event);

/* Reads `bytes` (a multiple of 16) from buf (16-byte aligned) with `workgroups` workgroups of 256
 * threads, grid-stride, four non-temporal 16-byte loads in flight per lane; sink: 64 dwords of device
 * scratch. */
int razer_probe_stream_read(const void *buf, size_t bytes, int workgroups, void *sink, void *hip_stream);

/* iters x 8 independent v_mfma_f32_32x32x16_bf16 per wavefront on `workgroups` workgroups of four
 * wavefronts, operands and accumulators in registers.  *flops (host, optional) receives the
 * floating-point operations of the launch, 2 * 32 * 32 * 16 per instruction. */
int razer_probe_mfma_bf16(int iters, int workgroups, void *sink, void *hip_stream, double *flops);

/* The same loop on the block-scaled FP4 x FP4 matrix instruction (v_mfma_scale_f32_32x32x64_f8f6f4, E8M0
 * scales of 2^0): the rate a two-pass FP4 realisation of the weight-activation mode (App. D.3) could at
 * most run at on this GPU.  2 * 32 * 32 * 64 flops per instruction. */
int razer_probe_mfma_fp4(int iters, int workgroups, void *sink, void *hip_stream, double *flops);

#ifdef __cplusplus
}
#endif
#endif /* RAZER_PROBE_H */
