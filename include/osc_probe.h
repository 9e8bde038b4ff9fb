/*
 * Matrix-core probe: a yardstick for the measurements, built into a library of its own
 * (libosc_probe.so) that only the benchmark loads.  No passage of the paper.
 *
 * Runs `workgroups` workgroups of eight wavefronts, each issuing `iters` x 8 FP4 block-scaled
 * MFMAs (v_mfma_scale_f32_32x32x64_f8f6f4, the instruction of the dual-path GEMM) on pseudo-random
 * register operands with nothing else in the loop, and reports through *flops (host) how many
 * floating-point operations that is.  Timed by the caller, it gives the matrix rate this machine
 * sustains at its real clocks, to be set beside the published peak.
 *   out     float (device), 4-byte aligned: never written in practice (keeps the result alive)
 *   stream  hipStream_t as void* (NULL = default stream)
 * Returns 0, -1 (null pointer), -2 (workgroups or iters not positive) or -6 (launch refused).
 */
#ifndef OSC_PROBE_H
#define OSC_PROBE_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif
int osc_probe_mfma_fp4(int32_t workgroups, int32_t iters, float *out, double *flops, void *stream);
#ifdef __cplusplus
}
#endif
#endif /* OSC_PROBE_H */
