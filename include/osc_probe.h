/*
 * Probes: yardsticks for the measurements, built into a library of their own (libosc_probe.so)
 * that only the benchmark loads.
 *
 * Matrix-core probe.  No passage of the paper.
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

/*
 * Streaming probe: a yardstick for the HBM-bound kernels.  No passage of the paper.
 *
 * Reads `bytes` bytes of `src` once, front to back, with 16-byte non-temporal loads, eight of them
 * in flight per lane, on `workgroups` workgroups of 256 threads that stride over the buffer, and does
 * nothing with them.  With loads_per_store = n > 0 it also writes one 16-byte non-temporal store per
 * n loads to `dst`, front to back (bytes / n bytes in all): n = 4 is the read/write mix of the fused
 * SwiGLU quantisers (the MXFP4 quantiser reads three bytes per byte written).  Timed by the caller over buffers larger than
 * the last-level cache, it gives the rate a bare streaming loop reaches on this machine, to be set
 * beside the published 8 TB/s.
 *   src    device, 16-byte aligned, `bytes` bytes (a multiple of 32768)
 *   dst    device, 16-byte aligned, at least bytes / n + 4096 bytes when n > 0; with n = 0 at least
 *          16 bytes (never written in practice: keeps the loads alive)
 *   loads_per_store  0 (read only), or a divisor of 8
 *   stream hipStream_t as void* (NULL = default stream)
 * Returns 0, -1 (null pointer), -2 (sizes or loads_per_store out of range), -4 (alignment) or -6
 * (launch refused).
 */
int osc_probe_stream(const void *src, void *dst, int64_t bytes, int32_t loads_per_store, int32_t workgroups,
                     void *stream);
#ifdef __cplusplus
}
#endif
#endif /* OSC_PROBE_H */
