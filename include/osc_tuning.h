/*
 * libosc -- kernel-choice overrides for tests and tuning.  Not part of the product interface:
 * the settings change which kernel serves a call, never its result (the parity tests force
 * every kernel through these knobs to show exactly that).  Process-wide; -1 restores the
 * library's own choice.  No entry point of osc.h reads the environment.
 */
#ifndef OSC_TUNING_H
#define OSC_TUNING_H

#ifdef __cplusplus
extern "C" {
#endif

enum {
    OSC_TUNE_GEMM_TILE = 0,        /* tile rows / 64 of the GEMM kernels: 1, 2 or 4 */
    OSC_TUNE_GEMM_KERNEL = 1,      /* 0 staged, 1 DMA, 2 persistent, 3 skinny (ignored where a kernel
                                      cannot serve the shape) */
    OSC_TUNE_GROUPED_ONE_TILE = 2, /* 1: grouped 8-bit GEMMs keep one tile per workgroup */
    OSC_TUNE_SWIGLU_TABLE = 3,     /* 0 / 1: SwiGLU fusions evaluate silu per element / look it up */
    OSC_TUNE_GEMM_KSPLIT = 4       /* 0 / 1: dual-path 64 x 128 tiles never / always split their K loop over two wavefront groups */
};

/* Errors: OSC_ERR_UNSUPPORTED for an unknown knob.  Any negative value means "automatic". */
int osc_tuning_set(int knob, int value);
/* The current setting (-1 = automatic, also for an unknown knob). */
int osc_tuning_get(int knob);

#ifdef __cplusplus
}
#endif
#endif /* OSC_TUNING_H */
