// Measurement aid: what the matrix core of this machine sustains on the instruction the dual-path
// GEMM uses (v_mfma_scale_f32_32x32x64_f8f6f4 on FP4 operands), with nothing else in the loop.
// Sustained clocks sit below the published peak and fall further with the switching activity of
// the operands, so the probe runs on pseudo-random register contents.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/osc_probe.h"

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int PROBE_THREADS = 512;  // eight wavefronts: two per SIMD, as in the GEMM

__global__ void __launch_bounds__(PROBE_THREADS) probe_mfma_fp4_kernel(int iters, uint32_t seed, float* out) {
    uint32_t x = seed ^ (blockIdx.x * 2654435761u) ^ (threadIdx.x * 40503u);
    auto next = [&]() { x = x * 1664525u + 1013904223u; return (int)x; };
    v8i a[4], b[2];
    for (int i = 0; i < 4; ++i) a[i] = (v8i){next(), next(), next(), next(), 0, 0, 0, 0};
    for (int j = 0; j < 2; ++j) b[j] = (v8i){next(), next(), next(), next(), 0, 0, 0, 0};
    v16f acc[4][2];
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 2; ++j)
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[i], b[j], acc[i][j], 4, 4, 0, 120, 0, 120);
        // keep the operands changing a little so the loop cannot be hoisted
        asm volatile("" : "+v"(a[0]), "+v"(b[0]));
    }
    float s = 0.0f;
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 2; ++j)
            for (int e = 0; e < 16; ++e) s += acc[i][j][e];
    if (s == 12345.678f) out[0] = s;  // never true in practice; keeps the accumulators alive
}

}  // namespace

extern "C" int osc_probe_mfma_fp4(int32_t workgroups, int32_t iters, float* out, double* flops, void* stream) {
    if (workgroups <= 0 || iters <= 0) return -2;
    if (!out || !flops) return -1;
    // 8 wavefronts x 8 MFMAs of 32x32x64 per iteration (4 x 2 operand fragments), 2 flops per multiply-add
    *flops = (double)workgroups * 8.0 * 8.0 * (double)iters * 2.0 * 32.0 * 32.0 * 64.0;
    hipLaunchKernelGGL(probe_mfma_fp4_kernel, dim3(workgroups), dim3(PROBE_THREADS), 0,
                       reinterpret_cast<hipStream_t>(stream), iters, 12345u, out);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}
