// Measurement aids.  The streaming probe: what a bare loop of 16-byte loads (and stores) reaches on this
// machine's memory.  The matrix-core probe: what the matrix core of this machine sustains on the instruction the dual-path
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

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// One trip of a workgroup: 256 threads x 8 loads of 16 bytes = 32 KB of src, and, with WR = n > 0, 8 / n
// stores of 16 bytes per thread = 32 / n KB of dst.
template <int WR>
__global__ void __launch_bounds__(256) probe_stream_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                           int64_t n16) {
    constexpr int U = 8;
    u32x4 acc = {0u, 0u, 0u, 0u};
    const int64_t stride = (int64_t)gridDim.x * 256 * U;
    for (int64_t i0 = (int64_t)blockIdx.x * 256 * U; i0 + 256 * U <= n16; i0 += stride) {
        u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(src + i0 + threadIdx.x + 256 * u);
        if constexpr (WR > 0) {
            u32x4* d = dst + i0 / WR + threadIdx.x;
#pragma unroll
            for (int u = 0; u < U; u += WR) {
                u32x4 a = v[u];
#pragma unroll
                for (int k = 1; k < WR; ++k) a ^= v[u + k];
                __builtin_nontemporal_store(a, d + 256 * (u / WR));
            }
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) acc ^= v[u];
        }
    }
    if (WR == 0 && acc.x == 0x12345678u && acc.y == 0x9abcdef0u && acc.z == 7u) dst[0] = acc;  // never true in practice
}

}  // namespace

extern "C" int osc_probe_stream(const void* src, void* dst, int64_t bytes, int32_t loads_per_store, int32_t workgroups,
                                void* stream) {
    if (!src || !dst) return -1;
    const int n = loads_per_store;
    if (bytes <= 0 || bytes % 32768 != 0 || workgroups <= 0 || !(n == 0 || n == 1 || n == 2 || n == 4 || n == 8)) return -2;
    if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15) return -4;
    const u32x4* s = static_cast<const u32x4*>(src);
    u32x4* d = static_cast<u32x4*>(dst);
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const dim3 g(workgroups), b(256);
    const int64_t n16 = bytes / 16;
    switch (n) {
        case 0: hipLaunchKernelGGL(probe_stream_kernel<0>, g, b, 0, st, s, d, n16); break;
        case 1: hipLaunchKernelGGL(probe_stream_kernel<1>, g, b, 0, st, s, d, n16); break;
        case 2: hipLaunchKernelGGL(probe_stream_kernel<2>, g, b, 0, st, s, d, n16); break;
        case 4: hipLaunchKernelGGL(probe_stream_kernel<4>, g, b, 0, st, s, d, n16); break;
        default: hipLaunchKernelGGL(probe_stream_kernel<8>, g, b, 0, st, s, d, n16); break;
    }
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

extern "C" int osc_probe_mfma_fp4(int32_t workgroups, int32_t iters, float* out, double* flops, void* stream) {
    if (workgroups <= 0 || iters <= 0) return -2;
    if (!out || !flops) return -1;
    // 8 wavefronts x 8 MFMAs of 32x32x64 per iteration (4 x 2 operand fragments), 2 flops per multiply-add
    *flops = (double)workgroups * 8.0 * 8.0 * (double)iters * 2.0 * 32.0 * 32.0 * 64.0;
    hipLaunchKernelGGL(probe_mfma_fp4_kernel, dim3(workgroups), dim3(PROBE_THREADS), 0,
                       reinterpret_cast<hipStream_t>(stream), iters, 12345u, out);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}
