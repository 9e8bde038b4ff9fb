// Global -> LDS DMA, counted waits and the LDS image of 128-byte operand lines shared by the GEMM
// kernels (device code only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace osc {

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// s_waitcnt vmcnt(N): at most N vector memory operations of this wavefront still in flight
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);
}

__device__ __forceinline__ void load_to_lds16(const uint8_t* src, uint8_t* lds_wave_base) {
    // each lane's 16 bytes land at lds_wave_base + 16 * lane
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
}

// Rows of 128 bytes: 16-byte piece `c` (0..7) of row `r` sits at piece position c ^ swz8(r), so the
// lanes of one LDS access (consecutive rows, same piece) spread over all banks.
__device__ __forceinline__ int swz8(int r) { return (r & 7) ^ ((r >> 3) & 1); }
__device__ __forceinline__ int st128_off(int row, int piece) { return row * 128 + ((piece ^ swz8(row)) << 4); }

}  // namespace osc
