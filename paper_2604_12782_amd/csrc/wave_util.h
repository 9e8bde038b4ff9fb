// 64-lane reductions and the row/segment work split shared by the streaming kernels (device code only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace osc {

// 64-lane reductions on the vector ALU alone (DPP inside each row of 16 lanes, then four lane
// reads).
__device__ __forceinline__ uint64_t dpp_u64(uint64_t v, const int ctrl_sel) {
    const int lo = (int)(uint32_t)v, hi = (int)(uint32_t)(v >> 32);
    int l2, h2;
    switch (ctrl_sel) {
        case 0: l2 = __builtin_amdgcn_mov_dpp(lo, 0xB1, 0xF, 0xF, true); h2 = __builtin_amdgcn_mov_dpp(hi, 0xB1, 0xF, 0xF, true); break;    // lane ^ 1
        case 1: l2 = __builtin_amdgcn_mov_dpp(lo, 0x4E, 0xF, 0xF, true); h2 = __builtin_amdgcn_mov_dpp(hi, 0x4E, 0xF, 0xF, true); break;    // lane ^ 2
        case 2: l2 = __builtin_amdgcn_mov_dpp(lo, 0x141, 0xF, 0xF, true); h2 = __builtin_amdgcn_mov_dpp(hi, 0x141, 0xF, 0xF, true); break;  // 7 - lane
        default: l2 = __builtin_amdgcn_mov_dpp(lo, 0x140, 0xF, 0xF, true); h2 = __builtin_amdgcn_mov_dpp(hi, 0x140, 0xF, 0xF, true); break; // 15 - lane
    }
    return (uint64_t)(uint32_t)h2 << 32 | (uint32_t)l2;
}
__device__ __forceinline__ uint64_t lane_u64(uint64_t v, const int l) {
    return (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), l) << 32 |
           (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, l);
}
__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const uint64_t u = dpp_u64(v, s);
        v = u > v ? u : v;
    }
    const uint64_t a = lane_u64(v, 0), b = lane_u64(v, 16), c = lane_u64(v, 32), d = lane_u64(v, 48);
    const uint64_t ab = a > b ? a : b, cd = c > d ? c : d;
    return ab > cd ? ab : cd;
}
__device__ __forceinline__ uint64_t wave_sum_u64(uint64_t v) {
#pragma unroll
    for (int s = 0; s < 4; ++s) v += dpp_u64(v, s);
    return (lane_u64(v, 0) + lane_u64(v, 16)) + (lane_u64(v, 32) + lane_u64(v, 48));
}


__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
    v = max(v, (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true));
    v = max(v, (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true));
    v = max(v, (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x141, 0xF, 0xF, true));
    v = max(v, (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x140, 0xF, 0xF, true));
    const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)v, 0), b = (uint32_t)__builtin_amdgcn_readlane((int)v, 16);
    const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)v, 32), d = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
    return max(max(a, b), max(c, d));
}

// ---- work split of the row-streaming kernels: (row, 1024-channel segment) items --------------
constexpr int SEG_CHUNKS = 128;             // chunks per segment (two per lane)
constexpr int SEG_CH = SEG_CHUNKS * 8;      // channels per segment


struct QItem {
    int m, seg;
};
// linear work item (four per workgroup trip) -> (row, segment).  A block of 32 rows is
// 32*nseg items; XCD x = workgroup % 8 owns blocks x, x+8, ...
__device__ __forceinline__ QItem quant_item(int wg, int wave, int nseg, int M) {
    const int per_block = 8 * nseg;          // workgroups per 32-row block
    const int x = wg & 7, s = wg >> 3;
    const int block = x + 8 * (s / per_block);
    const int it = (s % per_block) * 4 + wave;  // item within the block, row-major (row, segment)
    QItem q;
    q.m = block * 32 + it / nseg;
    q.seg = it % nseg;
    if (q.m >= M) q.m = -1;
    return q;
}


}  // namespace osc
