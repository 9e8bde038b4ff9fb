// Dual-path GEMM (Section 3.3.1, Eq. dual-path) and FP8 W8A8 GEMM (Section 3.4) on the CDNA4
// matrix cores, single and grouped (mixture-of-experts) forms, one kernel template.
//
// Operands.  Every operand is a row-major byte matrix whose rows run along the reduction axis
// (FP4 codes: K/2 bytes per row, FP8 codes: K bytes, bf16 branch: 2*K_o bytes).  The reduction
// axis is consumed 64 bytes per row per step: 128 FP4 channels = four scale groups = one scale
// word of the row-block-major scale layout (see osc.h), 64 FP8 channels, or 32 bf16 channels.
//
// Matrix-core operand layout (32x32 tiles, 64-lane wavefront, lane = 32*q + r):
//   v_mfma_scale_f32_32x32x64_f8f6f4, FP4: lane holds row r, 32 consecutive elements (16 bytes) of
//     reduction block q and, in one byte of its scale register picked by op_sel, their E8M0 scale.
//     FP8: lane holds 32 bytes of block q; unit scales, row/column scales applied in the epilogue.
//   v_mfma_f32_32x32x16_bf16: lane holds row r, 8 consecutive bf16 (16 bytes) of block q.
//   Result register i of lane (q, r'): row 8*(i/4) + 4*q + i%4, column r'.
// The hardware only pairs lane-block q of A with lane-block q of B, so how the reduction axis is
// dealt to (q, instruction) is free as long as both operands agree.  Here lanes of block q take
// bytes [32q, 32q+32) of the 64-byte step, i.e. 16-byte pieces 2q and 2q+1, and piece I feeds
// MFMA I; the FP4 scale word is shifted right by 16q bits so that byte I is the scale of piece I.
//
// The kernels share these conventions; the host picks one per call (launch_gemm):
//   gemm_kernel        register-staged (global -> VGPR -> LDS -> MFMA), 64-byte steps, any legal
//                      shape (ragged rows through a block of zeros), grouped and row-mapped problems;
//   gemm_dma2_kernel   global -> LDS by DMA in whole 128-byte lines, two LDS stages; dual path, FP8 and
//                      MXFP8, grouped and row-mapped problems; needs 128-byte row pitches.  Tiles of
//                      256x256 and 128x256 on eight wavefronts, 128x128 and 64x128 on four; a launch of
//                      at most one 64x128 tile per CU splits every tile's K loop over two wavefront groups;
//   gemm_dma2g_kernel  the same stages on persistent workgroups for grouped 8-bit problems;
//   gemm_pipe2_kernel  the same data path, persistent workgroups, slot-pinned instruction order,
//                      early buffer release; one problem (dual path, FP8 or MXFP8) of more than one whole
//                      256x256 tile per CU (a ragged row tail goes to the DMA kernel);
//   gemm_skinny_kernel M <= 64 (decode) and other launches of at most 512 blocks of 32x32 outputs: one
//                      workgroup per 32 output channels streams the weights once, its wavefronts split
//                      the reduction axis;
//   gemm_ring_kernel   a four-slot ring of half stages with two wavefront groups in anti-phase; never
//                      chosen by the launcher, reachable through the tuning override only.
#include <cstdio>
#include <cstdlib>
#include <type_traits>

#include "osc_internal.h"
#include "lds_dma.h"

namespace osc {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int GT = 256;  // 4 wavefronts, arranged 2 x 2 over the workgroup tile
enum { MODE_DUAL = 0, MODE_FP8 = 1, MODE_MX8 = 2 };  // MX8: E4M3 codes with E8M0 block scales on both operands

struct KArgs {
    const uint8_t* Xq;
    const uint8_t* Xs;
    const float* xs;
    const uint8_t* B;
    int64_t bpitch;  // bytes per row of B
    const int32_t* row_map;
    const int32_t* off;
    int E;
    const uint8_t* Wpack;
    size_t pack_stride, off_q, off_s, off_l, off_z;
    int64_t wlpitch;  // bytes per row of W_L^T
    int M, N, K, K_o;
    void* Y;
    int y_bf16;
    int64_t ldy;
    int tiles_n;
    // grouped problems, which rows of an expert this launch covers: 0 = all of them; 1 = its first
    // (n + BM/2) / BM tiles (an expert whose last tile would be less than half full leaves those rows
    // out); 2 = the rows that a mode-1 launch with tiles of grp_bm rows left out
    int grp_mode, grp_bm;
};



struct TilePos {
    int m0, n0, row_begin, row_end;
    const uint8_t* wp;
    bool valid;
};

// Workgroups are dealt round-robin to the 8 XCDs; renumber so that each XCD owns a contiguous
// run of tiles and its L2 sees neighbouring tiles.  Single problem: tiles walk down bands of 8
// m-tiles.  Grouped: m-tiles are numbered expert by expert (the grid is an upper bound).
template <int BM, int BN>
__device__ __forceinline__ TilePos tile_at(const KArgs& a, int tile);

template <int BM, int BN>
__device__ __forceinline__ TilePos locate_tile(const KArgs& a) {
    int tile = blockIdx.x;
    if (a.off) {
        // grouped: XCD x takes m-tiles x, x+8, ... and walks the n-tiles of each in turn (they share
        // the activation rows).  The surplus m-tiles at the end of the numbering (the grid is an
        // upper bound, a multiple of 8 m-tiles) are then spread over all XCDs.
        const int x = tile & 7, sidx = tile >> 3;
        tile = ((sidx / a.tiles_n) * 8 + x) * a.tiles_n + sidx % a.tiles_n;
    } else {
        const int per = gridDim.x >> 3;
        if (tile < (per << 3)) tile = (tile & 7) * per + (tile >> 3);
    }
    return tile_at<BM, BN>(a, tile);
}

// position of tile number `tile` (numbered so that neighbours share operand panels)
template <int BM, int BN>
__device__ __forceinline__ TilePos tile_at(const KArgs& a, int tile) {
    TilePos p;
    p.row_begin = 0;
    p.row_end = a.M;
    p.wp = a.Wpack;
    p.valid = true;
    int tm_idx, tn_idx;
    if (a.off) {
        // m-tiles are numbered expert by expert.  Every wavefront finds the expert of m-tile j by
        // itself: 64 experts at a time, one per lane, prefix sum of their tile counts, first lane
        // whose running total exceeds j.  (A serial walk over the offsets costs one dependent
        // memory round trip per expert.)
        tn_idx = tile % a.tiles_n;
        const int j = tile / a.tiles_n;
        const int lane = threadIdx.x & 63;
        int before = 0, e_found = -1, j_in = 0;
        for (int e0 = 0; e0 < a.E; e0 += 64) {
            const int e = e0 + lane;
            int b = e < a.E ? a.off[e] : 0;
            int n = e < a.E ? a.off[e + 1] - b : 0;
            if (a.grp_mode == 1) {
                n = min(n, (n + BM / 2) / BM * BM);
            } else if (a.grp_mode == 2) {
                const int skip = min(n, (n + a.grp_bm / 2) / a.grp_bm * a.grp_bm);
                b += skip;
                n -= skip;
            }
            const int te = (n + BM - 1) / BM;
            int ps = te;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int v = __shfl_up(ps, d);
                if (lane >= d) ps += v;
            }
            const int total = __shfl(ps, 63);
            if (j < before + total) {
                const int l = __ffsll((unsigned long long)__ballot(before + ps > j)) - 1;
                e_found = e0 + l;
                j_in = j - (before + __shfl(ps, l) - __shfl(te, l));
                p.row_begin = __shfl(b, l);
                p.row_end = p.row_begin + __shfl(n, l);
                break;
            }
            before += total;
        }
        e_found = __builtin_amdgcn_readfirstlane(e_found);
        j_in = __builtin_amdgcn_readfirstlane(j_in);
        p.row_begin = __builtin_amdgcn_readfirstlane(p.row_begin);
        p.row_end = __builtin_amdgcn_readfirstlane(p.row_end);
        if (e_found < 0) {  // surplus workgroup (the grid is an upper bound)
            p.valid = false;
            e_found = 0;
        }
        tm_idx = j_in;
        p.wp += (size_t)e_found * a.pack_stride;
    } else {
        const int tiles_m = (a.M + BM - 1) / BM;
        const int band = tile / (8 * a.tiles_n), within = tile - band * 8 * a.tiles_n;
        const int rows = min(8, tiles_m - band * 8);
        tm_idx = band * 8 + within % rows;
        tn_idx = within / rows;
    }
    p.m0 = p.row_begin + tm_idx * BM;
    p.n0 = tn_idx * BN;
    return p;
}

// LDS_SCALES (FP8, tiles entirely inside Y): the row scales of the tile's BM rows and the column scales of
// its BN columns are read from `tile_scales` in LDS (BM + BN floats) instead of global memory.
template <int MODE, int TM, int TN, int WN = 2, bool LDS_SCALES = false>
__device__ __forceinline__ void store_result(const KArgs& a, const TilePos& tp, v16f (&acc)[TM][TN],
                                             const float* tile_scales = nullptr) {
    constexpr int BM = 64 * TM, BN = 32 * TN * WN;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave / WN, wn = wave % WN, q = lane >> 5, r = lane & 31;
    const int m0 = tp.m0, n0 = tp.n0, row_end = tp.row_end;
    const uint8_t* wp = tp.wp;
    // ---- epilogue ---------------------------------------------------------------------------
    // Result register k of lane (q, r): row 8*(k/4) + 4*q + k%4, column r of its 32x32 tile.
    // fp32: every register is one 128-byte row segment per half-wave.  bf16: neighbouring lanes
    // swap one register of each pair so that every lane owns two adjacent columns of one row and
    // writes them as one 32-bit word (even lanes row k, odd lanes row k+1).
    const float* wsc = (MODE == MODE_FP8) ? reinterpret_cast<const float*>(wp + a.off_s) : nullptr;
    const int odd = r & 1;
    const int wu_m = __builtin_amdgcn_readfirstlane(wm), wu_n = __builtin_amdgcn_readfirstlane(wn);
    // byte offset of this lane's four columns inside a 32x32 result tile: row 4q + r%4, columns 4(r/4) ..
    const uint32_t yoff8 = 2u * (uint32_t)((4 * q + (r & 3)) * (int)a.ldy + (r & ~3));
    const bool hi2 = (r & 2) != 0;
    // 16-byte stores of eight bf16 columns need rows that keep 16-byte alignment
    const bool wide16 = (a.ldy & 7) == 0 && (reinterpret_cast<uintptr_t>(a.Y) & 15) == 0;
    // byte selector of step 2: even lanes [own.lo, other.lo], odd lanes [other.hi, own.hi]
    const uint32_t sel12 = odd ? 0x03020706u : 0x05040100u;
    auto store_tile = [&](auto kind_tag) __attribute__((always_inline)) {
        // 2: tile entirely inside Y, no bounds tests; 1: all columns inside, rows tested (ragged
        // last tile of a problem or an expert); 0: everything tested, 2-byte stores
        constexpr int KIND = decltype(kind_tag)::value;
        constexpr bool FULL = KIND == 2;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int rbase = m0 + wm * (TM * 32) + i * 32 + 4 * q;
            float xr[16];
            if (MODE == MODE_FP8) {
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    const int row = rbase + 8 * (k >> 2) + (k & 3);
                    if constexpr (LDS_SCALES) xr[k] = tile_scales[row - m0];
                    else xr[k] = a.xs[FULL ? row : min(row, row_end - 1)];
                }
            }
            if constexpr (KIND >= 1 && TN % 2 == 0) {
                if (a.y_bf16 && wide16) {
                    // 16-byte stores: the two exchange rounds described below, on two neighbouring tiles,
                    // then a third between lanes l and l^4: lanes of even column groups complete eight
                    // adjacent columns of the left tile, the others of the right tile, so one store
                    // instruction writes eight rows of 128 contiguous bytes.
                    const bool lo4 = (r & 4) != 0;
                    const uint32_t yoff16 = 2u * (uint32_t)((4 * q + (r & 3)) * (int)a.ldy + (r & ~3) + (lo4 ? 28 : 0));
#pragma unroll
                    for (int jp = 0; jp < TN; jp += 2) {
                        u32x2 o[2][4];
#pragma unroll
                        for (int s2 = 0; s2 < 2; ++s2) {
                            const int j = jp + s2;
                            float cs = 1.0f;
                            if (MODE == MODE_FP8) cs = LDS_SCALES ? tile_scales[BM + wn * (TN * 32) + j * 32 + r] : wsc[n0 + wn * (TN * 32) + j * 32 + r];
                            uint32_t P[8], W[8];
#pragma unroll
                            for (int k = 0; k < 8; ++k) {
                                const float v0 = (MODE == MODE_FP8) ? acc[i][j][2 * k] * (xr[2 * k] * cs) : acc[i][j][2 * k];
                                const float v1 = (MODE == MODE_FP8) ? acc[i][j][2 * k + 1] * (xr[2 * k + 1] * cs)
                                                                     : acc[i][j][2 * k + 1];
                                const v2f pair = {v0, v1};
                                P[k] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pair, v2bf));
                            }
#pragma unroll
                            for (int k = 0; k < 8; ++k) {
                                const uint32_t Q = (uint32_t)__builtin_amdgcn_mov_dpp((int)P[k], 0xB1, 0xF, 0xF, true);
                                W[k] = __builtin_amdgcn_perm(Q, P[k], sel12);
                            }
#pragma unroll
                            for (int h = 0; h < 4; ++h) {
                                const uint32_t ra = (uint32_t)__builtin_amdgcn_mov_dpp((int)W[2 * h], 0x4E, 0xF, 0xF, true);
                                const uint32_t rb = (uint32_t)__builtin_amdgcn_mov_dpp((int)W[2 * h + 1], 0x4E, 0xF, 0xF, true);
                                o[s2][h] = (u32x2){hi2 ? rb : W[2 * h], hi2 ? W[2 * h + 1] : ra};
                            }
                        }
                        uint8_t* const ybase = reinterpret_cast<uint8_t*>(a.Y) +
                            2 * ((int64_t)(m0 + wu_m * (TM * 32) + i * 32) * a.ldy + n0 + wu_n * (TN * 32) + jp * 32);
#pragma unroll
                        for (int h = 0; h < 4; ++h) {
                            // lane + 4 sends its left-tile words down, lane - 4 its right-tile words up
                            const uint32_t dx = (uint32_t)__builtin_amdgcn_mov_dpp((int)o[0][h].x, 0x104, 0xF, 0xF, true);
                            const uint32_t dy = (uint32_t)__builtin_amdgcn_mov_dpp((int)o[0][h].y, 0x104, 0xF, 0xF, true);
                            const uint32_t ux = (uint32_t)__builtin_amdgcn_mov_dpp((int)o[1][h].x, 0x114, 0xF, 0xF, true);
                            const uint32_t uy = (uint32_t)__builtin_amdgcn_mov_dpp((int)o[1][h].y, 0x114, 0xF, 0xF, true);
                            const u32x4 out = {lo4 ? ux : o[0][h].x, lo4 ? uy : o[0][h].y, lo4 ? o[1][h].x : dx,
                                               lo4 ? o[1][h].y : dy};
                            uint8_t* const hbase = ybase + 2 * (int64_t)(8 * h) * a.ldy;
                            if (FULL || rbase + 8 * h + (r & 3) < row_end)
                                __builtin_nontemporal_store(out, reinterpret_cast<u32x4*>(hbase + yoff16));
                        }
                    }
                    continue;
                }
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = n0 + wn * (TN * 32) + j * 32 + r;
                float cs = 1.0f;
                if (MODE == MODE_FP8) cs = LDS_SCALES ? tile_scales[BM + col - n0] : wsc[FULL ? col : min(col, a.N - 1)];
                float v[16];
#pragma unroll
                for (int k = 0; k < 16; ++k)
                    v[k] = (MODE == MODE_FP8) ? acc[i][j][k] * (xr[k] * cs) : acc[i][j][k];
                if (a.y_bf16 && KIND >= 1) {
                    // 8-byte stores: two rounds of exchanges inside each quad of lanes turn "one column,
                    // sixteen rows per lane" into "four adjacent columns of one row per lane".
                    //  1. pairs of result registers (rows R, R+1 of column c) are rounded to packed bf16;
                    //  2. lanes c, c^1 swap halves: even lanes get row R, odd lanes row R+1, columns c&~1, +1;
                    //  3. lanes l, l^2 swap words of register pairs (k, k+2): lanes 0,1 of a quad complete
                    //     rows R, R+1, lanes 2,3 rows R+2, R+3, columns 4b .. 4b+3.
                    // Each step runs over all registers of the tile before the next one starts, so the
                    // single wavefront of a SIMD always has independent instructions to issue.
                    uint8_t* const ybase = reinterpret_cast<uint8_t*>(a.Y) +
                        2 * ((int64_t)(m0 + wu_m * (TM * 32) + i * 32) * a.ldy + n0 + wu_n * (TN * 32) + j * 32);
                    uint32_t P[8], W[8];
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        const v2f pair = {v[2 * k], v[2 * k + 1]};
                        P[k] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pair, v2bf));
                    }
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        const uint32_t Q = (uint32_t)__builtin_amdgcn_mov_dpp((int)P[k], 0xB1, 0xF, 0xF, true);
                        W[k] = __builtin_amdgcn_perm(Q, P[k], sel12);
                    }
#pragma unroll
                    for (int h = 0; h < 4; ++h) {
                        // both words cross to lane l^2; each lane keeps one of its own and one of the other's
                        // (every crossing has a single use, so it folds into the select that consumes it)
                        const uint32_t ra = (uint32_t)__builtin_amdgcn_mov_dpp((int)W[2 * h], 0x4E, 0xF, 0xF, true);
                        const uint32_t rb = (uint32_t)__builtin_amdgcn_mov_dpp((int)W[2 * h + 1], 0x4E, 0xF, 0xF, true);
                        const u32x2 out = {hi2 ? rb : W[2 * h], hi2 ? W[2 * h + 1] : ra};
                        uint8_t* const hbase = ybase + 2 * (int64_t)(8 * h) * a.ldy;
                        if (FULL || rbase + 8 * h + (r & 3) < row_end)
                            __builtin_nontemporal_store(out, reinterpret_cast<u32x2*>(hbase + yoff8));
                    }
                } else if (a.y_bf16) {
                    uint16_t* Y = reinterpret_cast<uint16_t*>(a.Y);
#pragma unroll
                    for (int k = 0; k < 16; k += 2) {
                        const float send = odd ? v[k] : v[k + 1];
                        // neighbour lane's value: DPP quad_perm [1,0,3,2]
                        const float recv = __builtin_bit_cast(
                            float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), 0xB1, 0xF, 0xF, false));
                        const float lo = odd ? recv : v[k], hi = odd ? v[k + 1] : recv;
                        const int row = rbase + 8 * (k >> 2) + (k & 3) + odd;
                        const int c0 = col - odd;
                        uint16_t* dst = Y + (int64_t)row * a.ldy + c0;
                        const uint32_t word =
                            (uint32_t)f32_to_bf16_rne(lo) | ((uint32_t)f32_to_bf16_rne(hi) << 16);
                        if (row < row_end) {
                            if (c0 < a.N) dst[0] = (uint16_t)word;
                            if (c0 + 1 < a.N) dst[1] = (uint16_t)(word >> 16);
                        }
                    }
                } else {
                    float* Y = reinterpret_cast<float*>(a.Y);
#pragma unroll
                    for (int k = 0; k < 16; ++k) {
                        const int row = rbase + 8 * (k >> 2) + (k & 3);
                        if (FULL || (row < row_end && (KIND == 1 || col < a.N))) Y[(int64_t)row * a.ldy + col] = v[k];
                    }
                }
            }
        }
    };
    // 32-bit stores of bf16 pairs need an even leading dimension and a 4-byte aligned Y
    const bool cols = (n0 + BN <= a.N) &&
                      (!a.y_bf16 || (((a.ldy & 3) == 0) && ((reinterpret_cast<uintptr_t>(a.Y) & 7) == 0)));
    if (cols && m0 + BM <= row_end)
        store_tile(std::integral_constant<int, 2>{});
    else if (cols)
        store_tile(std::integral_constant<int, 1>{});
    else
        store_tile(std::integral_constant<int, 0>{});
}

// ------------------------------------------------------------------------------------------
// Ring kernel.  Per step every row contributes 64 contiguous bytes (FP4: 128 channels = four
// scale groups = one scale word; FP8: 64 channels; bf16: 32 channels).  Lanes of block q take
// bytes [32q, 32q+32) of the step, i.e. 16-byte pieces 2q and 2q+1; piece I feeds MFMA I.  The
// FP4 scale word is shifted right by 16q bits so that byte I is again the scale of piece I.
//
// LDS holds four stages of (BM + BN) rows x 64 bytes.  In step s a workgroup computes from stage
// s % 4 and refills stage (s+3) % 4, which every wave left before the barrier that ended step
// s-1, with the operands of step s+3.  Those loads are spread between the MFMAs of the step (a
// wave that issued them in one burst would sit in the memory queue instead of feeding the matrix
// core).  The barrier that ends step s first waits for the loads issued during step s-1, so the
// operands of step s+2 are published there; a load has between one and two steps to land.
// ------------------------------------------------------------------------------------------

// piece `c` (0..3) of stage row `r` sits at piece position c ^ ((r >> 2) & 3): the 16 lanes of one
// LDS access phase (consecutive rows, same piece) then cover all 64 banks
__device__ __forceinline__ int ring_off(int row, int piece) {
    return row * 64 + ((piece ^ ((row >> 2) & 3)) << 4);
}

// Scheduling hint for one half step: ND LDS reads, NW LDS writes and NV VMEM operations spread
// evenly between NM MFMAs (the compiler would otherwise bunch them).
template <int NM, int ND, int NW, int NV, int K = 0>
__device__ __forceinline__ void spread_hint() {
    constexpr int G = (ND > NW ? ND : NW) > 0 ? (ND > NW ? ND : NW) : 1;
    if constexpr (K < G) {
        constexpr int m = NM / G + (K < NM % G ? 1 : 0);
        constexpr int d = ND / G + (K < ND % G ? 1 : 0);
        constexpr int w = NW / G + (K < NW % G ? 1 : 0);
        constexpr int v = NV / G + (K < NV % G ? 1 : 0);
        if constexpr (m > 0) __builtin_amdgcn_sched_group_barrier(0x008, m, 0);
        if constexpr (d > 0) __builtin_amdgcn_sched_group_barrier(0x100, d, 0);
        if constexpr (w > 0) __builtin_amdgcn_sched_group_barrier(0x200, w, 0);
        if constexpr (v > 0) __builtin_amdgcn_sched_group_barrier(0x020, v, 0);
        spread_hint<NM, ND, NW, NV, K + 1>();
    }
}

// RAGGED = false needs every operand row to be a whole number of 64-byte steps; RAGGED = true
// redirects, lane by lane, the pieces past the end of a row to a block of zeros in the packed
// weight (address arithmetic only: nothing may depend on a loaded value before it is used, or
// the compiler waits for the load right after issuing it).
template <int MODE, int TM, int TN, bool RAGGED>
__global__ void __launch_bounds__(GT) gemm_kernel(KArgs a) {
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr int STG = (BM + BN) * 64;        // bytes per LDS stage
    constexpr int LA = BM / 64, LB = BN / 64;  // 16-byte loads per thread and step
    constexpr int NSC = (MODE == MODE_DUAL) ? TM + TN : 0;  // scale words per lane and step
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1, q = lane >> 5, r = lane & 31;
    const TilePos tp = locate_tile<BM, BN>(a);
    if (!tp.valid) return;
    const int m0 = tp.m0, n0 = tp.n0, row_end = tp.row_end;
    const uint8_t* wp = tp.wp;

    const int Kg4 = ((a.K >> 5) + 3) >> 2;
    const int rowbytes = (MODE == MODE_DUAL) ? (a.K >> 1) : a.K;
    const int nA = (rowbytes + 63) >> 6;                                  // steps of the main phase
    const int nB = (MODE == MODE_DUAL) ? ((a.K_o * 2 + 63) >> 6) : 0;     // steps of the bf16 branch
    const int nS = nA + nB;
    const int validB_a = (int)a.bpitch, validB_b = (int)a.wlpitch;  // bytes per row in the bf16 phase

    // ---- global -> registers: thread t owns stage position (row (t >> 2) + 64 i, piece t & 3) ----
    const int c4 = (t & 3) ^ ((t >> 4) & 3);  // reduction-axis piece stored at that position
    // 32-bit byte offsets of this thread's piece in each operand (the launcher checks that they fit)
    uint32_t oa[LA], ob[LB], oa2[LA], ob2[LB];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        int g = min(m0 + (t >> 2) + 64 * i, row_end - 1);
        if (MODE == MODE_DUAL && a.row_map) g = a.row_map[g];
        oa[i] = (uint32_t)g * (uint32_t)rowbytes + c4 * 16;
        oa2[i] = (uint32_t)g * (uint32_t)a.bpitch + c4 * 16;
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        const int n = min(n0 + (t >> 2) + 64 * i, a.N - 1);
        ob[i] = (uint32_t)n * (uint32_t)rowbytes + c4 * 16;
        ob2[i] = (uint32_t)n * (uint32_t)a.wlpitch + c4 * 16;
    }
    const uint8_t* wq = wp + a.off_q;
    const uint8_t* wl = wp + a.off_l;
    const uint8_t* zeros = wp + a.off_z;  // 256 bytes of zeros at the end of every packed weight

    // ---- scale words: one per (row, step) -----------------------------------------------------
    uint32_t so_a[TM], so_b[TN];
    if (MODE == MODE_DUAL) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            int g = min(m0 + wm * (TM * 32) + i * 32 + r, row_end - 1);
            if (a.row_map) g = a.row_map[g];
            so_a[i] = (uint32_t)(g >> 5) * (uint32_t)Kg4 * 128u + (g & 31) * 4;
        }
#pragma unroll
        for (int i = 0; i < TN; ++i) {
            const int n = min(n0 + wn * (TN * 32) + i * 32 + r, a.N - 1);
            so_b[i] = (uint32_t)(n >> 5) * (uint32_t)Kg4 * 128u + (n & 31) * 4;
        }
    }
    const uint8_t* wsb = wp + a.off_s;

    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int k = 0; k < 16; ++k) acc[i][j][k] = 0.0f;

    const int ra0 = wm * (TM * 32) + r, rb0 = BM + wn * (TN * 32) + r;  // stage rows of tile 0

    // Macros rather than closures: the compiler keeps arrays that closures capture, when those
    // closures are expanded in several loops, in scratch memory.
    //
    // Operands of step T_ of a phase into a register set.  A step past the end of the phase
    // re-reads the last one (the data is never used); with RAGGED, pieces past the end of a row
    // come from the block of zeros.
#define OSC_LOAD(T_, NSTEP_, ABASE_, BBASE_, OA_, OB_, AVALID_, BVALID_, RA_, RB_)                   \
    {                                                                                                \
        const int T__ = min((T_), (NSTEP_)-1);                                                       \
        const uint8_t* ab__ = (ABASE_) + T__ * 64;                                                   \
        const uint8_t* bb__ = (BBASE_) + T__ * 64;                                                   \
        if (RAGGED) {                                                                                \
            const bool ina__ = T__ * 64 + c4 * 16 < (AVALID_), inb__ = T__ * 64 + c4 * 16 < (BVALID_); \
            _Pragma("unroll") for (int i = 0; i < LA; ++i) RA_[i] =                                  \
                *reinterpret_cast<const u32x4*>(ina__ ? ab__ + OA_[i] : zeros);                      \
            _Pragma("unroll") for (int i = 0; i < LB; ++i) RB_[i] =                                  \
                *reinterpret_cast<const u32x4*>(inb__ ? bb__ + OB_[i] : zeros);                      \
        } else {                                                                                     \
            _Pragma("unroll") for (int i = 0; i < LA; ++i) RA_[i] =                                  \
                *reinterpret_cast<const u32x4*>(ab__ + OA_[i]);                                      \
            _Pragma("unroll") for (int i = 0; i < LB; ++i) RB_[i] =                                  \
                *reinterpret_cast<const u32x4*>(bb__ + OB_[i]);                                      \
        }                                                                                            \
    }
#define OSC_LOAD_MAIN(T_, RA_, RB_) OSC_LOAD(T_, nA, a.Xq, wq, oa, ob, rowbytes, rowbytes, RA_, RB_)
#define OSC_LOAD_BRANCH(T_, RA_, RB_) OSC_LOAD(T_, nB, a.B, wl, oa2, ob2, validB_a, validB_b, RA_, RB_)
    // step S_ of the whole sequence (main phase, then bf16 branch); nothing to load past its end
#define OSC_LOAD_ANY(S_, RA_, RB_)                 \
    {                                              \
        if ((S_) < nA) {                           \
            OSC_LOAD_MAIN((S_), RA_, RB_)          \
        } else if ((S_) < nS) {                    \
            OSC_LOAD_BRANCH((S_)-nA, RA_, RB_)     \
        }                                          \
    }
    // a register set into LDS stage STG_
#define OSC_PUT(STG_, RA_, RB_)                                                                       \
    {                                                                                                 \
        uint8_t* st__ = lds + (STG_)*STG + t * 16;                                                    \
        _Pragma("unroll") for (int i = 0; i < LA; ++i) *reinterpret_cast<u32x4*>(st__ + i * 4096) = RA_[i]; \
        _Pragma("unroll") for (int i = 0; i < LB; ++i)                                                \
            *reinterpret_cast<u32x4*>(st__ + BM * 64 + i * 4096) = RB_[i];                            \
    }
    // fragments of piece P_ from stage STG_
#define OSC_FRAGS(STG_, P_, FA_, FB_)                                                                 \
    {                                                                                                 \
        const uint8_t* st__ = lds + (STG_)*STG;                                                       \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) FA_[i] =                                       \
            *reinterpret_cast<const u32x4*>(st__ + ring_off(ra0 + 32 * i, (P_)));                     \
        _Pragma("unroll") for (int j = 0; j < TN; ++j) FB_[j] =                                       \
            *reinterpret_cast<const u32x4*>(st__ + ring_off(rb0 + 32 * j, (P_)));                     \
    }
    // scale words of step T_ (a step past the end re-reads the last one and is never used; the
    // scale bytes of groups past K/32 inside the last word are zero by layout)
#define OSC_SCALES(T_, SA_, SB_)                                                                      \
    {                                                                                                 \
        const uint32_t o__ = (uint32_t)min((T_), Kg4 - 1) * 128u;                                     \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) SA_[i] =                                       \
            *reinterpret_cast<const int*>(a.Xs + o__ + so_a[i]);                                      \
        _Pragma("unroll") for (int i = 0; i < TN; ++i) SB_[i] =                                       \
            *reinterpret_cast<const int*>(wsb + o__ + so_b[i]);                                       \
    }
#define OSC_MFMA_FP4(I_, FA_, FB_, SA_, SB_)                                                          \
    {                                                                                                 \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) {                                              \
            const v8i av__ = {(int)FA_[i].x, (int)FA_[i].y, (int)FA_[i].z, (int)FA_[i].w, 0, 0, 0, 0}; \
            _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                          \
                const v8i bv__ = {(int)FB_[j].x, (int)FB_[j].y, (int)FB_[j].z, (int)FB_[j].w, 0, 0, 0, 0}; \
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av__, bv__, acc[i][j], 4, 4, I_, \
                                                                            SA_[i], I_, SB_[j]);      \
            }                                                                                         \
        }                                                                                             \
    }
#define OSC_MFMA_BF16(FA_, FB_)                                                                       \
    {                                                                                                 \
        _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                \
            _Pragma("unroll") for (int j = 0; j < TN; ++j) acc[i][j] =                                \
                __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, FA_[i]),             \
                                                        __builtin_bit_cast(v8bf, FB_[j]), acc[i][j], 0, 0, 0); \
    }
    // FP8: one MFMA per tile pair and step; tile pairs [LO_, HI_)
#define OSC_MFMA_FP8(LO_, HI_, FA_, GA_, FB_, GB_)                                                    \
    {                                                                                                 \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) {                                              \
            const v8i av__ = {(int)FA_[i].x, (int)FA_[i].y, (int)FA_[i].z, (int)FA_[i].w,             \
                              (int)GA_[i].x, (int)GA_[i].y, (int)GA_[i].z, (int)GA_[i].w};            \
            _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                          \
                if (i * TN + j < (LO_) || i * TN + j >= (HI_)) continue;                              \
                const v8i bv__ = {(int)FB_[j].x, (int)FB_[j].y, (int)FB_[j].z, (int)FB_[j].w,         \
                                  (int)GB_[j].x, (int)GB_[j].y, (int)GB_[j].z, (int)GB_[j].w};        \
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av__, bv__, acc[i][j], 0, 0, 0, \
                                                                            0x7f7f7f7f, 0, 0x7f7f7f7f); \
            }                                                                                         \
        }                                                                                             \
    }

    // ---- prologue: step 0 in LDS, step 1 in registers ------------------------------------------
    // Two register sets hold operands in flight.  At the top of a step, set W holds the operands
    // of the next step (written to LDS during this step) and set L is free (receives the loads of
    // the step after the next).
    u32x4 ra0s[LA], rb0s[LB], ra1s[LA], rb1s[LB];
    int sn_a[TM], sn_b[TN];
    OSC_LOAD_ANY(0, ra0s, rb0s)
    OSC_LOAD_ANY(1, ra1s, rb1s)
    if (MODE == MODE_DUAL && nA > 0) OSC_SCALES(0, sn_a, sn_b)
    OSC_PUT(0, ra0s, rb0s)
    __syncthreads();
    int stg = 0;  // stage of the current step; the next one is (stg + 1) % 3

#define OSC_NEXT_STAGE (stg == 2 ? 0 : stg + 1)
    // One step of the FP4 phase.  LOADER_(step, set) fetches the operands two steps ahead into set
    // L; set W goes to the next LDS stage.
#define OSC_STEP_FP4(S_, LOADER_, RLA_, RLB_, RWA_, RWB_)                              \
    {                                                                                  \
        u32x4 fa0[TM], fb0[TN], fa1[TM], fb1[TN];                                      \
        int sa[TM], sb[TN];                                                            \
        OSC_FRAGS(stg, 2 * q, fa0, fb0)                                                \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) sa[i] = (unsigned)sn_a[i] >> (16 * q); \
        _Pragma("unroll") for (int i = 0; i < TN; ++i) sb[i] = (unsigned)sn_b[i] >> (16 * q); \
        OSC_SCALES((S_) + 1, sn_a, sn_b)                                               \
        LOADER_((S_) + 2, RLA_, RLB_)                                                  \
        OSC_FRAGS(stg, 2 * q + 1, fa1, fb1)                                            \
        OSC_MFMA_FP4(0, fa0, fb0, sa, sb)                                              \
        spread_hint<TM * TN, TM + TN, 0, NSC + LA + LB>();                             \
        OSC_PUT(OSC_NEXT_STAGE, RWA_, RWB_)                                            \
        OSC_MFMA_FP4(1, fa1, fb1, sa, sb)                                              \
        spread_hint<TM * TN, 0, LA + LB, 0>();                                         \
        __syncthreads();                                                               \
        stg = OSC_NEXT_STAGE;                                                          \
    }
#define OSC_STEP_BF16(S_, RLA_, RLB_, RWA_, RWB_)                                      \
    {                                                                                  \
        u32x4 fa0[TM], fb0[TN], fa1[TM], fb1[TN];                                      \
        OSC_FRAGS(stg, 2 * q, fa0, fb0)                                                \
        OSC_LOAD_BRANCH((S_) + 2 - nA, RLA_, RLB_)                                     \
        OSC_FRAGS(stg, 2 * q + 1, fa1, fb1)                                            \
        OSC_MFMA_BF16(fa0, fb0)                                                        \
        spread_hint<TM * TN, TM + TN, 0, LA + LB>();                                   \
        OSC_PUT(OSC_NEXT_STAGE, RWA_, RWB_)                                            \
        OSC_MFMA_BF16(fa1, fb1)                                                        \
        spread_hint<TM * TN, 0, LA + LB, 0>();                                         \
        __syncthreads();                                                               \
        stg = OSC_NEXT_STAGE;                                                          \
    }
#define OSC_STEP_FP8(S_, RLA_, RLB_, RWA_, RWB_)                                       \
    {                                                                                  \
        u32x4 fa0[TM], fb0[TN], fa1[TM], fb1[TN];                                      \
        OSC_FRAGS(stg, 2 * q, fa0, fb0)                                                \
        OSC_FRAGS(stg, 2 * q + 1, fa1, fb1)                                            \
        OSC_LOAD_MAIN((S_) + 2, RLA_, RLB_)                                            \
        OSC_MFMA_FP8(0, (TM * TN) / 2, fa0, fa1, fb0, fb1)                             \
        spread_hint<(TM * TN) / 2, 0, 0, LA + LB>();                                   \
        OSC_PUT(OSC_NEXT_STAGE, RWA_, RWB_)                                            \
        OSC_MFMA_FP8((TM * TN) / 2, TM * TN, fa0, fa1, fb0, fb1)                       \
        spread_hint<TM * TN - (TM * TN) / 2, 0, LA + LB, 0>();                         \
        __syncthreads();                                                               \
        stg = OSC_NEXT_STAGE;                                                          \
    }
    // after an odd step the roles of the two sets are swapped: move the live one back to set 1
#define OSC_RESET_SETS                                                       \
    {                                                                        \
        _Pragma("unroll") for (int i = 0; i < LA; ++i) ra1s[i] = ra0s[i];    \
        _Pragma("unroll") for (int i = 0; i < LB; ++i) rb1s[i] = rb0s[i];    \
    }

    // Two steps per trip so that the register sets alternate statically.
    if (MODE == MODE_FP8) {
        int s = 0;
#pragma unroll 1
        for (; s + 1 < nA; s += 2) {
            OSC_STEP_FP8(s, ra0s, rb0s, ra1s, rb1s)
            OSC_STEP_FP8(s + 1, ra1s, rb1s, ra0s, rb0s)
        }
        if (s < nA) OSC_STEP_FP8(s, ra0s, rb0s, ra1s, rb1s)
    } else {
        int s = 0;
        // Path A: block-scaled FP4.  Its last two steps already load the bf16 branch.
#pragma unroll 1
        for (; s + 3 < nA; s += 2) {
            OSC_STEP_FP4(s, OSC_LOAD_MAIN, ra0s, rb0s, ra1s, rb1s)
            OSC_STEP_FP4(s + 1, OSC_LOAD_MAIN, ra1s, rb1s, ra0s, rb0s)
        }
        if (s + 2 < nA) {  // odd remainder: one more step that still loads the main phase
            OSC_STEP_FP4(s, OSC_LOAD_MAIN, ra0s, rb0s, ra1s, rb1s)
            OSC_RESET_SETS
            ++s;
        }
        if (s + 1 < nA) {
            OSC_STEP_FP4(s, OSC_LOAD_ANY, ra0s, rb0s, ra1s, rb1s)
            OSC_STEP_FP4(s + 1, OSC_LOAD_ANY, ra1s, rb1s, ra0s, rb0s)
            s += 2;
        } else if (s < nA) {
            OSC_STEP_FP4(s, OSC_LOAD_ANY, ra0s, rb0s, ra1s, rb1s)
            OSC_RESET_SETS
            ++s;
        }
        // Path B: bf16 branch into the same accumulators
#pragma unroll 1
        for (; s + 1 < nS; s += 2) {
            OSC_STEP_BF16(s, ra0s, rb0s, ra1s, rb1s)
            OSC_STEP_BF16(s + 1, ra1s, rb1s, ra0s, rb0s)
        }
        if (s < nS) OSC_STEP_BF16(s, ra0s, rb0s, ra1s, rb1s)
    }
    store_result<MODE, TM, TN>(a, tp, acc);
}


// ------------------------------------------------------------------------------------------
// DMA variant with full cache lines: every row contributes 128 contiguous bytes per stage (one
// DMA instruction then covers 8 rows x 128 bytes; with 64-byte row segments the DMA path was
// measured at half the L2 throughput).  Two LDS stages of (BM + BN) rows x 128 bytes.  A stage is
// consumed as two 64-byte half steps, laid out as in the other kernels (lanes of block q take
// pieces 2q and 2q+1 of the half step).  The loads of the next stage are spread between the
// MFMAs of the first three quarters of the current one; the stage ends with "all loads landed"
// and one barrier.  Needs operand rows that are whole 128-byte stages.
// ------------------------------------------------------------------------------------------

constexpr int dma2_scale_bytes(int BM, int BN) { return ((BM + BN) / 32 * 256 + 1023) / 1024 * 1024; }

template <int MODE, int TM, int TN, int WN, int KS = 1>
__global__ void __launch_bounds__(128 * WN * KS) gemm_dma2_kernel(KArgs a) {
    // KS = 2 (dual path and FP8, small tiles): two groups of 2 x WN wavefronts share a tile and split its reduction
    // axis, group g taking stages g, g + 2, ... through LDS stages of its own; the partial sums meet in LDS
    // at the end.  A launch of at most one small tile per CU leaves one wavefront on every SIMD, and a stage
    // is then a chain of latencies (LDS read, eight MFMAs, barrier) with nothing to overlap it; the second
    // group fills those gaps and halves the number of stages each wavefront walks through.
    static_assert(KS == 1 || (KS == 2 && WN == 2 && (MODE == MODE_DUAL || MODE == MODE_FP8)), "K split: two groups, dual path or FP8");
    // 2 x WN wavefronts; WN = 4 puts two wavefronts on every SIMD: while one waits for its LDS
    // reads or sits between two dependent MFMAs the other keeps the matrix core busy
    constexpr int NWV = 2 * WN;                // wavefronts
    constexpr int RPP = NWV * 8;               // stage rows that one DMA pass of the workgroup fills
    constexpr int BM = 64 * TM, BN = 32 * TN * WN;
    constexpr int STG = (BM + BN) * 128;
    constexpr int LA = BM / RPP, LB = BN / RPP;  // DMA loads per thread and stage
    constexpr int NBLK = (BM + BN) / 32;      // 32-row blocks of a stage
    constexpr int NSB = (NBLK + NWV - 1) / NWV;  // scale DMA loads per wave and stage (one block each)
    static_assert(BM % RPP == 0 && BN % RPP == 0, "tile does not split over the wavefronts");
    // bytes of scale words per stage: [block][half step][32 rows][4], rounded up to whole 1 KB requests
    constexpr int SCL = dma2_scale_bytes(BM, BN);
    constexpr int NREQ = (NBLK + 3) / 4;       // 16-byte scale requests per stage (four blocks each)
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_all[];
    const int grp = KS > 1 ? __builtin_amdgcn_readfirstlane((int)threadIdx.x / (128 * WN)) : 0;
    uint8_t* const lds = lds_all + grp * (2 * STG + 2 * SCL);  // this group's two stages and their scale words
    uint8_t* const scl = lds + 2 * STG;        // scale words of the two stages

    const int t = KS > 1 ? (int)threadIdx.x % (128 * WN) : (int)threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave / WN, wn = wave % WN, q = lane >> 5, r = lane & 31;
    const TilePos tp = locate_tile<BM, BN>(a);
    if (!tp.valid) return;
    const int m0 = tp.m0, n0 = tp.n0, row_end = tp.row_end;
    const uint8_t* wp = tp.wp;

    const int Kg4 = ((a.K >> 5) + 3) >> 2;
    const int rowbytes = (MODE == MODE_DUAL) ? (a.K >> 1) : a.K;
    const int nTA = rowbytes >> 7;                                       // stages of the main phase
    const int nTB = (MODE == MODE_DUAL) ? ((a.K_o * 2 + 127) >> 7) : 0;  // stages of the bf16 branch
    const int nT = nTA + nTB;

    // thread t fills stage position (row (t >> 3) + RPP i, piece position t & 7)
    const int c8 = (t & 7) ^ swz8(t >> 3);
    uint32_t oa[LA], ob[LB];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        int g = min(m0 + (t >> 3) + RPP * i, row_end - 1);
        if (MODE == MODE_DUAL && a.row_map) g = a.row_map[g];
        oa[i] = (uint32_t)g;
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) ob[i] = (uint32_t)min(n0 + (t >> 3) + RPP * i, a.N - 1);
    const uint8_t* wq = wp + a.off_q;
    const uint8_t* wl = wp + a.off_l;
    // Scale words travel through LDS as well (a register load in the loop would make the compiler
    // wait for "all vector memory", which includes the DMA loads just issued).  Wave w moves blocks
    // w*NSB .. w*NSB+NSB-1: lanes 0-31 fetch the word of the first half step of their row, lanes
    // 32-63 that of the second.
    // (MXFP8: one scale word per row and 128-byte stage; both lane halves fetch that word.)
    uint32_t sco[NSB];
    if (MODE == MODE_DUAL || MODE == MODE_MX8) {
#pragma unroll
        for (int k = 0; k < NSB; ++k) {
            const int b = min(wave * NSB + k, NBLK - 1);
            int g;
            if (b < BM / 32) {
                g = min(m0 + 32 * b + r, row_end - 1);
                if (a.row_map) g = a.row_map[g];
            } else {
                g = min(n0 + 32 * (b - BM / 32) + r, a.N - 1);
            }
            sco[k] = (uint32_t)(g >> 5) * (uint32_t)Kg4 * 128u + (g & 31) * 4 + (MODE == MODE_DUAL ? q * 128 : 0);
        }
    }
    const uint8_t* wsb = wp + a.off_s;
    // Dual path, one problem, rows not mapped: a stage's scale words are whole 256-byte blocks of the
    // row-block-major layout, and lane l of wavefront w < NREQ fetches piece l % 16 of block 4w + l / 16 with
    // one 16-byte request (a request costs the memory pipeline the same whatever its width: three or four
    // per stage and workgroup instead of one per block and lane half).  Blocks past the last valid row or
    // channel repeat the last valid one; their rows are never stored.
    const bool use16 = MODE == MODE_DUAL && !a.off && !a.row_map;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const uint8_t* sc16_src = nullptr;
    if (use16) {
        const int blk = min(4 * min(wave_u, NREQ - 1) + (lane >> 4), NBLK - 1);
        const bool isa = blk < BM / 32;
        const int gb = isa ? min((m0 >> 5) + blk, (row_end - 1) >> 5) : min((n0 >> 5) + blk - BM / 32, (a.N - 1) >> 5);
        sc16_src = (isa ? a.Xs : wsb) + ((size_t)gb * (uint32_t)Kg4 * 128u + (uint32_t)(lane & 15) * 16u);
    }

    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int k = 0; k < 16; ++k) acc[i][j][k] = 0.0f;
    const int ra0 = wm * (TM * 32) + r, rb0 = BM + wn * (TN * 32) + r;

    // loads [LO_, HI_) of the A rows and of the B rows of stage T_ of a phase into LDS buffer BUF_
#define OSC_D2(T_, ABASE_, APITCH_, BBASE_, BPITCH_, BUF_, ALO_, AHI_, BLO_, BHI_)                   \
    {                                                                                                \
        uint8_t* st__ = lds + (BUF_)*STG + wave * 1024;                                              \
        const uint32_t o__ = (uint32_t)(T_)*128u + c8 * 16;                                          \
        _Pragma("unroll") for (int i = (ALO_); i < (AHI_); ++i)                                      \
            load_to_lds16((ABASE_) + (oa[i] * (uint32_t)(APITCH_) + o__), st__ + i * (RPP * 128));          \
        _Pragma("unroll") for (int i = (BLO_); i < (BHI_); ++i)                                      \
            load_to_lds16((BBASE_) + (ob[i] * (uint32_t)(BPITCH_) + o__), st__ + BM * 128 + i * (RPP * 128)); \
    }
    // stage S_ of the whole sequence (main phase, then bf16 branch); nothing past the end
#define OSC_D2_ANY(S_, BUF_, ALO_, AHI_, BLO_, BHI_)                                                  \
    {                                                                                                 \
        if ((S_) < nTA) {                                                                             \
            OSC_D2((S_), a.Xq, rowbytes, wq, rowbytes, BUF_, ALO_, AHI_, BLO_, BHI_)                  \
        } else if ((S_) < nT) {                                                                       \
            OSC_D2((S_)-nTA, a.B, a.bpitch, wl, a.wlpitch, BUF_, ALO_, AHI_, BLO_, BHI_)              \
        }                                                                                             \
    }
#define OSC_D2_MAIN(S_, BUF_, ALO_, AHI_, BLO_, BHI_) OSC_D2((S_), a.Xq, rowbytes, wq, rowbytes, BUF_, ALO_, AHI_, BLO_, BHI_)
#define OSC_D2_BRANCH(S_, BUF_, ALO_, AHI_, BLO_, BHI_) \
    { if ((S_) < nT) OSC_D2((S_)-nTA, a.B, a.bpitch, wl, a.wlpitch, BUF_, ALO_, AHI_, BLO_, BHI_) }
    // fragments of piece P_ (0..7) from buffer BUF_
#define OSC_F2(BUF_, P_, FA_, FB_)                                                                    \
    {                                                                                                 \
        const uint8_t* st__ = lds + (BUF_)*STG;                                                       \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) FA_[i] =                                       \
            *reinterpret_cast<const u32x4*>(st__ + st128_off(ra0 + 32 * i, (P_)));                    \
        _Pragma("unroll") for (int j = 0; j < TN; ++j) FB_[j] =                                       \
            *reinterpret_cast<const u32x4*>(st__ + st128_off(rb0 + 32 * j, (P_)));                    \
    }

    // scale words of stage T_ (half steps 2T_, 2T_+1) into scale buffer BUF_
#define OSC_D2_SCALES(T_, BUF_)                                                                       \
    {                                                                                                 \
        const uint32_t o__ = (MODE == MODE_DUAL ? (uint32_t)min(2 * (T_), Kg4 - 2) : (uint32_t)min((T_), Kg4 - 1)) * 128u; \
        if (use16) {                                                                                  \
            if (wave_u < NREQ) load_to_lds16(sc16_src + o__, scl + (BUF_)*SCL + wave_u * 1024);       \
        } else                                                                                        \
        _Pragma("unroll") for (int k = 0; k < NSB; ++k) {                                             \
            const int b__ = wave * NSB + k;                                                           \
            if (NBLK % NWV != 0 && b__ >= NBLK) continue;                                             \
            const uint8_t* src__ = (b__ < BM / 32 ? a.Xs : wsb) + (o__ + sco[k]);                     \
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src__,    \
                                             (__attribute__((address_space(3))) void*)(scl + (BUF_)*SCL + b__ * 256), \
                                             4, 0, 0);                                                \
        }                                                                                             \
    }
    // this lane's scale words of half step H_ of buffer BUF_, byte I = scale of piece 2q+I
#define OSC_D2_READ_SCALES(BUF_, H_, SA_, SB_)                                                        \
    {                                                                                                 \
        const uint8_t* sc__ = scl + (BUF_)*SCL + (H_)*128 + r * 4;                                    \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) SA_[i] =                                       \
            *reinterpret_cast<const uint32_t*>(sc__ + (wm * TM + i) * 256) >> ((MODE == MODE_MX8 ? 8 : 16) * q); \
        _Pragma("unroll") for (int j = 0; j < TN; ++j) SB_[j] =                                       \
            *reinterpret_cast<const uint32_t*>(sc__ + (BM / 32 + wn * TN + j) * 256) >> ((MODE == MODE_MX8 ? 8 : 16) * q); \
    }

    // ---- prologue ---------------------------------------------------------------------------------
    if ((MODE == MODE_DUAL || MODE == MODE_MX8) && grp < nTA) OSC_D2_SCALES(grp, 0)
    OSC_D2_ANY(grp, 0, 0, LA, 0, LB)
    wait_vmcnt<0>();
    __syncthreads();
    u32x4 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
    int buf = 0;

    // One FP4 stage = two half steps x two pieces.  REFILL_(stage, buffer, alo, ahi, blo, bhi)
    // issues part of the next stage's loads.
#define D2_R1A ((LA * 3 + 7) / 8)
#define D2_R1B ((LB * 3 + 7) / 8)
#define D2_R2A ((LA * 6 + 7) / 8)
#define D2_R2B ((LB * 6 + 7) / 8)
#define OSC_D2_STAGE_FP4(T_, REFILL_)                                                          \
    {                                                                                          \
        int sa[TM], sb[TN], ta[TM], tb[TN];                                                    \
        OSC_F2(buf, 2 * q, fa0, fb0)                                                           \
        OSC_D2_READ_SCALES(buf, 0, sa, sb)                                                     \
        if ((T_) + KS < nTA) OSC_D2_SCALES((T_) + KS, buf ^ 1)                                   \
        REFILL_((T_) + KS, buf ^ 1, 0, D2_R1A, 0, D2_R1B)                                       \
        OSC_F2(buf, 2 * q + 1, fa1, fb1)                                                       \
        OSC_MFMA_FP4(0, fa0, fb0, sa, sb)                                                      \
        spread_hint<TM * TN, TM + TN, 0, NSB + D2_R1A + D2_R1B>();                             \
        REFILL_((T_) + KS, buf ^ 1, D2_R1A, D2_R2A, D2_R1B, D2_R2B)                             \
        OSC_F2(buf, 4 + 2 * q, fa0, fb0)                                                       \
        OSC_D2_READ_SCALES(buf, 1, ta, tb)                                                     \
        OSC_MFMA_FP4(1, fa1, fb1, sa, sb)                                                      \
        spread_hint<TM * TN, 2 * (TM + TN), 0, D2_R2A - D2_R1A + D2_R2B - D2_R1B>();           \
        REFILL_((T_) + KS, buf ^ 1, D2_R2A, LA, D2_R2B, LB)                                     \
        OSC_F2(buf, 4 + 2 * q + 1, fa1, fb1)                                                   \
        OSC_MFMA_FP4(0, fa0, fb0, ta, tb)                                                      \
        spread_hint<TM * TN, TM + TN, 0, LA - D2_R2A + LB - D2_R2B>();                         \
        OSC_MFMA_FP4(1, fa1, fb1, ta, tb)                                                      \
        __builtin_amdgcn_sched_barrier(0);                                                     \
        wait_vmcnt<0>();                                                                       \
        __syncthreads();                                                                       \
        __builtin_amdgcn_sched_barrier(0);                                                     \
        buf ^= 1;                                                                              \
    }
#define OSC_D2_STAGE_BF16(T_)                                                                  \
    {                                                                                          \
        OSC_F2(buf, 2 * q, fa0, fb0)                                                           \
        OSC_D2_BRANCH((T_) + KS, buf ^ 1, 0, LA / 2, 0, LB / 2)                                 \
        OSC_F2(buf, 2 * q + 1, fa1, fb1)                                                       \
        OSC_MFMA_BF16(fa0, fb0)                                                                \
        spread_hint<TM * TN, TM + TN, 0, LA / 2 + LB / 2>();                                   \
        OSC_D2_BRANCH((T_) + KS, buf ^ 1, LA / 2, LA, LB / 2, LB)                               \
        OSC_F2(buf, 4 + 2 * q, fa0, fb0)                                                       \
        OSC_MFMA_BF16(fa1, fb1)                                                                \
        spread_hint<TM * TN, TM + TN, 0, LA - LA / 2 + LB - LB / 2>();                         \
        OSC_F2(buf, 4 + 2 * q + 1, fa1, fb1)                                                   \
        OSC_MFMA_BF16(fa0, fb0)                                                                \
        spread_hint<TM * TN, TM + TN, 0, 0>();                                                 \
        OSC_MFMA_BF16(fa1, fb1)                                                                \
        __builtin_amdgcn_sched_barrier(0);                                                     \
        wait_vmcnt<0>();                                                                       \
        __syncthreads();                                                                       \
        __builtin_amdgcn_sched_barrier(0);                                                     \
        buf ^= 1;                                                                              \
    }
    // FP8 stage: 128 channels = two MFMAs per tile pair (pieces 2q,2q+1 and 4+2q,4+2q+1)
#define OSC_D2_STAGE_FP8(T_)                                                                   \
    {                                                                                          \
        u32x4 ga0[TM], gb0[TN], ga1[TM], gb1[TN];                                              \
        OSC_F2(buf, 2 * q, fa0, fb0)                                                           \
        OSC_F2(buf, 2 * q + 1, ga0, gb0)                                                       \
        if ((T_) + KS < nT) OSC_D2_MAIN((T_) + KS, buf ^ 1, 0, LA, 0, LB / 2)                    \
        OSC_F2(buf, 4 + 2 * q, fa1, fb1)                                                       \
        OSC_F2(buf, 4 + 2 * q + 1, ga1, gb1)                                                   \
        OSC_MFMA_FP8(0, TM * TN, fa0, ga0, fb0, gb0)                                           \
        spread_hint<TM * TN, 2 * (TM + TN), 0, LA + LB / 2>();                                 \
        if ((T_) + KS < nT) OSC_D2_MAIN((T_) + KS, buf ^ 1, 0, 0, LB / 2, LB)                    \
        OSC_MFMA_FP8(0, TM * TN, fa1, ga1, fb1, gb1)                                           \
        spread_hint<TM * TN, 0, 0, LB - LB / 2>();                                             \
        __builtin_amdgcn_sched_barrier(0);                                                     \
        wait_vmcnt<0>();                                                                       \
        __syncthreads();                                                                       \
        __builtin_amdgcn_sched_barrier(0);                                                     \
        buf ^= 1;                                                                              \
    }

    // FP8 stage with one pair of fragment sets, for two wavefronts per SIMD (the other wavefront
    // covers the wait between the two halves; 2 % faster there than the four-set stage)
#define OSC_D2_STAGE_FP8_LEAN(T_)                                                              \
    {                                                                                          \
        OSC_F2(buf, 2 * q, fa0, fb0)                                                           \
        OSC_F2(buf, 2 * q + 1, fa1, fb1)                                                       \
        if ((T_) + 1 < nT) OSC_D2_MAIN((T_) + 1, buf ^ 1, 0, LA, 0, LB)                        \
        OSC_MFMA_FP8(0, TM * TN, fa0, fa1, fb0, fb1)                                           \
        __builtin_amdgcn_sched_barrier(0);                                                     \
        OSC_F2(buf, 4 + 2 * q, fa0, fb0)                                                       \
        OSC_F2(buf, 4 + 2 * q + 1, fa1, fb1)                                                   \
        OSC_MFMA_FP8(0, TM * TN, fa0, fa1, fb0, fb1)                                           \
        __builtin_amdgcn_sched_barrier(0);                                                     \
        wait_vmcnt<0>();                                                                       \
        __syncthreads();                                                                       \
        __builtin_amdgcn_sched_barrier(0);                                                     \
        buf ^= 1;                                                                              \
    }

    // MXFP8 stage.  With 8-bit operands the 32x32x64 instruction takes, from lane half q, elements
    // 16q .. 16q+15 of each of its two 32-element scale blocks (registers 0-3: block 0, registers
    // 4-7: block 1), and the scale of block b from the lanes of half b.  So the MFMA that handles
    // groups 2h and 2h+1 of the line gets, in lane half q, piece 4h+q (first registers) and piece
    // 4h+2+q (last registers), and the scale word shifted right by 8q bits has the scale this half
    // must supply (group 2h+q) in byte 2h.
#define OSC_MFMA_MX8(I_, FA_, GA_, FB_, GB_, SA_, SB_)                                                \
    {                                                                                                 \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) {                                              \
            const v8i av__ = {(int)FA_[i].x, (int)FA_[i].y, (int)FA_[i].z, (int)FA_[i].w,             \
                              (int)GA_[i].x, (int)GA_[i].y, (int)GA_[i].z, (int)GA_[i].w};            \
            _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                          \
                const v8i bv__ = {(int)FB_[j].x, (int)FB_[j].y, (int)FB_[j].z, (int)FB_[j].w,         \
                                  (int)GB_[j].x, (int)GB_[j].y, (int)GB_[j].z, (int)GB_[j].w};        \
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av__, bv__, acc[i][j], 0, 0, I_, \
                                                                            SA_[i], I_, SB_[j]);      \
            }                                                                                         \
        }                                                                                             \
    }
#define OSC_D2_STAGE_MX8(T_)                                                                   \
    {                                                                                          \
        u32x4 ga0[TM], gb0[TN], ga1[TM], gb1[TN];                                              \
        int sa[TM], sb[TN];                                                                    \
        OSC_F2(buf, q, fa0, fb0)                                                               \
        OSC_F2(buf, 2 + q, ga0, gb0)                                                           \
        OSC_D2_READ_SCALES(buf, 0, sa, sb)                                                     \
        if ((T_) + 1 < nT) {                                                                   \
            OSC_D2_SCALES((T_) + 1, buf ^ 1)                                                   \
            OSC_D2_MAIN((T_) + 1, buf ^ 1, 0, LA, 0, LB / 2)                                   \
        }                                                                                      \
        OSC_F2(buf, 4 + q, fa1, fb1)                                                           \
        OSC_F2(buf, 6 + q, ga1, gb1)                                                           \
        OSC_MFMA_MX8(0, fa0, ga0, fb0, gb0, sa, sb)                                            \
        spread_hint<TM * TN, 2 * (TM + TN), 0, NSB + LA + LB / 2>();                           \
        if ((T_) + 1 < nT) OSC_D2_MAIN((T_) + 1, buf ^ 1, 0, 0, LB / 2, LB)                    \
        OSC_MFMA_MX8(2, fa1, ga1, fb1, gb1, sa, sb)                                            \
        spread_hint<TM * TN, 0, 0, LB - LB / 2>();                                             \
        __builtin_amdgcn_sched_barrier(0);                                                     \
        wait_vmcnt<0>();                                                                       \
        __syncthreads();                                                                       \
        __builtin_amdgcn_sched_barrier(0);                                                     \
        buf ^= 1;                                                                              \
    }
    // the same stage with one pair of fragment sets, for two wavefronts per SIMD (the other
    // wavefront covers the wait between the two halves, and four sets do not fit 256 registers)
#define OSC_D2_STAGE_MX8_LEAN(T_)                                                              \
    {                                                                                          \
        int sa[TM], sb[TN];                                                                    \
        OSC_F2(buf, q, fa0, fb0)                                                               \
        OSC_F2(buf, 2 + q, fa1, fb1)                                                           \
        OSC_D2_READ_SCALES(buf, 0, sa, sb)                                                     \
        if ((T_) + 1 < nT) {                                                                   \
            OSC_D2_SCALES((T_) + 1, buf ^ 1)                                                   \
            OSC_D2_MAIN((T_) + 1, buf ^ 1, 0, LA, 0, LB)                                       \
        }                                                                                      \
        OSC_MFMA_MX8(0, fa0, fa1, fb0, fb1, sa, sb)                                            \
        __builtin_amdgcn_sched_barrier(0);                                                     \
        OSC_F2(buf, 4 + q, fa0, fb0)                                                           \
        OSC_F2(buf, 6 + q, fa1, fb1)                                                           \
        OSC_MFMA_MX8(2, fa0, fa1, fb0, fb1, sa, sb)                                            \
        __builtin_amdgcn_sched_barrier(0);                                                     \
        wait_vmcnt<0>();                                                                       \
        __syncthreads();                                                                       \
        __builtin_amdgcn_sched_barrier(0);                                                     \
        buf ^= 1;                                                                              \
    }

    if (MODE == MODE_MX8 && WN == 4) {
#pragma unroll 1
        for (int T = 0; T < nT; ++T) OSC_D2_STAGE_MX8_LEAN(T)
    } else if (MODE == MODE_MX8) {
#pragma unroll 1
        for (int T = 0; T < nT; ++T) OSC_D2_STAGE_MX8(T)
    } else if (MODE == MODE_FP8 && WN == 4) {
#pragma unroll 1
        for (int T = 0; T < nT; ++T) OSC_D2_STAGE_FP8_LEAN(T)
    } else if (MODE == MODE_FP8) {
#pragma unroll 1
        for (int T = grp; T < nT; T += KS) OSC_D2_STAGE_FP8(T)
        if constexpr (KS > 1) {
            if (grp == 1 && (nT & 1)) __syncthreads();
        }
    } else {
        int T = grp;
#pragma unroll 1
        for (; T + KS < nTA; T += KS) OSC_D2_STAGE_FP4(T, OSC_D2_MAIN)
        if (T < nTA) {
            OSC_D2_STAGE_FP4(T, OSC_D2_ANY)
            T += KS;
        }
#pragma unroll 1
        for (; T < nT; T += KS) OSC_D2_STAGE_BF16(T)
        if constexpr (KS > 1) {
            // every stage ends in a workgroup barrier: the group with one stage fewer keeps the count even
            if (grp == 1 && (nT & 1)) __syncthreads();
        }
    }
    if constexpr (KS > 1) {
        // partial sums of group 1 -> LDS -> group 0 (every group has waited for its own last DMA request)
        constexpr int GT_ = 128 * WN;
        __syncthreads();
        float* const red = reinterpret_cast<float*>(lds_all);
        if (grp == 1) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int k2 = 0; k2 < 16; ++k2) red[((i * TN + j) * 16 + k2) * GT_ + t] = acc[i][j][k2];
        }
        __syncthreads();
        if (grp != 0) return;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int k2 = 0; k2 < 16; ++k2) acc[i][j][k2] += red[((i * TN + j) * 16 + k2) * GT_ + t];
    }
    store_result<MODE, TM, TN, WN>(a, tp, acc);
}

// ------------------------------------------------------------------------------------------
// The DMA kernel above for grouped 8-bit problems (FP8, MXFP8) with persistent workgroups.  An
// expert's tile is a few stages long (K = 768: six), its weights are used by no other tile and come
// from HBM, so a workgroup that handles one tile spends a third of its time before the first and
// after the last MFMA.  Here a workgroup walks tiles v, v + grid, ... : the experts' row ranges and running tile
// counts are put into LDS once, so finding a tile is a short binary search there; when the K
// loop of a tile ends, both LDS stages are free and the first two stages of the next tile are
// requested, then the results are stored, and the next K loop starts on operands that have
// landed.  Measured on the MoE shape (T = 32768, 128 experts, 2048 x 768): FP8 109.6 -> 104 us,
// MXFP8 102.5 -> 97.3 us; the dual path with its row map gained nothing from the same scheme
// (131 us either way) and keeps one tile per workgroup.
// ------------------------------------------------------------------------------------------
template <int MODE, int TM, int TN, int WN>
__global__ void __launch_bounds__(128 * WN) gemm_dma2g_kernel(KArgs a, int ntiles) {
    static_assert(MODE != MODE_DUAL, "8-bit modes only (no row map, no bf16 branch)");
    constexpr int NWV = 2 * WN;
    constexpr int RPP = NWV * 8;
    constexpr int BM = 64 * TM, BN = 32 * TN * WN;
    constexpr int STG = (BM + BN) * 128;
    constexpr int LA = BM / RPP, LB = BN / RPP;
    constexpr int NBLK = (BM + BN) / 32;
    constexpr int NSB = (NBLK + NWV - 1) / NWV;
    static_assert(BM % RPP == 0 && BN % RPP == 0, "tile does not split over the wavefronts");
    constexpr int SCL = NBLK * 256;
    constexpr bool use16 = false;  // (the 16-byte scale requests of the DMA kernel are for single problems)
    constexpr int NREQ = 0, wave_u = 0;
    const uint8_t* const sc16_src = nullptr;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    uint8_t* const scl = lds + 2 * STG;
    // per expert, behind the two stages and their scale words: first tile number, first row, rows
    int* const cum_l = reinterpret_cast<int*>(scl + 2 * SCL);  // [E + 1]
    int* const eb_l = cum_l + a.E + 1;                          // [E]
    int* const en_l = eb_l + a.E;                               // [E]

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave / WN, wn = wave % WN, q = lane >> 5, r = lane & 31;
    const int Kg4 = ((a.K >> 5) + 3) >> 2;
    const int rowbytes = (MODE == MODE_DUAL) ? (a.K >> 1) : a.K;
    const int nTA = rowbytes >> 7;
    const int nTB = (MODE == MODE_DUAL) ? ((a.K_o * 2 + 127) >> 7) : 0;
    const int nT = nTA + nTB;
    const int c8 = (t & 7) ^ swz8(t >> 3);

    // rows of every expert that this launch covers (see KArgs::grp_mode) and the running tile count
    for (int e = t; e < a.E; e += 128 * WN) {
        int b = a.off[e];
        int n = a.off[e + 1] - b;
        if (a.grp_mode == 1) {
            n = min(n, (n + BM / 2) / BM * BM);
        } else if (a.grp_mode == 2) {
            const int skip = min(n, (n + a.grp_bm / 2) / a.grp_bm * a.grp_bm);
            b += skip;
            n -= skip;
        }
        eb_l[e] = b;
        en_l[e] = n;
    }
    __syncthreads();
    if (wave == 0) {
        int before = 0;
        for (int e0 = 0; e0 < a.E; e0 += 64) {
            const int e = e0 + lane;
            const int te = e < a.E ? (en_l[e] + BM - 1) / BM : 0;
            int ps = te;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int u = __shfl_up(ps, d);
                if (lane >= d) ps += u;
            }
            if (e < a.E) cum_l[e] = before + ps - te;
            before += __shfl(ps, 63);
        }
        if (lane == 0) cum_l[a.E] = before;
    }
    __syncthreads();
    // tile number v of the numbering of locate_tile() -> position: a binary search over the running
    // tile counts (a few dependent LDS reads of uniform addresses, nothing kept in registers)
    auto find_tile = [&](int v) -> TilePos {
        TilePos p;
        p.valid = false;
        p.m0 = p.n0 = p.row_begin = p.row_end = 0;
        p.wp = a.Wpack;
        if (v >= ntiles) return p;
        const int x = v & 7, sidx = v >> 3;
        const int j = (sidx / a.tiles_n) * 8 + x;  // m-tile, counted over all experts
        if (j >= cum_l[a.E]) return p;
        // the last expert whose first tile number is <= j: experts without tiles share that number with
        // their successor, so the last one is the one that owns tile j
        int lo = 0, hi = a.E - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (cum_l[mid] <= j) lo = mid; else hi = mid - 1;
        }
        const int e = __builtin_amdgcn_readfirstlane(lo);
        p.row_begin = __builtin_amdgcn_readfirstlane(eb_l[e]);
        p.row_end = p.row_begin + __builtin_amdgcn_readfirstlane(en_l[e]);
        p.m0 = p.row_begin + (j - __builtin_amdgcn_readfirstlane(cum_l[e])) * BM;
        p.n0 = (sidx % a.tiles_n) * BN;
        p.wp = a.Wpack + (size_t)e * a.pack_stride;
        p.valid = true;
        return p;
    };

    int v = blockIdx.x;
    TilePos tp = find_tile(v);
    if (!tp.valid) return;  // m-tiles are numbered in order: nothing valid follows an invalid one

    uint32_t oa[LA], ob[LB], sco[NSB];
    const uint8_t *wq, *wl, *wsb;
    int m0, n0, row_end;
    int buf = 0;
    // the first two stages of tile TP_ into buffers buf and buf ^ 1
#define D2G_START(TP_)                                                                                \
    {                                                                                                 \
        m0 = (TP_).m0;                                                                                \
        n0 = (TP_).n0;                                                                                \
        row_end = (TP_).row_end;                                                                      \
        wq = (TP_).wp + a.off_q;                                                                      \
        wl = (TP_).wp + a.off_l;                                                                      \
        wsb = (TP_).wp + a.off_s;                                                                     \
        _Pragma("unroll") for (int i = 0; i < LA; ++i) oa[i] = (uint32_t)min(m0 + (t >> 3) + RPP * i, row_end - 1); \
        _Pragma("unroll") for (int i = 0; i < LB; ++i) ob[i] = (uint32_t)min(n0 + (t >> 3) + RPP * i, a.N - 1);     \
        if (MODE == MODE_MX8) {                                                                       \
            _Pragma("unroll") for (int k = 0; k < NSB; ++k) {                                         \
                const int b = min(wave * NSB + k, NBLK - 1);                                          \
                const int g = b < BM / 32 ? min(m0 + 32 * b + r, row_end - 1)                         \
                                          : min(n0 + 32 * (b - BM / 32) + r, a.N - 1);                \
                sco[k] = (uint32_t)(g >> 5) * (uint32_t)Kg4 * 128u + (g & 31) * 4;                    \
            }                                                                                         \
            OSC_D2_SCALES(0, buf)                                                                     \
        }                                                                                             \
        OSC_D2_ANY(0, buf, 0, LA, 0, LB)                                                              \
        if (MODE == MODE_MX8 && 1 < nTA) OSC_D2_SCALES(1, buf ^ 1)                                    \
        OSC_D2_ANY(1, buf ^ 1, 0, LA, 0, LB)                                                          \
    }

    D2G_START(tp)
    wait_vmcnt<0>();
    __syncthreads();

    v16f acc[TM][TN];
    u32x4 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
    const int ra0 = wm * (TM * 32) + r, rb0 = BM + wn * (TN * 32) + r;

#pragma unroll 1
    for (;;) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int k = 0; k < 16; ++k) acc[i][j][k] = 0.0f;
        const TilePos nxt = find_tile(v + (int)gridDim.x);
        // stage 0: its operands and those of stage 1 are in LDS; stage number nT switches every request off
        if (MODE == MODE_MX8) {
            OSC_D2_STAGE_MX8_LEAN(nT)
#pragma unroll 1
            for (int T = 1; T < nT; ++T) OSC_D2_STAGE_MX8_LEAN(T)
        } else {
            OSC_D2_STAGE_FP8_LEAN(nT)
#pragma unroll 1
            for (int T = 1; T < nT; ++T) OSC_D2_STAGE_FP8_LEAN(T)
        }
        const TilePos ctp = tp;
        if (nxt.valid) D2G_START(nxt)
        __builtin_amdgcn_sched_barrier(0);
        store_result<MODE, TM, TN, WN>(a, ctp, acc);
        if (!nxt.valid) break;
        tp = nxt;
        v += (int)gridDim.x;
        wait_vmcnt<0>();
        __syncthreads();
    }
#undef D2G_START
}



// ------------------------------------------------------------------------------------------
// Persistent pipelined kernel for one problem made of whole tiles (M % BM == 0,
// N % BN == 0, no row map).  Same operands and LDS image as the DMA kernel above, but
//  (1) the order of every instruction of a stage is pinned: a stage is a row of slots, one MFMA per
//      slot, and every LDS read and DMA load is tied to a slot and fenced there (sched_barrier).
//      Left alone, the compiler hoists all memory operations of a stage above its MFMAs (or sinks
//      the MFMAs below the last branch of the loop body) and the matrix core idles while they issue;
//  (2) a stage releases its LDS buffer early.  Stage T computes from buffer T % 2:
//        group 0 (piece 2q,     set X, scales S0): reads piece 4+2q+1 into set Z and scales S1
//        group 1 (piece 2q+1,   set Y):            reads piece 4+2q into set X
//        slot A_AT: every wave has read the whole stage -> barrier -> the loads of stage T+2 start
//                   flowing into the buffer, spread evenly over the rest of the stage
//        group 2 (piece 4+2q,   set X, scales S1)
//        slot B_AT: loads of stage T+1 have landed (vmcnt leaves the younger ones in flight) -> barrier
//        group 3 (piece 4+2q+1, set Z): reads pieces 2q, 2q+1 of stage T+1 into X, Y and scales S0
//      so a load has about one to 1.3 stages to land and the first MFMA of a stage never waits;
//  (3) one workgroup per compute unit walks a list of tiles, and the stream of loads runs ahead of
//      the stream of MFMAs across tile borders: the load cursor (tile, stage) is two stages ahead of
//      the compute cursor, so while the last two stages of a tile are computed the first two of the
//      next tile arrive, and the result stores of a tile drain under the next tile's main loop.
// Every stage moves the same number of loads (a bf16 branch stage carries idle scale loads; past
// the last tile the last stage is fetched again into a buffer nobody reads), so the wait before the
// second barrier of a stage is a compile-time count and the stage has no branch.  Addresses are a
// uniform base per (tile, stage, 32-row block) plus one per-thread 32-bit offset.  XCD x
// (= workgroup % 8) owns the x-th eighth of the tile list; its workgroups take neighbouring tiles
// at any time (8 m-tiles x 4 n-tiles with 32 workgroups).
// The description above is the dual path's stage (256 FP4 or 64 bf16 channels, four MFMA groups).  The 8-bit
// modes (per-token FP8, MXFP8) keep (1)-(3), the load stream and the barriers, with a stage of 128 channels
// = two MFMA steps and a register plan of their own, described at PIPE8_STAGE.
// ------------------------------------------------------------------------------------------
#define NBLK_OF(BM_, BN_) (((BM_) + (BN_)) / 32)
template <int MODE, int TM, int TN, int WN>
__global__ void __launch_bounds__(128 * WN) gemm_pipe2_kernel(KArgs a, int ntiles) {
    static_assert(MODE == MODE_DUAL || ((MODE == MODE_FP8 || MODE == MODE_MX8) && TM == 4 && TN == 4),
                  "dual path, or 8-bit operands on 4 x 4 blocks per wavefront");
    constexpr bool DUAL = MODE == MODE_DUAL, MX = MODE == MODE_MX8;
    constexpr bool BLKSC = DUAL || MX;  // block scales travel with the stages
    constexpr int NWV = 2 * WN, RPP = NWV * 8;  // wavefronts (2 x WN); stage rows per DMA pass
    constexpr int BM = 64 * TM, BN = 32 * TN * WN;
    constexpr int STG = (BM + BN) * 128;
    constexpr int LA = BM / RPP, LB = BN / RPP;
    // per stage and wavefront: dual path and MXFP8, NSB 32-row blocks of scale words (MXFP8: one word per row
    // and stage, fetched by both lane halves); FP8, NSB 64-float blocks of the tile's row and column scales
    // for the epilogue (fetched with every stage so that all stages move the same number of loads; two copies
    // in LDS, by parity of the tile's position in this workgroup's list)
    // (dual path with four scale blocks per wavefront that all belong to one operand: one 16-byte request per
    // lane fetches the four 256-byte blocks at once; a request costs the memory pipeline the same whatever its width)
    constexpr bool SC16 = DUAL && NBLK_OF(BM, BN) % (4 * NWV) == 0 && (BM / 32) % 4 == 0;
    constexpr int NBLK = (BM + BN) / 32, NSB = SC16 ? NBLK / NWV / 4 : BLKSC ? NBLK / NWV : (BM + BN) / 64 / NWV,
                  SCL = BLKSC ? NBLK * 256 : (BM + BN) * 4;
    static_assert(BLKSC || (BM + BN) % (64 * NWV) == 0, "tile scales do not split over the wavefronts");
    static_assert(BM % RPP == 0 && BN % RPP == 0 && NBLK % NWV == 0, "tile does not split over the wavefronts");
    constexpr int NT = TM * TN, NSLOT = 4 * NT, NRD = 2 * (TM + TN), NLD = NSB + LA + LB;
    // Three register sets: X holds piece 2q, then 4+2q, then piece 2q of the next stage; Y holds piece
    // 2q+1; Z holds piece 4+2q+1.  Reads: Z in group 0, X again in group 1 (after group 0 consumed
    // it), and X, Y of the next stage in group 3.
    constexpr int HR = TM + TN;                       // 16-byte reads per piece
    constexpr int RPS = (HR + NT - 1) / NT;           // reads per slot
    // group 1 reads two fragments per slot and the free point follows two slots behind the last of them: the
    // earlier the buffer is released, the longer the next loads have to land (one read per slot and four slots
    // of slack, i.e. slot 28 instead of 22 of 64: 2.8 % slower at 8192 x 4096 x 4096)
    constexpr int RPS1 = 2;
    constexpr int A_AT = NT + (HR + RPS1 - 1) / RPS1 + 2;  // free point: the reads of group 1 have landed
    constexpr int B_AT = 3 * NT - 1;           // (slots 43 .. 55 of 64: within 0.5 %, 43 is 2 % slower)
    // loads: spread evenly over the LW slots behind the free point; load l goes to slot A_AT + 1 + l * LW / NLD
    constexpr int LW = NSLOT - A_AT - 1;
    constexpr int LPS = NLD / LW + 2;  // upper bound of loads in one slot
    static_assert(LW >= 2, "no room for the loads");
    constexpr int RPS2 = (2 * HR + NSLOT - B_AT - 2) / (NSLOT - B_AT - 1);
    constexpr int N_BEFORE_B = []() {
        int n = 0;
        for (int l = 0; l < NLD; ++l)
            if (A_AT + 1 + l * LW / NLD <= B_AT) ++n;
        return n;
    }();
    // FP8 stage (128 channels): 2 NT slots of one MFMA each, see PIPE8_STAGE below
    constexpr int F8_SLOT = 2 * NT;
    constexpr int F8_A_AT = NT;                // the last read of the stage (slot NT - 3) has landed
    constexpr int F8_B_AT = NT + NT / 2 - 1;
    constexpr int F8_LW = F8_SLOT - F8_A_AT - 1 > 0 ? F8_SLOT - F8_A_AT - 1 : 1;  // (only the 4 x 4 form is built for FP8)
    constexpr int F8_LPS = NLD / F8_LW + 2;
    constexpr int F8_N_BEFORE_B = []() {
        int n = 0;
        for (int l = 0; l < NLD; ++l)
            if (F8_A_AT + 1 + l * F8_LW / NLD <= F8_B_AT) ++n;
        return n;
    }();
    static_assert(DUAL || (F8_B_AT > F8_A_AT && F8_SLOT - F8_B_AT - 1 >= 2 * TN), "FP8 stage: no room for the next stage's reads");
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    uint8_t* const scl = lds + 2 * STG;

    const int t = threadIdx.x, lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave / WN, wn = wave % WN, q = lane >> 5, r = lane & 31;
    const int Kg4 = ((a.K >> 5) + 3) >> 2;
    const int rowbytes = DUAL ? a.K >> 1 : a.K;
    const int nTA = rowbytes >> 7;
    const int nTB = DUAL ? (a.K_o * 2 + 127) >> 7 : 0;
    const int nT = nTA + nTB;  // >= 3 (checked on the host)
    const int ra0 = wm * (TM * 32) + r, rb0 = BM + wn * (TN * 32) + r;
    const int tiles_m = a.M / BM;

    // this workgroup's tiles: first, first + step, ... below last
    const int per = (ntiles + 7) >> 3;
    const int xcd = blockIdx.x & 7;
    const int step = (gridDim.x + 7 - xcd) >> 3;  // workgroups on this XCD
    const int last = min(ntiles, (xcd + 1) * per);
    int ctile = xcd * per + (blockIdx.x >> 3);    // compute cursor
    if (ctile >= last) return;

    // per-thread parts of the addresses: row (t >> 3) of a block of RPP rows, 16-byte piece c8
    const uint32_t c8 = (uint32_t)((t & 7) ^ swz8(t >> 3)) * 16u;
    const uint32_t vo_main = (uint32_t)(t >> 3) * (uint32_t)rowbytes + c8;       // FP4 phase, both operands
    const uint32_t vo_ba = (uint32_t)(t >> 3) * (uint32_t)a.bpitch + c8;         // branch phase, B rows
    const uint32_t vo_bw = (uint32_t)(t >> 3) * (uint32_t)a.wlpitch + c8;        // branch phase, W_L rows
    const uint32_t vo_s = (uint32_t)(r * 4 + (DUAL ? q * 128 : 0));               // scale word of row r (dual path: of half step q)
    // 16-byte form: lane l fetches piece l % 16 of the 256 bytes (two half steps x 32 rows x 4) of block l / 16
    const uint32_t vo_s16 = (uint32_t)(lane >> 4) * ((uint32_t)Kg4 * 128u) + (uint32_t)(lane & 15) * 16u;
    const uint8_t* const wq = a.Wpack + a.off_q;
    const uint8_t* const wl = a.Wpack + a.off_l;
    const uint8_t* const wsb = a.Wpack + a.off_s;
    const float* const wcs = reinterpret_cast<const float*>(wsb);  // FP8: column scales

    // ---- load cursor: tile (m0, n0), stage lT; uniform bases of the stage's first 32-row blocks ----
    int lT = 0, lm0, ln0;
    int lpar = 0;              // FP8: which copy of the tile scales the load cursor's tile writes
    int nm0 = 0, nn0 = 0;      // position of this workgroup's tile after the one under the load cursor
    bool hasnext;
    const uint8_t *pa, *pb, *psa = nullptr, *psb = nullptr;  // A rows, B rows, A scale block, B scale block at this stage
    uint32_t sa32, sb32;                 // bytes between consecutive blocks of RPP rows
    uint32_t voa, vob;                   // per-thread offsets in use
#define PIPE2_TILE_POS(TILE_, M0_, N0_)                                                              \
    {                                                                                                \
        const int band__ = (TILE_) / (8 * a.tiles_n), within__ = (TILE_)-band__ * 8 * a.tiles_n;     \
        const int rows__ = min(8, tiles_m - band__ * 8);                                             \
        M0_ = (band__ * 8 + within__ % rows__) * BM;                                                 \
        N0_ = (within__ / rows__) * BN;                                                              \
    }
#define PIPE2_STAGE_SETUP                                                                            \
    {                                                                                                \
        /* selects only: a branch here would split the stage into basic blocks, and the compiler     \
           then sinks every MFMA of the stage below the last of them */                              \
        const bool fp4__ = lT < nTA;                                                                 \
        const uint32_t ko__ = (uint32_t)(fp4__ ? lT : lT - nTA) * 128u;                              \
        const uint32_t pitcha__ = fp4__ ? (uint32_t)rowbytes : (uint32_t)a.bpitch;                   \
        const uint32_t pitchb__ = fp4__ ? (uint32_t)rowbytes : (uint32_t)a.wlpitch;                  \
        sa32 = (uint32_t)RPP * pitcha__;                                                                       \
        sb32 = (uint32_t)RPP * pitchb__;                                                                       \
        pa = (fp4__ ? a.Xq : a.B) + ((size_t)lm0 * pitcha__ + ko__);                                 \
        pb = (fp4__ ? wq : wl) + ((size_t)ln0 * pitchb__ + ko__);                                    \
        voa = fp4__ ? vo_main : vo_ba;                                                               \
        vob = fp4__ ? vo_main : vo_bw;                                                               \
        if (BLKSC) {                                                                                 \
            const uint32_t so__ = (uint32_t)(DUAL ? min(2 * lT, Kg4 - 2) : min(lT, Kg4 - 1)) * 128u; \
            psa = a.Xs + ((size_t)(lm0 >> 5) * (uint32_t)Kg4 * 128u + so__);                         \
            psb = wsb + ((size_t)(ln0 >> 5) * (uint32_t)Kg4 * 128u + so__);                          \
        }                                                                                            \
    }
    // advance the load cursor by one stage; at the end of a tile it moves to (nm0, nn0), the next
    // tile of this workgroup, or, if there is none, stays on the last stage
#define PIPE2_ADVANCE                                                                                \
    {                                                                                                \
        const bool wrap__ = lT + 1 == nT;                                                            \
        const bool jump__ = wrap__ && hasnext;                                                       \
        lT = wrap__ ? (hasnext ? 0 : lT) : lT + 1;                                                   \
        lpar ^= jump__ ? 1 : 0;                                                                      \
        lm0 = jump__ ? nm0 : lm0;                                                                    \
        ln0 = jump__ ? nn0 : ln0;                                                                    \
        PIPE2_STAGE_SETUP                                                                            \
    }
    // load number L_ (0..NLD-1) of the stage under the load cursor into buffer BUF_
#define PIPE2_LOAD(L_, BUF_)                                                                         \
    {                                                                                                \
        if ((L_) < NSB && SC16) {                                                                    \
            const int b__ = (wave * NSB + (L_)) * 4;                                                 \
            const uint8_t* src__ = (b__ < BM / 32 ? psa + (size_t)b__ * ((uint32_t)Kg4 * 128u)       \
                                                  : psb + (size_t)(b__ - BM / 32) * ((uint32_t)Kg4 * 128u)) + vo_s16; \
            load_to_lds16(src__, scl + (BUF_)*SCL + b__ * 256);                                      \
        } else if ((L_) < NSB && BLKSC) {                                                            \
            const int b__ = wave * NSB + (L_);                                                       \
            const uint8_t* src__ = (b__ < BM / 32 ? psa + (size_t)b__ * ((uint32_t)Kg4 * 128u)       \
                                                  : psb + (size_t)(b__ - BM / 32) * ((uint32_t)Kg4 * 128u)) + vo_s; \
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src__,   \
                                             (__attribute__((address_space(3))) void*)(scl + (BUF_)*SCL + b__ * 256), \
                                             4, 0, 0);                                               \
        } else if ((L_) < NSB) {                                                                     \
            const int b__ = wave * NSB + (L_);                                                       \
            const float* src__ = (b__ < BM / 64 ? a.xs + (lm0 + b__ * 64) : wcs + (ln0 + (b__ - BM / 64) * 64)) + lane; \
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src__,   \
                                             (__attribute__((address_space(3))) void*)(scl + lpar * SCL + b__ * 256), \
                                             4, 0, 0);                                               \
        } else if ((L_) < NSB + LA) {                                                                \
            const int i__ = (L_)-NSB;                                                                \
            load_to_lds16(pa + (size_t)i__ * sa32 + voa, lds + (BUF_)*STG + wave * 1024 + i__ * (RPP * 128)); \
        } else {                                                                                     \
            const int i__ = (L_)-NSB - LA;                                                           \
            load_to_lds16(pb + (size_t)i__ * sb32 + vob,                                             \
                          lds + (BUF_)*STG + wave * 1024 + BM * 128 + i__ * (RPP * 128));                   \
        }                                                                                            \
    }

    // scale word number R_ (0..TM+TN-1) of half step H_
#define PIPE_READ_SCALE(R_, BUF_, H_, SA_, SB_)                                                         \
    {                                                                                                   \
        /* a 16-bit read at byte 2q of the word: byte I of the register = scale of piece 2q+I, no shift */ \
        const uint8_t* sc__ = scl + (BUF_)*SCL + (H_)*128 + r * 4 + 2 * q;                              \
        if ((R_) < TM)                                                                                  \
            SA_[(R_) < TM ? (R_) : 0] = *reinterpret_cast<const uint16_t*>(sc__ + (wm * TM + (R_)) * 256); \
        else                                                                                            \
            SB_[(R_) >= TM ? (R_)-TM : 0] =                                                             \
                *reinterpret_cast<const uint16_t*>(sc__ + (BM / 32 + wn * TN + (R_)-TM) * 256);         \
    }
#define PIPE_MFMA_FP4(N_, FA_, FB_, SA_, SB_, SEL_)                                                     \
    {                                                                                                   \
        const int i__ = (N_) / TN, j__ = (N_) % TN;                                                     \
        const v8i av__ = {(int)FA_[i__].x, (int)FA_[i__].y, (int)FA_[i__].z, (int)FA_[i__].w, 0, 0, 0, 0}; \
        const v8i bv__ = {(int)FB_[j__].x, (int)FB_[j__].y, (int)FB_[j__].z, (int)FB_[j__].w, 0, 0, 0, 0}; \
        acc[i__][j__] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av__, bv__, acc[i__][j__], 4, 4, SEL_, \
                                                                        SA_[i__], SEL_, SB_[j__]);      \
    }
#define PIPE_MFMA_BF16(N_, FA_, FB_)                                                                    \
    {                                                                                                   \
        const int i__ = (N_) / TN, j__ = (N_) % TN;                                                     \
        acc[i__][j__] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, FA_[i__]),     \
                                                                __builtin_bit_cast(v8bf, FB_[j__]),     \
                                                                acc[i__][j__], 0, 0, 0);                \
    }
    // read number R_ (0..TM+TN-1) of piece P_ from buffer BUF_ into set SA_/SB_
#define PIPE_READ1(R_, BUF_, P_, SA_, SB_)                                                             \
    {                                                                                                  \
        const uint8_t* st__ = lds + (BUF_)*STG;                                                        \
        const u32x4 v__ = *reinterpret_cast<const u32x4*>(                                             \
            st__ + st128_off(((R_) < TM ? ra0 + 32 * (R_) : rb0 + 32 * ((R_)-TM)), (P_)));             \
        if ((R_) < TM) SA_[(R_) < TM ? (R_) : 0] = v__;                                                \
        else SB_[(R_) >= TM ? (R_)-TM : 0] = v__;                                                      \
    }
    u32x4 Xa[TM], Xb[TN], Ya[TM], Yb[TN], Za[TM], Zb[TN];
    int s0a[TM], s0b[TN], s1a[TM], s1b[TN];
    // 8-bit modes: a lane's fragment of a 64-channel MFMA step is two pieces (32 bytes).  One set for the A
    // fragments (block i is read again as soon as its last MFMA of the step has been issued; the last
    // block has a second set, A8x, for its step-1 fragment), two for the B fragments (every block of a
    // step is in use until the step ends).
    u32x4 A8[TM][2], Bp[TN][2], Bq[TN][2], A8x[2];
    // MXFP8: this lane's scale bytes of the stage (byte 2 KS_ = scale of MFMA step KS_) and the words of the next
    int m8a[TM], m8b[TN];
    uint32_t m8an[TM], m8bn[TN];
    v16f acc[TM][TN];
    // half H_ (0, 1) of the fragment of 32-row block I_ / J_ for MFMA step KS_ (0, 1) of buffer BUF_
    // (per-token FP8: lane half q supplies bytes 32q .. 32q+31 of the step, pieces 2q and 2q+1; MXFP8: elements
    // 16q .. 16q+15 of each of the step's two scale blocks, pieces q and 2+q, see the DMA kernel)
#define PIPE8_PIECE(KS_, H_) (MX ? 4 * (KS_) + q + 2 * (H_) : 4 * (KS_) + 2 * q + (H_))
#define PIPE8_RA(I_, BUF_, KS_, H_)                                                                     \
    A8[I_][H_] = *reinterpret_cast<const u32x4*>(lds + (BUF_)*STG + st128_off(ra0 + 32 * (I_), PIPE8_PIECE(KS_, H_)));
#define PIPE8_RB(SET_, J_, BUF_, KS_, H_)                                                               \
    SET_[J_][H_] = *reinterpret_cast<const u32x4*>(lds + (BUF_)*STG + st128_off(rb0 + 32 * (J_), PIPE8_PIECE(KS_, H_)));
    // scale word number R_ (0..TM+TN-1) of the stage in buffer BUF_
#define PIPE8_READ_SCALE(R_, BUF_)                                                                      \
    {                                                                                                   \
        const uint8_t* sc__ = scl + (BUF_)*SCL + r * 4;                                                 \
        if ((R_) < TM) m8an[(R_) < TM ? (R_) : 0] = *reinterpret_cast<const uint32_t*>(sc__ + (wm * TM + (R_)) * 256); \
        else m8bn[(R_) >= TM ? (R_)-TM : 0] = *reinterpret_cast<const uint32_t*>(sc__ + (BM / 32 + wn * TN + (R_)-TM) * 256); \
    }
#define PIPE8_TAKE_SCALES                                                                               \
    {                                                                                                   \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) m8a[i] = (int)(m8an[i] >> (8 * q));              \
        _Pragma("unroll") for (int j = 0; j < TN; ++j) m8b[j] = (int)(m8bn[j] >> (8 * q));              \
    }
#define PIPE8_MFMA(N_, BS_, KS_)                                                                        \
    {                                                                                                   \
        const int i__ = (N_) / TN, j__ = (N_) % TN;                                                     \
        const bool x__ = (KS_) == 1 && i__ == TM - 1;                                                   \
        const u32x4 a0__ = x__ ? A8x[0] : A8[i__][0], a1__ = x__ ? A8x[1] : A8[i__][1];                 \
        const v8i av__ = {(int)a0__.x, (int)a0__.y, (int)a0__.z, (int)a0__.w,                           \
                          (int)a1__.x, (int)a1__.y, (int)a1__.z, (int)a1__.w};                          \
        const v8i bv__ = {(int)BS_[j__][0].x, (int)BS_[j__][0].y, (int)BS_[j__][0].z, (int)BS_[j__][0].w, \
                          (int)BS_[j__][1].x, (int)BS_[j__][1].y, (int)BS_[j__][1].z, (int)BS_[j__][1].w}; \
        if (MX)                                                                                         \
            acc[i__][j__] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av__, bv__, acc[i__][j__], 0, 0, 2 * (KS_), \
                                                                            m8a[i__], 2 * (KS_), m8b[j__]); \
        else                                                                                            \
            acc[i__][j__] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av__, bv__, acc[i__][j__], 0, 0, 0, \
                                                                            0x7f7f7f7f, 0, 0x7f7f7f7f); \
    }

    // ---- prologue: the first two stages of the first tile ---------------------------------------
    PIPE2_TILE_POS(ctile, lm0, ln0)
    hasnext = false;  // the first two stages belong to the first tile (nT >= 3)
    PIPE2_STAGE_SETUP
#pragma unroll
    for (int l = 0; l < NLD; ++l) PIPE2_LOAD(l, 0)
    PIPE2_ADVANCE
#pragma unroll
    for (int l = 0; l < NLD; ++l) PIPE2_LOAD(l, 1)
    PIPE2_ADVANCE
    wait_vmcnt<0>();
    __syncthreads();
    if constexpr (DUAL) {
#pragma unroll
        for (int rd = 0; rd < HR; ++rd) PIPE_READ1(rd, 0, 2 * q, Xa, Xb)
#pragma unroll
        for (int rd = 0; rd < HR; ++rd) PIPE_READ1(rd, 0, 2 * q + 1, Ya, Yb)
#pragma unroll
        for (int rd = 0; rd < TM + TN; ++rd) PIPE_READ_SCALE(rd, 0, 0, s0a, s0b)
    }
    int buf = 0;
    int cpar = 0;  // FP8: which copy of the tile scales the tile under the compute cursor reads

#define PIPE2_FENCE __builtin_amdgcn_sched_barrier(0);
#define PIPE2_GROUP(G_, FP4_)                                                                          \
    {                                                                                                  \
        _Pragma("unroll") for (int n__ = 0; n__ < NT; ++n__) {                                         \
            constexpr int g__ = (G_);                                                                  \
            const int k = g__ * NT + n__;                                                              \
            if (FP4_) {                                                                                \
                if (g__ == 0) PIPE_MFMA_FP4(n__, Xa, Xb, s0a, s0b, 0)                                  \
                else if (g__ == 1) PIPE_MFMA_FP4(n__, Ya, Yb, s0a, s0b, 1)                             \
                else if (g__ == 2) PIPE_MFMA_FP4(n__, Xa, Xb, s1a, s1b, 0)                             \
                else PIPE_MFMA_FP4(n__, Za, Zb, s1a, s1b, 1)                                           \
            } else {                                                                                   \
                if (g__ == 0) PIPE_MFMA_BF16(n__, Xa, Xb)                                              \
                else if (g__ == 1) PIPE_MFMA_BF16(n__, Ya, Yb)                                         \
                else if (g__ == 2) PIPE_MFMA_BF16(n__, Xa, Xb)                                         \
                else PIPE_MFMA_BF16(n__, Za, Zb)                                                       \
            }                                                                                          \
            /* group 0: piece 4+2q+1 -> Z, scales of the second half -> S1 */                          \
            if (g__ == 0) {                                                                            \
                _Pragma("unroll") for (int u = 0; u < RPS; ++u)                                        \
                    if (n__ * RPS + u < HR) PIPE_READ1(n__ * RPS + u, buf, 4 + 2 * q + 1, Za, Zb)      \
                if (FP4_ && n__ < HR) PIPE_READ_SCALE(n__, buf, 1, s1a, s1b)                           \
            }                                                                                          \
            /* group 1: piece 4+2q -> X (group 0 has consumed piece 2q) */                             \
            if (g__ == 1) {                                                                            \
                _Pragma("unroll") for (int u = 0; u < RPS1; ++u)                                       \
                    if (n__ * RPS1 + u < HR) PIPE_READ1(n__ * RPS1 + u, buf, 4 + 2 * q, Xa, Xb)        \
            }                                                                                          \
            if (k == A_AT) {                                                                           \
                PIPE2_FENCE                                                                            \
                __builtin_amdgcn_s_waitcnt(0xC07F); /* lgkmcnt(0): this wave has read the whole stage */ \
                __builtin_amdgcn_s_barrier();                                                          \
                PIPE2_FENCE                                                                            \
            }                                                                                          \
            if (k > A_AT) {                                                                            \
                const int l0__ = ((k - A_AT - 1) * NLD + LW - 1) / LW, l1__ = ((k - A_AT) * NLD + LW - 1) / LW; \
                _Pragma("unroll") for (int u = 0; u < LPS; ++u)                                        \
                    if (l0__ + u < l1__ && l0__ + u < NLD) PIPE2_LOAD(l0__ + u, buf)                   \
            }                                                                                          \
            if (k == B_AT) {                                                                           \
                PIPE2_FENCE                                                                            \
                wait_vmcnt<N_BEFORE_B>();                                                              \
                __builtin_amdgcn_s_barrier();                                                          \
                PIPE2_FENCE                                                                            \
            }                                                                                          \
            /* group 3: pieces 2q, 2q+1 of the next stage -> X, Y; its first scales -> S0 */           \
            if (k > B_AT) {                                                                            \
                _Pragma("unroll") for (int u = 0; u < RPS2; ++u) {                                     \
                    const int rd__ = (k - B_AT - 1) * RPS2 + u;                                        \
                    if (rd__ < HR) PIPE_READ1(rd__, buf ^ 1, 2 * q, Xa, Xb)                            \
                    else if (rd__ < 2 * HR) PIPE_READ1(rd__ - HR, buf ^ 1, 2 * q + 1, Ya, Yb)          \
                }                                                                                      \
                if (k - B_AT - 1 < HR) PIPE_READ_SCALE(k - B_AT - 1, buf ^ 1, 0, s0a, s0b)             \
            }                                                                                          \
            PIPE2_FENCE                                                                                \
        }                                                                                              \
    }
#define PIPE2_STAGE(FP4_)                                                                              \
    {                                                                                                  \
        PIPE2_GROUP(0, FP4_) PIPE2_GROUP(1, FP4_) PIPE2_GROUP(2, FP4_) PIPE2_GROUP(3, FP4_)            \
        PIPE2_ADVANCE                                                                                  \
        buf ^= 1;                                                                                      \
    }

    // FP8 stage: MFMA step 0 in slots 0 .. NT-1 (A8 x Bp), step 1 in slots NT .. 2NT-1 (A8 x Bq); slot
    // k = step * NT + i * TN + j.
    //   slots 0 .. 2TN-1:      Bq <- step 1
    //   slots (i+1) TN, +1:    block i < TM-1 of A <- step 1 (its step-0 MFMAs are slots i TN .. i TN + TN-1)
    //   slots NT-6, NT-5:      A8x <- step 1 of block TM-1 (a set of its own: waiting for that block's last
    //                          step-0 MFMA would keep the buffer busy four slots longer)
    //   slot F8_A_AT:          every wave has read the whole stage -> barrier -> loads of stage T+2
    //   slot F8_B_AT:          loads of stage T+1 have landed -> barrier
    //   behind it:             Bp and A <- step 0 of stage T+1: block TM-1 first (free since slot NT-1), then
    //                          blocks 0 .. TM-2 (block i is free after slot NT + i TN + TN-1 and is read in
    //                          slots F8_B_AT + 3 + 2i, + 4 + 2i)
#define PIPE8_STAGE                                                                                    \
    {                                                                                                  \
        _Pragma("unroll") for (int n__ = 0; n__ < NT; ++n__) {                                         \
            PIPE8_MFMA(n__, Bp, 0)                                                                     \
            if (n__ == NT - 6 || n__ == NT - 5)                                                        \
                A8x[n__ - (NT - 6)] = *reinterpret_cast<const u32x4*>(                                 \
                    lds + buf * STG + st128_off(ra0 + 32 * (TM - 1), PIPE8_PIECE(1, n__ - (NT - 6)))); \
            if (n__ < 2 * TN) PIPE8_RB(Bq, n__ / 2, buf, 1, n__ % 2)                                   \
            if (n__ >= TN && (n__ - TN) % TN < 2) PIPE8_RA((n__ - TN) / TN, buf, 1, (n__ - TN) % TN)   \
            PIPE2_FENCE                                                                                \
        }                                                                                              \
        _Pragma("unroll") for (int n__ = 0; n__ < NT; ++n__) {                                         \
            const int k = NT + n__;                                                                    \
            PIPE8_MFMA(n__, Bq, 1)                                                                     \
            if (k == F8_A_AT) {                                                                        \
                PIPE2_FENCE                                                                            \
                __builtin_amdgcn_s_waitcnt(0xC07F); /* lgkmcnt(0) */                                   \
                __builtin_amdgcn_s_barrier();                                                          \
                PIPE2_FENCE                                                                            \
            }                                                                                          \
            if (k > F8_A_AT) {                                                                         \
                const int l0__ = ((k - F8_A_AT - 1) * NLD + F8_LW - 1) / F8_LW,                        \
                          l1__ = ((k - F8_A_AT) * NLD + F8_LW - 1) / F8_LW;                            \
                _Pragma("unroll") for (int u = 0; u < F8_LPS; ++u)                                     \
                    if (l0__ + u < l1__ && l0__ + u < NLD) PIPE2_LOAD(l0__ + u, buf)                   \
            }                                                                                          \
            if (k == F8_B_AT) {                                                                        \
                PIPE2_FENCE                                                                            \
                wait_vmcnt<F8_N_BEFORE_B>();                                                           \
                __builtin_amdgcn_s_barrier();                                                          \
                PIPE2_FENCE                                                                            \
            }                                                                                          \
            if (k > F8_B_AT) {                                                                         \
                const int rd__ = k - F8_B_AT - 1;                                                      \
                if (rd__ < 2 * TN) PIPE8_RB(Bp, rd__ / 2, buf ^ 1, 0, rd__ % 2)                        \
                if (rd__ < 2) PIPE8_RA(TM - 1, buf ^ 1, 0, rd__)                                       \
                if (rd__ >= 2 && rd__ < 2 * TM) PIPE8_RA(rd__ / 2 - 1, buf ^ 1, 0, rd__ % 2)           \
                if (MX && rd__ < TM + TN) PIPE8_READ_SCALE(rd__, buf ^ 1)                              \
            }                                                                                          \
            PIPE2_FENCE                                                                                \
        }                                                                                              \
        if (MX) PIPE8_TAKE_SCALES                                                                      \
        PIPE2_ADVANCE                                                                                  \
        buf ^= 1;                                                                                      \
    }
    static_assert(DUAL || (NT + (TM - 2) * TN + TN - 1 < F8_B_AT + 3 + 2 * (TM - 2) && F8_B_AT + 2 * TM < F8_SLOT),
                  "8-bit stage: an A block is read before it is free");

#pragma unroll 1
    for (;;) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int k = 0; k < 16; ++k) acc[i][j][k] = 0.0f;
        // the load cursor is at stage 2 of this tile; it will cross into the next one (if any)
        hasnext = ctile + step < last;
        if (hasnext) PIPE2_TILE_POS(ctile + step, nm0, nn0)
        if constexpr (!DUAL) {
            // 8-bit modes: the first fragments of a tile are read here, again for every tile but the first
            // (the last stage of the tile before has read them already): 0.3 us per tile, and 70 registers
            // fewer are alive across the epilogue, which otherwise spills its results
#pragma unroll
            for (int i = 0; i < TM; ++i) { PIPE8_RA(i, buf, 0, 0) PIPE8_RA(i, buf, 0, 1) }
#pragma unroll
            for (int j = 0; j < TN; ++j) { PIPE8_RB(Bp, j, buf, 0, 0) PIPE8_RB(Bp, j, buf, 0, 1) }
            if constexpr (MX) {
#pragma unroll
                for (int rd = 0; rd < TM + TN; ++rd) PIPE8_READ_SCALE(rd, buf)
                PIPE8_TAKE_SCALES
            }
        }
        if constexpr (DUAL) {
#pragma unroll 1
            for (int T = 0; T < nTA; ++T) PIPE2_STAGE(1)
#pragma unroll 1
            for (int T = nTA; T < nT; ++T) PIPE2_STAGE(0)
        } else {
#pragma unroll 1
            for (int T = 0; T < nTA; ++T) PIPE8_STAGE
        }
        const bool done = !hasnext;
        if (done) wait_vmcnt<0>();  // the idle re-fetches of the last stage still target LDS
        TilePos ctp;
        PIPE2_TILE_POS(ctile, ctp.m0, ctp.n0)
        ctp.row_begin = 0;
        ctp.row_end = a.M;
        ctp.wp = a.Wpack;
        ctp.valid = true;
        if constexpr (BLKSC) {
            store_result<MODE, TM, TN, WN>(a, ctp, acc);
        } else {
            store_result<MODE, TM, TN, WN, true>(a, ctp, acc, reinterpret_cast<const float*>(scl + cpar * SCL));
            cpar ^= 1;
        }
        if (done) break;
        ctile += step;
    }
#undef NBLK_OF
#undef PIPE8_STAGE
#undef PIPE8_MFMA
#undef PIPE8_RA
#undef PIPE8_RB
#undef PIPE8_PIECE
#undef PIPE8_READ_SCALE
#undef PIPE8_TAKE_SCALES
#undef PIPE2_STAGE
#undef PIPE2_GROUP
#undef PIPE2_FENCE
}

template <int MODE, int TM, int TN, int WN = 2>
static int launch_pipe2(KArgs a, int64_t rows_total, bool grouped, hipStream_t st) {
    constexpr int BM = 64 * TM, BN = 32 * TN * WN;
    const size_t smem = (size_t)(BM + BN) * 128 * 2 + (MODE != MODE_FP8 ? (size_t)(BM + BN) / 32 * 256 * 2 : (size_t)(BM + BN) * 4 * 2);
    a.tiles_n = (int)((a.N + BN - 1) / BN);
    int64_t tiles_m = (rows_total + BM - 1) / BM;
    if (grouped) {  // upper bounds, whole rounds of the 8 XCDs
        if (a.grp_mode == 2) tiles_m = (int64_t)a.E * ((a.grp_bm / 2 + BM - 1) / BM);  // less than half a main tile each
        else tiles_m += a.E;                                                          // one ragged tile each
        tiles_m = (tiles_m + 7) / 8 * 8;
    }
    const int64_t ntiles = tiles_m * a.tiles_n;
    if (ntiles <= 0) return OSC_OK;
    if (ntiles > 0x7fffffff) return fail(OSC_ERR_UNSUPPORTED, "gemm: too many tiles");
    const int ncu = cu_count();
    if (ncu <= 0) return fail(OSC_ERR_HIP, "gemm: cannot read the number of compute units");
    const int per_cu = smem * 2 <= 160 * 1024 ? 2 : 1;  // workgroups that fit one CU's LDS
    const int64_t grid = ntiles < (int64_t)ncu * per_cu ? ntiles : (int64_t)ncu * per_cu;
    auto kern = gemm_pipe2_kernel<MODE, TM, TN, WN>;
    if (smem > 64 * 1024) {
        static unsigned char lds_done[MAX_DEVICES];
        static size_t lds_reserved[MAX_DEVICES];
        if (int rc = reserve_lds(reinterpret_cast<const void*>(kern), smem, lds_done, lds_reserved)) return rc;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(128 * WN), smem, st, a, (int)ntiles);
    return check_launch("gemm_pipe2_kernel");
}


// ------------------------------------------------------------------------------------------
// Ring kernel (dual path, one problem, eight wavefronts).  The reduction axis is staged in 64-byte
// row segments ("half stages": 128 FP4 channels = one scale word per row, or 32 bf16 channels of
// the branch) through a ring of four LDS slots, so a DMA load has two to three half stages to land
// instead of less than one stage of the two-slot kernels, at the price of half-line requests.
// The eight wavefronts form two groups of four (one wavefront of each group per SIMD) that run
// half an iteration apart: an iteration is a memory cluster (fragment and scale reads of the
// current half stage, DMA requests for the one three ahead) and a compute cluster (16 MFMAs), each
// closed by a workgroup barrier, and group 1 enters the loop one barrier late.  While one group
// feeds the matrix core the other one reads LDS and issues loads, and the barriers keep the two in
// that anti-phase.  A slot is refilled only after both groups have read it (the requests for half
// stage h+3 go to the slot of half stage h-1, which both groups left at least one barrier ago);
// a half stage is published by the counted wait every wavefront executes before a barrier.
// ------------------------------------------------------------------------------------------
template <int TM, int TN, int WN, bool PINGPONG>
__global__ void __launch_bounds__(128 * WN) gemm_ring_kernel(KArgs a) {
    constexpr int NWV = 2 * WN;
    constexpr int BM = 64 * TM, BN = 32 * TN * WN;
    constexpr int NS = 4;                        // ring slots
    constexpr int HSB = (BM + BN) * 64;          // operand bytes of a half stage
    constexpr int NBLK = (BM + BN) / 32;         // 32-row blocks (one 128-byte run of scale words each)
    constexpr int SCB = NBLK * 128;              // scale bytes of a half stage
    constexpr int LPT = (BM + BN) / 16 / NWV;    // operand DMA instructions per wavefront and half stage (16 rows each)
    constexpr int LPA = BM / 16 / NWV;           // of which on the A rows
    constexpr int SPT = NBLK / 2 / NWV;          // scale DMA instructions per wavefront (two blocks each)
    constexpr int NLD = LPT + SPT;
    static_assert((BM / 16) % NWV == 0 && (BN / 16) % NWV == 0 && (NBLK / 2) % NWV == 0, "tile does not split over the wavefronts");
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    uint8_t* const scl = lds + NS * HSB;

    const int t = threadIdx.x, lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave / WN, wn = wave % WN, q = lane >> 5, r = lane & 31;
    const TilePos tp = locate_tile<BM, BN>(a);
    const int m0 = tp.m0, n0 = tp.n0, row_end = tp.row_end;

    const int Kg4 = ((a.K >> 5) + 3) >> 2;
    const int rowbytes = a.K >> 1;
    const int nHA = rowbytes >> 6;                   // half stages of the FP4 phase
    const int nHB = (a.K_o * 2 + 63) >> 6;           // of the bf16 branch
    const int nH = nHA + nHB;                        // >= 3 (checked on the host)

    // ---- DMA addressing: lane l of instruction i moves the 16-byte piece at position l%4 of row 16*chunk + l/4 ----
    uint32_t grow[LPT];                              // global row of this lane for instruction i
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
        const int chunk = (i < LPA ? 0 : BM / 16) + wave + NWV * (i < LPA ? i : i - LPA);
        const int lrow = 16 * chunk + (lane >> 2) - (i < LPA ? 0 : BM);
        grow[i] = i < LPA ? (uint32_t)min(m0 + lrow, row_end - 1) : (uint32_t)min(n0 + lrow, a.N - 1);
    }
    // the piece stored at position p of stage row R is piece p ^ ((R >> 2) & 3) (ring_off)
    const uint32_t piece16 = (uint32_t)(((lane & 3) ^ ((lane >> 4) & 3)) << 4);
    uint32_t sco;                                    // scale word of this lane's row in its block, first half stage
    {
        const int b = 2 * wave + q;                  // block of this lane half
        const int g = b < BM / 32 ? min(m0 + 32 * b + r, row_end - 1) : min(n0 + 32 * (b - BM / 32) + r, a.N - 1);
        sco = (uint32_t)(g >> 5) * (uint32_t)Kg4 * 128u + (uint32_t)(g & 31) * 4u;
    }
    const bool sc_is_a = 2 * wave < BM / 32;         // both blocks of a wavefront lie on the same operand (BM/32 even)
    const uint8_t* const wq = tp.wp + a.off_q;
    const uint8_t* const wl = tp.wp + a.off_l;
    const uint8_t* const wsb = tp.wp + a.off_s;
    const uint8_t* const scbase = sc_is_a ? a.Xs : wsb;

    // ---- fragment addressing ----
    const int ra0 = wm * (TM * 32) + r, rb0 = BM + wn * (TN * 32) + r;
    const uint32_t fpos0 = (uint32_t)(((2 * q) ^ ((r >> 2) & 3)) << 4);   // position of piece 2q; piece 2q+1 sits at fpos0 ^ 16
    const uint32_t fa_off = (uint32_t)ra0 * 64u, fb_off = (uint32_t)rb0 * 64u;
    const uint32_t sa_off = (uint32_t)(wm * TM) * 128u + (uint32_t)r * 4u + 2u * q;
    const uint32_t sb_off = (uint32_t)(BM / 32 + wn * TN) * 128u + (uint32_t)r * 4u + 2u * q;

    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int k = 0; k < 16; ++k) acc[i][j][k] = 0.0f;

    // requests of half stage H_ (clamped to the last one: past the end the data goes to a slot nobody reads)
#define RING_LOAD(H_, SLOT_)                                                                              \
    {                                                                                                     \
        const int h__ = min((H_), nH - 1);                                                                \
        const bool fp4__ = h__ < nHA;                                                                     \
        const uint32_t ko__ = (uint32_t)(fp4__ ? h__ : h__ - nHA) * 64u + piece16;                        \
        const uint32_t pa__ = fp4__ ? (uint32_t)rowbytes : (uint32_t)a.bpitch;                            \
        const uint32_t pb__ = fp4__ ? (uint32_t)rowbytes : (uint32_t)a.wlpitch;                           \
        const uint8_t* ba__ = fp4__ ? a.Xq : a.B;                                                         \
        const uint8_t* bb__ = fp4__ ? wq : wl;                                                            \
        uint8_t* dst__ = lds + (SLOT_)*HSB + wave * 1024;                                                 \
        _Pragma("unroll") for (int i = 0; i < LPT; ++i) {                                                 \
            const uint8_t* src__ = (i < LPA ? ba__ + grow[i] * pa__ : bb__ + grow[i] * pb__) + ko__;      \
            load_to_lds16(src__, dst__ + (i < LPA ? i * (NWV * 1024) : BM * 64 + (i - LPA) * (NWV * 1024))); \
        }                                                                                                 \
        const uint32_t so__ = (uint32_t)min(h__, Kg4 - 1) * 128u + sco;                                   \
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(scbase + so__),  \
                                         (__attribute__((address_space(3))) void*)(scl + (SLOT_)*SCB + wave * 256), \
                                         4, 0, 0);                                                        \
    }
    // fragments of both pieces of this lane half and the two scale bytes that go with them
#define RING_READ(SLOT_, FA0_, FB0_, FA1_, FB1_, SA_, SB_)                                                \
    {                                                                                                     \
        const uint8_t* st__ = lds + (SLOT_)*HSB;                                                          \
        const uint8_t* sc__ = scl + (SLOT_)*SCB;                                                          \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) {                                                  \
            FA0_[i] = *reinterpret_cast<const u32x4*>(st__ + fa_off + i * 2048 + fpos0);                  \
            FA1_[i] = *reinterpret_cast<const u32x4*>(st__ + fa_off + i * 2048 + (fpos0 ^ 16u));          \
            SA_[i] = *reinterpret_cast<const uint16_t*>(sc__ + sa_off + i * 128);                         \
        }                                                                                                 \
        _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                                  \
            FB0_[j] = *reinterpret_cast<const u32x4*>(st__ + fb_off + j * 2048 + fpos0);                  \
            FB1_[j] = *reinterpret_cast<const u32x4*>(st__ + fb_off + j * 2048 + (fpos0 ^ 16u));          \
            SB_[j] = *reinterpret_cast<const uint16_t*>(sc__ + sb_off + j * 128);                         \
        }                                                                                                 \
    }

    // ---- prologue: half stages 0, 1, 2 requested; 0 published ----
    RING_LOAD(0, 0)
    RING_LOAD(1, 1)
    RING_LOAD(2, 2)
    wait_vmcnt<2 * NLD>();
    __syncthreads();
    if (PINGPONG && wm == 1) __builtin_amdgcn_s_barrier();   // group 1 runs half an iteration behind

    u32x4 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
    int sa[TM], sb[TN];
#define RING_ITER(H_, FP4_)                                                                               \
    {                                                                                                     \
        const int slot__ = (H_)&3;                                                                        \
        /* memory cluster */                                                                              \
        RING_READ(slot__, fa0, fb0, fa1, fb1, sa, sb)                                                     \
        RING_LOAD((H_) + 3, ((H_) + 3) & 3)                                                               \
        __builtin_amdgcn_sched_barrier(0);                                                                \
        __builtin_amdgcn_s_waitcnt(0xC07F); /* lgkmcnt(0): the fragments are in registers */              \
        if (PINGPONG) {                                                                                   \
            wait_vmcnt<2 * NLD>();                                                                        \
            __builtin_amdgcn_s_barrier();                                                                 \
        }                                                                                                 \
        __builtin_amdgcn_sched_barrier(0);                                                                \
        /* compute cluster */                                                                             \
        __builtin_amdgcn_s_setprio(1);                                                                    \
        if (FP4_) {                                                                                       \
            OSC_MFMA_FP4(0, fa0, fb0, sa, sb)                                                             \
            OSC_MFMA_FP4(1, fa1, fb1, sa, sb)                                                             \
        } else {                                                                                          \
            OSC_MFMA_BF16(fa0, fb0)                                                                       \
            OSC_MFMA_BF16(fa1, fb1)                                                                       \
        }                                                                                                 \
        __builtin_amdgcn_s_setprio(0);                                                                    \
        __builtin_amdgcn_sched_barrier(0);                                                                \
        wait_vmcnt<2 * NLD>();                                                                            \
        __builtin_amdgcn_s_barrier();                                                                     \
        __builtin_amdgcn_sched_barrier(0);                                                                \
    }
    int h = 0;
#pragma unroll 1
    for (; h < nHA; ++h) RING_ITER(h, true)
#pragma unroll 1
    for (; h < nH; ++h) RING_ITER(h, false)
    wait_vmcnt<0>();                                          // the idle requests of the last iterations still target LDS
    if (PINGPONG && wm == 0) __builtin_amdgcn_s_barrier();    // balances group 1's late start
#undef RING_ITER
#undef RING_READ
#undef RING_LOAD
    store_result<MODE_DUAL, TM, TN, WN>(a, tp, acc);
}

template <int TM, int TN, int WN, bool PINGPONG>
static int launch_ring(KArgs a, hipStream_t st) {
    constexpr int BM = 64 * TM, BN = 32 * TN * WN;
    const size_t smem = (size_t)4 * ((BM + BN) * 64 + (BM + BN) / 32 * 128);
    a.tiles_n = (int)((a.N + BN - 1) / BN);
    const int64_t grid = (int64_t)((a.M + BM - 1) / BM) * a.tiles_n;
    if (grid <= 0) return OSC_OK;
    if (grid > 0x7fffffff) return fail(OSC_ERR_UNSUPPORTED, "gemm: too many tiles");
    auto kern = gemm_ring_kernel<TM, TN, WN, PINGPONG>;
    static unsigned char lds_done[MAX_DEVICES];
    static size_t lds_reserved[MAX_DEVICES];
    if (int rc = reserve_lds(reinterpret_cast<const void*>(kern), smem, lds_done, lds_reserved)) return rc;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(128 * WN), smem, st, a);
    return check_launch("gemm_ring_kernel");
}

// ------------------------------------------------------------------------------------------
// Skinny kernel (M <= 64: decode batches, and other launches of few output blocks), dual path, FP8 and
// MXFP8.  The work is streaming the weights once, so the grid is as wide as it can be without splitting
// the reduction over workgroups: one workgroup per 32 output channels; its NW wavefronts take the
// 128-byte lines of the reduction axis in turn (FP4 lines, then bf16 branch lines) and never synchronise
// until the end: each wavefront moves its lines global -> LDS with the DMA path into a ring of DEPTH
// images of its own (whole 128-byte lines per row, so every request is a full cache line; the scale
// words of the 64 rows behind them), reads them back in the matrix-core layout, and the NW partial
// 32x32 results are summed through LDS in a fixed order.
// Inside a line, lanes of block q take bytes [64q, 64q+64): four 16-byte pieces, one MFMA each,
// and for FP4 exactly the four groups of scale word 2*line + q.
// MT = number of 32-row tiles of X per workgroup (blockIdx.y selects the group of MT tiles).
// ------------------------------------------------------------------------------------------
template <int MODE, int MT, int NW, int DEPTH>
__global__ void __launch_bounds__(64 * NW) gemm_skinny_kernel(KArgs a) {
    constexpr int ROWS = 32 + 32 * MT;      // rows of a line image: 32 weight rows, then the X rows
    constexpr int NSC = (MODE == MODE_FP8) ? 0 : 1 + MT;  // scale requests per line (one 256-byte run of words each)
    constexpr int IMG = ROWS * 128 + NSC * 256;  // bytes of a line image: the rows, then their scale words
    constexpr int NDMA = ROWS / 8;           // DMA instructions per line (8 rows each)
    constexpr int NREQ = NDMA + NSC;         // requests per line
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];  // [NW waves][DEPTH images], later the partial sums
    const int t = threadIdx.x, lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int q = lane >> 5, r = lane & 31;
    const int n0 = blockIdx.x * 32;
    const int mb = blockIdx.y * (32 * MT);  // first X row of this workgroup
    const int Kg4 = ((a.K >> 5) + 3) >> 2;
    const int rowbytes = (MODE == MODE_DUAL) ? (a.K >> 1) : a.K;
    const int nL = rowbytes >> 7;
    const int nLB = (MODE == MODE_DUAL) ? ((a.K_o * 2 + 127) >> 7) : 0;
    const int nLT = nL + nLB;
    uint8_t* const strip = lds + wave * (DEPTH * IMG);

    // DMA instruction i moves rows 8i .. 8i+7 of the image: lane -> row 8i + lane/8, piece position
    // lane%8, which holds piece (lane%8) ^ swz8(row) of the row
    uint32_t o_fp4[NDMA], o_br[NDMA];  // byte offset of this lane's 16 bytes in line 0, per phase
#pragma unroll
    for (int i = 0; i < NDMA; ++i) {
        const int row = 8 * i + (lane >> 3);
        const uint32_t piece = (uint32_t)((lane & 7) ^ swz8(row)) * 16u;
        if (row < 32) {
            const uint32_t g = (uint32_t)min(n0 + row, a.N - 1);
            o_fp4[i] = g * (uint32_t)rowbytes + piece;
            o_br[i] = g * (uint32_t)a.wlpitch + piece;
        } else {
            const uint32_t g = (uint32_t)min(mb + row - 32, a.M - 1);
            o_fp4[i] = g * (uint32_t)rowbytes + piece;
            o_br[i] = g * (uint32_t)a.bpitch + piece;
        }
    }
    const uint8_t* const wq = a.Wpack + a.off_q;
    const uint8_t* const wl = a.Wpack + a.off_l;
    // scale words of this lane's rows (weight row n0 + r, X rows 32m + r), word 2*line + q
    const int rowB = min(n0 + r, a.N - 1);
    // scale word of this lane's row: FP4 word 2*line + q (groups 4q .. 4q+3 of the line's eight);
    // MXFP8 word `line` of the row (four groups), shifted so that byte 2h is the scale of group 2h+q
    const int sq = (MODE == MODE_MX8) ? 0 : q * 128;
    const int sstep = (MODE == MODE_MX8) ? 128 : 256;  // bytes between the words of consecutive lines
    const uint8_t* const ws = a.Wpack + a.off_s + (size_t)(rowB >> 5) * Kg4 * 128 + (rowB & 31) * 4 + sq;
    const uint8_t* xs[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const int rowA = min(mb + 32 * m + r, a.M - 1);
        xs[m] = a.Xs + (size_t)(rowA >> 5) * Kg4 * 128 + (rowA & 31) * 4 + sq;
    }
    v16f acc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int k = 0; k < 16; ++k) acc[m][k] = 0.0f;

    // line L of the whole sequence into image IMG_ of this wave's strip (nothing past the end)
#define SKINNY_FETCH(L_, IMG_)                                                                          \
    {                                                                                                   \
        uint8_t* dst__ = strip + (IMG_)*IMG;                                                            \
        if ((L_) < nLT && MODE != MODE_FP8) {                                                           \
            /* scale words of the line: lane (q, r) fetches the word of its row; a line of the bf16     \
               branch fetches the last word again (never used), so every line is NREQ requests */       \
            const size_t so__ = (size_t)min((L_), nL - 1) * sstep;                                      \
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(ws + so__), \
                                             (__attribute__((address_space(3))) void*)(dst__ + ROWS * 128), 4, 0, 0); \
            _Pragma("unroll") for (int m = 0; m < MT; ++m)                                              \
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(xs[m] + so__), \
                                                 (__attribute__((address_space(3))) void*)(dst__ + ROWS * 128 + (1 + m) * 256), 4, 0, 0); \
        }                                                                                               \
        if ((L_) < nL) {                                                                                \
            _Pragma("unroll") for (int i = 0; i < NDMA; ++i)                                            \
                load_to_lds16((i < 4 ? wq : a.Xq) + ((size_t)(L_)*128 + o_fp4[i]), dst__ + i * 1024);   \
        } else if ((L_) < nLT) {                                                                        \
            _Pragma("unroll") for (int i = 0; i < NDMA; ++i)                                            \
                load_to_lds16((i < 4 ? wl : a.B) + ((size_t)((L_)-nL) * 128 + o_br[i]), dst__ + i * 1024); \
        }                                                                                               \
    }
    // consume line L from image IMG_
#define SKINNY_COMPUTE(L_, IMG_)                                                                        \
    {                                                                                                   \
        const uint8_t* src__ = strip + (IMG_)*IMG;                                                      \
        u32x4 fb__[4], fx__[MT][4];                                                                     \
        _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                                 \
            /* FP4 / bf16: pieces 4q .. 4q+3; 8-bit: pieces q, 2+q, 4+q, 6+q */                         \
            const int pc__ = (MODE == MODE_DUAL) ? 4 * q + i : 2 * i + q;                               \
            fb__[i] = *reinterpret_cast<const u32x4*>(src__ + st128_off(r, pc__));                      \
            _Pragma("unroll") for (int m = 0; m < MT; ++m)                                              \
                fx__[m][i] = *reinterpret_cast<const u32x4*>(src__ + st128_off(32 + 32 * m + r, pc__)); \
        }                                                                                               \
        if (MODE == MODE_FP8 || MODE == MODE_MX8) {                                                     \
            /* 128 channels = two MFMAs; MFMA h: registers 0-3 = piece 4h+q, registers 4-7 = piece      \
               4h+2+q (for 8-bit operands lane half q supplies elements 16q..16q+15 of both scale      \
               blocks, and the scale of block q) */                                                     \
            int sbm__ = 0x7f7f7f7f, sxm__[MT];                                                          \
            _Pragma("unroll") for (int m = 0; m < MT; ++m) sxm__[m] = 0x7f7f7f7f;                       \
            if (MODE == MODE_MX8) {                                                                     \
                sbm__ = *reinterpret_cast<const int*>(src__ + ROWS * 128 + lane * 4) >> (8 * q);        \
                _Pragma("unroll") for (int m = 0; m < MT; ++m)                                          \
                    sxm__[m] = *reinterpret_cast<const int*>(src__ + ROWS * 128 + (1 + m) * 256 + lane * 4) >> (8 * q); \
            }                                                                                           \
            SKINNY_F8(0) SKINNY_F8(1)                                                                   \
        } else if ((L_) < nL) {                                                                         \
            const int sb__ = *reinterpret_cast<const int*>(src__ + ROWS * 128 + lane * 4);              \
            int sx__[MT];                                                                               \
            _Pragma("unroll") for (int m = 0; m < MT; ++m)                                              \
                sx__[m] = *reinterpret_cast<const int*>(src__ + ROWS * 128 + (1 + m) * 256 + lane * 4); \
            SKINNY_FP4(0) SKINNY_FP4(1) SKINNY_FP4(2) SKINNY_FP4(3)                                     \
        } else {                                                                                        \
            _Pragma("unroll") for (int i = 0; i < 4; ++i)                                               \
                _Pragma("unroll") for (int m = 0; m < MT; ++m)                                          \
                    acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, fx__[m][i]), \
                                                                     __builtin_bit_cast(v8bf, fb__[i]), acc[m], 0, 0, 0); \
        }                                                                                               \
    }
#define SKINNY_F8(H_)                                                                                   \
    {                                                                                                   \
        const v8i bv__ = {(int)fb__[2 * (H_)].x, (int)fb__[2 * (H_)].y, (int)fb__[2 * (H_)].z, (int)fb__[2 * (H_)].w, \
                          (int)fb__[2 * (H_) + 1].x, (int)fb__[2 * (H_) + 1].y, (int)fb__[2 * (H_) + 1].z, (int)fb__[2 * (H_) + 1].w}; \
        _Pragma("unroll") for (int m = 0; m < MT; ++m) {                                                \
            const v8i av__ = {(int)fx__[m][2 * (H_)].x, (int)fx__[m][2 * (H_)].y, (int)fx__[m][2 * (H_)].z, (int)fx__[m][2 * (H_)].w, \
                              (int)fx__[m][2 * (H_) + 1].x, (int)fx__[m][2 * (H_) + 1].y, (int)fx__[m][2 * (H_) + 1].z, (int)fx__[m][2 * (H_) + 1].w}; \
            acc[m] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av__, bv__, acc[m], 0, 0, 2 * (H_), sxm__[m], 2 * (H_), sbm__); \
        }                                                                                               \
    }
#define SKINNY_FP4(I_)                                                                                  \
    {                                                                                                   \
        const v8i bv__ = {(int)fb__[I_].x, (int)fb__[I_].y, (int)fb__[I_].z, (int)fb__[I_].w, 0, 0, 0, 0}; \
        _Pragma("unroll") for (int m = 0; m < MT; ++m) {                                                \
            const v8i av__ = {(int)fx__[m][I_].x, (int)fx__[m][I_].y, (int)fx__[m][I_].z, (int)fx__[m][I_].w, 0, 0, 0, 0}; \
            acc[m] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av__, bv__, acc[m], 4, 4, I_, sx__[m], I_, sb__); \
        }                                                                                               \
    }
    // Lines wave, wave + NW, ...: DEPTH - 1 of them are in flight while one is consumed (a wavefront streams
    // a few dozen lines at most and a request to HBM outlasts the arithmetic of several lines, so the bytes
    // in flight set the streaming rate).  Everything a wavefront reads from LDS it wrote itself, so "my
    // requests up to this line have landed" is all the synchronisation needed: a counted wait that
    // leaves the younger lines in flight.  Every operand, the scale words included, travels by DMA:
    // a load into registers between the requests would make the compiler's own waits drain the queue.
    int L = wave, img = 0;
#pragma unroll
    for (int d = 0; d < DEPTH - 1; ++d) SKINNY_FETCH(L + d * NW, d)
#pragma unroll 1
    for (; L < nLT; L += NW) {
        const int ahead = (img + DEPTH - 1) % DEPTH;
        SKINNY_FETCH(L + (DEPTH - 1) * NW, ahead)
        const int younger = (nLT - 1 - L) / NW;  // lines of this wavefront after this one
        if (DEPTH > 2 && younger >= 2) wait_vmcnt<(DEPTH > 2 ? 2 : 1) * NREQ>();
        else if (younger >= 1) wait_vmcnt<NREQ>();
        else wait_vmcnt<0>();
        SKINNY_COMPUTE(L, img)
        img = img + 1 == DEPTH ? 0 : img + 1;
    }
#undef SKINNY_FP4
#undef SKINNY_F8
#undef SKINNY_COMPUTE
#undef SKINNY_FETCH

    // ---- sum the NW partial results in a fixed order, store -------------------------------------
    __syncthreads();  // every wave is done with its strip
    float* const red = reinterpret_cast<float*>(lds);  // [NW waves][MT][16][64]
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int k = 0; k < 16; ++k) red[((wave * MT + m) * 16 + k) * 64 + lane] = acc[m][k];
    __syncthreads();
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        // result register k of lane (q, r): row 8*(k/4) + 4q + k%4, column r; wave w finishes k = w, w+NW, ...
#pragma unroll
        for (int k0 = 0; k0 < 16; k0 += NW) {
            const int k = k0 + wave;
            if (k >= 16) break;
            float v = red[((0 * MT + m) * 16 + k) * 64 + lane];
#pragma unroll
            for (int w = 1; w < NW; ++w) v += red[((w * MT + m) * 16 + k) * 64 + lane];
            const int row = mb + 32 * m + 8 * (k >> 2) + 4 * q + (k & 3), col = n0 + r;
            if (MODE == MODE_FP8)  // per-token and per-channel scales
                v *= a.xs[min(row, a.M - 1)] * reinterpret_cast<const float*>(a.Wpack + a.off_s)[min(col, a.N - 1)];
            if (row < a.M && col < a.N) {
                if (a.y_bf16)
                    reinterpret_cast<uint16_t*>(a.Y)[(int64_t)row * a.ldy + col] = f32_to_bf16_rne(v);
                else
                    reinterpret_cast<float*>(a.Y)[(int64_t)row * a.ldy + col] = v;
            }
        }
    }
}

template <int MODE, int NW, int DEPTH>
static int launch_skinny_cfg(KArgs a, unsigned grid, unsigned mtiles, hipStream_t st) {
    constexpr size_t IMG = 64 * 128 + (MODE == MODE_FP8 ? 0 : 2 * 256);
    constexpr size_t smem = (size_t)NW * DEPTH * IMG;
    auto kern = gemm_skinny_kernel<MODE, 1, NW, DEPTH>;
    if (smem > 48 * 1024) {
        static unsigned char lds_done[MAX_DEVICES];
        static size_t lds_reserved[MAX_DEVICES];
        if (int rc = reserve_lds(reinterpret_cast<const void*>(kern), smem, lds_done, lds_reserved)) return rc;
    }
    hipLaunchKernelGGL(kern, dim3(grid, mtiles), dim3(64 * NW), smem, st, a);
    return check_launch("gemm_skinny_kernel");
}

template <int MODE>
static int launch_skinny(KArgs a, hipStream_t st) {
    const int64_t grid = (a.N + 31) / 32;
    if (grid <= 0) return OSC_OK;
    // LDS: a ring of three line images per wavefront (8.5 KB each: 32 weight rows, 32 X rows, their scale
    // words); the partial sums reuse the space.  33..64 rows: two workgroups per 32 output channels, one
    // per 32-row tile of X (the second pass over a weight row is an L2 hit).  The number of wavefronts
    // follows from how many workgroups a CU has to hold for the whole grid to be resident at once:
    //   grid <= CUs:       six wavefronts (153 KB), one workgroup per CU;
    //   grid <= 2 x CUs:   three wavefronts (76.5 KB), two per CU;
    //   larger grids:      two wavefronts (51 KB), three per CU (12288 output channels x two row tiles =
    //                      768 workgroups on 256 CUs).
    const unsigned mtiles = (unsigned)((a.M + 31) / 32);
    const int ncu = cu_count();
    if (ncu <= 0) return fail(OSC_ERR_HIP, "gemm: cannot read the number of compute units");
    if (grid * mtiles > 2 * (int64_t)ncu) return launch_skinny_cfg<MODE, 2, 3>(a, (unsigned)grid, mtiles, st);
    if (grid * mtiles <= (int64_t)ncu) return launch_skinny_cfg<MODE, 6, 3>(a, (unsigned)grid, mtiles, st);
    return launch_skinny_cfg<MODE, 3, 3>(a, (unsigned)grid, mtiles, st);
}

template <int MODE, int TM, int TN, bool RAGGED>
static int launch_cfg(KArgs a, int64_t rows_total, bool grouped, hipStream_t st) {
    constexpr int BM = 64 * TM, BN = 64 * TN;
    const size_t smem = (size_t)(BM + BN) * 64 * 3;
    a.tiles_n = (int)((a.N + BN - 1) / BN);
    int64_t tiles_m = (rows_total + BM - 1) / BM;
    if (grouped) {  // upper bounds, whole rounds of the 8 XCDs
        if (a.grp_mode == 2) tiles_m = (int64_t)a.E * ((a.grp_bm / 2 + BM - 1) / BM);  // less than half a main tile each
        else tiles_m += a.E;                                                          // one ragged tile each
        tiles_m = (tiles_m + 7) / 8 * 8;
    }
    const int64_t grid = tiles_m * a.tiles_n;
    if (grid <= 0) return OSC_OK;
    if (grid > 0x7fffffff) return fail(OSC_ERR_UNSUPPORTED, "gemm: too many tiles");
    auto kern = gemm_kernel<MODE, TM, TN, RAGGED>;
    if (smem > 64 * 1024) {
        static unsigned char lds_done[MAX_DEVICES];
        static size_t lds_reserved[MAX_DEVICES];
        if (int rc = reserve_lds(reinterpret_cast<const void*>(kern), smem, lds_done, lds_reserved)) return rc;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(GT), smem, st, a);
    return check_launch("gemm_kernel");
}

template <int MODE, int TM, int TN, int WN = 2, int KS = 1>
static int launch_dma2(KArgs a, int64_t rows_total, bool grouped, hipStream_t st) {
    constexpr int BM = 64 * TM, BN = 32 * TN * WN;
    const size_t smem = ((size_t)(BM + BN) * 128 * 2 + (size_t)dma2_scale_bytes(BM, BN) * 2) * KS;
    a.tiles_n = (int)((a.N + BN - 1) / BN);
    int64_t tiles_m = (rows_total + BM - 1) / BM;
    if (grouped) {  // upper bounds, whole rounds of the 8 XCDs
        if (a.grp_mode == 2) tiles_m = (int64_t)a.E * ((a.grp_bm / 2 + BM - 1) / BM);  // less than half a main tile each
        else tiles_m += a.E;                                                          // one ragged tile each
        tiles_m = (tiles_m + 7) / 8 * 8;
    }
    const int64_t grid = tiles_m * a.tiles_n;
    if (grid <= 0) return OSC_OK;
    if (grid > 0x7fffffff) return fail(OSC_ERR_UNSUPPORTED, "gemm: too many tiles");
    auto kern = gemm_dma2_kernel<MODE, TM, TN, WN, KS>;
    if (smem > 64 * 1024) {
        static unsigned char lds_done[MAX_DEVICES];
        static size_t lds_reserved[MAX_DEVICES];
        if (int rc = reserve_lds(reinterpret_cast<const void*>(kern), smem, lds_done, lds_reserved)) return rc;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(128 * WN * KS), smem, st, a);
    return check_launch("gemm_dma2_kernel");
}

// persistent form of the DMA kernel for grouped problems (at most 1024 experts, at least two stages)
template <int MODE, int TM, int TN, int WN>
static int launch_dma2g(KArgs a, int64_t rows_total, hipStream_t st) {
    constexpr int BM = 64 * TM, BN = 32 * TN * WN;
    const size_t smem = (size_t)(BM + BN) * 128 * 2 + (size_t)(BM + BN) / 32 * 256 * 2;
    a.tiles_n = (int)((a.N + BN - 1) / BN);
    int64_t tiles_m = (rows_total + BM - 1) / BM;
    if (a.grp_mode == 2) tiles_m = (int64_t)a.E * ((a.grp_bm / 2 + BM - 1) / BM);
    else tiles_m += a.E;
    tiles_m = (tiles_m + 7) / 8 * 8;
    const int64_t ntiles = tiles_m * a.tiles_n;
    if (ntiles <= 0) return OSC_OK;
    if (ntiles > 0x7fffffff) return fail(OSC_ERR_UNSUPPORTED, "gemm: too many tiles");
    const int ncu = cu_count();
    if (ncu <= 0) return fail(OSC_ERR_HIP, "gemm: cannot read the number of compute units");
    const int64_t cap = (int64_t)ncu / 8 * 8;  // whole rounds of the 8 XCDs
    const int64_t grid = ntiles < cap ? ntiles : cap;
    const size_t smem_all = smem + (size_t)(3 * a.E + 1) * 4;  // + the per-expert table
    auto kern = gemm_dma2g_kernel<MODE, TM, TN, WN>;
    {
        static unsigned char lds_done[MAX_DEVICES];
        static size_t lds_reserved[MAX_DEVICES];
        if (int rc = reserve_lds(reinterpret_cast<const void*>(kern), smem_all, lds_done, lds_reserved)) return rc;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(128 * WN), smem_all, st, a, (int)ntiles);
    return check_launch("gemm_dma2g_kernel");
}

template <int MODE>
static int launch_gemm(const GemmProblem& p, hipStream_t st) {
    KArgs a;
    a.Xq = p.Xq;
    a.Xs = p.Xs;
    a.xs = p.xs;
    a.B = reinterpret_cast<const uint8_t*>(p.B);
    a.bpitch = p.ldb * 2;
    a.row_map = p.row_map;
    a.off = p.expert_offsets;
    a.E = p.E;
    a.Wpack = p.Wpack;
    a.pack_stride = p.pack_stride;
    if (MODE == MODE_DUAL) {
        PackLayout L = pack_layout(p.N, p.K, p.K_o);
        a.off_q = L.off_q;
        a.off_s = L.off_s;
        a.off_l = L.off_l;
        a.off_z = L.off_z;
        a.wlpitch = L.ldwl * 2;
    } else if (MODE == MODE_MX8) {
        PackM8Layout L = packm8_layout(p.N, p.K);
        a.off_q = L.off_w;
        a.off_s = L.off_s;
        a.off_l = 0;
        a.off_z = L.off_z;
        a.wlpitch = 0;
    } else {
        Pack8Layout L = pack8_layout(p.N, p.K);
        a.off_q = L.off_w;
        a.off_s = L.off_s;
        a.off_l = 0;
        a.off_z = L.off_z;
        a.wlpitch = 0;
    }
    a.M = (int)p.M;
    a.N = (int)p.N;
    a.K = (int)p.K;
    a.K_o = p.K_o;
    a.Y = p.Y;
    a.y_bf16 = p.y_dtype == OSC_DT_BF16;
    a.ldy = p.ldy;
    a.tiles_n = 0;
    a.grp_mode = 0;
    a.grp_bm = 0;
    const bool grouped = p.expert_offsets != nullptr;
    const int64_t rowbytes = (MODE == MODE_DUAL) ? p.K / 2 : p.K;
    // the kernel addresses operand rows through 32-bit byte offsets (with a row_map the caller
    // guarantees the same for the rows it names)
    const int64_t lim = (int64_t)1 << 32;
    if (p.M * rowbytes >= lim || p.N * rowbytes >= lim || p.M * a.bpitch >= lim || p.N * a.wlpitch >= lim ||
        (p.M / 32 + 1) * ((p.K / 32 + 3) / 4) * 128 >= lim)
        return fail(OSC_ERR_UNSUPPORTED, "gemm: an operand of 4 GiB or more");
    const int64_t rows = grouped && p.E > 0 ? (p.M + p.E - 1) / p.E : p.M;  // rows per problem
    // Kernel and tile choice.
    //  - operand rows that are whole 128-byte lines: M <= 64 -> the skinny kernel; else 256x256 tiles
    //    when they give every CU at least one tile (dual path, one problem: the persistent kernel;
    //    otherwise the DMA kernel), else the DMA kernel with 128x128 tiles;
    //  - everything else: the staged kernel, 64x128 or 128x128 tiles, with per-lane zero fill when
    //    rows are not whole 64-byte steps.
    const int64_t t256 = ((rows + 255) / 256) * ((p.N + 255) / 256) * (grouped ? p.E : 1);
    const bool lines = rowbytes > 0 && rowbytes % 128 == 0 &&
                       (MODE != MODE_DUAL || p.K_o == 0 || a.bpitch % 128 == 0);
    const bool ragged = rowbytes % 64 != 0 || (MODE == MODE_DUAL && p.K_o > 0 && a.bpitch % 64 != 0);
    // 256-row tiles when they fill the chip, else 128x128, else (fewer than one tile per CU) 64x128
    const int64_t t128 = ((rows + 127) / 128) * ((p.N + 127) / 128) * (grouped ? p.E : 1);
    const int64_t t128_full = MODE == MODE_DUAL ? 512 : 257;  // measured crossover: two (8-bit: one) 128x128 tiles per CU
    // 256-row tiles also when they leave CUs idle but the 128 x 128 tiles would need a second round (two of
    // them are resident per CU): 1024 x 12288 x 4096 takes 42.7 us on 192 tiles of 256 x 256 and 51 us on 768
    // of 128 x 128, 768 x 12288 40 against 48 us; with one round of small tiles those are ahead (2048 x 4096:
    // 28.6 against 39 us).  Measured for single problems; grouped ones keep the plain rule.
    const int ncu_hint = cu_count();
    const bool second_round = !grouped && ncu_hint > 0 && t128 > 2 * (int64_t)ncu_hint;
    int tm = rows <= 64 ? 1 : (rows > 128 && (t256 >= 256 || second_round)) ? 4 : (t128 < t128_full ? 1 : 2);
    if (MODE == MODE_MX8 && !lines)  // implemented in the DMA and skinny kernels only
        return fail(OSC_ERR_UNSUPPORTED, "mxfp8 gemm: K must be a multiple of 128");
    int kind = lines ? 1 : 0;  // 0 = staged kernel, 1 = DMA kernel, 2 = persistent pipelined kernel, 3 = skinny kernel
    // persistent kernel: one dual-path problem, whole tiles along N, at least three stages; rows
    // past the last whole tile go to a second launch of the DMA kernel
    const bool pipe_ok = lines && !grouped && !p.row_map &&
                         (rowbytes / 128 + (MODE == MODE_DUAL ? (p.K_o * 2 + 127) / 128 : 0)) >= 3;
    // (with at most one tile per CU there is no next tile to run ahead into, and the eight wavefronts of the
    // DMA kernel are 6 % faster: 4096 x 4096 x 4096 in 46.5 against 49.4 us)
    if (kind == 1 && pipe_ok && tm == 4 && t256 > 256) kind = 2;
    // The weight-streaming kernel (one workgroup per 32 output channels and 32 rows) also wins for a few
    // hundred rows as long as its grid is resident at once (two workgroups per CU): a tiled launch of so
    // few tiles leaves most CUs idle (128 x 4096 x 4096: 11.8 us on 64 x 128 tiles, 6.8 us on 512 streaming
    // workgroups).  Beyond 512 workgroups it needs a second round (1024 x 1024 x 4096, 1024 workgroups:
    // 12.6 us) and the 64 x 128 tiles with their K loop split over two wavefront groups are ahead (9.9 us).
    const int64_t skinny_wgs = ((p.N + 31) / 32) * ((p.M + 31) / 32);
    const bool skinny_ok = lines && !grouped && !p.row_map && p.M >= 1 && (p.M <= 64 || skinny_wgs <= 512);
    if (skinny_ok) kind = 3;
    if (const int t_tile = tuning(TUNE_GEMM_TILE), t_kern = tuning(TUNE_GEMM_KERNEL); t_tile >= 0 || t_kern >= 0) {
        // test and tuning overrides (osc_tuning.h); a kernel that cannot serve the shape is not forced
        if (t_tile >= 0) tm = (t_tile == 1 || t_tile == 2 || t_tile == 4) ? t_tile : 2;
        int k2 = (t_kern >= 0 && t_kern <= 3) ? t_kern : kind;  // ids above 3 are handled before the launch below
        if (t_tile >= 0 && t_kern < 0 && k2 == 3) k2 = lines ? 1 : 0;  // a forced tile means a tiled kernel
        if ((k2 == 1 || k2 == 2) && !lines) k2 = 0;
        if (k2 == 2 && (tm == 1 || (MODE != MODE_DUAL && tm != 4))) k2 = 1;
        if (k2 == 2 && !pipe_ok) k2 = 1;
        if (k2 == 3 && !skinny_ok) k2 = 0;
        kind = k2;
    }
    if constexpr (MODE == MODE_DUAL) {
        // ring kernel (ids 4 and 5: with and without the two wavefront groups in anti-phase)
        const int t_kern = tuning(TUNE_GEMM_KERNEL);
        const bool ring_ok = lines && !grouped && !p.row_map && (rowbytes / 64 + (p.K_o * 2 + 63) / 64) >= 3 &&
                             (p.K_o == 0 || a.bpitch % 64 == 0) && p.M >= 1;
        if ((t_kern == 4 || t_kern == 5) && ring_ok)
            return t_kern == 4 ? launch_ring<4, 2, 4, true>(a, st) : launch_ring<4, 2, 4, false>(a, st);
    }
    if (kind == 3) return launch_skinny<MODE>(a, st);
    if (kind == 2 && p.N % (64 * tm) == 0 && p.M >= 64 * tm) {
        const int64_t m_full = p.M / (64 * tm) * (64 * tm);
        if (m_full < p.M) {  // ragged tail: rows m_full .. M-1 as a problem of their own
            GemmProblem tail = p;
            tail.M = p.M - m_full;
            tail.Xq = p.Xq + m_full * rowbytes;
            if (p.Xs) tail.Xs = p.Xs + (m_full / 32) * ((p.K / 32 + 3) / 4) * 128;
            if (p.xs) tail.xs = p.xs + m_full;
            tail.B = p.B ? p.B + m_full * p.ldb : nullptr;
            tail.Y = static_cast<uint8_t*>(p.Y) + m_full * p.ldy * (p.y_dtype == OSC_DT_BF16 ? 2 : 4);
            const int rc = launch_gemm<MODE>(tail, st);
            if (rc != OSC_OK) return rc;
        }
        a.M = (int)m_full;
        if constexpr (MODE == MODE_DUAL) {
            if (tm == 4) return launch_pipe2<MODE_DUAL, 4, 4>(a, m_full, grouped, st);
            return launch_pipe2<MODE_DUAL, 2, 2>(a, m_full, grouped, st);
        } else {
            return launch_pipe2<MODE, 4, 4>(a, m_full, grouped, st);
        }
    }

    if (kind >= 1 && grouped && tm == 4) {
        // experts in 256-row tiles, and what is left of an expert whose last tile would be less than
        // half full in 64-row tiles (an expert of 270 rows: one big tile and one small one, not two
        // big ones)
        a.grp_mode = 1;
        int rc;
        if constexpr (MODE != MODE_DUAL) {
            // 8-bit modes: persistent workgroups (the OSC_TUNE_GROUPED_ONE_TILE override keeps one tile each)
            const bool persistent = p.E >= 1 && p.E <= 1024 && !p.row_map && rowbytes / 128 >= 2 &&
                                    tuning(TUNE_GROUPED_ONE_TILE) != 1;
            rc = persistent ? launch_dma2g<MODE, 4, 2, 4>(a, p.M, st) : launch_dma2<MODE, 4, 2, 4>(a, p.M, grouped, st);
        } else {
            rc = launch_dma2<MODE, 4, 2, 4>(a, p.M, grouped, st);
        }
        if (rc != OSC_OK) return rc;
        a.grp_mode = 2;
        a.grp_bm = 256;
        return launch_dma2<MODE, 1, 2>(a, p.M, grouped, st);
    }
    if (kind >= 1) {
        // 256-row tiles run on eight wavefronts (2 x 4, 128x64 each): 6-8 % faster than four, the second
        // wavefront of a SIMD fills the issue gaps of the first
        if (tm == 4) return launch_dma2<MODE, 4, 2, 4>(a, p.M, grouped, st);
        if constexpr (MODE == MODE_DUAL || MODE == MODE_FP8) {
            // at most one 64 x 128 tile per CU: two groups of wavefronts per tile, each taking every second stage
            // (2048 x 1024 x 4096: 12.7 -> 11.0 us, 128 x 12288 x 4096: 16.8 -> 13.2 us; with more tiles than CUs
            // the doubled LDS footprint costs a round: 192 x 12288: 17.2 -> 23.9 us); the OSC_TUNE_GEMM_KSPLIT
            // override switches it off (0) or on (1) where the shape allows it
            const int ks = tuning(TUNE_GEMM_KSPLIT);
            const int64_t t64 = ((p.M + 63) / 64) * ((p.N + 127) / 128);
            const bool fits = !grouped && (rowbytes / 128 + (p.K_o * 2 + 127) / 128) >= 4;
            if (tm == 1 && fits && (ks == 1 || (ks != 0 && ncu_hint > 0 && t64 <= ncu_hint)))
                return launch_dma2<MODE, 1, 2, 2, 2>(a, p.M, grouped, st);
            // more 64 x 128 tiles than CUs but at most one 128 x 128 tile per CU: those, split the same way
            // (1024 x 4096 x 4096: 18.1 -> 16.5 us, 768 x 4096: 17.5 -> 14.5 us)
            if (fits && rows > 64 && ((tm == 2 && ks == 1) || (tm == 1 && ks < 0 && ncu_hint > 0 && t128 <= ncu_hint)))
                return launch_dma2<MODE, 2, 2, 2, 2>(a, p.M, grouped, st);
        }
        if (tm == 1) return launch_dma2<MODE, 1, 2>(a, p.M, grouped, st);
        // dual path, one problem: 128x256 tiles on eight wavefronts (64x64 each) beat two resident
        // workgroups of 128x128 by 4 % when they still give every CU a tile (8192x1024x4096: 29.1
        // against 30.3 us); the 8-bit modes gain nothing from them
        if constexpr (MODE == MODE_DUAL) {
            if (!grouped && ((p.M + 127) / 128) * ((p.N + 255) / 256) >= 256)
                return launch_dma2<MODE, 2, 2, 4>(a, p.M, grouped, st);
        }
        return launch_dma2<MODE, 2, 2>(a, p.M, grouped, st);
    }
    if constexpr (MODE == MODE_MX8) {
        return fail(OSC_ERR_UNSUPPORTED, "mxfp8 gemm: no kernel for this shape");
    } else {
    if (ragged) {
        if (tm == 1) return launch_cfg<MODE, 1, 2, true>(a, p.M, grouped, st);
        return launch_cfg<MODE, 2, 2, true>(a, p.M, grouped, st);
    }
    if (tm == 1) return launch_cfg<MODE, 1, 2, false>(a, p.M, grouped, st);
    return launch_cfg<MODE, 2, 2, false>(a, p.M, grouped, st);
    }
}

int launch_dual_gemm(const GemmProblem& p, hipStream_t st) { return launch_gemm<MODE_DUAL>(p, st); }
int launch_fp8_gemm(const GemmProblem& p, hipStream_t st) { return launch_gemm<MODE_FP8>(p, st); }
int launch_mxfp8_gemm(const GemmProblem& p, hipStream_t st) { return launch_gemm<MODE_MX8>(p, st); }

}  // namespace osc
