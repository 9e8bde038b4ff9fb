// Dual-path GEMM (Section 3.3.1, Eq. dual-path) and FP8 W8A8 GEMM (Section 3.4) on the CDNA4
// matrix cores, single and grouped (mixture-of-experts) forms.
//
// One kernel skeleton serves all of them.  Every operand is seen as a row-major byte matrix
// whose rows run along the reduction axis (FP4 codes: K/2 bytes per row, FP8 codes: K bytes,
// bf16 branch: 2*K_o bytes); the reduction axis is consumed 128 bytes per row per step.
//
// Matrix-core operand layout used (32x32 tiles, 64-lane wavefront, lane = 32*q + r):
//   v_mfma_scale_f32_32x32x64_f8f6f4, FP4: lane holds row r, 32 consecutive elements (16 bytes) of
//     reduction block q and, in one byte of its scale register picked by op_sel, their E8M0 scale.
//   v_mfma_f32_32x32x16_bf16: lane holds row r, 8 consecutive bf16 (16 bytes) of block q.
//   Result register i of lane (q, r'): row 8*(i/4) + 4*q + i%4, column r'.
// The hardware only pairs lane-block q of A with lane-block q of B, so the order in which the
// reduction axis is dealt to (q, instruction) is free as long as both operands agree.  Here
// the 128-byte step is split in two 64-byte halves, half q goes to lanes of block q, and the
// i-th 16-byte piece of the half feeds the i-th of four MFMAs.  For FP4 the four scale bytes of
// those pieces are then one aligned 32-bit word of the canonical [rows, K/32] scale matrix.
#include "osc_internal.h"

namespace osc {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int GT = 256;  // 4 wavefronts, arranged 2 x 2 over the workgroup tile
enum { MODE_DUAL = 0, MODE_FP8 = 1 };

struct KArgs {
    const uint8_t* Xq;
    const uint8_t* Xs;
    const float* xs;
    const uint16_t* B;
    int64_t ldb;
    const int32_t* row_map;
    const int32_t* off;
    int E;
    const uint8_t* Wpack;
    size_t pack_stride, off_q, off_s, off_l;
    int64_t ldwl;
    int M, N, K, K_o;
    void* Y;
    int y_bf16;
    int64_t ldy;
    int tiles_n;
};

// 16-byte piece `c` (0..7) of row `r` sits at piece c ^ swz(r): lanes of one LDS access
// (consecutive rows, same piece) then spread over all banks.
__device__ __forceinline__ int swz(int r) { return (r & 7) ^ ((r >> 3) & 1); }
__device__ __forceinline__ int lds_off(int r, int c) { return r * 128 + ((c ^ swz(r)) << 4); }

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <int MODE, int TM, int TN>
__global__ void __launch_bounds__(GT) gemm_kernel(KArgs a) {
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr int SA = BM / 32, SB = BN / 32;  // 16-byte load slots per thread and step
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    uint8_t* sA = lds;
    uint8_t* sB = lds + BM * 128;

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1, q = lane >> 5, r = lane & 31;

    // ---- which tile -----------------------------------------------------------------
    // Workgroups are dealt round-robin to the 8 XCDs; renumber so that each XCD owns a
    // contiguous run of tiles and its L2 sees neighbouring tiles.
    int tile = blockIdx.x;
    {
        const int per = gridDim.x >> 3;
        if (tile < (per << 3)) tile = (tile & 7) * per + (tile >> 3);
    }
    int row_begin = 0, row_end = a.M, tm_idx, tn_idx;
    const uint8_t* wp = a.Wpack;
    if (a.off) {  // grouped: m-tiles are numbered expert by expert
        tn_idx = tile % a.tiles_n;
        int j = tile / a.tiles_n, e = 0;
        for (; e < a.E; ++e) {
            const int b = a.off[e], n = a.off[e + 1] - b;
            const int te = (n + BM - 1) / BM;
            if (j < te) {
                row_begin = b;
                row_end = b + n;
                break;
            }
            j -= te;
        }
        if (e == a.E) return;  // surplus workgroup of the upper-bound grid
        tm_idx = j;
        wp += (size_t)e * a.pack_stride;
    } else {
        const int tiles_m = (a.M + BM - 1) / BM;
        const int band = tile / (8 * a.tiles_n), within = tile - band * 8 * a.tiles_n;
        const int rows = min(8, tiles_m - band * 8);
        tm_idx = band * 8 + within % rows;
        tn_idx = within / rows;
    }
    const int m0 = row_begin + tm_idx * BM, n0 = tn_idx * BN;

    // ---- per-thread source rows for the global -> LDS copies ------------------------------
    int arow[SA], brow[SB];
#pragma unroll
    for (int i = 0; i < SA; ++i) {
        int g = min(m0 + ((t + GT * i) >> 3), row_end - 1);
        arow[i] = (MODE == MODE_DUAL && a.row_map) ? a.row_map[g] : g;
    }
#pragma unroll
    for (int i = 0; i < SB; ++i) brow[i] = min(n0 + ((t + GT * i) >> 3), a.N - 1);
    const int c8 = t & 7;

    // rows whose fragments this lane feeds to the matrix cores
    int frow_a[TM], frow_b[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        int g = min(m0 + wm * (TM * 32) + i * 32 + r, row_end - 1);
        frow_a[i] = (MODE == MODE_DUAL && a.row_map) ? a.row_map[g] : g;
    }
#pragma unroll
    for (int i = 0; i < TN; ++i) frow_b[i] = min(n0 + wn * (TN * 32) + i * 32 + r, a.N - 1);

    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int k = 0; k < 16; ++k) acc[i][j][k] = 0.0f;

    u32x4 ra[SA], rb[SB];
    const u32x4 zero4 = {0u, 0u, 0u, 0u};

    auto gload = [&](const uint8_t* abase, int64_t apitch, int64_t avalid, const uint8_t* bbase,
                     int64_t bpitch, int64_t bvalid, int T) {
        const int64_t o = (int64_t)T * 128 + c8 * 16;
#pragma unroll
        for (int i = 0; i < SA; ++i)
            ra[i] = (o < avalid) ? *reinterpret_cast<const u32x4*>(abase + arow[i] * apitch + o) : zero4;
#pragma unroll
        for (int i = 0; i < SB; ++i)
            rb[i] = (o < bvalid) ? *reinterpret_cast<const u32x4*>(bbase + brow[i] * bpitch + o) : zero4;
    };
    auto lstore = [&]() {
#pragma unroll
        for (int i = 0; i < SA; ++i)
            *reinterpret_cast<u32x4*>(sA + lds_off((t + GT * i) >> 3, c8)) = ra[i];
#pragma unroll
        for (int i = 0; i < SB; ++i)
            *reinterpret_cast<u32x4*>(sB + lds_off((t + GT * i) >> 3, c8)) = rb[i];
    };
    auto frag = [&](const uint8_t* s, int row, int piece) {
        return *reinterpret_cast<const u32x4*>(s + lds_off(row, piece));
    };

    if (MODE == MODE_DUAL) {
        // ---- Path A: block-scaled FP4 ------------------------------------------------------
        const int Kg = a.K >> 5;
        const int64_t rowbytes = a.K >> 1;
        const int nA = (int)((rowbytes + 127) >> 7);
        const uint8_t* wq = wp + a.off_q;
        const uint8_t* ws = wp + a.off_s;
        const bool word_ok = (Kg & 3) == 0;
        auto scale_word = [&](const uint8_t* base, int row, int T) -> int {
            const int g0 = 8 * T + 4 * q;
            const uint8_t* p = base + (int64_t)row * Kg + g0;
            if (word_ok && g0 + 4 <= Kg) return *reinterpret_cast<const int*>(p);
            int v = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (g0 + k < Kg) v |= (int)p[k] << (8 * k);
            return v;
        };
        int sa_n[TM], sb_n[TN];
        gload(a.Xq, rowbytes, rowbytes, wq, rowbytes, rowbytes, 0);
#pragma unroll
        for (int i = 0; i < TM; ++i) sa_n[i] = scale_word(a.Xs, frow_a[i], 0);
#pragma unroll
        for (int i = 0; i < TN; ++i) sb_n[i] = scale_word(ws, frow_b[i], 0);
        for (int T = 0; T < nA; ++T) {
            int sa[TM], sb[TN];
            __syncthreads();
            lstore();
#pragma unroll
            for (int i = 0; i < TM; ++i) sa[i] = sa_n[i];
#pragma unroll
            for (int i = 0; i < TN; ++i) sb[i] = sb_n[i];
            __syncthreads();
            if (T + 1 < nA) {
                gload(a.Xq, rowbytes, rowbytes, wq, rowbytes, rowbytes, T + 1);
#pragma unroll
                for (int i = 0; i < TM; ++i) sa_n[i] = scale_word(a.Xs, frow_a[i], T + 1);
#pragma unroll
                for (int i = 0; i < TN; ++i) sb_n[i] = scale_word(ws, frow_b[i], T + 1);
            }
#define OSC_FP4_STEP(I)                                                                          \
    {                                                                                            \
        u32x4 fa[TM], fb[TN];                                                                    \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) fa[i] =                                   \
            frag(sA, wm * (TM * 32) + i * 32 + r, 4 * q + I);                                    \
        _Pragma("unroll") for (int j = 0; j < TN; ++j) fb[j] =                                   \
            frag(sB, wn * (TN * 32) + j * 32 + r, 4 * q + I);                                    \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) {                                         \
            const v8i av = {(int)fa[i].x, (int)fa[i].y, (int)fa[i].z, (int)fa[i].w, 0, 0, 0, 0}; \
            _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                     \
                const v8i bv = {(int)fb[j].x, (int)fb[j].y, (int)fb[j].z, (int)fb[j].w,          \
                                0,            0,            0,            0};                    \
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(                     \
                    av, bv, acc[i][j], 4, 4, I, sa[i], I, sb[j]);                                \
            }                                                                                    \
        }                                                                                        \
    }
            OSC_FP4_STEP(0)
            OSC_FP4_STEP(1)
            OSC_FP4_STEP(2)
            OSC_FP4_STEP(3)
#undef OSC_FP4_STEP
        }
        // ---- Path B: bf16 branch into the same accumulators --------------------------------
        if (a.K_o > 0) {
            const uint8_t* bsrc = reinterpret_cast<const uint8_t*>(a.B);
            const uint8_t* wl = wp + a.off_l;
            const int64_t ab = a.ldb * 2, wb = a.ldwl * 2;
            const int nB = (int)(((int64_t)a.K_o * 2 + 127) >> 7);
            gload(bsrc, ab, ab, wl, wb, wb, 0);
            for (int T = 0; T < nB; ++T) {
                __syncthreads();
                lstore();
                __syncthreads();
                if (T + 1 < nB) gload(bsrc, ab, ab, wl, wb, wb, T + 1);
#pragma unroll
                for (int I = 0; I < 4; ++I) {
                    u32x4 fa[TM], fb[TN];
#pragma unroll
                    for (int i = 0; i < TM; ++i) fa[i] = frag(sA, wm * (TM * 32) + i * 32 + r, 4 * q + I);
#pragma unroll
                    for (int j = 0; j < TN; ++j) fb[j] = frag(sB, wn * (TN * 32) + j * 32 + r, 4 * q + I);
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                __builtin_bit_cast(v8bf, fa[i]), __builtin_bit_cast(v8bf, fb[j]),
                                acc[i][j], 0, 0, 0);
                }
            }
        }
    } else {
        // ---- FP8: e4m3 x e4m3, unit block scales; row/column scales applied at the end -------
        const int64_t rowbytes = a.K;
        const int nA = (int)((rowbytes + 127) >> 7);
        const uint8_t* w8 = wp + a.off_q;
        gload(a.Xq, rowbytes, rowbytes, w8, rowbytes, rowbytes, 0);
        for (int T = 0; T < nA; ++T) {
            __syncthreads();
            lstore();
            __syncthreads();
            if (T + 1 < nA) gload(a.Xq, rowbytes, rowbytes, w8, rowbytes, rowbytes, T + 1);
#pragma unroll
            for (int I = 0; I < 2; ++I) {
                v8i fa[TM], fb[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    u32x4 lo = frag(sA, wm * (TM * 32) + i * 32 + r, 4 * q + 2 * I);
                    u32x4 hi = frag(sA, wm * (TM * 32) + i * 32 + r, 4 * q + 2 * I + 1);
                    fa[i] = (v8i){(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w,
                                  (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
                }
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    u32x4 lo = frag(sB, wn * (TN * 32) + j * 32 + r, 4 * q + 2 * I);
                    u32x4 hi = frag(sB, wn * (TN * 32) + j * 32 + r, 4 * q + 2 * I + 1);
                    fb[j] = (v8i){(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w,
                                  (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
                }
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                            fa[i], fb[j], acc[i][j], 0, 0, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
            }
        }
    }

    // ---- epilogue ---------------------------------------------------------------------------
    const float* wsc = (MODE == MODE_FP8) ? reinterpret_cast<const float*>(wp + a.off_s) : nullptr;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn * (TN * 32) + j * 32 + r;
            float cs = 1.0f;
            if (MODE == MODE_FP8 && col < a.N) cs = wsc[col];
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                const int row = m0 + wm * (TM * 32) + i * 32 + 8 * (k >> 2) + 4 * q + (k & 3);
                if (row < row_end && col < a.N) {
                    float v = acc[i][j][k];
                    if (MODE == MODE_FP8) v *= a.xs[row] * cs;
                    if (a.y_bf16)
                        reinterpret_cast<uint16_t*>(a.Y)[(int64_t)row * a.ldy + col] = f32_to_bf16_rne(v);
                    else
                        reinterpret_cast<float*>(a.Y)[(int64_t)row * a.ldy + col] = v;
                }
            }
        }
    }
}

template <int MODE, int TM, int TN>
static int launch_cfg(const KArgs& a, int tiles_m, hipStream_t st) {
    constexpr int BM = 64 * TM, BN = 64 * TN;
    const size_t smem = (size_t)(BM + BN) * 128;
    const int64_t grid = (int64_t)tiles_m * a.tiles_n;
    if (grid <= 0) return OSC_OK;
    if (grid > 0x7fffffff) return fail(OSC_ERR_UNSUPPORTED, "gemm: too many tiles");
    auto kern = gemm_kernel<MODE, TM, TN>;
    if (smem > 64 * 1024) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
            return fail(OSC_ERR_HIP, "gemm: cannot reserve %zu bytes of LDS", smem);
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(GT), smem, st, a);
    return check_launch("gemm_kernel");
}

template <int MODE>
static int launch_gemm(const GemmProblem& p, hipStream_t st) {
    KArgs a;
    a.Xq = p.Xq;
    a.Xs = p.Xs;
    a.xs = p.xs;
    a.B = p.B;
    a.ldb = p.ldb;
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
        a.ldwl = L.ldwl;
    } else {
        Pack8Layout L = pack8_layout(p.N, p.K);
        a.off_q = L.off_w;
        a.off_s = L.off_s;
        a.off_l = 0;
        a.ldwl = 0;
    }
    a.M = (int)p.M;
    a.N = (int)p.N;
    a.K = (int)p.K;
    a.K_o = p.K_o;
    a.Y = p.Y;
    a.y_bf16 = p.y_dtype == OSC_DT_BF16;
    a.ldy = p.ldy;
    // Tile choice: 128x128 workgroup tiles by default, 64-row tiles for short problems.
    const bool grouped = p.expert_offsets != nullptr;
    auto tiles_m_for = [&](int BM) -> int {
        int64_t tm = (p.M + BM - 1) / BM;
        if (grouped) tm += p.E;  // upper bound: every expert may add one ragged tile
        return (int)tm;
    };
    const int64_t rows = grouped && p.E > 0 ? (p.M + p.E - 1) / p.E : p.M;
    if (rows <= 64) {
        a.tiles_n = (int)((p.N + 127) / 128);
        return launch_cfg<MODE, 1, 2>(a, tiles_m_for(64), st);
    }
    a.tiles_n = (int)((p.N + 127) / 128);
    return launch_cfg<MODE, 2, 2>(a, tiles_m_for(128), st);
}

int launch_dual_gemm(const GemmProblem& p, hipStream_t st) { return launch_gemm<MODE_DUAL>(p, st); }
int launch_fp8_gemm(const GemmProblem& p, hipStream_t st) { return launch_gemm<MODE_FP8>(p, st); }

}  // namespace osc
