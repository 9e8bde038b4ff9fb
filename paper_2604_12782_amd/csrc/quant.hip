// Activation quantisers: OSC-enhanced MXFP4 (Section 3.2, Alg. 2) and per-token FP8 (Section 3.4).
// Both are HBM-bandwidth-bound row kernels: one workgroup walks whole rows with 16-byte loads.
#include "osc_internal.h"
#include "wave_util.h"

namespace osc {

typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int QT = 256;  // threads per workgroup

// ------------------------------------------------------------------------------------------
// MXFP4 + outlier gather.
//
// A row is cut into 16-byte chunks of 8 channels and into segments of 128 chunks (1024
// channels).  One wavefront converts one segment of one row at a time, two chunks per lane:
// chunk c of the segment belongs to lane c % 64, the four chunks of a 32-channel group sit in
// one quad of lanes (the group's amax is two DPP steps) and the sixteen chunks of four groups in
// one DPP row (their four scale codes leave as one 32-bit word of the row-block-major layout).
// The four wavefronts of a workgroup never wait for each other inside the loop.
//
// The suppression list becomes, once per workgroup, a table of AND masks (one 32-bit word per
// channel pair; zeroing protected channels is four ANDs per chunk, no branch) and the list of
// B columns that each segment owns (the list is ascending, so a segment owns a contiguous run).
// Every wavefront parks its raw segment in its own LDS strip; the lanes then pick the
// protected channels out of the strip and store the run of B columns themselves.
//
// Work is dealt so that the workgroups which the hardware places on one XCD hold 32 consecutive
// rows at a time: the 4-byte scale words of those rows share 128-byte lines and meet in that
// XCD's L2 before they are written back.
// ------------------------------------------------------------------------------------------
//
// GS is the size of a scale group: 32, or 64 (one more exchange: the two quads that hold a group
// of 64 agree on the larger amax, and its code is written for both of the group's blocks of 32).
template <int GS>
__global__ void __launch_bounds__(QT) quant_mxfp4_osc_kernel(
    const uint16_t* __restrict__ X, int M, int K, int64_t ldx, const int32_t* __restrict__ oidx,
    int K_o, uint8_t* __restrict__ Xq, uint8_t* __restrict__ Xs, uint16_t* __restrict__ B,
    int64_t ldb, int nseg, int total_wg) {
    extern __shared__ uint32_t smem[];
    const int Kg = K >> 5, Kg4 = (Kg + 3) >> 2;
    const int nchunk = K >> 3;
    const int t = threadIdx.x, lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);  // uniform: row and segment arithmetic stays on the scalar unit
    // LDS: strips [4][SEG_CHUNKS] x 16 B | keep [K/2] words | colstart [nseg+1] | oidx16 [K_o]
    u32x4* strip = reinterpret_cast<u32x4*>(smem) + wave * SEG_CHUNKS;
    uint32_t* keep = smem + 4 * SEG_CHUNKS * 4;
    int* colstart = reinterpret_cast<int*>(keep + (K >> 1));
    uint16_t* och = reinterpret_cast<uint16_t*>(colstart + nseg + 1);

    int wg = blockIdx.x;
    QItem cur = wg < total_wg ? quant_item(wg, wave, nseg, M) : QItem{-1, 0};
    u32x4 v0 = {0u, 0u, 0u, 0u}, v1 = {0u, 0u, 0u, 0u};
#define OSC_Q_LOAD(A0_, A1_, IT_)                                                              \
    do {                                                                                       \
        A0_ = (u32x4){0u, 0u, 0u, 0u};                                                         \
        A1_ = (u32x4){0u, 0u, 0u, 0u};                                                         \
        if ((IT_).m >= 0) {                                                                    \
            const u32x4* src_ = reinterpret_cast<const u32x4*>(X + (int64_t)(IT_).m * ldx);    \
            const int c_ = (IT_).seg * SEG_CHUNKS + lane;                                      \
            if (c_ < nchunk) A0_ = __builtin_nontemporal_load(src_ + c_);                      \
            if (c_ + 64 < nchunk) A1_ = __builtin_nontemporal_load(src_ + c_ + 64);            \
        }                                                                                      \
    } while (0)
    OSC_Q_LOAD(v0, v1, cur);  // in flight during the set-up

    if (K_o > 0) {
        for (int i = t; i < (K >> 1); i += QT) keep[i] = 0xffffffffu;
        __syncthreads();
        for (int o = t; o < K_o; o += QT) {
            const int c = oidx[o];
            const int prev = o ? oidx[o - 1] : -1;
            if (c >= 0 && c < K) atomicAnd(&keep[c >> 1], (c & 1) ? 0x0000ffffu : 0xffff0000u);
            och[o] = (uint16_t)c;
            // segments that start between the previous listed channel and this one start here
            for (int sgm = (prev < 0 ? -1 : prev / SEG_CH) + 1; sgm <= c / SEG_CH && sgm <= nseg; ++sgm)
                colstart[sgm] = o;
            if (o == K_o - 1)
                for (int sgm = c / SEG_CH + 1; sgm <= nseg; ++sgm) colstart[sgm] = K_o;
        }
        __syncthreads();
    }

    while (wg < total_wg) {
        const int wgn = wg + gridDim.x;
        const QItem nxt = wgn < total_wg ? quant_item(wgn, wave, nseg, M) : QItem{-1, 0};
        u32x4 n0, n1;
        OSC_Q_LOAD(n0, n1, nxt);  // next trip's loads fly while this one is converted
        if (cur.m >= 0) {
            const int m = cur.m;
            const int cbase = cur.seg * SEG_CHUNKS;
            uint32_t* dst = reinterpret_cast<uint32_t*>(Xq + (int64_t)m * (K >> 1));
            uint8_t* sdst = Xs + (int64_t)(m >> 5) * Kg4 * 128 + (m & 31) * 4;
            if (K_o > 0) {
                strip[lane] = v0;
                strip[lane + 64] = v1;
            }
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int c = cbase + lane + 64 * i;
                u32x4 w = i ? v1 : v0;
                if (K_o > 0 && c < nchunk) {  // steps 2-3 of Section 3.2: (back-up is the strip) zero
                    const u32x4 kp = *reinterpret_cast<const u32x4*>(keep + 4 * c);
                    w &= kp;
                }
                // amax of the group on bit patterns: for finite bf16 |x| orders like bits & 0x7fff
                u32x4 ab = w & 0x7fff7fffu;
                uint32_t a = max(max(ab.x & 0xffffu, ab.x >> 16), max(ab.y & 0xffffu, ab.y >> 16));
                a = max(a, max(max(ab.z & 0xffffu, ab.z >> 16), max(ab.w & 0xffffu, ab.w >> 16)));
                a = max(a, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)a, 0xB1, 0xF, 0xF, false));  // lane ^ 1
                a = max(a, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)a, 0x4E, 0xF, 0xF, false));  // lane ^ 2
                if (GS == 64)  // lane 7 - l of the same eight lanes sits in the group's other quad
                    a = max(a, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)a, 0x141, 0xF, 0xF, false));
                // shared exponent floor(log2 amax) - 2, clamped below: E8M0 code = max(E - 2, 0)
                const uint32_t code = (uint32_t)max((int)(a >> 7) - 2, 0);
                // four blocks of 32 (one DPP row of 16 lanes) -> one 32-bit scale word in the row's first lane;
                // chunks past the end of the row hold zeros, so their code is 0
                uint32_t word = code;
                word |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)code, 0x104, 0xF, 0xF, true) << 8;   // lane + 4
                word |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)code, 0x108, 0xF, 0xF, true) << 16;  // lane + 8
                word |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)code, 0x10C, 0xF, 0xF, true) << 24;  // lane + 12
                if ((lane & 15) == 0 && c < nchunk)
                    *reinterpret_cast<uint32_t*>(sdst + (c >> 4) * 128) = word;
                const float scale = __builtin_bit_cast(float, code << 23);
                // (scalars first: a bit cast applied to a vector component reads component 0)
                const uint32_t w0 = w.x, w1 = w.y, w2 = w.z, w3 = w.w;
                uint32_t out = 0;
                out = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(out, __builtin_bit_cast(v2bf, w0), scale, 0);
                out = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(out, __builtin_bit_cast(v2bf, w1), scale, 1);
                out = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(out, __builtin_bit_cast(v2bf, w2), scale, 2);
                out = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(out, __builtin_bit_cast(v2bf, w3), scale, 3);
                if (c < nchunk) __builtin_nontemporal_store(out, dst + c);
            }
            if (K_o > 0) {
                // The strip was written by this wavefront, and LDS runs a wavefront's operations in
                // order; the fences keep the compiler from moving the reads above the writes.
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                const uint16_t* raw = reinterpret_cast<const uint16_t*>(strip);
                uint16_t* brow = B + (int64_t)m * ldb;
                const int o1 = colstart[cur.seg + 1];
                for (int o = colstart[cur.seg] + lane; o < o1; o += 64)
                    brow[o] = raw[(int)och[o] - cur.seg * SEG_CH];
                if (cur.seg == nseg - 1)
                    for (int o = K_o + lane; o < (int)ldb; o += 64) brow[o] = 0;  // padding columns: +0
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
        }
        cur = nxt;
        v0 = n0;
        v1 = n1;
        wg = wgn;
    }
#undef OSC_Q_LOAD
}

// B columns of a table-free call still have to read +0 when the caller passes a buffer.
__global__ void zero_rows_kernel(uint16_t* B, int M, int64_t ldb) {
    int64_t n = (int64_t)M * (ldb >> 3);
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x)
        reinterpret_cast<u32x4*>(B)[i] = (u32x4){0u, 0u, 0u, 0u};
}

int launch_quant_mxfp4(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, const int32_t* oidx,
                       int32_t K_o, uint8_t* Xq, uint8_t* Xs, uint16_t* B, int64_t ldb,
                       hipStream_t st, int group) {
    if (group != 32 && group != 64) return fail(OSC_ERR_UNSUPPORTED, "quantize: scale group %d (32 or 64)", group);
    if (K % group) return fail(OSC_ERR_SHAPE, "quantize: K=%lld is not a multiple of the scale group %d", (long long)K, group);
    if (K > 65536) return fail(OSC_ERR_UNSUPPORTED, "quantize: K=%lld exceeds 65536", (long long)K);
    const int64_t nchunk = K / 8;
    const int nseg = (int)((nchunk + SEG_CHUNKS - 1) / SEG_CHUNKS);
    size_t smem = 4 * SEG_CHUNKS * 16;
    if (K_o > 0) smem += (size_t)(K / 2) * 4 + (size_t)(nseg + 1) * 4 + (size_t)K_o * 2;
    if (smem > 160 * 1024)
        return fail(OSC_ERR_UNSUPPORTED, "quantize: K=%lld with K_o=%d needs %zu bytes of LDS", (long long)K, (int)K_o, smem);
    auto kern = group == 64 ? quant_mxfp4_osc_kernel<64> : quant_mxfp4_osc_kernel<32>;
    if (smem > 48 * 1024) {
        // one flag set per kernel instantiation (scale groups of 32 and of 64)
        static unsigned char lds_done[2][MAX_DEVICES];
        static size_t lds_reserved[2][MAX_DEVICES];
        const int which = group == 64;
        if (int rc = reserve_lds(reinterpret_cast<const void*>(kern), smem, lds_done[which], lds_reserved[which])) return rc;
    }
    // 32-row blocks of 8*nseg workgroups each, dealt to XCDs in groups of eight blocks
    const int64_t blocks = (M + 31) / 32;
    const int64_t total_wg = (blocks + 7) / 8 * 8 * (8 * nseg);
    if (total_wg > 0x7fffffff) return fail(OSC_ERR_UNSUPPORTED, "quantize: M=%lld too large", (long long)M);
    // eight workgroups per compute unit; sixteen when every one of them still gets eight items or more
    // (M = 32768 at K = 4096: 63.1 -> 61.3 us; at M = 8192 the smaller grid is ahead, 17.9 against 18.6 us)
    const int64_t cap = total_wg >= 8 * 4096 ? 4096 : 2048;
    int grid = (int)(total_wg < cap ? total_wg : cap);
    if (K_o == 0 && B && ldb > 0)
        hipLaunchKernelGGL(zero_rows_kernel, dim3(grid), dim3(QT), 0, st, B, (int)M, ldb);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(QT), smem, st, X, (int)M, (int)K, ldx, oidx,
                       (int)K_o, Xq, Xs, B, ldb, nseg, (int)total_wg);
    return check_launch("quant_mxfp4_osc_kernel");
}

// ------------------------------------------------------------------------------------------
// "Dynamic" protection (Section 4.2; Table 3, note 3): the protected element of every group is
// found at run time, token by token.  Same work split as the kernel above, no table: the sort key
// (magnitude bits << 5) | (31 - position) makes "largest magnitude, lowest position" one unsigned
// maximum over the group's quad of lanes; the owning lane moves that element into the dense
// backup row Bd (every lane stores its 16-byte chunk of Bd: zeros but for that element) and
// zeroes it; the rest is quantised as in Alg. 2.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(QT) quant_mxfp4_dynamic_kernel(const uint16_t* __restrict__ X, int M, int K,
                                                                 int64_t ldx, uint8_t* __restrict__ Xq,
                                                                 uint8_t* __restrict__ Xs,
                                                                 uint16_t* __restrict__ Bd, int64_t ldb,
                                                                 uint8_t* __restrict__ idx, int nseg,
                                                                 int total_wg) {
    const int Kg = K >> 5, Kg4 = (Kg + 3) >> 2;
    const int nchunk = K >> 3;
    const int t = threadIdx.x, lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);  // uniform: row and segment arithmetic stays on the scalar unit
    const uint32_t kbase = 31u - (uint32_t)((lane & 3) * 8);
    for (int wg = blockIdx.x; wg < total_wg; wg += gridDim.x) {
        const QItem cur = quant_item(wg, wave, nseg, M);
        if (cur.m < 0) continue;
        const int m = cur.m;
        const u32x4* src = reinterpret_cast<const u32x4*>(X + (int64_t)m * ldx);
        uint32_t* dst = reinterpret_cast<uint32_t*>(Xq + (int64_t)m * (K >> 1));
        uint8_t* sdst = Xs + (int64_t)(m >> 5) * Kg4 * 128 + (m & 31) * 4;
        u32x4* bdst = reinterpret_cast<u32x4*>(Bd + (int64_t)m * ldb);
        u32x4 v[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int c = cur.seg * SEG_CHUNKS + lane + 64 * i;
            v[i] = (u32x4){0u, 0u, 0u, 0u};
            if (c < nchunk) v[i] = __builtin_nontemporal_load(src + c);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int c = cur.seg * SEG_CHUNKS + lane + 64 * i;
            uint32_t w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
            // Eq. 2 at run time: position of the group's largest magnitude
            uint32_t k = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                k = max(k, ((w[e] & 0x7fffu) << 5) | (kbase - 2 * e));
                k = max(k, (((w[e] >> 16) & 0x7fffu) << 5) | (kbase - 2 * e - 1));
            }
            k = max(k, (uint32_t)__builtin_amdgcn_mov_dpp((int)k, 0xB1, 0xF, 0xF, true));  // lane ^ 1
            k = max(k, (uint32_t)__builtin_amdgcn_mov_dpp((int)k, 0x4E, 0xF, 0xF, true));  // lane ^ 2
            const int jstar = 31 - (int)(k & 31u);
            // back-up and zero (steps 2-3 of Section 3.2, with the index of this token)
            uint32_t b[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int p0 = (lane & 3) * 8 + 2 * e;  // position of the low half of word e
                const uint32_t mask = jstar == p0 ? 0x0000ffffu : jstar == p0 + 1 ? 0xffff0000u : 0u;
                b[e] = w[e] & mask;
                w[e] &= ~mask;
            }
            if (c < nchunk) __builtin_nontemporal_store((u32x4){b[0], b[1], b[2], b[3]}, bdst + c);
            // scale of what is left
            const uint32_t a0 = w[0] & 0x7fff7fffu, a1 = w[1] & 0x7fff7fffu, a2 = w[2] & 0x7fff7fffu,
                           a3 = w[3] & 0x7fff7fffu;
            uint32_t a = max(max(a0 & 0xffffu, a0 >> 16), max(a1 & 0xffffu, a1 >> 16));
            a = max(a, max(max(a2 & 0xffffu, a2 >> 16), max(a3 & 0xffffu, a3 >> 16)));
            a = max(a, (uint32_t)__builtin_amdgcn_mov_dpp((int)a, 0xB1, 0xF, 0xF, true));
            a = max(a, (uint32_t)__builtin_amdgcn_mov_dpp((int)a, 0x4E, 0xF, 0xF, true));
            const uint32_t code = (uint32_t)max((int)(a >> 7) - 2, 0);
            uint32_t word = code, iword = (uint32_t)jstar;
            word |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)code, 0x104, 0xF, 0xF, true) << 8;
            word |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)code, 0x108, 0xF, 0xF, true) << 16;
            word |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)code, 0x10C, 0xF, 0xF, true) << 24;
            iword |= (uint32_t)__builtin_amdgcn_update_dpp(0, jstar, 0x104, 0xF, 0xF, true) << 8;
            iword |= (uint32_t)__builtin_amdgcn_update_dpp(0, jstar, 0x108, 0xF, 0xF, true) << 16;
            iword |= (uint32_t)__builtin_amdgcn_update_dpp(0, jstar, 0x10C, 0xF, 0xF, true) << 24;
            if ((lane & 15) == 0 && c < nchunk) {
                *reinterpret_cast<uint32_t*>(sdst + (c >> 4) * 128) = word;
                if (idx) {
                    // four positions of four consecutive groups; a row's last word may be partly past Kg
                    uint8_t* ip = idx + (int64_t)m * Kg + (c >> 2);
                    const int left = Kg - (c >> 2);
                    if (left >= 4 && ((Kg & 3) == 0)) *reinterpret_cast<uint32_t*>(ip) = iword;
                    else
                        for (int e = 0; e < 4 && e < left; ++e) ip[e] = (uint8_t)(iword >> (8 * e));
                }
            }
            const float scale = __builtin_bit_cast(float, code << 23);
            uint32_t out = 0;
            out = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(out, __builtin_bit_cast(v2bf, w[0]), scale, 0);
            out = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(out, __builtin_bit_cast(v2bf, w[1]), scale, 1);
            out = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(out, __builtin_bit_cast(v2bf, w[2]), scale, 2);
            out = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(out, __builtin_bit_cast(v2bf, w[3]), scale, 3);
            if (c < nchunk) __builtin_nontemporal_store(out, dst + c);
        }
        // padding columns of Bd (ldb > K): +0, written by the wavefront of the last segment
        if (cur.seg == nseg - 1)
            for (int64_t o = K + lane; o < ldb; o += 64) Bd[(int64_t)m * ldb + o] = 0;
    }
}

int launch_quant_mxfp4_dynamic(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, uint8_t* Xq, uint8_t* Xs,
                               uint16_t* Bd, int64_t ldb, uint8_t* idx, hipStream_t st) {
    if (K > 65536) return fail(OSC_ERR_UNSUPPORTED, "quantize: K=%lld exceeds 65536", (long long)K);
    const int64_t nchunk = K / 8;
    const int nseg = (int)((nchunk + SEG_CHUNKS - 1) / SEG_CHUNKS);
    const int64_t blocks = (M + 31) / 32;
    const int64_t total_wg = (blocks + 7) / 8 * 8 * (8 * nseg);
    if (total_wg > 0x7fffffff) return fail(OSC_ERR_UNSUPPORTED, "quantize: M=%lld too large", (long long)M);
    const int64_t cap = 4096;
    const int grid = (int)(total_wg < cap ? total_wg : cap);
    hipLaunchKernelGGL(quant_mxfp4_dynamic_kernel, dim3(grid), dim3(QT), 0, st, X, (int)M, (int)K, ldx, Xq, Xs,
                       Bd, ldb, idx, nseg, (int)total_wg);
    return check_launch("quant_mxfp4_dynamic_kernel");
}

// Row-block-major scales -> plain [rows, K/32].
__global__ void scales_to_rowmajor_kernel(const uint8_t* __restrict__ S, int64_t rows, int Kg,
                                          uint8_t* __restrict__ out) {
    const int Kg4 = (Kg + 3) >> 2;
    const int64_t total = rows * Kg;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t m = i / Kg;
        const int g = (int)(i - m * Kg);
        out[i] = S[((m >> 5) * Kg4 + (g >> 2)) * 128 + (m & 31) * 4 + (g & 3)];
    }
}

int launch_scales_to_rowmajor(const uint8_t* S, int64_t rows, int64_t K, uint8_t* out, hipStream_t st) {
    const int64_t total = rows * (K / 32);
    if (total == 0) return OSC_OK;
    int grid = (int)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
    hipLaunchKernelGGL(scales_to_rowmajor_kernel, dim3(grid), dim3(256), 0, st, S, rows, (int)(K / 32), out);
    return check_launch("scales_to_rowmajor_kernel");
}

// ------------------------------------------------------------------------------------------
// Per-token FP8 (e4m3).  The row lives in registers between the amax reduction and the
// conversion, so X is read once.
// ------------------------------------------------------------------------------------------
template <int CPT>
__global__ void __launch_bounds__(QT) quant_fp8_kernel(const uint16_t* __restrict__ X, int M, int K,
                                                       int64_t ldx, uint8_t* __restrict__ X8,
                                                       float* __restrict__ xs) {
    __shared__ uint32_t red[QT / 64];
    const int t = threadIdx.x;
    const int nchunk = K >> 3;
    for (int m = blockIdx.x; m < M; m += gridDim.x) {
        const u32x4* src = reinterpret_cast<const u32x4*>(X + (int64_t)m * ldx);
        u32x4 v[CPT];
        uint32_t a = 0;
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            int c = t + QT * i;
            if (c < nchunk) {
                v[i] = __builtin_nontemporal_load(src + c);
                uint32_t w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
                for (int k = 0; k < 4; ++k) a = max(a, max(w[k] & 0x7fffu, (w[k] >> 16) & 0x7fffu));
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) a = max(a, (uint32_t)__shfl_xor((int)a, off));
        __syncthreads();  // red[] of the previous row is no longer read
        if ((t & 63) == 0) red[t >> 6] = a;
        __syncthreads();
        a = max(max(red[0], red[1]), max(red[2], red[3]));
        const float amax = __builtin_bit_cast(float, a << 16);
        float scale = 1.0f, inv = 1.0f;
        if (amax >= 0x1p-100f) {
            scale = __fdiv_rn(amax, 448.0f);
            inv = __fdiv_rn(448.0f, amax);
        }
        if (t == 0) xs[m] = scale;
        u32x2* dst = reinterpret_cast<u32x2*>(X8 + (int64_t)m * K);
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            int c = t + QT * i;
            if (c < nchunk) {
                uint32_t w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
                float p[8];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    float lo = __builtin_bit_cast(float, w[k] << 16);
                    float hi = __builtin_bit_cast(float, w[k] & 0xffff0000u);
                    // one rounded multiply each; the clamp realises saturation at +-448
                    p[2 * k] = fminf(fmaxf(__fmul_rn(lo, inv), -448.0f), 448.0f);
                    p[2 * k + 1] = fminf(fmaxf(__fmul_rn(hi, inv), -448.0f), 448.0f);
                }
                int r0 = 0, r1 = 0;
                r0 = __builtin_amdgcn_cvt_pk_fp8_f32(p[0], p[1], r0, false);
                r0 = __builtin_amdgcn_cvt_pk_fp8_f32(p[2], p[3], r0, true);
                r1 = __builtin_amdgcn_cvt_pk_fp8_f32(p[4], p[5], r1, false);
                r1 = __builtin_amdgcn_cvt_pk_fp8_f32(p[6], p[7], r1, true);
                __builtin_nontemporal_store((u32x2){(uint32_t)r0, (uint32_t)r1}, dst + c);
            }
        }
    }
}

int launch_quant_fp8(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, uint8_t* X8, float* xs,
                     hipStream_t st) {
    const int64_t nchunk = K / 8;
    const int cpt = (int)((nchunk + QT - 1) / QT);
    int grid = (int)(M < 4096 ? M : 4096);
#define OSC_QLAUNCH(C) \
    hipLaunchKernelGGL(quant_fp8_kernel<C>, dim3(grid), dim3(QT), 0, st, X, (int)M, (int)K, ldx, X8, xs)
    if (cpt <= 1) OSC_QLAUNCH(1);
    else if (cpt <= 2) OSC_QLAUNCH(2);
    else if (cpt <= 4) OSC_QLAUNCH(4);
    else if (cpt <= 8) OSC_QLAUNCH(8);
    else if (cpt <= 16) OSC_QLAUNCH(16);
    else return fail(OSC_ERR_UNSUPPORTED, "fp8 quantize: K=%lld exceeds 32768", (long long)K);
#undef OSC_QLAUNCH
    return check_launch("quant_fp8_kernel");
}

// ------------------------------------------------------------------------------------------
// MXFP8 (E4M3 elements, one E8M0 scale per 32 channels): the 8-bit micro-scaling form of the W_2
// fallback (Section 3.4; Section 4.1, implementation details).  Same work split as the MXFP4
// kernel (one wavefront per 1024-channel segment of a row, no barriers), no table.  Scale
// exponent floor(log2 amax) - 8 in integer arithmetic on the bf16 exponent field; elements are
// x * 2^-e (exact), clamped to +-448 (the conversion instruction does not saturate) and rounded to
// nearest even by v_cvt_pk_fp8_f32.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(QT) quant_mxfp8_kernel(const uint16_t* __restrict__ X, int M, int K,
                                                         int64_t ldx, uint8_t* __restrict__ Xq,
                                                         uint8_t* __restrict__ Xs, int nseg, int total_wg) {
    const int Kg = K >> 5, Kg4 = (Kg + 3) >> 2;
    const int nchunk = K >> 3;
    const int t = threadIdx.x, lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);  // uniform: row and segment arithmetic stays on the scalar unit
    for (int wg = blockIdx.x; wg < total_wg; wg += gridDim.x) {
        const QItem it = quant_item(wg, wave, nseg, M);
        if (it.m < 0) continue;  // uniform over the wavefront
        const int m = it.m;
        const u32x4* src = reinterpret_cast<const u32x4*>(X + (int64_t)m * ldx);
        const int c0 = it.seg * SEG_CHUNKS + lane;
        u32x4 v[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};
        if (c0 < nchunk) v[0] = __builtin_nontemporal_load(src + c0);
        if (c0 + 64 < nchunk) v[1] = __builtin_nontemporal_load(src + c0 + 64);
        u32x2* dst = reinterpret_cast<u32x2*>(Xq + (int64_t)m * K);
        uint8_t* sdst = Xs + (int64_t)(m >> 5) * Kg4 * 128 + (m & 31) * 4;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int c = c0 + 64 * i;
            const u32x4 w = v[i];
            const u32x4 ab = w & 0x7fff7fffu;
            uint32_t a = max(max(ab.x & 0xffffu, ab.x >> 16), max(ab.y & 0xffffu, ab.y >> 16));
            a = max(a, max(max(ab.z & 0xffffu, ab.z >> 16), max(ab.w & 0xffffu, ab.w >> 16)));
            a = max(a, (uint32_t)__builtin_amdgcn_mov_dpp((int)a, 0xB1, 0xF, 0xF, true));  // lane ^ 1
            a = max(a, (uint32_t)__builtin_amdgcn_mov_dpp((int)a, 0x4E, 0xF, 0xF, true));  // lane ^ 2
            const uint32_t code = (uint32_t)max((int)(a >> 7) - 8, 0);  // E8M0 code = max(E - 8, 0)
            uint32_t word = code;
            word |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)code, 0x104, 0xF, 0xF, true) << 8;   // lane + 4
            word |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)code, 0x108, 0xF, 0xF, true) << 16;  // lane + 8
            word |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)code, 0x10C, 0xF, 0xF, true) << 24;  // lane + 12
            if ((lane & 15) == 0 && c < nchunk) *reinterpret_cast<uint32_t*>(sdst + (c >> 4) * 128) = word;
            // 2^-(code - 127): exponent field 254 - code (8 .. 254)
            const float inv = __builtin_bit_cast(float, (254u - code) << 23);
            const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
            float p[8];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float lo = __builtin_bit_cast(float, ww[k] << 16);
                const float hi = __builtin_bit_cast(float, ww[k] & 0xffff0000u);
                p[2 * k] = fminf(fmaxf(__fmul_rn(lo, inv), -448.0f), 448.0f);
                p[2 * k + 1] = fminf(fmaxf(__fmul_rn(hi, inv), -448.0f), 448.0f);
            }
            int r0 = 0, r1 = 0;
            r0 = __builtin_amdgcn_cvt_pk_fp8_f32(p[0], p[1], r0, false);
            r0 = __builtin_amdgcn_cvt_pk_fp8_f32(p[2], p[3], r0, true);
            r1 = __builtin_amdgcn_cvt_pk_fp8_f32(p[4], p[5], r1, false);
            r1 = __builtin_amdgcn_cvt_pk_fp8_f32(p[6], p[7], r1, true);
            if (c < nchunk) __builtin_nontemporal_store((u32x2){(uint32_t)r0, (uint32_t)r1}, dst + c);
        }
    }
}

int launch_quant_mxfp8(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, uint8_t* Xq, uint8_t* Xs,
                       hipStream_t st) {
    const int64_t nchunk = K / 8;
    const int nseg = (int)((nchunk + SEG_CHUNKS - 1) / SEG_CHUNKS);
    const int64_t blocks = (M + 31) / 32;
    const int64_t total_wg = (blocks + 7) / 8 * 8 * (8 * nseg);
    if (total_wg > 0x7fffffff) return fail(OSC_ERR_UNSUPPORTED, "quantize: M=%lld too large", (long long)M);
    const int grid = (int)(total_wg < 4096 ? total_wg : 4096);
    hipLaunchKernelGGL(quant_mxfp8_kernel, dim3(grid), dim3(QT), 0, st, X, (int)M, (int)K, ldx, Xq, Xs, nseg,
                       (int)total_wg);
    return check_launch("quant_mxfp8_kernel");
}

// ------------------------------------------------------------------------------------------
// Offline: W_L gather.  WLt[n][o] = W[n][oidx[o]], zero padded to ldwl columns.
// ------------------------------------------------------------------------------------------
__global__ void gather_wl_kernel(const uint16_t* __restrict__ W, int64_t N, int64_t ldw,
                                 const int32_t* __restrict__ oidx, int K_o, uint16_t* __restrict__ WLt,
                                 int64_t ldwl) {
    int64_t total = N * ldwl;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        int64_t n = i / ldwl;
        int o = (int)(i - n * ldwl);
        WLt[i] = (o < K_o) ? W[n * ldw + oidx[o]] : (uint16_t)0;
    }
}
__global__ void unpack_wl_kernel(const uint16_t* __restrict__ WLt, int64_t ldwl, int64_t N, int K_o,
                                 uint16_t* __restrict__ WL) {
    int64_t total = (int64_t)K_o * N;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        int64_t o = i / N, n = i - o * N;
        WL[i] = WLt[n * ldwl + o];
    }
}

int launch_gather_wl(const uint16_t* W, int64_t N, int64_t K, int64_t ldw, const int32_t* oidx,
                     int32_t K_o, uint16_t* WLt, int64_t ldwl, hipStream_t st) {
    (void)K;
    if (N * ldwl == 0) return OSC_OK;
    int grid = (int)((N * ldwl + 255) / 256 < 4096 ? (N * ldwl + 255) / 256 : 4096);
    hipLaunchKernelGGL(gather_wl_kernel, dim3(grid), dim3(256), 0, st, W, N, ldw, oidx, (int)K_o, WLt, ldwl);
    return check_launch("gather_wl_kernel");
}
int launch_unpack_wl(const uint16_t* WLt, int64_t ldwl, int64_t N, int32_t K_o, uint16_t* WL,
                     hipStream_t st) {
    if ((int64_t)K_o * N == 0) return OSC_OK;
    int64_t total = (int64_t)K_o * N;
    int grid = (int)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
    hipLaunchKernelGGL(unpack_wl_kernel, dim3(grid), dim3(256), 0, st, WLt, ldwl, N, (int)K_o, WL);
    return check_launch("unpack_wl_kernel");
}

}  // namespace osc
