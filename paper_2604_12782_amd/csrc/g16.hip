// 4-bit formats whose scale group is 16 channels (Section 3.1: G in {16, 32, 64}; Table 2, row
// G = 16; NVFP4 is named in the abstract and the conclusion): the OSC-enhanced quantiser (Alg. 2)
// and the dual-path layer (Eq. dual-path) for
//   format 0: E2M1 elements, one E8M0 scale per 16 channels (shared exponent floor(log2 amax) - 2);
//   format 1: NVFP4 - E2M1 elements, one E4M3 scale per 16 channels, one single-precision scale per
//             tensor, each step one IEEE single-precision operation (see osc.h).
// The matrix core scales blocks of 32 with powers of two only, so neither format can be multiplied
// as 4-bit operands.  What the formats buy is bytes: in the weight-bound (decode) regime of Table 2
// the layer streams 0.56 bytes per weight instead of 1.  The GEMM here is that regime's kernel: the
// 4-bit codes travel through HBM, L2 and LDS as they are and are expanded to bf16 in registers with
// their scale folded in (E2M1 x E8M0 and E2M1 x E4M3 are exact in bf16), then multiplied on the bf16
// (NVFP4: fp16) matrix core into fp32; the tensor scales are applied once, before the bf16 branch is added.
#include "osc_internal.h"
#include "lds_dma.h"
#include "wave_util.h"

namespace osc {

typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int QT16 = 256;

// ------------------------------------------------------------------------------------------
// Quantiser: the work split, the table expansion and the gather of quant_mxfp4_osc_kernel (one
// wavefront per 1024-channel segment of a row, two 16-byte chunks per lane); a block of 16 channels
// is two neighbouring lanes, its scale byte leaves as one of four in a 32-bit word (plain row-major
// [M, K/16], so K must be a multiple of 64).
// ------------------------------------------------------------------------------------------
template <int FMT>
__global__ void __launch_bounds__(QT16) quant_fp4_g16_kernel(
    const uint16_t* __restrict__ X, int M, int K, int64_t ldx, const int32_t* __restrict__ oidx, int K_o, float ts,
    uint8_t* __restrict__ Xq, uint8_t* __restrict__ Xs, uint16_t* __restrict__ B, int64_t ldb, int nseg, int total_wg) {
    extern __shared__ uint32_t smem[];
    const int nchunk = K >> 3;
    const int t = threadIdx.x, lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);
    u32x4* strip = reinterpret_cast<u32x4*>(smem) + wave * SEG_CHUNKS;
    uint32_t* keep = smem + 4 * SEG_CHUNKS * 4;
    int* colstart = reinterpret_cast<int*>(keep + (K >> 1));
    uint16_t* och = reinterpret_cast<uint16_t*>(colstart + nseg + 1);
    if (K_o > 0) {
        for (int i = t; i < (K >> 1); i += QT16) keep[i] = 0xffffffffu;
        for (int i = t; i <= nseg; i += QT16) colstart[i] = K_o;
        __syncthreads();
        for (int o = t; o < K_o; o += QT16) {
            const int c = oidx[o];
            const int prev = o ? oidx[o - 1] : -1;
            if (c >= 0 && c < K) atomicAnd(&keep[c >> 1], (c & 1) ? 0x0000ffffu : 0xffff0000u);
            och[o] = (uint16_t)c;
            for (int sgm = (prev < 0 ? -1 : prev / SEG_CH) + 1; sgm <= c / SEG_CH && sgm <= nseg; ++sgm) colstart[sgm] = o;
        }
        __syncthreads();
    }
    const float d6 = __fmul_rn(6.0f, ts);
    for (int wg = blockIdx.x; wg < total_wg; wg += gridDim.x) {
        const QItem cur = quant_item(wg, wave, nseg, M);
        if (cur.m < 0) continue;
        const int m = cur.m, cbase = cur.seg * SEG_CHUNKS;
        const u32x4* src = reinterpret_cast<const u32x4*>(X + (int64_t)m * ldx);
        uint32_t* dst = reinterpret_cast<uint32_t*>(Xq + (int64_t)m * (K >> 1));
        uint32_t* sdst = reinterpret_cast<uint32_t*>(Xs + (int64_t)m * (K >> 4));
        u32x4 v[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int c = cbase + lane + 64 * i;
            v[i] = (u32x4){0u, 0u, 0u, 0u};
            if (c < nchunk) v[i] = __builtin_nontemporal_load(src + c);
        }
        if (K_o > 0) {
            strip[lane] = v[0];
            strip[lane + 64] = v[1];
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int c = cbase + lane + 64 * i;
            u32x4 w = v[i];
            if (K_o > 0 && c < nchunk) w &= *reinterpret_cast<const u32x4*>(keep + 4 * c);  // steps 2-3 of Section 3.2
            const u32x4 ab = w & 0x7fff7fffu;
            uint32_t a = max(max(ab.x & 0xffffu, ab.x >> 16), max(ab.y & 0xffffu, ab.y >> 16));
            a = max(a, max(max(ab.z & 0xffffu, ab.z >> 16), max(ab.w & 0xffffu, ab.w >> 16)));
            a = max(a, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)a, 0xB1, 0xF, 0xF, false));  // the block's other lane
            uint32_t code, out = 0;
            const uint32_t w4[4] = {w.x, w.y, w.z, w.w};
            if (FMT == 0) {
                code = (uint32_t)max((int)(a >> 7) - 2, 0);
                const float scale = __builtin_bit_cast(float, code << 23);
                out = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(out, __builtin_bit_cast(v2bf, w4[0]), scale, 0);
                out = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(out, __builtin_bit_cast(v2bf, w4[1]), scale, 1);
                out = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(out, __builtin_bit_cast(v2bf, w4[2]), scale, 2);
                out = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(out, __builtin_bit_cast(v2bf, w4[3]), scale, 3);
            } else {
                const float amax = __builtin_bit_cast(float, a << 16);
                const float q = fminf(__fdiv_rn(amax, d6), 448.0f);
                code = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(q, q, 0, false) & 0xffu;
                const float sval = __builtin_amdgcn_cvt_f32_fp8((int)code, 0);
                const float inv = sval == 0.0f ? 0.0f : __fdiv_rn(1.0f, __fmul_rn(ts, sval));
                float lo[4], hi[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    lo[k] = __fmul_rn(__builtin_bit_cast(float, w4[k] << 16), inv);
                    hi[k] = __fmul_rn(__builtin_bit_cast(float, w4[k] & 0xffff0000u), inv);
                }
                out = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(out, lo[0], hi[0], 1.0f, 0);
                out = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(out, lo[1], hi[1], 1.0f, 1);
                out = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(out, lo[2], hi[2], 1.0f, 2);
                out = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(out, lo[3], hi[3], 1.0f, 3);
            }
            // four blocks (eight lanes) -> one 32-bit word in the first of the eight lanes
            uint32_t word = code;
            word |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)code, 0x102, 0xF, 0xF, true) << 8;   // lane + 2
            word |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)code, 0x104, 0xF, 0xF, true) << 16;  // lane + 4
            word |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)code, 0x106, 0xF, 0xF, true) << 24;  // lane + 6
            if ((lane & 7) == 0 && c < nchunk) sdst[c >> 3] = word;
            if (c < nchunk) __builtin_nontemporal_store(out, dst + c);
        }
        if (B) {
            uint16_t* brow = B + (int64_t)m * ldb;
            if (K_o > 0) {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                const uint16_t* raw = reinterpret_cast<const uint16_t*>(strip);
                const int o1 = colstart[cur.seg + 1];
                for (int o = colstart[cur.seg] + lane; o < o1; o += 64) brow[o] = raw[(int)och[o] - cur.seg * SEG_CH];
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
            if (cur.seg == nseg - 1)
                for (int o = K_o + lane; o < (int)ldb; o += 64) brow[o] = 0;  // padding columns: +0
        }
    }
}

int launch_quant_fp4_g16(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, const int32_t* oidx, int32_t K_o, int fmt,
                         float ts, uint8_t* Xq, uint8_t* Xs, uint16_t* B, int64_t ldb, hipStream_t st) {
    const int64_t nchunk = K / 8;
    const int nseg = (int)((nchunk + SEG_CHUNKS - 1) / SEG_CHUNKS);
    size_t smem = 4 * SEG_CHUNKS * 16;
    if (K_o > 0) smem += (size_t)(K / 2) * 4 + (size_t)(nseg + 1) * 4 + (size_t)K_o * 2;
    if (smem > 160 * 1024)
        return fail(OSC_ERR_UNSUPPORTED, "quantize: K=%lld with K_o=%d needs %zu bytes of LDS", (long long)K, (int)K_o, smem);
    auto kern = fmt == 0 ? quant_fp4_g16_kernel<0> : quant_fp4_g16_kernel<1>;
    if (smem > 48 * 1024) {
        static unsigned char lds_done[2][MAX_DEVICES];
        static size_t lds_reserved[2][MAX_DEVICES];
        if (int rc = reserve_lds(reinterpret_cast<const void*>(kern), smem, lds_done[fmt], lds_reserved[fmt])) return rc;
    }
    const int64_t blocks = (M + 31) / 32;
    const int64_t total_wg = (blocks + 7) / 8 * 8 * (8 * nseg);
    if (total_wg > 0x7fffffff) return fail(OSC_ERR_UNSUPPORTED, "quantize: M=%lld too large", (long long)M);
    const int grid = (int)(total_wg < 2048 ? total_wg : 2048);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(QT16), smem, st, X, (int)M, (int)K, ldx, oidx, (int)K_o, ts, Xq, Xs, B, ldb,
                       nseg, (int)total_wg);
    return check_launch("quant_fp4_g16_kernel");
}

// ------------------------------------------------------------------------------------------
// Streaming GEMM.  One workgroup per 32 output channels and 32 rows of X; its wavefronts take the
// 128-byte lines of the reduction axis in turn (256 four-bit channels = 16 scale blocks per row and
// line, then the bf16 lines of the branch) and never synchronise until the end.  A wavefront moves
// a line global -> LDS by DMA into a strip of its own (codes in whole 128-byte lines, the 16 scale
// bytes of every row beside them), expands it in registers and multiplies.
// K order inside a line: the bf16 matrix core pairs lane half q of one operand with lane half q of
// the other, nothing else, so a lane takes the 16 contiguous bytes [32j + 16q, +16) of its row for
// the four MFMAs 4j .. 4j+3 (dword t feeds MFMA 4j+t); those 32 channels are scale blocks 4j+2q and
// 4j+2q+1, applied during the expansion.
// ------------------------------------------------------------------------------------------
template <int FMT>
__device__ __forceinline__ float scale16_f32(uint32_t byte) {
    if (FMT == 0) return __builtin_bit_cast(float, byte ? byte << 23 : 0x00400000u);  // 2^(byte - 127)
    return __builtin_amdgcn_cvt_f32_fp8((int)byte, 0);
}
// Expansion of 16 bytes of codes (32 channels, scale blocks s0 | s1) into four operand registers
// sets of 8 values each, the block scale folded in.
//   format 0: the conversion instruction multiplies by a power of two (it takes only the exponent of
//             its scale operand, which is all an E8M0 scale has): E2M1 x 2^e, exact in bf16.
//   format 1: an E4M3 scale has a mantissa, so the codes become fp16 (exact) and are multiplied by the
//             scale as packed fp16: an E2M1 value times an E4M3 value has at most six significant bits
//             and lies in [2^-10, 2688], exact in fp16; the main phase then runs on the fp16 matrix
//             core (the bf16 branch keeps the bf16 one; both accumulate into the same fp32 registers).
typedef _Float16 v2h __attribute__((ext_vector_type(2)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
template <int FMT>
struct Operand;
template <>
struct Operand<0> {
    typedef v8bf type;
};
template <>
struct Operand<1> {
    typedef v8h type;
};
template <int FMT>
__device__ __forceinline__ void expand32(const u32x4 c, uint32_t sbytes, typename Operand<FMT>::type (&out)[4]) {
    const float s0 = scale16_f32<FMT>(sbytes & 0xffu), s1 = scale16_f32<FMT>((sbytes >> 8) & 0xffu);
    const uint32_t w[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const float s = t < 2 ? s0 : s1;
        if constexpr (FMT == 0) {
            const v2bf p0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w[t], s, 0), p1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w[t], s, 1),
                       p2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w[t], s, 2), p3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w[t], s, 3);
            out[t] = (v8bf){p0.x, p0.y, p1.x, p1.y, p2.x, p2.y, p3.x, p3.y};
        } else {
            const _Float16 sh = (_Float16)s;  // exact: every E4M3 value is an fp16 value
            const v2h ss = {sh, sh};
            const v2h p0 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w[t], 1.0f, 0) * ss, p1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w[t], 1.0f, 1) * ss,
                      p2 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w[t], 1.0f, 2) * ss, p3 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w[t], 1.0f, 3) * ss;
            out[t] = (v8h){p0.x, p0.y, p1.x, p1.y, p2.x, p2.y, p3.x, p3.y};
        }
    }
}

struct G16Args {
    const uint8_t* Xq;
    const uint8_t* Xs;
    const uint8_t* B;
    int64_t bpitch;
    const uint8_t* Wq;
    const uint8_t* Ws;
    const uint8_t* WL;
    int64_t wlpitch;
    int M, N, K, K_o;
    float ts;  // product of the two tensor scales (1 for format 0)
    void* Y;
    int y_bf16;
    int64_t ldy;
};

template <int FMT, int NW>
__global__ void __launch_bounds__(64 * NW) gemm_g16_kernel(G16Args a) {
    constexpr int IMG = 64 * 128 + 64 * 16;  // codes of 32 weight rows and 32 X rows, then their scale bytes
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int t = threadIdx.x, lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int q = lane >> 5, r = lane & 31;
    const int n0 = blockIdx.x * 32, mb = blockIdx.y * 32;
    const int rowbytes = a.K >> 1, srow = a.K >> 4;
    const int nL = rowbytes >> 7;
    const int nLB = (a.K_o * 2 + 127) >> 7;
    const int nLT = nL + nLB;
    uint8_t* const strip = lds + wave * (2 * IMG);

    // DMA instruction i (0..7) moves rows 8i .. 8i+7 of the image (rows 0-31 weights, 32-63 X): lane ->
    // row 8i + lane/8, piece position lane%8 holding piece (lane%8) ^ swz8(row); instruction 8 moves
    // the 16 scale bytes of row `lane`
    uint32_t o_fp4[8], o_br[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int row = 8 * i + (lane >> 3);
        const uint32_t piece = (uint32_t)((lane & 7) ^ swz8(row)) * 16u;
        const uint32_t g = row < 32 ? (uint32_t)min(n0 + row, a.N - 1) : (uint32_t)min(mb + row - 32, a.M - 1);
        o_fp4[i] = g * (uint32_t)rowbytes + piece;
        o_br[i] = g * (uint32_t)(row < 32 ? a.wlpitch : a.bpitch) + piece;
    }
    const uint32_t o_sc = (lane < 32 ? (uint32_t)min(n0 + lane, a.N - 1) : (uint32_t)min(mb + lane - 32, a.M - 1)) * (uint32_t)srow;
    const uint8_t* const sc_base = lane < 32 ? a.Ws : a.Xs;

    v16f acc;
#pragma unroll
    for (int k = 0; k < 16; ++k) acc[k] = 0.0f;

#define G16_FETCH(L_, IMG_)                                                                              \
    {                                                                                                    \
        uint8_t* dst__ = strip + (IMG_)*IMG;                                                             \
        if ((L_) < nL) {                                                                                 \
            _Pragma("unroll") for (int i = 0; i < 8; ++i)                                                \
                load_to_lds16((i < 4 ? a.Wq : a.Xq) + ((size_t)(L_)*128 + o_fp4[i]), dst__ + i * 1024);  \
            load_to_lds16(sc_base + ((size_t)(L_)*16 + o_sc), dst__ + 8192);                             \
        } else if ((L_) < nLT) {                                                                         \
            _Pragma("unroll") for (int i = 0; i < 8; ++i)                                                \
                load_to_lds16((i < 4 ? a.WL : a.B) + ((size_t)((L_)-nL) * 128 + o_br[i]), dst__ + i * 1024); \
            load_to_lds16(sc_base + o_sc, dst__ + 8192); /* keeps the count of requests per line fixed */ \
        }                                                                                                \
    }
    bool scaled = FMT == 0;  // the tensor scales go on once, before the first branch line
    int L = wave, img = 0;
    G16_FETCH(L, 0)
#pragma unroll 1
    for (; L < nLT; L += NW) {
        G16_FETCH(L + NW, img ^ 1)
        if (L + NW < nLT) wait_vmcnt<9>(); else wait_vmcnt<0>();
        const uint8_t* src = strip + img * IMG;
        if (L < nL) {
            const u32x4 sw = *reinterpret_cast<const u32x4*>(src + 8192 + r * 16);
            const u32x4 sx = *reinterpret_cast<const u32x4*>(src + 8192 + (32 + r) * 16);
            const uint32_t swv[4] = {sw.x, sw.y, sw.z, sw.w}, sxv[4] = {sx.x, sx.y, sx.z, sx.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const u32x4 cw = *reinterpret_cast<const u32x4*>(src + st128_off(r, 2 * j + q));
                const u32x4 cx = *reinterpret_cast<const u32x4*>(src + st128_off(32 + r, 2 * j + q));
                typename Operand<FMT>::type fw[4], fx[4];
                expand32<FMT>(cw, swv[j] >> (16 * q), fw);
                expand32<FMT>(cx, sxv[j] >> (16 * q), fx);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    if constexpr (FMT == 0) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[k], fw[k], acc, 0, 0, 0);
                    else acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(fx[k], fw[k], acc, 0, 0, 0);
                }
            }
        } else {
            if (!scaled) {
#pragma unroll
                for (int k = 0; k < 16; ++k) acc[k] *= a.ts;
                scaled = true;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const u32x4 fw = *reinterpret_cast<const u32x4*>(src + st128_off(r, 4 * q + i));
                const u32x4 fx = *reinterpret_cast<const u32x4*>(src + st128_off(32 + r, 4 * q + i));
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, fx), __builtin_bit_cast(v8bf, fw), acc, 0, 0, 0);
            }
        }
        img ^= 1;
    }
#undef G16_FETCH
    if (!scaled) {
#pragma unroll
        for (int k = 0; k < 16; ++k) acc[k] *= a.ts;
    }
    // ---- sum the NW partial results in a fixed order, store ----
    __syncthreads();
    float* const red = reinterpret_cast<float*>(lds);  // [NW][16][64]
#pragma unroll
    for (int k = 0; k < 16; ++k) red[(wave * 16 + k) * 64 + lane] = acc[k];
    __syncthreads();
#pragma unroll
    for (int k0 = 0; k0 < 16; k0 += NW) {
        const int k = k0 + wave;
        if (k >= 16) break;
        float v = red[k * 64 + lane];
#pragma unroll
        for (int w = 1; w < NW; ++w) v += red[(w * 16 + k) * 64 + lane];
        const int row = mb + 8 * (k >> 2) + 4 * q + (k & 3), col = n0 + r;
        if (row < a.M && col < a.N) {
            if (a.y_bf16)
                reinterpret_cast<uint16_t*>(a.Y)[(int64_t)row * a.ldy + col] = f32_to_bf16_rne(v);
            else
                reinterpret_cast<float*>(a.Y)[(int64_t)row * a.ldy + col] = v;
        }
    }
}

int launch_dual_gemm_g16(const uint8_t* Xq, const uint8_t* Xs, float xts, const uint16_t* B, int64_t ldb, const uint8_t* Wq,
                         const uint8_t* Ws, const uint16_t* WLt, int64_t ldwl, float wts, int64_t M, int64_t N, int64_t K,
                         int32_t K_o, int fmt, void* Y, int y_dtype, int64_t ldy, hipStream_t st) {
    G16Args a;
    a.Xq = Xq;
    a.Xs = Xs;
    a.B = reinterpret_cast<const uint8_t*>(B);
    a.bpitch = ldb * 2;
    a.Wq = Wq;
    a.Ws = Ws;
    a.WL = reinterpret_cast<const uint8_t*>(WLt);
    a.wlpitch = ldwl * 2;
    a.M = (int)M;
    a.N = (int)N;
    a.K = (int)K;
    a.K_o = K_o;
    a.ts = fmt == 0 ? 1.0f : xts * wts;
    a.Y = Y;
    a.y_bf16 = y_dtype == OSC_DT_BF16;
    a.ldy = ldy;
    const int64_t lim = (int64_t)1 << 32;
    if (M * (K / 2) >= lim || N * (K / 2) >= lim || M * a.bpitch >= lim || N * a.wlpitch >= lim)
        return fail(OSC_ERR_UNSUPPORTED, "gemm: an operand of 4 GiB or more");
    const dim3 grid((unsigned)((N + 31) / 32), (unsigned)((M + 31) / 32));
    const int ncu = cu_count();
    if (ncu <= 0) return fail(OSC_ERR_HIP, "gemm: cannot read the number of compute units");
    constexpr int IMG = 64 * 128 + 64 * 16;
    // eight wavefronts when the grid leaves CUs idle, four otherwise (two workgroups per CU)
    const bool wide = (int64_t)grid.x * grid.y <= ncu;
    const size_t smem = (size_t)(wide ? 8 : 4) * 2 * IMG;
#define G16_LAUNCH(F_, NW_)                                                                               \
    {                                                                                                     \
        auto kern = gemm_g16_kernel<F_, NW_>;                                                             \
        static unsigned char lds_done[MAX_DEVICES];                                                       \
        static size_t lds_reserved[MAX_DEVICES];                                                          \
        if (int rc = reserve_lds(reinterpret_cast<const void*>(kern), smem, lds_done, lds_reserved)) return rc; \
        hipLaunchKernelGGL(kern, grid, dim3(64 * NW_), smem, st, a);                                      \
    }
    if (fmt == 0) {
        if (wide) G16_LAUNCH(0, 8) else G16_LAUNCH(0, 4)
    } else {
        if (wide) G16_LAUNCH(1, 8) else G16_LAUNCH(1, 4)
    }
#undef G16_LAUNCH
    return check_launch("gemm_g16_kernel");
}

}  // namespace osc
