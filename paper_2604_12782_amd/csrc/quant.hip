// Activation quantisers: OSC-enhanced MXFP4 (Section 3.2, Alg. 2) and per-token FP8 (Section 3.4).
// Both are HBM-bandwidth-bound row kernels: one workgroup walks whole rows with 16-byte loads.
#include "osc_internal.h"

namespace osc {

typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int QT = 256;  // threads per workgroup

// ------------------------------------------------------------------------------------------
// MXFP4 + outlier gather.
//
// A row is cut into 16-byte chunks of 8 channels; chunk c belongs to thread c % 256 and the four
// chunks of a 32-channel group sit in four neighbouring lanes, so the group's amax is two
// cross-lane steps.  The suppression list is turned, once per workgroup, into one 32-bit mask
// per group plus the column of B where the group's first protected channel goes; protected
// values are parked in LDS at their column and the B row leaves with 16-byte stores.
//
// CPT = chunks per thread held in registers (row length <= 256*8*CPT channels).
// ------------------------------------------------------------------------------------------
template <int CPT>
__global__ void __launch_bounds__(QT) quant_mxfp4_osc_kernel(
    const uint16_t* __restrict__ X, int M, int K, int64_t ldx, const int32_t* __restrict__ oidx,
    int K_o, uint8_t* __restrict__ Xq, uint8_t* __restrict__ Xs, uint16_t* __restrict__ B,
    int64_t ldb) {
    extern __shared__ uint32_t smem[];
    const int Kg = K >> 5, Kg4 = (Kg + 3) >> 2;
    const int nchunk = K >> 3;
    uint32_t* mask = smem;                                     // [Kg]
    int* first = reinterpret_cast<int*>(smem + Kg);            // [Kg]
    uint16_t* stage = reinterpret_cast<uint16_t*>(smem + ((2 * Kg + 3) & ~3));  // [ldb], 16-byte aligned
    const int t = threadIdx.x;

    int m = blockIdx.x;
    u32x4 v[CPT];
    auto load_row = [&](int row) {
        const u32x4* src = reinterpret_cast<const u32x4*>(X + (int64_t)row * ldx);
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            int c = t + QT * i;
            if (c < nchunk) v[i] = __builtin_nontemporal_load(src + c);
        }
    };
    if (m < M) load_row(m);  // in flight while the table is set up

    if (K_o > 0) {
        for (int g = t; g < Kg; g += QT) {
            mask[g] = 0u;
            first[g] = 0x7fffffff;
        }
        for (int o = t; o < (int)(ldb >> 1); o += QT)
            reinterpret_cast<uint32_t*>(stage)[o] = 0u;  // padding columns stay +0
        __syncthreads();
        for (int o = t; o < K_o; o += QT) {
            int c = oidx[o];
            atomicOr(&mask[c >> 5], 1u << (c & 31));
            atomicMin(&first[c >> 5], o);
        }
        __syncthreads();
    }

    for (; m < M; m += gridDim.x) {
        uint32_t packed[CPT];
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            int c = t + QT * i;
            if (c < nchunk) {
                uint32_t w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
                const int g = c >> 2, sub = c & 3;
                if (K_o > 0) {
                    const uint32_t gm = mask[g];
                    const uint32_t mb = (gm >> (8 * sub)) & 0xffu;
                    if (mb) {  // steps 2-3 of Section 3.2: back up, then zero
                        const int base = first[g];
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            if (mb & (1u << j)) {
                                int col = base + __builtin_popcount(gm & ((1u << (8 * sub + j)) - 1u));
                                uint32_t word = w[j >> 1];
                                stage[col] = (uint16_t)((j & 1) ? (word >> 16) : (word & 0xffffu));
                                w[j >> 1] = (j & 1) ? (word & 0x0000ffffu) : (word & 0xffff0000u);
                            }
                        }
                    }
                }
                // amax of the group on bit patterns: for finite bf16, |x| orders like bits & 0x7fff
                uint32_t a = 0;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    uint32_t lo = w[k] & 0x7fffu, hi = (w[k] >> 16) & 0x7fffu;
                    a = max(a, max(lo, hi));
                }
                a = max(a, (uint32_t)__shfl_xor((int)a, 1));
                a = max(a, (uint32_t)__shfl_xor((int)a, 2));
                // shared exponent floor(log2 amax) - 2, clamped below: E8M0 code = max(E - 2, 0)
                int code = max((int)(a >> 7) - 2, 0);
                {   // four groups (16 lanes) -> one 32-bit word of the row-block-major scale layout
                    const int g0 = g & ~3;
                    uint32_t word = (uint32_t)code;
                    uint32_t c1 = (uint32_t)__shfl_down(code, 4, 16);
                    uint32_t c2 = (uint32_t)__shfl_down(code, 8, 16);
                    uint32_t c3 = (uint32_t)__shfl_down(code, 12, 16);
                    if (g0 + 1 < Kg) word |= c1 << 8;
                    if (g0 + 2 < Kg) word |= c2 << 16;
                    if (g0 + 3 < Kg) word |= c3 << 24;
                    if ((c & 15) == 0)
                        *reinterpret_cast<uint32_t*>(Xs + ((int64_t)(m >> 5) * Kg4 + (g >> 2)) * 128 + (m & 31) * 4) = word;
                }
                float scale = __builtin_bit_cast(float, (uint32_t)code << 23);
                uint32_t out = 0;
                out = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(out, __builtin_bit_cast(v2bf, w[0]), scale, 0);
                out = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(out, __builtin_bit_cast(v2bf, w[1]), scale, 1);
                out = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(out, __builtin_bit_cast(v2bf, w[2]), scale, 2);
                out = __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(out, __builtin_bit_cast(v2bf, w[3]), scale, 3);
                packed[i] = out;
            }
        }
        const int mn = m + gridDim.x;
        if (mn < M) load_row(mn);  // next row's loads overlap this row's stores
        uint32_t* dst = reinterpret_cast<uint32_t*>(Xq + (int64_t)m * (K >> 1));
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            int c = t + QT * i;
            if (c < nchunk) __builtin_nontemporal_store(packed[i], dst + c);
        }
        if (K_o > 0) {
            __syncthreads();
            u32x4* bdst = reinterpret_cast<u32x4*>(B + (int64_t)m * ldb);
            for (int i = t; i < (int)(ldb >> 3); i += QT)
                __builtin_nontemporal_store(reinterpret_cast<const u32x4*>(stage)[i], bdst + i);
            __syncthreads();
        }
    }
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
                       hipStream_t st) {
    const int64_t Kg = K / 32;
    const int64_t nchunk = K / 8;
    const int cpt = (int)((nchunk + QT - 1) / QT);
    size_t smem = (size_t)((2 * Kg + 3) & ~(int64_t)3) * 4 + (K_o > 0 ? (size_t)ldb * 2 : 0);
    if (smem > 60 * 1024) return fail(OSC_ERR_UNSUPPORTED, "quantize: K=%lld / ldb=%lld too large for the table in LDS", (long long)K, (long long)ldb);
    int grid = (int)(M < 2048 ? M : 2048);
    if (K_o == 0 && B && ldb > 0)
        hipLaunchKernelGGL(zero_rows_kernel, dim3(grid), dim3(QT), 0, st, B, (int)M, ldb);
#define OSC_QLAUNCH(C)                                                                           \
    hipLaunchKernelGGL(quant_mxfp4_osc_kernel<C>, dim3(grid), dim3(QT), smem, st, X, (int)M, (int)K, \
                       ldx, oidx, (int)K_o, Xq, Xs, B, ldb)
    if (cpt <= 1) OSC_QLAUNCH(1);
    else if (cpt <= 2) OSC_QLAUNCH(2);
    else if (cpt <= 4) OSC_QLAUNCH(4);
    else if (cpt <= 8) OSC_QLAUNCH(8);
    else return fail(OSC_ERR_UNSUPPORTED, "quantize: K=%lld exceeds 16384", (long long)K);
#undef OSC_QLAUNCH
    return check_launch("quant_mxfp4_osc_kernel");
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
