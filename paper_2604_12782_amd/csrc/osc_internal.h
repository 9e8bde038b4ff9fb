// Internal declarations shared by the translation units of libosc (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/osc.h"

namespace osc {

int fail(int code, const char* fmt, ...);  // records the thread-local message, returns code
int check_launch(const char* what);        // hipGetLastError -> OSC_OK / OSC_ERR_HIP

// Kernel-choice overrides (osc_tuning.h): process-wide, -1 = automatic.  Read with relaxed loads.
enum { TUNE_GEMM_TILE = 0, TUNE_GEMM_KERNEL = 1, TUNE_GROUPED_ONE_TILE = 2, TUNE_SWIGLU_TABLE = 3, TUNE_GEMM_KSPLIT = 4, TUNE_COUNT = 5 };
int tuning(int knob);
// number of compute units of the current device (cached per device); <= 0 on error
int cu_count();
// hipFuncAttributeMaxDynamicSharedMemorySize, issued once per (kernel, device); `done` is the
// caller's per-kernel flag array, one entry per device
constexpr int MAX_DEVICES = 64;
int reserve_lds(const void* kernel, size_t bytes, unsigned char (&done)[MAX_DEVICES], size_t (&reserved)[MAX_DEVICES]);

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Layout of a packed dual-path weight: three sections, each 256-byte aligned.
struct PackLayout {
    size_t off_q;   // uint8 [N, K/2]   MXFP4 codes, K-major
    size_t off_s;   // E8M0 scales, row-block-major (scale_bytes(N, K) bytes)
    size_t off_l;   // bf16  [N, ldwl]  W_L transposed (K_o-major), zero padded to ldwl
    int64_t ldwl;   // round_up(K_o, 64)
    size_t off_z;   // 256 bytes of zeros (stand-in for anything past the end of an operand row)
    size_t total;
};
PackLayout pack_layout(int64_t N, int64_t K, int32_t K_o);
// bytes of a row-block-major E8M0 scale tensor: [ceil(rows/32)][ceil(K/128)][32][4]
inline size_t scale_bytes(int64_t rows, int64_t K) {
    return (size_t)((rows + 31) / 32) * (size_t)((K / 32 + 3) / 4) * 128;
}
int launch_scales_to_rowmajor(const uint8_t* S, int64_t rows, int64_t K, uint8_t* out, hipStream_t st);

// Layout of a packed FP8 weight.
struct Pack8Layout {
    size_t off_w;  // uint8 [N, K]
    size_t off_s;  // float [N]
    size_t off_z;  // 256 bytes of zeros
    size_t total;
};
Pack8Layout pack8_layout(int64_t N, int64_t K);

// Layout of a packed MXFP8 weight.
struct PackM8Layout {
    size_t off_w;  // uint8 [N, K] E4M3 codes
    size_t off_s;  // E8M0 scales, row-block-major (scale_bytes(N, K) bytes)
    size_t off_z;  // 256 bytes of zeros
    size_t total;
};
PackM8Layout packm8_layout(int64_t N, int64_t K);

// kernels' host launchers (each enqueues on `st`, returns OSC_OK / OSC_ERR_HIP)
int launch_quant_mxfp4(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, const int32_t* oidx,
                       int32_t K_o, uint8_t* Xq, uint8_t* Xs, uint16_t* B, int64_t ldb,
                       hipStream_t st, int group = 32);
int launch_quant_mxfp4_dynamic(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, uint8_t* Xq, uint8_t* Xs,
                               uint16_t* Bd, int64_t ldb, uint8_t* idx, hipStream_t st);
int launch_rmsnorm_quant_mxfp4(const uint16_t* X, const uint16_t* gamma, float eps, int64_t M, int64_t K, int64_t ldx,
                               const int32_t* oidx, int32_t K_o, uint8_t* Xq, uint8_t* Xs, uint16_t* B, int64_t ldb,
                               uint16_t* Xn, hipStream_t st);
int launch_swiglu_quant_mxfp8(const uint16_t* G, const uint16_t* U, int64_t M, int64_t K, int64_t ldg, int64_t ldu,
                              uint8_t* Xq, uint8_t* Xs, uint16_t* Yn, hipStream_t st);
int launch_swiglu_quant_fp8(const uint16_t* G, const uint16_t* U, int64_t M, int64_t K, int64_t ldg, int64_t ldu,
                            uint8_t* X8, float* xs, uint16_t* Yn, hipStream_t st);
int launch_quant_fp8(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, uint8_t* X8, float* xs,
                     hipStream_t st);
int launch_quant_mxfp8(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, uint8_t* Xq, uint8_t* Xs,
                       hipStream_t st);
int launch_gather_wl(const uint16_t* W, int64_t N, int64_t K, int64_t ldw, const int32_t* oidx,
                     int32_t K_o, uint16_t* WLt, int64_t ldwl, hipStream_t st);
int launch_unpack_wl(const uint16_t* WLt, int64_t ldwl, int64_t N, int32_t K_o, uint16_t* WL,
                     hipStream_t st);

int launch_profile_abs_sum(const uint16_t* X, int64_t S, int64_t H, int64_t ldx, double* abs_sum,
                           hipStream_t st);
int launch_profile_threshold(const double* abs_sum, int64_t count, float alpha, float* T, hipStream_t st);
int launch_profile_hist(const uint16_t* X, int64_t S, int64_t H, int64_t ldx, int32_t G, const float* T,
                        uint32_t* hist, hipStream_t st);
int launch_profile_table(const uint32_t* hist, int32_t Kg, int32_t G, int32_t R, int16_t* table,
                         uint32_t* n_total, uint32_t* n_hit, float* density, float* cbar, hipStream_t st);

constexpr int64_t PROFILE_STATIC_MAX_H = 16384;  // widest activation the allocation-free profiling call takes
size_t profile_scratch_bytes(int64_t H);
int launch_profile_calibrate_static(const uint16_t* X, int64_t S, int64_t H, int64_t ldx, int32_t G, float alpha,
                                    int32_t R, int16_t* table, uint32_t* n_total, uint32_t* n_hit, float* density,
                                    float* cbar, float* T_out, hipStream_t st);
int launch_profile_calibrate(const uint16_t* X, int64_t S, int64_t H, int64_t ldx, int32_t G, float alpha, int32_t R,
                             int16_t* table, uint32_t* n_total, uint32_t* n_hit, float* density, float* cbar,
                             float* T_out, uint8_t* scratch, hipStream_t st);

// 4-bit formats with a scale per 16 channels (g16.hip)
struct Pack16Layout {
    size_t off_q;   // uint8 [N, K/2]   E2M1 codes
    size_t off_s;   // uint8 [N, K/16]  scale bytes, plain row-major
    size_t off_l;   // bf16  [N, ldwl]  W_L transposed, zero padded
    int64_t ldwl;   // round_up(K_o, 64)
    size_t off_z;   // 256 bytes of zeros
    size_t total;
};
Pack16Layout pack16_layout(int64_t N, int64_t K, int32_t K_o);
int launch_quant_fp4_g16(const uint16_t* X, int64_t M, int64_t K, int64_t ldx, const int32_t* oidx, int32_t K_o, int fmt,
                         float ts, uint8_t* Xq, uint8_t* Xs, uint16_t* B, int64_t ldb, hipStream_t st);
int launch_dual_gemm_g16(const uint8_t* Xq, const uint8_t* Xs, float xts, const uint16_t* B, int64_t ldb, const uint8_t* Wq,
                         const uint8_t* Ws, const uint16_t* WLt, int64_t ldwl, float wts, int64_t M, int64_t N, int64_t K,
                         int32_t K_o, int fmt, void* Y, int y_dtype, int64_t ldy, hipStream_t st);

struct GemmProblem {
    // activations
    const uint8_t* Xq;   // dual: codes [*, K/2]; fp8, mxfp8: codes [*, K]
    const uint8_t* Xs;   // dual, mxfp8: E8M0 scales, row-block-major
    const float* xs;     // fp8: per-row scale
    const uint16_t* B;   // dual: gathered bf16 [*, ldb]
    int64_t ldb;
    const int32_t* row_map;         // grouped dual: routed row -> activation row (or null)
    const int32_t* expert_offsets;  // grouped: [E+1] (or null)
    int32_t E;
    // weights (first expert; experts are pack_stride bytes apart)
    const uint8_t* Wpack;
    size_t pack_stride;
    int64_t M, N, K;
    int32_t K_o;
    void* Y;
    int y_dtype;
    int64_t ldy;
};
int launch_dual_gemm(const GemmProblem& p, hipStream_t st);
int launch_fp8_gemm(const GemmProblem& p, hipStream_t st);
int launch_mxfp8_gemm(const GemmProblem& p, hipStream_t st);

}  // namespace osc
