// C ABI of libosc: argument checking and dispatch.  Every check runs on the host before
// anything is enqueued, so the error paths need no GPU.
#include <cstdarg>
#include <cstdio>

#include "osc_internal.h"

namespace osc {

static thread_local char g_err[256] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

int check_launch(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(OSC_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return OSC_OK;
}

PackLayout pack_layout(int64_t N, int64_t K, int32_t K_o) {
    PackLayout L;
    L.ldwl = ((int64_t)K_o + 63) / 64 * 64;
    L.off_q = 0;
    L.off_s = align_up((size_t)N * (size_t)(K / 2), 256);
    L.off_l = align_up(L.off_s + scale_bytes(N, K), 256);
    L.off_z = align_up(L.off_l + (size_t)N * (size_t)L.ldwl * 2, 256);
    L.total = L.off_z + 256;
    return L;
}

Pack8Layout pack8_layout(int64_t N, int64_t K) {
    Pack8Layout L;
    L.off_w = 0;
    L.off_s = align_up((size_t)N * (size_t)K, 256);
    L.off_z = align_up(L.off_s + (size_t)N * 4, 256);
    L.total = L.off_z + 256;
    return L;
}

PackM8Layout packm8_layout(int64_t N, int64_t K) {
    PackM8Layout L;
    L.off_w = 0;
    L.off_s = align_up((size_t)N * (size_t)K, 256);
    L.off_z = align_up(L.off_s + scale_bytes(N, K), 256);
    L.total = L.off_z + 256;
    return L;
}

Pack16Layout pack16_layout(int64_t N, int64_t K, int32_t K_o) {
    Pack16Layout L;
    L.ldwl = ((int64_t)K_o + 63) / 64 * 64;
    L.off_q = 0;
    L.off_s = align_up((size_t)N * (size_t)(K / 2), 256);
    L.off_l = align_up(L.off_s + (size_t)N * (size_t)(K / 16), 256);
    L.off_z = align_up(L.off_l + (size_t)N * (size_t)L.ldwl * 2, 256);
    L.total = L.off_z + 256;
    return L;
}

}  // namespace osc

using namespace osc;

#define REQUIRE(cond, code, ...) \
    do {                         \
        if (!(cond)) return fail(code, __VA_ARGS__); \
    } while (0)

extern "C" {

const char* osc_last_error(void) { return g_err; }
int osc_version(void) { return 100; }

int osc_table_to_index_g(const int16_t* table, int32_t Kg, int32_t R, int32_t G, int32_t* oidx, int32_t* K_o) {
    REQUIRE(table && oidx && K_o, OSC_ERR_NULL, "osc_table_to_index: null pointer");
    REQUIRE(Kg >= 0 && R >= 0, OSC_ERR_SHAPE, "osc_table_to_index: Kg=%d R=%d", Kg, R);
    REQUIRE(G == 16 || G == 32 || G == 64, OSC_ERR_UNSUPPORTED, "osc_table_to_index: group size %d (16, 32 or 64)", G);
    REQUIRE((int64_t)Kg * G <= 0x7fffffff, OSC_ERR_UNSUPPORTED, "osc_table_to_index: more than 2^31-1 channels");
    int32_t n = 0;
    for (int32_t g = 0; g < Kg; ++g) {
        uint64_t seen = 0;
        for (int32_t s = 0; s < R; ++s) {
            const int j = table[(int64_t)g * R + s];
            if (j == -1) continue;
            REQUIRE(j >= 0 && j < G, OSC_ERR_TABLE, "osc_table_to_index: group %d holds index %d", g, j);
            REQUIRE(!(seen >> j & 1u), OSC_ERR_TABLE, "osc_table_to_index: group %d repeats index %d", g, j);
            seen |= (uint64_t)1 << j;
        }
        while (seen) {
            const int j = __builtin_ctzll(seen);
            seen &= seen - 1;
            oidx[n++] = g * G + j;
        }
    }
    *K_o = n;
    return OSC_OK;
}

int osc_table_to_index(const int16_t* table, int32_t Kg, int32_t R, int32_t* oidx, int32_t* K_o) {
    return osc_table_to_index_g(table, Kg, R, 32, oidx, K_o);
}

size_t osc_packed_weight_bytes(int64_t N, int64_t K, int32_t K_o) {
    if (N < 0 || K < 0 || K % 32 || K_o < 0) return 0;
    return pack_layout(N, K, K_o).total;
}

size_t osc_packed_weight_fp8_bytes(int64_t N, int64_t K) {
    if (N < 0 || K < 0) return 0;
    return pack8_layout(N, K).total;
}

static int check_mx_shape(const char* who, int64_t rows, int64_t K, int64_t ld, int32_t K_o) {
    REQUIRE(rows >= 0 && K >= 0 && K_o >= 0, OSC_ERR_SHAPE, "%s: negative extent", who);
    REQUIRE(K % 32 == 0, OSC_ERR_SHAPE, "%s: K=%lld is not a multiple of 32", who, (long long)K);
    REQUIRE(ld >= K, OSC_ERR_SHAPE, "%s: leading dimension %lld < K=%lld", who, (long long)ld, (long long)K);
    REQUIRE(K_o <= K, OSC_ERR_SHAPE, "%s: K_o=%d > K", who, K_o);
    REQUIRE(rows <= 0x7fffffff && K <= 0x7fffffff, OSC_ERR_UNSUPPORTED, "%s: extent above 2^31-1", who);
    return OSC_OK;
}

int osc_pack_weight_g(const void* W, int64_t N, int64_t K, int64_t ldw, const int32_t* oidx,
                      int32_t K_o, int32_t G, void* Wpack, void* stream) {
    REQUIRE(G == 32 || G == 64, OSC_ERR_UNSUPPORTED, "osc_pack_weight: scale group %d (32 or 64)", G);
    int rc = check_mx_shape("osc_pack_weight", N, K, ldw, K_o);
    if (rc) return rc;
    REQUIRE(K % G == 0, OSC_ERR_SHAPE, "osc_pack_weight: K=%lld is not a multiple of G=%d", (long long)K, G);
    if (N == 0) return OSC_OK;
    REQUIRE(W && Wpack && (K_o == 0 || oidx), OSC_ERR_NULL, "osc_pack_weight: null pointer");
    REQUIRE(ldw % 8 == 0 && aligned(W, 16) && aligned(Wpack, 256), OSC_ERR_UNSUPPORTED,
            "osc_pack_weight: W rows must be 16-byte aligned and Wpack 256-byte aligned");
    PackLayout L = pack_layout(N, K, K_o);
    uint8_t* base = static_cast<uint8_t*>(Wpack);
    if (K > 0) {
        rc = launch_quant_mxfp4(static_cast<const uint16_t*>(W), N, K, ldw, nullptr, 0, base + L.off_q,
                                base + L.off_s, nullptr, 0, as_stream(stream), G);
        if (rc) return rc;
    }
    if (hipMemsetAsync(base + L.off_z, 0, 256, as_stream(stream)) != hipSuccess)
        return fail(OSC_ERR_HIP, "osc_pack_weight: cannot clear the zero block");
    return launch_gather_wl(static_cast<const uint16_t*>(W), N, K, ldw, oidx, K_o,
                            reinterpret_cast<uint16_t*>(base + L.off_l), L.ldwl, as_stream(stream));
}

int osc_pack_weight(const void* W, int64_t N, int64_t K, int64_t ldw, const int32_t* oidx,
                    int32_t K_o, void* Wpack, void* stream) {
    return osc_pack_weight_g(W, N, K, ldw, oidx, K_o, 32, Wpack, stream);
}

int osc_unpack_weight(const void* Wpack, int64_t N, int64_t K, int32_t K_o, uint8_t* Wq, uint8_t* Ws,
                      void* WL, void* stream) {
    int rc = check_mx_shape("osc_unpack_weight", N, K, K, K_o);
    if (rc) return rc;
    if (N == 0) return OSC_OK;
    REQUIRE(Wpack, OSC_ERR_NULL, "osc_unpack_weight: null pointer");
    PackLayout L = pack_layout(N, K, K_o);
    const uint8_t* base = static_cast<const uint8_t*>(Wpack);
    hipStream_t st = as_stream(stream);
    if (Wq && K > 0 &&
        hipMemcpyAsync(Wq, base + L.off_q, (size_t)N * (K / 2), hipMemcpyDeviceToDevice, st) != hipSuccess)
        return fail(OSC_ERR_HIP, "osc_unpack_weight: copy of codes failed");
    if (Ws && K > 0) {
        rc = launch_scales_to_rowmajor(base + L.off_s, N, K, Ws, st);
        if (rc) return rc;
    }
    if (WL)
        return launch_unpack_wl(reinterpret_cast<const uint16_t*>(base + L.off_l), L.ldwl, N, K_o,
                                static_cast<uint16_t*>(WL), st);
    return OSC_OK;
}

size_t osc_act_scale_bytes(int64_t M, int64_t K) {
    if (M < 0 || K < 0 || K % 32) return 0;
    return scale_bytes(M, K);
}

int osc_unpack_act_scales(const uint8_t* Xs, int64_t M, int64_t K, uint8_t* out, void* stream) {
    int rc = check_mx_shape("osc_unpack_act_scales", M, K, K, 0);
    if (rc) return rc;
    if (M == 0 || K == 0) return OSC_OK;
    REQUIRE(Xs && out, OSC_ERR_NULL, "osc_unpack_act_scales: null pointer");
    return launch_scales_to_rowmajor(Xs, M, K, out, as_stream(stream));
}

int osc_pack_weight_fp8(const void* W, int64_t N, int64_t K, int64_t ldw, void* W8pack, void* stream) {
    REQUIRE(N >= 0 && K >= 0, OSC_ERR_SHAPE, "osc_pack_weight_fp8: negative extent");
    REQUIRE(ldw >= K, OSC_ERR_SHAPE, "osc_pack_weight_fp8: ldw < K");
    REQUIRE(K % 16 == 0, OSC_ERR_SHAPE, "osc_pack_weight_fp8: K=%lld is not a multiple of 16", (long long)K);
    REQUIRE(N <= 0x7fffffff && K <= 0x7fffffff, OSC_ERR_UNSUPPORTED, "osc_pack_weight_fp8: extent above 2^31-1");
    if (N == 0) return OSC_OK;
    REQUIRE(W && W8pack, OSC_ERR_NULL, "osc_pack_weight_fp8: null pointer");
    REQUIRE(ldw % 8 == 0 && aligned(W, 16) && aligned(W8pack, 256), OSC_ERR_UNSUPPORTED,
            "osc_pack_weight_fp8: W rows must be 16-byte aligned and W8pack 256-byte aligned");
    Pack8Layout L = pack8_layout(N, K);
    uint8_t* base = static_cast<uint8_t*>(W8pack);
    if (hipMemsetAsync(base + L.off_z, 0, 256, as_stream(stream)) != hipSuccess)
        return fail(OSC_ERR_HIP, "osc_pack_weight_fp8: cannot clear the zero block");
    return launch_quant_fp8(static_cast<const uint16_t*>(W), N, K, ldw, base + L.off_w,
                            reinterpret_cast<float*>(base + L.off_s), as_stream(stream));
}

int osc_unpack_weight_fp8(const void* W8pack, int64_t N, int64_t K, uint8_t* W8, float* ws, void* stream) {
    REQUIRE(N >= 0 && K >= 0, OSC_ERR_SHAPE, "osc_unpack_weight_fp8: negative extent");
    if (N == 0) return OSC_OK;
    REQUIRE(W8pack, OSC_ERR_NULL, "osc_unpack_weight_fp8: null pointer");
    Pack8Layout L = pack8_layout(N, K);
    const uint8_t* base = static_cast<const uint8_t*>(W8pack);
    hipStream_t st = as_stream(stream);
    if (W8 && K > 0 &&
        hipMemcpyAsync(W8, base + L.off_w, (size_t)N * K, hipMemcpyDeviceToDevice, st) != hipSuccess)
        return fail(OSC_ERR_HIP, "osc_unpack_weight_fp8: copy of codes failed");
    if (ws && hipMemcpyAsync(ws, base + L.off_s, (size_t)N * 4, hipMemcpyDeviceToDevice, st) != hipSuccess)
        return fail(OSC_ERR_HIP, "osc_unpack_weight_fp8: copy of scales failed");
    return OSC_OK;
}

size_t osc_packed_weight_mxfp8_bytes(int64_t N, int64_t K) {
    if (N < 0 || K < 0 || K % 32) return 0;
    return packm8_layout(N, K).total;
}

int osc_pack_weight_mxfp8(const void* W, int64_t N, int64_t K, int64_t ldw, void* Wpack, void* stream) {
    int rc = check_mx_shape("osc_pack_weight_mxfp8", N, K, ldw, 0);
    if (rc) return rc;
    if (N == 0 || K == 0) return OSC_OK;
    REQUIRE(W && Wpack, OSC_ERR_NULL, "osc_pack_weight_mxfp8: null pointer");
    REQUIRE(ldw % 8 == 0 && aligned(W, 16) && aligned(Wpack, 256), OSC_ERR_UNSUPPORTED,
            "osc_pack_weight_mxfp8: W rows must be 16-byte aligned and Wpack 256-byte aligned");
    PackM8Layout L = packm8_layout(N, K);
    uint8_t* base = static_cast<uint8_t*>(Wpack);
    if (hipMemsetAsync(base + L.off_z, 0, 256, as_stream(stream)) != hipSuccess)
        return fail(OSC_ERR_HIP, "osc_pack_weight_mxfp8: cannot clear the zero block");
    return launch_quant_mxfp8(static_cast<const uint16_t*>(W), N, K, ldw, base + L.off_w, base + L.off_s,
                              as_stream(stream));
}

int osc_unpack_weight_mxfp8(const void* Wpack, int64_t N, int64_t K, uint8_t* W8, uint8_t* Ws, void* stream) {
    int rc = check_mx_shape("osc_unpack_weight_mxfp8", N, K, K, 0);
    if (rc) return rc;
    if (N == 0 || K == 0) return OSC_OK;
    REQUIRE(Wpack, OSC_ERR_NULL, "osc_unpack_weight_mxfp8: null pointer");
    PackM8Layout L = packm8_layout(N, K);
    const uint8_t* base = static_cast<const uint8_t*>(Wpack);
    hipStream_t st = as_stream(stream);
    if (W8 && hipMemcpyAsync(W8, base + L.off_w, (size_t)N * K, hipMemcpyDeviceToDevice, st) != hipSuccess)
        return fail(OSC_ERR_HIP, "osc_unpack_weight_mxfp8: copy of codes failed");
    if (Ws) return launch_scales_to_rowmajor(base + L.off_s, N, K, Ws, st);
    return OSC_OK;
}

int osc_quantize_act(const void* X, int64_t M, int64_t K, int64_t ldx, const int32_t* oidx, int32_t K_o,
                     int fmt, uint8_t* Xq, void* Xs, void* B, int64_t ldb, void* stream) {
    REQUIRE(fmt == OSC_FMT_MXFP4_OSC || fmt == OSC_FMT_FP8_E4M3_TOKEN || fmt == OSC_FMT_MXFP8 ||
                fmt == OSC_FMT_MXFP4_OSC_G64, OSC_ERR_UNSUPPORTED,
            "osc_quantize_act: unknown format %d", fmt);
    if (fmt == OSC_FMT_MXFP8) {
        int rc8 = check_mx_shape("osc_quantize_act", M, K, ldx, 0);
        if (rc8) return rc8;
        if (M == 0 || K == 0) return OSC_OK;
        REQUIRE(X && Xq && Xs, OSC_ERR_NULL, "osc_quantize_act: null pointer");
        REQUIRE(ldx % 8 == 0 && aligned(X, 16) && aligned(Xq, 8) && aligned(Xs, 4), OSC_ERR_UNSUPPORTED,
                "osc_quantize_act: misaligned pointer or ldx %% 8 != 0");
        return launch_quant_mxfp8(static_cast<const uint16_t*>(X), M, K, ldx, Xq, static_cast<uint8_t*>(Xs),
                                  as_stream(stream));
    }
    if (fmt == OSC_FMT_FP8_E4M3_TOKEN) {
        REQUIRE(M >= 0 && K >= 0, OSC_ERR_SHAPE, "osc_quantize_act: negative extent");
        REQUIRE(ldx >= K, OSC_ERR_SHAPE, "osc_quantize_act: ldx < K");
        REQUIRE(K % 8 == 0, OSC_ERR_SHAPE, "osc_quantize_act: FP8 needs K %% 8 == 0, got %lld", (long long)K);
        REQUIRE(M <= 0x7fffffff && K <= 0x7fffffff, OSC_ERR_UNSUPPORTED, "osc_quantize_act: extent above 2^31-1");
        if (M == 0) return OSC_OK;
        REQUIRE(Xq && Xs && (X || K == 0), OSC_ERR_NULL, "osc_quantize_act: null pointer");
        REQUIRE(ldx % 8 == 0 && aligned(X, 16) && aligned(Xq, 8) && aligned(Xs, 4), OSC_ERR_UNSUPPORTED,
                "osc_quantize_act: misaligned pointer or ldx %% 8 != 0");
        return launch_quant_fp8(static_cast<const uint16_t*>(X), M, K, ldx, Xq, static_cast<float*>(Xs),
                                as_stream(stream));
    }
    int rc = check_mx_shape("osc_quantize_act", M, K, ldx, K_o);
    if (rc) return rc;
    const int group = fmt == OSC_FMT_MXFP4_OSC_G64 ? 64 : 32;
    REQUIRE(K % group == 0, OSC_ERR_SHAPE, "osc_quantize_act: K=%lld is not a multiple of the scale group %d",
            (long long)K, group);
    REQUIRE(K_o == 0 || ldb >= K_o, OSC_ERR_SHAPE, "osc_quantize_act: ldb=%lld < K_o=%d", (long long)ldb, K_o);
    if (M == 0 || K == 0) return OSC_OK;
    REQUIRE(X && Xq && Xs, OSC_ERR_NULL, "osc_quantize_act: null pointer");
    REQUIRE(K_o == 0 || (oidx && B), OSC_ERR_NULL, "osc_quantize_act: K_o > 0 needs oidx and B");
    REQUIRE(ldx % 8 == 0 && aligned(X, 16) && aligned(Xq, 4) && aligned(Xs, 4), OSC_ERR_UNSUPPORTED,
            "osc_quantize_act: misaligned pointer or ldx %% 8 != 0");
    if (B) {
        REQUIRE(ldb >= 0, OSC_ERR_SHAPE, "osc_quantize_act: negative ldb");
        REQUIRE(ldb % 8 == 0 && aligned(B, 16), OSC_ERR_UNSUPPORTED,
                "osc_quantize_act: B must be 16-byte aligned with ldb %% 8 == 0");
    }
    return launch_quant_mxfp4(static_cast<const uint16_t*>(X), M, K, ldx, oidx, K_o, Xq,
                              static_cast<uint8_t*>(Xs), static_cast<uint16_t*>(B), B ? ldb : 0,
                              as_stream(stream), group);
}

int osc_rmsnorm_quantize_act(const void* X, const void* gamma, float eps, int64_t M, int64_t K, int64_t ldx,
                             const int32_t* oidx, int32_t K_o, uint8_t* Xq, void* Xs, void* B, int64_t ldb, void* Xn,
                             void* stream) {
    int rc = check_mx_shape("osc_rmsnorm_quantize_act", M, K, ldx, K_o);
    if (rc) return rc;
    REQUIRE(K_o == 0 || ldb >= K_o, OSC_ERR_SHAPE, "osc_rmsnorm_quantize_act: ldb=%lld < K_o=%d", (long long)ldb, K_o);
    REQUIRE(eps >= 0.0f, OSC_ERR_SHAPE, "osc_rmsnorm_quantize_act: negative eps");
    if (M == 0 || K == 0) return OSC_OK;
    REQUIRE(X && gamma && Xq && Xs, OSC_ERR_NULL, "osc_rmsnorm_quantize_act: null pointer");
    REQUIRE(K_o == 0 || (oidx && B), OSC_ERR_NULL, "osc_rmsnorm_quantize_act: K_o > 0 needs oidx and B");
    REQUIRE(ldx % 8 == 0 && aligned(X, 16) && aligned(gamma, 16) && aligned(Xq, 4) && aligned(Xs, 4) && aligned(Xn, 16),
            OSC_ERR_UNSUPPORTED, "osc_rmsnorm_quantize_act: misaligned pointer or ldx %% 8 != 0");
    if (B) {
        REQUIRE(ldb >= 0, OSC_ERR_SHAPE, "osc_rmsnorm_quantize_act: negative ldb");
        REQUIRE(ldb % 8 == 0 && aligned(B, 16), OSC_ERR_UNSUPPORTED,
                "osc_rmsnorm_quantize_act: B must be 16-byte aligned with ldb %% 8 == 0");
    }
    return launch_rmsnorm_quant_mxfp4(static_cast<const uint16_t*>(X), static_cast<const uint16_t*>(gamma), eps, M, K,
                                      ldx, oidx, K_o, Xq, static_cast<uint8_t*>(Xs), static_cast<uint16_t*>(B),
                                      B ? ldb : 0, static_cast<uint16_t*>(Xn), as_stream(stream));
}

int osc_swiglu_quantize_act(const void* G, const void* U, int64_t M, int64_t K, int64_t ldg, int64_t ldu,
                            uint8_t* Xq, void* Xs, void* Yn, void* stream) {
    int rc = check_mx_shape("osc_swiglu_quantize_act", M, K, ldg, 0);
    if (rc) return rc;
    REQUIRE(ldu >= K, OSC_ERR_SHAPE, "osc_swiglu_quantize_act: ldu=%lld < K=%lld", (long long)ldu, (long long)K);
    if (M == 0 || K == 0) return OSC_OK;
    REQUIRE(G && U && Xq && Xs, OSC_ERR_NULL, "osc_swiglu_quantize_act: null pointer");
    REQUIRE(ldg % 8 == 0 && ldu % 8 == 0 && aligned(G, 16) && aligned(U, 16) && aligned(Xq, 8) && aligned(Xs, 4) &&
                aligned(Yn, 16),
            OSC_ERR_UNSUPPORTED, "osc_swiglu_quantize_act: misaligned pointer or leading dimension");
    return launch_swiglu_quant_mxfp8(static_cast<const uint16_t*>(G), static_cast<const uint16_t*>(U), M, K, ldg, ldu,
                                     Xq, static_cast<uint8_t*>(Xs), static_cast<uint16_t*>(Yn), as_stream(stream));
}

int osc_swiglu_quantize_act_fp8(const void* G, const void* U, int64_t M, int64_t K, int64_t ldg, int64_t ldu,
                                uint8_t* X8, float* xs, void* Yn, void* stream) {
    REQUIRE(M >= 0 && K >= 0, OSC_ERR_SHAPE, "osc_swiglu_quantize_act_fp8: negative extent");
    REQUIRE(ldg >= K && ldu >= K, OSC_ERR_SHAPE, "osc_swiglu_quantize_act_fp8: leading dimension below K=%lld", (long long)K);
    REQUIRE(K % 8 == 0, OSC_ERR_SHAPE, "osc_swiglu_quantize_act_fp8: K=%lld is not a multiple of 8", (long long)K);
    REQUIRE(M <= 0x7fffffff && K <= 0x7fffffff, OSC_ERR_UNSUPPORTED, "osc_swiglu_quantize_act_fp8: extent above 2^31-1");
    if (M == 0) return OSC_OK;
    REQUIRE(X8 && xs && ((G && U) || K == 0), OSC_ERR_NULL, "osc_swiglu_quantize_act_fp8: null pointer");
    REQUIRE(ldg % 8 == 0 && ldu % 8 == 0 && aligned(G, 16) && aligned(U, 16) && aligned(X8, 8) && aligned(xs, 4) &&
                aligned(Yn, 16),
            OSC_ERR_UNSUPPORTED, "osc_swiglu_quantize_act_fp8: misaligned pointer or leading dimension");
    return launch_swiglu_quant_fp8(static_cast<const uint16_t*>(G), static_cast<const uint16_t*>(U), M, K, ldg, ldu,
                                   X8, xs, static_cast<uint16_t*>(Yn), as_stream(stream));
}

int osc_quantize_act_dynamic(const void* X, int64_t M, int64_t K, int64_t ldx, uint8_t* Xq, void* Xs, void* Bd,
                             int64_t ldb, uint8_t* idx, void* stream) {
    int rc = check_mx_shape("osc_quantize_act_dynamic", M, K, ldx, 0);
    if (rc) return rc;
    REQUIRE(ldb >= K, OSC_ERR_SHAPE, "osc_quantize_act_dynamic: ldb=%lld < K=%lld", (long long)ldb, (long long)K);
    if (M == 0 || K == 0) return OSC_OK;
    REQUIRE(X && Xq && Xs && Bd, OSC_ERR_NULL, "osc_quantize_act_dynamic: null pointer");
    REQUIRE(ldx % 8 == 0 && aligned(X, 16) && aligned(Xq, 4) && aligned(Xs, 4) && ldb % 8 == 0 && aligned(Bd, 16) &&
                aligned(idx, 4),
            OSC_ERR_UNSUPPORTED, "osc_quantize_act_dynamic: misaligned pointer or leading dimension");
    return launch_quant_mxfp4_dynamic(static_cast<const uint16_t*>(X), M, K, ldx, Xq, static_cast<uint8_t*>(Xs),
                                      static_cast<uint16_t*>(Bd), ldb, idx, as_stream(stream));
}

static int check_gemm_common(const char* who, int64_t M, int64_t N, int64_t K, const void* Y, int y_dtype,
                             int64_t ldy) {
    REQUIRE(M >= 0 && N >= 0 && K >= 0, OSC_ERR_SHAPE, "%s: negative extent", who);
    REQUIRE(y_dtype == OSC_DT_F32 || y_dtype == OSC_DT_BF16, OSC_ERR_UNSUPPORTED, "%s: unknown y_dtype %d", who, y_dtype);
    REQUIRE(ldy >= N, OSC_ERR_SHAPE, "%s: ldy=%lld < N=%lld", who, (long long)ldy, (long long)N);
    REQUIRE(M <= 0x7fffffff && N <= 0x7fffffff && K <= 0x7fffffff, OSC_ERR_UNSUPPORTED, "%s: extent above 2^31-1", who);
    if (M > 0 && N > 0) REQUIRE(Y, OSC_ERR_NULL, "%s: Y is null", who);
    return OSC_OK;
}

static int dual_common(const char* who, const uint8_t* Xq, const uint8_t* Xs, const void* B, int64_t ldb,
                       const int32_t* row_map, const int32_t* off, int32_t E, int64_t M, const void* Wpack,
                       int64_t N, int64_t K, int32_t K_o, void* Y, int y_dtype, int64_t ldy, void* stream) {
    int rc = check_gemm_common(who, M, N, K, Y, y_dtype, ldy);
    if (rc) return rc;
    REQUIRE(K % 32 == 0, OSC_ERR_SHAPE, "%s: K=%lld is not a multiple of 32", who, (long long)K);
    REQUIRE(K_o >= 0 && K_o <= K, OSC_ERR_SHAPE, "%s: K_o=%d out of range", who, K_o);
    REQUIRE(K_o == 0 || ldb >= K_o, OSC_ERR_SHAPE, "%s: ldb=%lld < K_o=%d", who, (long long)ldb, K_o);
    if (M == 0 || N == 0) return OSC_OK;
    REQUIRE(Wpack && (K == 0 || (Xq && Xs)) && (K_o == 0 || B), OSC_ERR_NULL, "%s: null pointer", who);
    REQUIRE(aligned(Xq, 16) && aligned(Xs, 4) && aligned(Wpack, 256), OSC_ERR_UNSUPPORTED,
            "%s: Xq must be 16-byte aligned, Xs 4-byte aligned and Wpack 256-byte aligned", who);
    REQUIRE(K_o == 0 || (ldb % 8 == 0 && aligned(B, 16)), OSC_ERR_UNSUPPORTED,
            "%s: B must be 16-byte aligned with ldb %% 8 == 0", who);
    GemmProblem p{};
    p.Xq = Xq;
    p.Xs = Xs;
    p.B = static_cast<const uint16_t*>(B);
    p.ldb = K_o ? ldb : 0;
    p.row_map = row_map;
    p.expert_offsets = off;
    p.E = E;
    p.Wpack = static_cast<const uint8_t*>(Wpack);
    p.pack_stride = pack_layout(N, K, K_o).total;
    p.M = M;
    p.N = N;
    p.K = K;
    p.K_o = K_o;
    p.Y = Y;
    p.y_dtype = y_dtype;
    p.ldy = ldy;
    return launch_dual_gemm(p, as_stream(stream));
}

int osc_dual_gemm(const uint8_t* Xq, const uint8_t* Xs, const void* B, int64_t ldb, const void* Wpack,
                  int64_t M, int64_t N, int64_t K, int32_t K_o, void* Y, int y_dtype, int64_t ldy,
                  void* stream) {
    return dual_common("osc_dual_gemm", Xq, Xs, B, ldb, nullptr, nullptr, 0, M, Wpack, N, K, K_o, Y, y_dtype,
                       ldy, stream);
}

int osc_grouped_dual_gemm(const uint8_t* Xq, const uint8_t* Xs, const void* B, int64_t ldb,
                          const int32_t* row_map, const int32_t* expert_offsets, int32_t E, int64_t T,
                          const void* Wpack, int64_t N, int64_t K, int32_t K_o, void* Y, int y_dtype,
                          int64_t ldy, void* stream) {
    REQUIRE(E >= 0, OSC_ERR_SHAPE, "osc_grouped_dual_gemm: E=%d", E);
    REQUIRE(expert_offsets, OSC_ERR_NULL, "osc_grouped_dual_gemm: expert_offsets is null");
    if (E == 0) return OSC_OK;
    return dual_common("osc_grouped_dual_gemm", Xq, Xs, B, ldb, row_map, expert_offsets, E, T, Wpack, N, K, K_o,
                       Y, y_dtype, ldy, stream);
}

int osc_mxfp8_gemm(const uint8_t* X8, const uint8_t* Xs, const void* Wpack, int64_t M, int64_t N, int64_t K,
                   const int32_t* expert_offsets, int32_t E, void* Y, int y_dtype, int64_t ldy, void* stream) {
    int rc = check_gemm_common("osc_mxfp8_gemm", M, N, K, Y, y_dtype, ldy);
    if (rc) return rc;
    REQUIRE(K % 32 == 0, OSC_ERR_SHAPE, "osc_mxfp8_gemm: K=%lld is not a multiple of 32", (long long)K);
    REQUIRE(!expert_offsets || E >= 0, OSC_ERR_SHAPE, "osc_mxfp8_gemm: E=%d", E);
    if (M == 0 || N == 0 || (expert_offsets && E == 0)) return OSC_OK;
    REQUIRE(Wpack && (K == 0 || (X8 && Xs)), OSC_ERR_NULL, "osc_mxfp8_gemm: null pointer");
    REQUIRE(K % 128 == 0, OSC_ERR_UNSUPPORTED,
            "osc_mxfp8_gemm: K=%lld: only whole 128-channel lines are implemented", (long long)K);
    REQUIRE(aligned(X8, 16) && aligned(Xs, 4) && aligned(Wpack, 256), OSC_ERR_UNSUPPORTED,
            "osc_mxfp8_gemm: X8 must be 16-byte, Xs 4-byte and Wpack 256-byte aligned");
    GemmProblem p{};
    p.Xq = X8;
    p.Xs = Xs;
    p.expert_offsets = expert_offsets;
    p.E = expert_offsets ? E : 0;
    p.Wpack = static_cast<const uint8_t*>(Wpack);
    p.pack_stride = packm8_layout(N, K).total;
    p.M = M;
    p.N = N;
    p.K = K;
    p.K_o = 0;
    p.Y = Y;
    p.y_dtype = y_dtype;
    p.ldy = ldy;
    return launch_mxfp8_gemm(p, as_stream(stream));
}

int osc_fp8_gemm(const uint8_t* X8, const float* xs, const void* W8pack, int64_t M, int64_t N, int64_t K,
                 const int32_t* expert_offsets, int32_t E, void* Y, int y_dtype, int64_t ldy, void* stream) {
    int rc = check_gemm_common("osc_fp8_gemm", M, N, K, Y, y_dtype, ldy);
    if (rc) return rc;
    REQUIRE(K % 16 == 0, OSC_ERR_SHAPE, "osc_fp8_gemm: K=%lld is not a multiple of 16", (long long)K);
    REQUIRE(!expert_offsets || E >= 0, OSC_ERR_SHAPE, "osc_fp8_gemm: E=%d", E);
    if (M == 0 || N == 0 || (expert_offsets && E == 0)) return OSC_OK;
    REQUIRE(W8pack && xs && (K == 0 || X8), OSC_ERR_NULL, "osc_fp8_gemm: null pointer");
    REQUIRE(aligned(X8, 16) && aligned(W8pack, 256), OSC_ERR_UNSUPPORTED,
            "osc_fp8_gemm: X8 must be 16-byte aligned and W8pack 256-byte aligned");
    GemmProblem p{};
    p.Xq = X8;
    p.xs = xs;
    p.expert_offsets = expert_offsets;
    p.E = expert_offsets ? E : 0;
    p.Wpack = static_cast<const uint8_t*>(W8pack);
    p.pack_stride = pack8_layout(N, K).total;
    p.M = M;
    p.N = N;
    p.K = K;
    p.K_o = 0;
    p.Y = Y;
    p.y_dtype = y_dtype;
    p.ldy = ldy;
    return launch_fp8_gemm(p, as_stream(stream));
}

// ---- offline profiling -------------------------------------------------------------------

static int check_profile_x(const char* who, const void* X, int64_t S, int64_t H, int64_t ldx) {
    REQUIRE(S >= 0 && H >= 0, OSC_ERR_SHAPE, "%s: negative extent", who);
    REQUIRE(H % 8 == 0, OSC_ERR_SHAPE, "%s: H=%lld is not a multiple of 8", who, (long long)H);
    REQUIRE(ldx >= H, OSC_ERR_SHAPE, "%s: ldx=%lld < H=%lld", who, (long long)ldx, (long long)H);
    REQUIRE(H <= 0x7fffffff, OSC_ERR_UNSUPPORTED, "%s: H above 2^31-1", who);
    if (S == 0 || H == 0) return OSC_OK;
    REQUIRE(X, OSC_ERR_NULL, "%s: null pointer", who);
    REQUIRE(ldx % 8 == 0 && aligned(X, 16), OSC_ERR_UNSUPPORTED, "%s: X rows must be 16-byte aligned", who);
    return OSC_OK;
}

int osc_profile_abs_sum(const void* X, int64_t S, int64_t H, int64_t ldx, double* abs_sum, void* stream) {
    int rc = check_profile_x("osc_profile_abs_sum", X, S, H, ldx);
    if (rc) return rc;
    REQUIRE(abs_sum, OSC_ERR_NULL, "osc_profile_abs_sum: null pointer");
    REQUIRE(aligned(abs_sum, 8), OSC_ERR_UNSUPPORTED, "osc_profile_abs_sum: misaligned abs_sum");
    if (S == 0 || H == 0) return OSC_OK;
    return launch_profile_abs_sum(static_cast<const uint16_t*>(X), S, H, ldx, abs_sum, as_stream(stream));
}

int osc_profile_threshold(const double* abs_sum, int64_t count, float alpha, float* T, void* stream) {
    REQUIRE(abs_sum && T, OSC_ERR_NULL, "osc_profile_threshold: null pointer");
    REQUIRE(count > 0, OSC_ERR_SHAPE, "osc_profile_threshold: count=%lld", (long long)count);
    REQUIRE(aligned(abs_sum, 8) && aligned(T, 4), OSC_ERR_UNSUPPORTED, "osc_profile_threshold: misaligned pointer");
    return launch_profile_threshold(abs_sum, count, alpha, T, as_stream(stream));
}

int osc_profile_hist(const void* X, int64_t S, int64_t H, int64_t ldx, int32_t G, const float* T,
                     uint32_t* hist, void* stream) {
    int rc = check_profile_x("osc_profile_hist", X, S, H, ldx);
    if (rc) return rc;
    REQUIRE(G == 16 || G == 32 || G == 64, OSC_ERR_UNSUPPORTED, "osc_profile_hist: group size %d (16, 32 or 64)", G);
    REQUIRE(H % G == 0, OSC_ERR_SHAPE, "osc_profile_hist: H=%lld is not a multiple of G=%d", (long long)H, G);
    if (S == 0 || H == 0) return OSC_OK;
    REQUIRE(T && hist, OSC_ERR_NULL, "osc_profile_hist: null pointer");
    REQUIRE(aligned(T, 4) && aligned(hist, 4), OSC_ERR_UNSUPPORTED, "osc_profile_hist: misaligned pointer");
    return launch_profile_hist(static_cast<const uint16_t*>(X), S, H, ldx, G, T, hist, as_stream(stream));
}

int osc_profile_table(const uint32_t* hist, int32_t Kg, int32_t G, int32_t R, int16_t* table,
                      uint32_t* n_total, uint32_t* n_hit, float* density, float* cbar, void* stream) {
    REQUIRE(Kg >= 0 && R >= 0, OSC_ERR_SHAPE, "osc_profile_table: Kg=%d R=%d", Kg, R);
    REQUIRE(G >= 1 && G <= 64, OSC_ERR_UNSUPPORTED, "osc_profile_table: group size %d (1..64)", G);
    REQUIRE((Kg == 0 || hist) && (Kg == 0 || R == 0 || table), OSC_ERR_NULL, "osc_profile_table: null pointer");
    if (Kg == 0 && !cbar) return OSC_OK;
    return launch_profile_table(hist, Kg, G, R, table, n_total, n_hit, density, cbar, as_stream(stream));
}

// ---- 4-bit formats with a scale per 16 channels -----------------------------------------------

static int check_g16(const char* who, int64_t R, int64_t K, int64_t ld, int32_t K_o, int fmt16, float ts) {
    REQUIRE(R >= 0 && K >= 0 && K_o >= 0, OSC_ERR_SHAPE, "%s: negative extent", who);
    REQUIRE(K % 64 == 0, OSC_ERR_SHAPE, "%s: K=%lld is not a multiple of 64", who, (long long)K);
    REQUIRE(ld >= K, OSC_ERR_SHAPE, "%s: leading dimension %lld < K=%lld", who, (long long)ld, (long long)K);
    REQUIRE(K_o <= K, OSC_ERR_SHAPE, "%s: K_o=%d exceeds K", who, K_o);
    REQUIRE(fmt16 == OSC_FMT16_E8M0 || fmt16 == OSC_FMT16_NVFP4, OSC_ERR_UNSUPPORTED, "%s: unknown format %d", who, fmt16);
    REQUIRE(K <= 65536, OSC_ERR_UNSUPPORTED, "%s: K=%lld exceeds 65536", who, (long long)K);
    if (fmt16 == OSC_FMT16_NVFP4)
        REQUIRE(ts >= 0x1p-100f && ts <= 0x1p100f, OSC_ERR_SHAPE, "%s: tensor scale %g outside [2^-100, 2^100]", who, (double)ts);
    return OSC_OK;
}

int osc_quantize_act_g16(const void* X, int64_t M, int64_t K, int64_t ldx, const int32_t* oidx, int32_t K_o, int fmt16,
                         float tensor_scale, uint8_t* Xq, uint8_t* Xs16, void* B, int64_t ldb, void* stream) {
    int rc = check_g16("osc_quantize_act_g16", M, K, ldx, K_o, fmt16, tensor_scale);
    if (rc) return rc;
    REQUIRE(K_o == 0 || ldb >= K_o, OSC_ERR_SHAPE, "osc_quantize_act_g16: ldb=%lld < K_o=%d", (long long)ldb, K_o);
    if (M == 0 || K == 0) return OSC_OK;
    REQUIRE(X && Xq && Xs16 && (K_o == 0 || (oidx && B)), OSC_ERR_NULL, "osc_quantize_act_g16: null pointer");
    REQUIRE(ldx % 8 == 0 && aligned(X, 16) && aligned(Xq, 4) && aligned(Xs16, 4), OSC_ERR_UNSUPPORTED,
            "osc_quantize_act_g16: X rows must be 16-byte aligned, Xq and Xs16 4-byte aligned");
    REQUIRE(!B || (aligned(B, 2) && ldb >= 0), OSC_ERR_UNSUPPORTED, "osc_quantize_act_g16: misaligned B");
    return launch_quant_fp4_g16(static_cast<const uint16_t*>(X), M, K, ldx, oidx, K_o, fmt16, tensor_scale, Xq, Xs16,
                                static_cast<uint16_t*>(B), B ? ldb : 0, as_stream(stream));
}

size_t osc_packed_weight_g16_bytes(int64_t N, int64_t K, int32_t K_o) {
    if (N < 0 || K < 0 || K % 64 || K_o < 0) return 0;
    return pack16_layout(N, K, K_o).total;
}

int osc_pack_weight_g16(const void* W, int64_t N, int64_t K, int64_t ldw, const int32_t* oidx, int32_t K_o, int fmt16,
                        float tensor_scale, void* Wpack, void* stream) {
    int rc = check_g16("osc_pack_weight_g16", N, K, ldw, K_o, fmt16, tensor_scale);
    if (rc) return rc;
    if (N == 0) return OSC_OK;
    REQUIRE(W && Wpack && (K_o == 0 || oidx), OSC_ERR_NULL, "osc_pack_weight_g16: null pointer");
    REQUIRE(ldw % 8 == 0 && aligned(W, 16) && aligned(Wpack, 256), OSC_ERR_UNSUPPORTED,
            "osc_pack_weight_g16: W rows must be 16-byte aligned and Wpack 256-byte aligned");
    const Pack16Layout L = pack16_layout(N, K, K_o);
    uint8_t* base = static_cast<uint8_t*>(Wpack);
    if (K > 0) {
        rc = launch_quant_fp4_g16(static_cast<const uint16_t*>(W), N, K, ldw, nullptr, 0, fmt16, tensor_scale, base + L.off_q,
                                  base + L.off_s, nullptr, 0, as_stream(stream));
        if (rc) return rc;
    }
    if (hipMemsetAsync(base + L.off_z, 0, 256, as_stream(stream)) != hipSuccess)
        return fail(OSC_ERR_HIP, "osc_pack_weight_g16: cannot clear the zero block");
    return launch_gather_wl(static_cast<const uint16_t*>(W), N, K, ldw, oidx, K_o, reinterpret_cast<uint16_t*>(base + L.off_l),
                            L.ldwl, as_stream(stream));
}

int osc_unpack_weight_g16(const void* Wpack, int64_t N, int64_t K, int32_t K_o, uint8_t* Wq, uint8_t* Ws16, void* WL,
                          void* stream) {
    REQUIRE(N >= 0 && K >= 0 && K % 64 == 0 && K_o >= 0, OSC_ERR_SHAPE, "osc_unpack_weight_g16: bad shape");
    if (N == 0) return OSC_OK;
    REQUIRE(Wpack, OSC_ERR_NULL, "osc_unpack_weight_g16: null pointer");
    const Pack16Layout L = pack16_layout(N, K, K_o);
    const uint8_t* base = static_cast<const uint8_t*>(Wpack);
    hipStream_t st = as_stream(stream);
    if (Wq && K > 0 && hipMemcpyAsync(Wq, base + L.off_q, (size_t)N * (K / 2), hipMemcpyDeviceToDevice, st) != hipSuccess)
        return fail(OSC_ERR_HIP, "osc_unpack_weight_g16: copy of codes failed");
    if (Ws16 && K > 0 && hipMemcpyAsync(Ws16, base + L.off_s, (size_t)N * (K / 16), hipMemcpyDeviceToDevice, st) != hipSuccess)
        return fail(OSC_ERR_HIP, "osc_unpack_weight_g16: copy of scales failed");
    if (WL) return launch_unpack_wl(reinterpret_cast<const uint16_t*>(base + L.off_l), L.ldwl, N, K_o, static_cast<uint16_t*>(WL), st);
    return OSC_OK;
}

int osc_dual_gemm_g16(const uint8_t* Xq, const uint8_t* Xs16, float x_tensor_scale, const void* B, int64_t ldb,
                      const void* Wpack, float w_tensor_scale, int64_t M, int64_t N, int64_t K, int32_t K_o, int fmt16,
                      void* Y, int y_dtype, int64_t ldy, void* stream) {
    int rc = check_g16("osc_dual_gemm_g16", M, K, K, K_o, fmt16, x_tensor_scale);
    if (rc) return rc;
    if (fmt16 == OSC_FMT16_NVFP4)
        REQUIRE(w_tensor_scale >= 0x1p-100f && w_tensor_scale <= 0x1p100f, OSC_ERR_SHAPE,
                "osc_dual_gemm_g16: weight tensor scale %g outside [2^-100, 2^100]", (double)w_tensor_scale);
    REQUIRE(N >= 0 && ldy >= N, OSC_ERR_SHAPE, "osc_dual_gemm_g16: N=%lld ldy=%lld", (long long)N, (long long)ldy);
    REQUIRE(y_dtype == OSC_DT_F32 || y_dtype == OSC_DT_BF16, OSC_ERR_UNSUPPORTED, "osc_dual_gemm_g16: y_dtype %d", y_dtype);
    REQUIRE(K % 256 == 0 && K > 0, OSC_ERR_UNSUPPORTED,
            "osc_dual_gemm_g16: K=%lld must be a positive multiple of 256 (whole 128-byte lines of codes)", (long long)K);
    REQUIRE(K_o == 0 || (ldb >= K_o && ldb % 64 == 0), OSC_ERR_UNSUPPORTED,
            "osc_dual_gemm_g16: ldb=%lld must be a multiple of 64 and at least K_o=%d", (long long)ldb, K_o);
    if (M == 0 || N == 0) return OSC_OK;
    REQUIRE(Xq && Xs16 && Wpack && Y && (K_o == 0 || B), OSC_ERR_NULL, "osc_dual_gemm_g16: null pointer");
    REQUIRE(aligned(Xq, 16) && aligned(Xs16, 16) && aligned(Wpack, 256) && (!B || aligned(B, 16)), OSC_ERR_UNSUPPORTED,
            "osc_dual_gemm_g16: operands must be 16-byte aligned (the packed weight 256-byte)");
    const Pack16Layout L = pack16_layout(N, K, K_o);
    const uint8_t* base = static_cast<const uint8_t*>(Wpack);
    return launch_dual_gemm_g16(Xq, Xs16, x_tensor_scale, static_cast<const uint16_t*>(B), K_o ? ldb : 0, base + L.off_q,
                                base + L.off_s, reinterpret_cast<const uint16_t*>(base + L.off_l), L.ldwl, w_tensor_scale, M,
                                N, K, K_o, fmt16, Y, y_dtype, ldy, as_stream(stream));
}

size_t osc_profile_workspace_bytes(int64_t H) { return H < 0 ? 0 : profile_scratch_bytes(H); }

static int check_calibrate(const char* who, const void* X, int64_t S, int64_t H, int64_t ldx, int32_t G, int32_t R,
                           const int16_t* table) {
    int rc = check_profile_x(who, X, S, H, ldx);
    if (rc) return rc;
    REQUIRE(G == 16 || G == 32 || G == 64, OSC_ERR_UNSUPPORTED, "%s: group size %d (16, 32 or 64)", who, G);
    REQUIRE(H % G == 0, OSC_ERR_SHAPE, "%s: H=%lld is not a multiple of G=%d", who, (long long)H, G);
    REQUIRE(S > 0 && H > 0, OSC_ERR_SHAPE, "%s: empty calibration piece (S=%lld, H=%lld)", who, (long long)S, (long long)H);
    REQUIRE(R >= 0, OSC_ERR_SHAPE, "%s: R=%d", who, R);
    REQUIRE(R == 0 || table, OSC_ERR_NULL, "%s: null table", who);
    return OSC_OK;
}

int osc_profile_calibrate(const void* X, int64_t S, int64_t H, int64_t ldx, int32_t G, float alpha, int32_t R,
                          int16_t* table, uint32_t* n_total, uint32_t* n_hit, float* density, float* cbar,
                          float* T_out, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_calibrate("osc_profile_calibrate", X, S, H, ldx, G, R, table);
    if (rc) return rc;
    REQUIRE(workspace, OSC_ERR_NULL, "osc_profile_calibrate: null workspace");
    REQUIRE(aligned(workspace, 256), OSC_ERR_UNSUPPORTED, "osc_profile_calibrate: workspace must be 256-byte aligned");
    REQUIRE(workspace_bytes >= profile_scratch_bytes(H), OSC_ERR_WORKSPACE,
            "osc_profile_calibrate: workspace of %zu bytes, %zu needed", workspace_bytes, profile_scratch_bytes(H));
    return launch_profile_calibrate(static_cast<const uint16_t*>(X), S, H, ldx, G, alpha, R, table, n_total, n_hit,
                                    density, cbar, T_out, static_cast<uint8_t*>(workspace), as_stream(stream));
}

int osc_profile_calibrate_static(const void* X, int64_t S, int64_t H, int64_t ldx, int32_t G, float alpha, int32_t R,
                                 int16_t* table, uint32_t* n_total, uint32_t* n_hit, float* density, float* cbar,
                                 float* T_out, void* stream) {
    int rc = check_calibrate("osc_profile_calibrate_static", X, S, H, ldx, G, R, table);
    if (rc) return rc;
    REQUIRE(H <= PROFILE_STATIC_MAX_H, OSC_ERR_UNSUPPORTED,
            "osc_profile_calibrate_static: H=%lld exceeds the %lld channels its fixed scratch array holds "
            "(use osc_profile_calibrate with a workspace)", (long long)H, (long long)PROFILE_STATIC_MAX_H);
    return launch_profile_calibrate_static(static_cast<const uint16_t*>(X), S, H, ldx, G, alpha, R, table, n_total,
                                           n_hit, density, cbar, T_out, as_stream(stream));
}

}  // extern "C"
