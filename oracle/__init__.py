"""CPU oracle for the OSC dual-path linear layer -- TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes front end of ``osc_ref.c`` (see that file's header for what
each function computes and which passage of the paper it follows).  Only the
tests, the smoke check and the benchmark's ``cpu_baseline`` leg import this
package.  It shares nothing with, and never imports, the HIP library.

All bf16 tensors are numpy ``uint16`` arrays holding the bf16 bit patterns.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "osc_ref.c")
# OSC_ORACLE_SANITIZE=1 (set by tests/test_oracle_sanitized.py for a child process that preloads the
# sanitizer runtimes) selects a second build of the same source with address and undefined-behaviour
# checks compiled in
_SANITIZE = os.environ.get("OSC_ORACLE_SANITIZE") == "1"
_LIB = os.path.join(_HERE, "liboscref_san.so" if _SANITIZE else "liboscref.so")


def build(force=False):
    """Compile osc_ref.c with gcc (plain C, OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        flags = (["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                  "-fno-omit-frame-pointer"] if _SANITIZE else ["-O2"])
        subprocess.check_call(
            ["gcc", *flags, "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC", _SRC, "-lm",
             "-o", _LIB])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.ref_e2m1_decode.restype = C.c_double
        _lib.ref_e2m1_decode.argtypes = [C.c_int]
        _lib.ref_e2m1_encode.argtypes = [C.c_double, C.c_int]
        _lib.ref_e8m0_code_for_amax.argtypes = [C.c_double]
        _lib.ref_e8m0_code_for_amax_e4m3.argtypes = [C.c_double]
        _lib.ref_e4m3_decode.restype = C.c_double
        _lib.ref_e4m3_decode.argtypes = [C.c_int]
        _lib.ref_e4m3_encode.argtypes = [C.c_float]
    return _lib


class OracleError(RuntimeError):
    pass


def _check(rc, what):
    if rc != 0:
        raise OracleError(f"{what} failed with code {rc}")


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _c(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


i64 = C.c_int64
i32 = C.c_int32

# ---- scalar codecs ---------------------------------------------------------


def e2m1_decode(code):
    return lib().ref_e2m1_decode(int(code))


def e2m1_encode(v, negative=None):
    if negative is None:
        negative = bool(np.signbit(v))
    return lib().ref_e2m1_encode(float(v), int(negative))


def e8m0_code_for_amax(amax):
    return lib().ref_e8m0_code_for_amax(float(amax))


def e8m0_code_for_amax_e4m3(amax):
    """E8M0 code of an MXFP8 (E4M3 elements) block whose largest magnitude is amax."""
    return lib().ref_e8m0_code_for_amax_e4m3(float(amax))


def e4m3_decode(code):
    return lib().ref_e4m3_decode(int(code))


def e4m3_encode(v):
    return lib().ref_e4m3_encode(float(np.float32(v)))


# ---- table -----------------------------------------------------------------


def table_to_index(table, G=32):
    """table[Kg, R] int16 (local index in a group of G channels, or -1) -> ascending channel
    ids int32[K_o]."""
    table = _c(table, np.int16)
    Kg, R = table.shape
    oidx = np.zeros(max(Kg * min(R, G), 1), np.int32)
    ko = i32(0)
    _check(lib().ref_table_to_index_g(_p(table), i32(Kg), i32(R), i32(G), _p(oidx), C.byref(ko)),
           "ref_table_to_index_g")
    return oidx[:ko.value].copy()


# ---- quantisers --------------------------------------------------------------


def quantize_mxfp4_osc(X, oidx=None, ldb=None, G=32):
    """Alg. 2.  X uint16[M, K] -> (Xq uint8[M, K/2], Xs uint8[M, K/32], B uint16[M, ldb]).
    G = 64: one shared exponent per 64 channels, stored in both of its blocks of 32."""
    X = _c(X, np.uint16)
    M, K = X.shape
    oidx = np.zeros(0, np.int32) if oidx is None else _c(oidx, np.int32)
    K_o = int(oidx.shape[0])
    if ldb is None:
        ldb = (K_o + 31) // 32 * 32
    Xq = np.empty((M, K // 2), np.uint8)
    Xs = np.empty((M, K // 32), np.uint8)
    B = np.empty((M, ldb), np.uint16)
    _check(lib().ref_quantize_mxfp4_osc_g(_p(X), i64(M), i64(K), i64(K), _p(oidx), i32(K_o), i32(G),
                                          _p(Xq), _p(Xs), _p(B), i64(ldb)), "ref_quantize_mxfp4_osc_g")
    return Xq, Xs, B


def quantize_mxfp4_dynamic(X, ldb=None):
    """Dynamic protection: X uint16[M, K] -> (Xq, Xs, Bd uint16[M, ldb] dense, idx uint8[M, K/32])."""
    X = _c(X, np.uint16)
    M, K = X.shape
    if ldb is None:
        ldb = K
    Xq = np.empty((M, K // 2), np.uint8)
    Xs = np.empty((M, K // 32), np.uint8)
    Bd = np.empty((M, ldb), np.uint16)
    idx = np.empty((M, K // 32), np.uint8)
    _check(lib().ref_quantize_mxfp4_dynamic(_p(X), i64(M), i64(K), i64(K), _p(Xq), _p(Xs), _p(Bd), i64(ldb),
                                            _p(idx)), "ref_quantize_mxfp4_dynamic")
    return Xq, Xs, Bd, idx


def rmsnorm(X, gamma, eps=1e-6):
    """Order-free RMSNorm (see ref_rmsnorm): X uint16[M, K], gamma uint16[K] -> Y uint16[M, K]."""
    X, gamma = _c(X, np.uint16), _c(gamma, np.uint16)
    M, K = X.shape
    Y = np.empty((M, K), np.uint16)
    lib().ref_rmsnorm.argtypes = [C.c_void_p, C.c_void_p, C.c_double, i64, i64, i64, C.c_void_p]
    _check(lib().ref_rmsnorm(_p(X), _p(gamma), float(np.float32(eps)), M, K, K, _p(Y)), "ref_rmsnorm")
    return Y


def swiglu(G, U):
    """bf16(bf16(silu(G)) * U) with the fixed single-precision silu of ref_swiglu; uint16[M, K] each."""
    G, U = _c(G, np.uint16), _c(U, np.uint16)
    M, K = G.shape
    Y = np.empty((M, K), np.uint16)
    lib().ref_swiglu.argtypes = [C.c_void_p, C.c_void_p, i64, i64, i64, i64, C.c_void_p]
    _check(lib().ref_swiglu(_p(G), _p(U), M, K, K, K, _p(Y)), "ref_swiglu")
    return Y


def rmsnorm_plain(X, gamma, eps=1e-6, mid_round=False):
    """Textbook RMSNorm in double precision, one rounding to bf16 at the end; mid_round also rounds
    the normalised value to bf16 before the product with gamma (see ref_rmsnorm_plain)."""
    X, gamma = _c(X, np.uint16), _c(gamma, np.uint16)
    M, K = X.shape
    Y = np.empty((M, K), np.uint16)
    lib().ref_rmsnorm_plain.argtypes = [C.c_void_p, C.c_void_p, C.c_double, i64, i64, i64, C.c_int, C.c_void_p]
    _check(lib().ref_rmsnorm_plain(_p(X), _p(gamma), float(np.float32(eps)), M, K, K, int(mid_round), _p(Y)),
           "ref_rmsnorm_plain")
    return Y


def swiglu_plain(G, U, mid_round=False):
    """Textbook silu(G) * U in double precision, one rounding to bf16 at the end; mid_round also
    rounds silu(G) to bf16 before the product."""
    G, U = _c(G, np.uint16), _c(U, np.uint16)
    M, K = G.shape
    Y = np.empty((M, K), np.uint16)
    lib().ref_swiglu_plain.argtypes = [C.c_void_p, C.c_void_p, i64, i64, i64, i64, C.c_int, C.c_void_p]
    _check(lib().ref_swiglu_plain(_p(G), _p(U), M, K, K, K, int(mid_round), _p(Y)), "ref_swiglu_plain")
    return Y


def gather_wl(W, oidx):
    """W uint16[N, K] -> W_L uint16[K_o, N] (rows of the unquantised weight)."""
    W = _c(W, np.uint16)
    N, K = W.shape
    oidx = _c(oidx, np.int32)
    WL = np.empty((oidx.shape[0], N), np.uint16)
    _check(lib().ref_gather_wl(_p(W), i64(N), i64(K), i64(K), _p(oidx), i32(oidx.shape[0]),
                               _p(WL)), "ref_gather_wl")
    return WL


def quantize_fp8_rows(X):
    """X uint16[M, K] -> (X8 uint8[M, K] e4m3 codes, scale float32[M])."""
    X = _c(X, np.uint16)
    M, K = X.shape
    X8 = np.empty((M, K), np.uint8)
    xs = np.empty(M, np.float32)
    _check(lib().ref_quantize_fp8_rows(_p(X), i64(M), i64(K), i64(K), _p(X8), _p(xs)),
           "ref_quantize_fp8_rows")
    return X8, xs


def quantize_mxfp8(X):
    """X uint16[M, K] -> (Xq uint8[M, K] e4m3 codes, Xs uint8[M, K/32] E8M0 codes)."""
    X = _c(X, np.uint16)
    M, K = X.shape
    Xq = np.empty((M, K), np.uint8)
    Xs = np.empty((M, K // 32), np.uint8)
    _check(lib().ref_quantize_mxfp8(_p(X), i64(M), i64(K), i64(K), _p(Xq), _p(Xs)), "ref_quantize_mxfp8")
    return Xq, Xs


FMT16_E8M0, FMT16_NVFP4 = 0, 1


def quantize_fp4_g16(X, oidx=None, ldb=None, fmt=FMT16_E8M0, tensor_scale=1.0):
    """Alg. 2 with scale groups of 16 channels.  fmt 0: E8M0 scale per 16; fmt 1: NVFP4 (E4M3 scale per
    16, single-precision tensor scale given by the caller).
    -> (Xq uint8[M, K/2], Xs16 uint8[M, K/16], B uint16[M, ldb])."""
    X = _c(X, np.uint16)
    M, K = X.shape
    oidx = np.zeros(0, np.int32) if oidx is None else _c(oidx, np.int32)
    K_o = len(oidx)
    if ldb is None:
        ldb = K_o
    Xq = np.empty((M, K // 2), np.uint8)
    Xs = np.empty((M, K // 16), np.uint8)
    B = np.zeros((M, ldb), np.uint16)
    lib().ref_quantize_fp4_g16.argtypes = [C.c_void_p, i64, i64, i64, C.c_void_p, i32, C.c_int, C.c_float,
                                           C.c_void_p, C.c_void_p, C.c_void_p, i64]
    _check(lib().ref_quantize_fp4_g16(_p(X), M, K, K, _p(oidx) if K_o else None, K_o, fmt,
                                      float(np.float32(tensor_scale)), _p(Xq), _p(Xs), _p(B) if ldb else None, ldb),
           "ref_quantize_fp4_g16")
    return Xq, Xs, B


def dual_gemm_g16(Xq, Xs16, B, Wq, Ws16, WL, fmt=FMT16_E8M0, x_tensor_scale=1.0, w_tensor_scale=1.0):
    """Eq. (dual-path) on operands with one scale per 16 channels, in double."""
    Xq, Xs16, Wq, Ws16 = (_c(a, np.uint8) for a in (Xq, Xs16, Wq, Ws16))
    M, N = Xq.shape[0], Wq.shape[0]
    K = Xq.shape[1] * 2
    assert Wq.shape[1] * 2 == K and Xs16.shape == (M, K // 16) and Ws16.shape == (N, K // 16)
    K_o = 0 if WL is None else int(WL.shape[0])
    if K_o:
        B, WL = _c(B, np.uint16), _c(WL, np.uint16)
        ldb = B.shape[1]
    else:
        B, WL, ldb = None, None, 0
    Y = np.empty((M, N), np.float64)
    lib().ref_dual_gemm_g16.argtypes = [C.c_void_p, C.c_void_p, C.c_float, C.c_void_p, i64, C.c_void_p, C.c_void_p,
                                        C.c_float, C.c_void_p, i64, i64, i64, i32, C.c_int, C.c_void_p, i64]
    _check(lib().ref_dual_gemm_g16(_p(Xq), _p(Xs16), float(np.float32(x_tensor_scale)), _p(B), ldb, _p(Wq), _p(Ws16),
                                   float(np.float32(w_tensor_scale)), _p(WL), M, N, K, K_o, fmt, _p(Y), N),
           "ref_dual_gemm_g16")
    return Y


# ---- GEMMs -------------------------------------------------------------------


def dual_gemm(Xq, Xs, B, Wq, Ws, WL):
    """Eq. (dual-path) in double.  B uint16[M, ldb>=K_o], WL uint16[K_o, N]."""
    Xq, Xs, Wq, Ws = (_c(a, np.uint8) for a in (Xq, Xs, Wq, Ws))
    M, N = Xq.shape[0], Wq.shape[0]
    K = Xq.shape[1] * 2
    assert Wq.shape[1] * 2 == K and Xs.shape == (M, K // 32) and Ws.shape == (N, K // 32)
    K_o = 0 if WL is None else int(WL.shape[0])
    if K_o:
        B, WL = _c(B, np.uint16), _c(WL, np.uint16)
        ldb = B.shape[1]
        assert WL.shape[1] == N and B.shape[0] == M
    else:
        B, WL, ldb = None, None, 0
    Y = np.empty((M, N), np.float64)
    _check(lib().ref_dual_gemm(_p(Xq), _p(Xs), _p(B), i64(ldb), _p(Wq), _p(Ws), _p(WL), i64(M),
                               i64(N), i64(K), i32(K_o), _p(Y), i64(N)), "ref_dual_gemm")
    return Y


def grouped_dual_gemm(Xq, Xs, B, row_map, offsets, Wq, Ws, WL):
    """E experts: Wq uint8[E, N, K/2], Ws uint8[E, N, K/32], WL uint16[E, K_o, N]."""
    Xq, Xs, Wq, Ws = (_c(a, np.uint8) for a in (Xq, Xs, Wq, Ws))
    offsets = _c(offsets, np.int32)
    E, N = Wq.shape[0], Wq.shape[1]
    K = Xq.shape[1] * 2
    K_o = 0 if WL is None else int(WL.shape[1])
    if K_o:
        B, WL = _c(B, np.uint16), _c(WL, np.uint16)
        ldb = B.shape[1]
    else:
        B, WL, ldb = None, None, 0
    row_map = None if row_map is None else _c(row_map, np.int32)
    T = int(offsets[-1])
    Y = np.zeros((T, N), np.float64)
    _check(lib().ref_grouped_dual_gemm(_p(Xq), _p(Xs), _p(B), i64(ldb), _p(row_map), _p(offsets),
                                       i32(E), _p(Wq), _p(Ws), _p(WL), i64(N), i64(K), i32(K_o),
                                       _p(Y), i64(N)), "ref_grouped_dual_gemm")
    return Y


def fp8_gemm(X8, xs, W8, ws):
    X8, W8 = _c(X8, np.uint8), _c(W8, np.uint8)
    xs, ws = _c(xs, np.float32), _c(ws, np.float32)
    M, K = X8.shape
    N = W8.shape[0]
    assert W8.shape[1] == K
    Y = np.empty((M, N), np.float64)
    _check(lib().ref_fp8_gemm(_p(X8), _p(xs), _p(W8), _p(ws), i64(M), i64(N), i64(K), _p(Y),
                              i64(N)), "ref_fp8_gemm")
    return Y


def mxfp8_gemm(Xq, Xs, Wq, Ws):
    Xq, Xs, Wq, Ws = (_c(a, np.uint8) for a in (Xq, Xs, Wq, Ws))
    M, K = Xq.shape
    N = Wq.shape[0]
    assert Wq.shape[1] == K and Xs.shape == (M, K // 32) and Ws.shape == (N, K // 32)
    Y = np.empty((M, N), np.float64)
    _check(lib().ref_mxfp8_gemm(_p(Xq), _p(Xs), _p(Wq), _p(Ws), i64(M), i64(N), i64(K), _p(Y), i64(N)),
           "ref_mxfp8_gemm")
    return Y


def grouped_fp8_gemm(X8, xs, offsets, W8, ws):
    """W8 uint8[E, N, K], ws float32[E, N]; rows [off[e], off[e+1]) use expert e."""
    X8, W8 = _c(X8, np.uint8), _c(W8, np.uint8)
    xs, ws = _c(xs, np.float32), _c(ws, np.float32)
    offsets = _c(offsets, np.int32)
    E, N, K = W8.shape
    T = int(offsets[-1])
    Y = np.zeros((T, N), np.float64)
    _check(lib().ref_grouped_fp8_gemm(_p(X8), _p(xs), _p(offsets), i32(E), _p(W8), _p(ws), i64(N),
                                      i64(K), _p(Y), i64(N)), "ref_grouped_fp8_gemm")
    return Y


def profile_threshold(X, alpha=5.0):
    """Eq. 1: alpha * mean |X| over the whole [S, H] activation tensor (bf16 bits), in double."""
    X = _c(X, np.uint16)
    S, H = X.shape
    T = C.c_double(0.0)
    lib().ref_profile_threshold.argtypes = [C.c_void_p, i64, i64, i64, C.c_double, C.c_void_p]
    _check(lib().ref_profile_threshold(_p(X), S, H, H, float(alpha), C.byref(T)), "ref_profile_threshold")
    return T.value


def profile_hist(X, T, G=32, hist=None):
    """Eq. 2-3: counts [H/G, G] of the per-token group argmax positions whose magnitude exceeds T.
    Adds into ``hist`` when given."""
    X = _c(X, np.uint16)
    S, H = X.shape
    if hist is None:
        hist = np.zeros((H // G, G), np.uint32)
    assert hist.dtype == np.uint32 and hist.flags.c_contiguous and hist.shape == (H // G, G)
    lib().ref_profile_hist.argtypes = [C.c_void_p, i64, i64, i64, i32, C.c_double, C.c_void_p]
    _check(lib().ref_profile_hist(_p(X), S, H, H, G, float(T), _p(hist)), "ref_profile_hist")
    return hist


def profile_table(hist, R=1):
    """Alg. 1 table + Eq. 4 statistics from counts [Kg, G].
    Returns (table int16 [Kg, R], n_total, n_hit, density float64 [Kg], cbar)."""
    hist = _c(hist, np.uint32)
    Kg, G = hist.shape
    table = np.full((Kg, max(R, 0)), -1, np.int16)
    n_total, n_hit = np.zeros(Kg, np.uint32), np.zeros(Kg, np.uint32)
    density = np.zeros(Kg, np.float64)
    cbar = C.c_double(0.0)
    lib().ref_profile_table.argtypes = [C.c_void_p, i32, i32, i32] + [C.c_void_p] * 5
    _check(lib().ref_profile_table(_p(hist), Kg, G, R, _p(table), _p(n_total), _p(n_hit), _p(density),
                                   C.byref(cbar)), "ref_profile_table")
    return table, n_total, n_hit, density, cbar.value


def num_threads():
    return int(lib().ref_num_threads())
