"""ctypes binding of libosc.  Argument marshalling only: torch tensors in, torch tensors out,
each function named after the C entry point it calls (see include/osc.h for the contract).

bf16 tensors may be torch.bfloat16 or raw torch.uint16/int16 bit patterns.
"""
import ctypes as C
import os

import numpy as np
import torch

OSC_DT_F32, OSC_DT_BF16 = 0, 1
OSC_FMT_MXFP4_OSC, OSC_FMT_FP8_E4M3_TOKEN, OSC_FMT_MXFP8, OSC_FMT_MXFP4_OSC_G64 = 0, 1, 2, 3
OSC_FMT16_E8M0, OSC_FMT16_NVFP4 = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libosc.so")
_lib = None

i64, i32, vp, sz = C.c_int64, C.c_int32, C.c_void_p, C.c_size_t
_SIGS = {
    "osc_last_error": (C.c_char_p, []),
    "osc_version": (C.c_int, []),
    "osc_table_to_index": (C.c_int, [vp, i32, i32, vp, vp]),
    "osc_table_to_index_g": (C.c_int, [vp, i32, i32, i32, vp, vp]),
    "osc_packed_weight_bytes": (sz, [i64, i64, i32]),
    "osc_pack_weight_g": (C.c_int, [vp, i64, i64, i64, vp, i32, i32, vp, vp]),
    "osc_pack_weight": (C.c_int, [vp, i64, i64, i64, vp, i32, vp, vp]),
    "osc_unpack_weight": (C.c_int, [vp, i64, i64, i32, vp, vp, vp, vp]),
    "osc_packed_weight_fp8_bytes": (sz, [i64, i64]),
    "osc_pack_weight_fp8": (C.c_int, [vp, i64, i64, i64, vp, vp]),
    "osc_unpack_weight_fp8": (C.c_int, [vp, i64, i64, vp, vp, vp]),
    "osc_packed_weight_mxfp8_bytes": (sz, [i64, i64]),
    "osc_pack_weight_mxfp8": (C.c_int, [vp, i64, i64, i64, vp, vp]),
    "osc_unpack_weight_mxfp8": (C.c_int, [vp, i64, i64, vp, vp, vp]),
    "osc_mxfp8_gemm": (C.c_int, [vp, vp, vp, i64, i64, i64, vp, i32, vp, C.c_int, i64, vp]),
    "osc_act_scale_bytes": (sz, [i64, i64]),
    "osc_unpack_act_scales": (C.c_int, [vp, i64, i64, vp, vp]),
    "osc_quantize_act": (C.c_int, [vp, i64, i64, i64, vp, i32, C.c_int, vp, vp, vp, i64, vp]),
    "osc_dual_gemm": (C.c_int, [vp, vp, vp, i64, vp, i64, i64, i64, i32, vp, C.c_int, i64, vp]),
    "osc_fp8_gemm": (C.c_int, [vp, vp, vp, i64, i64, i64, vp, i32, vp, C.c_int, i64, vp]),
    "osc_rmsnorm_quantize_act": (C.c_int, [vp, vp, C.c_float, i64, i64, i64, vp, i32, vp, vp, vp, i64, vp, vp]),
    "osc_swiglu_quantize_act": (C.c_int, [vp, vp, i64, i64, i64, i64, vp, vp, vp, vp]),
    "osc_swiglu_quantize_act_fp8": (C.c_int, [vp, vp, i64, i64, i64, i64, vp, vp, vp, vp]),
    "osc_quantize_act_dynamic": (C.c_int, [vp, i64, i64, i64, vp, vp, vp, i64, vp, vp]),
    "osc_tuning_set": (C.c_int, [C.c_int, C.c_int]),
    "osc_tuning_get": (C.c_int, [C.c_int]),
    "osc_profile_abs_sum": (C.c_int, [vp, i64, i64, i64, vp, vp]),
    "osc_profile_threshold": (C.c_int, [vp, i64, C.c_float, vp, vp]),
    "osc_profile_hist": (C.c_int, [vp, i64, i64, i64, i32, vp, vp, vp]),
    "osc_profile_table": (C.c_int, [vp, i32, i32, i32, vp, vp, vp, vp, vp, vp]),
    "osc_profile_workspace_bytes": (sz, [i64]),
    "osc_profile_calibrate": (C.c_int, [vp, i64, i64, i64, i32, C.c_float, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]),
    "osc_profile_calibrate_static": (C.c_int, [vp, i64, i64, i64, i32, C.c_float, i32, vp, vp, vp, vp, vp, vp, vp]),
    "osc_quantize_act_g16": (C.c_int, [vp, i64, i64, i64, vp, i32, C.c_int, C.c_float, vp, vp, vp, i64, vp]),
    "osc_packed_weight_g16_bytes": (sz, [i64, i64, i32]),
    "osc_pack_weight_g16": (C.c_int, [vp, i64, i64, i64, vp, i32, C.c_int, C.c_float, vp, vp]),
    "osc_unpack_weight_g16": (C.c_int, [vp, i64, i64, i32, vp, vp, vp, vp]),
    "osc_dual_gemm_g16": (C.c_int, [vp, vp, C.c_float, vp, i64, vp, C.c_float, i64, i64, i64, i32, C.c_int, vp, C.c_int,
                                    i64, vp]),
    "osc_grouped_dual_gemm": (C.c_int, [vp, vp, vp, i64, vp, vp, i32, i64, vp, i64, i64, i32, vp,
                                        C.c_int, i64, vp]),
}


class OscError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libosc error {code}: {msg}")
        self.code = code


def lib_path():
    return _LIB_PATH


def lib():
    """The loaded C library; raises if it has not been built (there is no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise OSError(f"{_LIB_PATH} is missing: run `python paper_2604_12782_amd/build.py` "
                          "(or __graft_entry__.build()) first")
        _lib = C.CDLL(_LIB_PATH)
        for name, (res, args) in _SIGS.items():
            fn = getattr(_lib, name)
            fn.restype, fn.argtypes = res, args
    return _lib


def osc_last_error():
    return lib().osc_last_error().decode()


def osc_version():
    return lib().osc_version()


def _check(rc):
    if rc != 0:
        raise OscError(rc, osc_last_error())


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _rows16(t):
    assert t.dim() == 2 and t.stride(1) == 1 and t.element_size() == 2, "need a 2-D bf16 tensor"
    return t


def osc_table_to_index(table):
    """table: int16 [Kg, R] (host; numpy or torch) -> int32 numpy array of channel ids."""
    table = np.ascontiguousarray(np.asarray(table), dtype=np.int16)
    Kg, R = table.shape
    oidx = np.zeros(max(Kg * min(R, 32), 1), np.int32)
    n = i32(0)
    _check(lib().osc_table_to_index(table.ctypes.data, Kg, R, oidx.ctypes.data, C.addressof(n)))
    return oidx[:n.value].copy()


def osc_table_to_index_g(table, G):
    """table: int16 [Kg, R] of local indices in groups of G channels -> int32 numpy array of channel ids."""
    table = np.ascontiguousarray(np.asarray(table), dtype=np.int16)
    Kg, R = table.shape
    oidx = np.zeros(max(Kg * min(R, max(G, 1)), 1), np.int32)
    n = i32(0)
    _check(lib().osc_table_to_index_g(table.ctypes.data, Kg, R, G, oidx.ctypes.data, C.addressof(n)))
    return oidx[:n.value].copy()


def osc_packed_weight_bytes(N, K, K_o):
    return lib().osc_packed_weight_bytes(N, K, K_o)


def osc_packed_weight_fp8_bytes(N, K):
    return lib().osc_packed_weight_fp8_bytes(N, K)


def osc_pack_weight(W, oidx, out=None):
    """W bf16 [N, K] (device), oidx int32 [K_o] (device) -> packed weight (uint8 tensor)."""
    W = _rows16(W)
    N, K = W.shape
    K_o = 0 if oidx is None else int(oidx.numel())
    if out is None:
        out = torch.empty(osc_packed_weight_bytes(N, K, K_o), dtype=torch.uint8, device=W.device)
    _check(lib().osc_pack_weight(_ptr(W), N, K, W.stride(0), _ptr(oidx) if K_o else None, K_o,
                                 _ptr(out), _stream()))
    return out


def osc_pack_weight_g(W, oidx, G, out=None):
    """osc_pack_weight with scale groups of G (32 or 64) channels."""
    W = _rows16(W)
    N, K = W.shape
    K_o = 0 if oidx is None else int(oidx.numel())
    if out is None:
        out = torch.empty(osc_packed_weight_bytes(N, K, K_o), dtype=torch.uint8, device=W.device)
    _check(lib().osc_pack_weight_g(_ptr(W), N, K, W.stride(0), _ptr(oidx) if K_o else None, K_o, G,
                                   _ptr(out), _stream()))
    return out


def osc_unpack_weight(Wpack, N, K, K_o):
    dev = Wpack.device
    Wq = torch.empty((N, K // 2), dtype=torch.uint8, device=dev)
    Ws = torch.empty((N, K // 32), dtype=torch.uint8, device=dev)
    WL = torch.empty((K_o, N), dtype=torch.uint16, device=dev)
    _check(lib().osc_unpack_weight(_ptr(Wpack), N, K, K_o, _ptr(Wq), _ptr(Ws), _ptr(WL), _stream()))
    return Wq, Ws, WL


def osc_pack_weight_fp8(W, out=None):
    W = _rows16(W)
    N, K = W.shape
    if out is None:
        out = torch.empty(osc_packed_weight_fp8_bytes(N, K), dtype=torch.uint8, device=W.device)
    _check(lib().osc_pack_weight_fp8(_ptr(W), N, K, W.stride(0), _ptr(out), _stream()))
    return out


def osc_unpack_weight_fp8(W8pack, N, K):
    dev = W8pack.device
    W8 = torch.empty((N, K), dtype=torch.uint8, device=dev)
    ws = torch.empty(N, dtype=torch.float32, device=dev)
    _check(lib().osc_unpack_weight_fp8(_ptr(W8pack), N, K, _ptr(W8), _ptr(ws), _stream()))
    return W8, ws


def osc_packed_weight_mxfp8_bytes(N, K):
    return lib().osc_packed_weight_mxfp8_bytes(N, K)


def osc_pack_weight_mxfp8(W, out=None):
    W = _rows16(W)
    N, K = W.shape
    if out is None:
        out = torch.empty(osc_packed_weight_mxfp8_bytes(N, K), dtype=torch.uint8, device=W.device)
    _check(lib().osc_pack_weight_mxfp8(_ptr(W), N, K, W.stride(0), _ptr(out), _stream()))
    return out


def osc_unpack_weight_mxfp8(Wpack, N, K):
    dev = Wpack.device
    W8 = torch.empty((N, K), dtype=torch.uint8, device=dev)
    Ws = torch.empty((N, K // 32), dtype=torch.uint8, device=dev)
    _check(lib().osc_unpack_weight_mxfp8(_ptr(Wpack), N, K, _ptr(W8), _ptr(Ws), _stream()))
    return W8, Ws


def osc_act_scale_bytes(M, K):
    return lib().osc_act_scale_bytes(M, K)


def osc_unpack_act_scales(Xs, M, K):
    """Row-block-major scale tensor -> plain uint8 [M, K/32]."""
    out = torch.empty((M, K // 32), dtype=torch.uint8, device=Xs.device)
    _check(lib().osc_unpack_act_scales(_ptr(Xs), M, K, _ptr(out), _stream()))
    return out


def osc_quantize_act(X, oidx=None, fmt=OSC_FMT_MXFP4_OSC, ldb=None, out=None):
    """X bf16 [M, K] (device).  MXFP4_OSC, MXFP4_OSC_G64 -> (Xq uint8 [M,K/2], Xs uint8 row-block-major
    scales, B uint16 [M,ldb]);
    FP8_E4M3_TOKEN -> (X8 uint8 [M,K], xs float32 [M]);
    MXFP8 -> (X8 uint8 [M,K], Xs uint8 row-block-major scales).  `out` may hold preallocated outputs."""
    X = _rows16(X)
    M, K = X.shape
    dev = X.device
    if fmt == OSC_FMT_MXFP8:
        X8, Xs = out if out is not None else (torch.empty((M, K), dtype=torch.uint8, device=dev),
                                              torch.empty(osc_act_scale_bytes(M, K), dtype=torch.uint8, device=dev))
        _check(lib().osc_quantize_act(_ptr(X), M, K, X.stride(0), None, 0, fmt, _ptr(X8), _ptr(Xs),
                                      None, 0, _stream()))
        return X8, Xs
    if fmt == OSC_FMT_FP8_E4M3_TOKEN:
        X8, xs = out if out is not None else (torch.empty((M, K), dtype=torch.uint8, device=dev),
                                              torch.empty(M, dtype=torch.float32, device=dev))
        _check(lib().osc_quantize_act(_ptr(X), M, K, X.stride(0), None, 0, fmt, _ptr(X8), _ptr(xs),
                                      None, 0, _stream()))
        return X8, xs
    K_o = 0 if oidx is None else int(oidx.numel())
    if out is not None:
        Xq, Xs, B = out
        ldb = 0 if B is None else B.stride(0)
    else:
        if ldb is None:
            ldb = (K_o + 63) // 64 * 64
        Xq = torch.empty((M, K // 2), dtype=torch.uint8, device=dev)
        Xs = torch.empty(osc_act_scale_bytes(M, K), dtype=torch.uint8, device=dev)
        B = torch.empty((M, ldb), dtype=torch.uint16, device=dev) if ldb else None
    _check(lib().osc_quantize_act(_ptr(X), M, K, X.stride(0), _ptr(oidx) if K_o else None, K_o, fmt,
                                  _ptr(Xq), _ptr(Xs), _ptr(B), ldb, _stream()))
    return Xq, Xs, B


def _y(M, N, y_dtype, dev, out):
    if out is not None:
        return out
    return torch.empty((M, N), dtype=torch.float32 if y_dtype == OSC_DT_F32 else torch.bfloat16,
                       device=dev)


def osc_dual_gemm(Xq, Xs, B, Wpack, N, K, K_o, y_dtype=OSC_DT_F32, out=None):
    M = Xq.shape[0]
    Y = _y(M, N, y_dtype, Xq.device, out)
    _check(lib().osc_dual_gemm(_ptr(Xq), _ptr(Xs), _ptr(B), 0 if B is None else B.stride(0),
                               _ptr(Wpack), M, N, K, K_o, _ptr(Y), y_dtype, Y.stride(0) if M else N,
                               _stream()))
    return Y


def osc_fp8_gemm(X8, xs, W8pack, N, K, expert_offsets=None, y_dtype=OSC_DT_F32, out=None):
    M = X8.shape[0]
    Y = _y(M, N, y_dtype, X8.device, out)
    E = 0 if expert_offsets is None else int(expert_offsets.numel()) - 1
    _check(lib().osc_fp8_gemm(_ptr(X8), _ptr(xs), _ptr(W8pack), M, N, K, _ptr(expert_offsets), E,
                              _ptr(Y), y_dtype, Y.stride(0) if M else N, _stream()))
    return Y


def osc_mxfp8_gemm(X8, Xs, Wpack, N, K, expert_offsets=None, y_dtype=OSC_DT_F32, out=None):
    M = X8.shape[0]
    Y = _y(M, N, y_dtype, X8.device, out)
    E = 0 if expert_offsets is None else int(expert_offsets.numel()) - 1
    _check(lib().osc_mxfp8_gemm(_ptr(X8), _ptr(Xs), _ptr(Wpack), M, N, K, _ptr(expert_offsets), E,
                                _ptr(Y), y_dtype, Y.stride(0) if M else N, _stream()))
    return Y


def osc_grouped_dual_gemm(Xq, Xs, B, row_map, expert_offsets, T, Wpack, N, K, K_o,
                          y_dtype=OSC_DT_F32, out=None):
    Y = _y(T, N, y_dtype, Xq.device, out)
    E = int(expert_offsets.numel()) - 1
    _check(lib().osc_grouped_dual_gemm(_ptr(Xq), _ptr(Xs), _ptr(B), 0 if B is None else B.stride(0),
                                       _ptr(row_map), _ptr(expert_offsets), E, T, _ptr(Wpack), N, K,
                                       K_o, _ptr(Y), y_dtype, Y.stride(0) if T else N, _stream()))
    return Y


def osc_profile_abs_sum(X, abs_sum=None):
    """abs_sum (float64 [1], device) += sum |X|; a zeroed accumulator is made when none is given."""
    X = _rows16(X)
    if abs_sum is None:
        abs_sum = torch.zeros(1, dtype=torch.float64, device=X.device)
    _check(lib().osc_profile_abs_sum(_ptr(X), X.shape[0], X.shape[1], X.stride(0), _ptr(abs_sum), _stream()))
    return abs_sum


def osc_profile_threshold(abs_sum, count, alpha=5.0, out=None):
    """T (float32 [1], device) = alpha * abs_sum / count."""
    if out is None:
        out = torch.empty(1, dtype=torch.float32, device=abs_sum.device)
    _check(lib().osc_profile_threshold(_ptr(abs_sum), count, alpha, _ptr(out), _stream()))
    return out


def osc_profile_hist(X, T, G=32, hist=None):
    """hist (uint32 as int32 [H/G, G], device) += per-token group-argmax counts above T (device float)."""
    X = _rows16(X)
    S, H = X.shape
    if hist is None:
        hist = torch.zeros((H // G, G), dtype=torch.int32, device=X.device)
    _check(lib().osc_profile_hist(_ptr(X), S, H, X.stride(0), G, _ptr(T), _ptr(hist), _stream()))
    return hist


def osc_profile_table(hist, R=1):
    """-> (table int16 [Kg, R], n_total int32 [Kg], n_hit int32 [Kg], density float32 [Kg], cbar float32 [1])."""
    Kg, G = hist.shape
    dev = hist.device
    table = torch.empty((Kg, R), dtype=torch.int16, device=dev)
    n_total = torch.empty(Kg, dtype=torch.int32, device=dev)
    n_hit = torch.empty(Kg, dtype=torch.int32, device=dev)
    density = torch.empty(Kg, dtype=torch.float32, device=dev)
    cbar = torch.empty(1, dtype=torch.float32, device=dev)
    _check(lib().osc_profile_table(_ptr(hist), Kg, G, R, _ptr(table), _ptr(n_total), _ptr(n_hit), _ptr(density),
                                   _ptr(cbar), _stream()))
    return table, n_total, n_hit, density, cbar


def osc_profile_workspace_bytes(H):
    return lib().osc_profile_workspace_bytes(H)


def _calibrate_outputs(H, G, R, dev, out):
    if out is not None:
        return out
    Kg = H // G
    return (torch.empty((Kg, R), dtype=torch.int16, device=dev), torch.empty(Kg, dtype=torch.int32, device=dev),
            torch.empty(Kg, dtype=torch.int32, device=dev), torch.empty(Kg, dtype=torch.float32, device=dev),
            torch.empty(1, dtype=torch.float32, device=dev), torch.empty(1, dtype=torch.float32, device=dev))


def osc_profile_calibrate(X, G=32, alpha=5.0, R=1, workspace=None, out=None):
    """Alg. 1 in one call -> (table, n_total, n_hit, density, cbar, T).  `workspace`: uint8 device
    tensor of osc_profile_workspace_bytes(H) bytes (allocated here when not given)."""
    X = _rows16(X)
    S, H = X.shape
    if workspace is None:
        workspace = torch.empty(osc_profile_workspace_bytes(H), dtype=torch.uint8, device=X.device)
    o = _calibrate_outputs(H, G, R, X.device, out)
    _check(lib().osc_profile_calibrate(_ptr(X), S, H, X.stride(0), G, alpha, R, *[_ptr(t) for t in o], _ptr(workspace),
                                       workspace.numel(), _stream()))
    return o


def osc_profile_calibrate_static(X, G=32, alpha=5.0, R=1, out=None):
    """osc_profile_calibrate on the library's own fixed scratch array (H <= 16384); with `out` given
    (the six output tensors) the call allocates nothing at all."""
    X = _rows16(X)
    S, H = X.shape
    o = _calibrate_outputs(H, G, R, X.device, out)
    _check(lib().osc_profile_calibrate_static(_ptr(X), S, H, X.stride(0), G, alpha, R, *[_ptr(t) for t in o], _stream()))
    return o


def osc_quantize_act_g16(X, oidx=None, fmt16=OSC_FMT16_E8M0, tensor_scale=1.0, ldb=None, out=None):
    """4-bit quantiser with one scale per 16 channels -> (Xq uint8 [M, K/2], Xs16 uint8 [M, K/16], B or None)."""
    X = _rows16(X)
    M, K = X.shape
    dev = X.device
    K_o = 0 if oidx is None else int(oidx.numel())
    if ldb is None:
        ldb = (K_o + 63) // 64 * 64
    if out is not None:
        Xq, Xs, B = out
    else:
        Xq = torch.empty((M, K // 2), dtype=torch.uint8, device=dev)
        Xs = torch.empty((M, K // 16), dtype=torch.uint8, device=dev)
        B = torch.empty((M, ldb), dtype=torch.uint16, device=dev) if ldb else None
    _check(lib().osc_quantize_act_g16(_ptr(X), M, K, X.stride(0), _ptr(oidx), K_o, fmt16, float(tensor_scale), _ptr(Xq),
                                      _ptr(Xs), _ptr(B), ldb, _stream()))
    return Xq, Xs, B


def osc_packed_weight_g16_bytes(N, K, K_o):
    return lib().osc_packed_weight_g16_bytes(N, K, K_o)


def osc_pack_weight_g16(W, oidx=None, fmt16=OSC_FMT16_E8M0, tensor_scale=1.0, out=None):
    W = _rows16(W)
    N, K = W.shape
    K_o = 0 if oidx is None else int(oidx.numel())
    if out is None:
        out = torch.empty(osc_packed_weight_g16_bytes(N, K, K_o), dtype=torch.uint8, device=W.device)
    _check(lib().osc_pack_weight_g16(_ptr(W), N, K, W.stride(0), _ptr(oidx), K_o, fmt16, float(tensor_scale), _ptr(out),
                                     _stream()))
    return out


def osc_unpack_weight_g16(Wpack, N, K, K_o):
    dev = Wpack.device
    Wq = torch.empty((N, K // 2), dtype=torch.uint8, device=dev)
    Ws = torch.empty((N, K // 16), dtype=torch.uint8, device=dev)
    WL = torch.empty((K_o, N), dtype=torch.uint16, device=dev) if K_o else None
    _check(lib().osc_unpack_weight_g16(_ptr(Wpack), N, K, K_o, _ptr(Wq), _ptr(Ws), _ptr(WL), _stream()))
    return Wq, Ws, WL


def osc_dual_gemm_g16(Xq, Xs16, B, Wpack, N, K, K_o, fmt16=OSC_FMT16_E8M0, x_tensor_scale=1.0, w_tensor_scale=1.0,
                      y_dtype=OSC_DT_F32, out=None):
    M = Xq.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=torch.bfloat16 if y_dtype == OSC_DT_BF16 else torch.float32, device=Xq.device)
    _check(lib().osc_dual_gemm_g16(_ptr(Xq), _ptr(Xs16), float(x_tensor_scale), _ptr(B), 0 if B is None else B.stride(0),
                                   _ptr(Wpack), float(w_tensor_scale), M, N, K, K_o, fmt16, _ptr(out), y_dtype,
                                   out.stride(0), _stream()))
    return out


def osc_quantize_act_dynamic(X, ldb=None, want_idx=True, out=None):
    """Dynamic protection -> (Xq, Xs, Bd uint16 [M, ldb] dense, idx uint8 [M, K/32] or None)."""
    X = _rows16(X)
    M, K = X.shape
    dev = X.device
    if ldb is None:
        ldb = K
    if out is not None:
        Xq, Xs, Bd, idx = out
    else:
        Xq = torch.empty((M, K // 2), dtype=torch.uint8, device=dev)
        Xs = torch.empty(osc_act_scale_bytes(M, K), dtype=torch.uint8, device=dev)
        Bd = torch.empty((M, ldb), dtype=torch.uint16, device=dev)
        idx = torch.empty((M, K // 32), dtype=torch.uint8, device=dev) if want_idx else None
    _check(lib().osc_quantize_act_dynamic(_ptr(X), M, K, X.stride(0), _ptr(Xq), _ptr(Xs), _ptr(Bd), ldb, _ptr(idx),
                                          _stream()))
    return Xq, Xs, Bd, idx


def osc_rmsnorm_quantize_act(X, gamma, eps=1e-6, oidx=None, ldb=None, want_norm=False, out=None):
    """RMSNorm + OSC quantiser in one pass -> (Xq, Xs, B, Xn or None)."""
    X = _rows16(X)
    M, K = X.shape
    dev = X.device
    K_o = 0 if oidx is None else int(oidx.numel())
    if out is not None:
        Xq, Xs, B, Xn = out
        ldb = 0 if B is None else B.stride(0)
    else:
        if ldb is None:
            ldb = (K_o + 63) // 64 * 64
        Xq = torch.empty((M, K // 2), dtype=torch.uint8, device=dev)
        Xs = torch.empty(osc_act_scale_bytes(M, K), dtype=torch.uint8, device=dev)
        B = torch.empty((M, ldb), dtype=torch.uint16, device=dev) if ldb else None
        Xn = torch.empty((M, K), dtype=torch.uint16, device=dev) if want_norm else None
    _check(lib().osc_rmsnorm_quantize_act(_ptr(X), _ptr(gamma), eps, M, K, X.stride(0), _ptr(oidx), K_o, _ptr(Xq),
                                          _ptr(Xs), _ptr(B), ldb, _ptr(Xn), _stream()))
    return Xq, Xs, B, Xn


OSC_TUNE_GEMM_TILE, OSC_TUNE_GEMM_KERNEL, OSC_TUNE_GROUPED_ONE_TILE, OSC_TUNE_SWIGLU_TABLE = 0, 1, 2, 3
OSC_TUNE_GEMM_KSPLIT = 4


def osc_tuning_set(knob, value):
    """Kernel-choice override for tests and tuning (include/osc_tuning.h); value < 0 = automatic."""
    _check(lib().osc_tuning_set(knob, -1 if value is None else int(value)))


def osc_tuning_get(knob):
    return lib().osc_tuning_get(knob)


def osc_swiglu_quantize_act(G, U, want_y=False, out=None):
    """SwiGLU + MXFP8 quantiser in one pass -> (Xq uint8 [M, K], Xs, Yn uint16 [M, K] or None)."""
    G, U = _rows16(G), _rows16(U)
    M, K = G.shape
    assert U.shape == G.shape
    dev = G.device
    if out is not None:
        Xq, Xs, Yn = out
    else:
        Xq = torch.empty((M, K), dtype=torch.uint8, device=dev)
        Xs = torch.empty(osc_act_scale_bytes(M, K), dtype=torch.uint8, device=dev)
        Yn = torch.empty((M, K), dtype=torch.uint16, device=dev) if want_y else None
    _check(lib().osc_swiglu_quantize_act(_ptr(G), _ptr(U), M, K, G.stride(0), U.stride(0), _ptr(Xq), _ptr(Xs),
                                         _ptr(Yn), _stream()))
    return Xq, Xs, Yn


def osc_swiglu_quantize_act_fp8(G, U, want_y=False, out=None):
    """SwiGLU + per-token FP8 quantiser in one pass -> (X8 uint8 [M, K], xs float32 [M], Yn uint16 [M, K] or None)."""
    G, U = _rows16(G), _rows16(U)
    M, K = G.shape
    assert U.shape == G.shape
    dev = G.device
    if out is not None:
        X8, xs, Yn = out
    else:
        X8 = torch.empty((M, K), dtype=torch.uint8, device=dev)
        xs = torch.empty(M, dtype=torch.float32, device=dev)
        Yn = torch.empty((M, K), dtype=torch.uint16, device=dev) if want_y else None
    _check(lib().osc_swiglu_quantize_act_fp8(_ptr(G), _ptr(U), M, K, G.stride(0), U.stride(0), _ptr(X8), _ptr(xs),
                                             _ptr(Yn), _stream()))
    return X8, xs, Yn
