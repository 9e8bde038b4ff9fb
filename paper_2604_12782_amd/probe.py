"""ctypes binding of libosc_probe.so, the benchmark's yardsticks (include/osc_probe.h).
Not part of the product path: only bench.py loads it."""
import ctypes as C
import os

import torch

_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libosc_probe.so")
_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_PATH):
            raise OSError(f"{_PATH} is missing: run `python paper_2604_12782_amd/build.py` first")
        _lib = C.CDLL(_PATH)
        _lib.osc_probe_mfma_fp4.restype = C.c_int
        _lib.osc_probe_mfma_fp4.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.osc_probe_stream.restype = C.c_int
        _lib.osc_probe_stream.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_void_p]
    return _lib


def osc_probe_mfma_fp4(workgroups, iters, out=None):
    """Enqueues the matrix-core probe; returns the number of floating-point operations it performs."""
    if out is None:
        out = torch.zeros(1, dtype=torch.float32, device="cuda")
    flops = C.c_double(0.0)
    rc = lib().osc_probe_mfma_fp4(workgroups, iters, out.data_ptr(), C.addressof(flops),
                                  torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError(f"osc_probe_mfma_fp4 failed with {rc}")
    return flops.value


def osc_probe_stream(src, dst, loads_per_store=0, workgroups=8192):
    """Enqueues the streaming probe over the whole of `src` (a device tensor); returns the bytes it moves."""
    nbytes = src.numel() * src.element_size()
    rc = lib().osc_probe_stream(src.data_ptr(), dst.data_ptr(), nbytes, loads_per_store, workgroups,
                                torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError(f"osc_probe_stream failed with {rc}")
    return nbytes + (nbytes // loads_per_store if loads_per_store else 0)
