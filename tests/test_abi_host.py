"""CPU-only checks of the C ABI: the library loads, exports every symbol the header declares,
and rejects bad arguments on the host before anything is launched (no GPU needed)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2604_12782_amd as osc
from paper_2604_12782_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(osc.lib_path()):
        from paper_2604_12782_amd import build
        build.build()
    return osc.lib()


def declared_symbols(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(osc_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound(lib):
    headers = sorted(h for h in os.listdir(os.path.join(ROOT, "include")) if h.endswith(".h"))
    assert headers == ["osc.h", "osc_probe.h", "osc_tuning.h"]
    names = declared_symbols("osc.h") + declared_symbols("osc_tuning.h")
    assert {"osc_quantize_act", "osc_dual_gemm", "osc_fp8_gemm", "osc_grouped_dual_gemm"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared but not exported"
        assert n in binding._SIGS, f"{n} has no ctypes signature"
        assert hasattr(osc, n), f"{n} has no Python binding of the same name"
    assert osc.osc_version() >= 100
    # the matrix-core yardstick lives in a library of its own that only the benchmark loads
    from paper_2604_12782_amd import probe
    for n in declared_symbols("osc_probe.h"):
        assert hasattr(probe.lib(), n) and hasattr(probe, n), n
        assert not hasattr(osc, n), f"{n} belongs to the probe library, not to the product"


def test_tuning_knobs_host(lib):
    for k in range(5):
        assert osc.osc_tuning_get(k) == -1
        osc.osc_tuning_set(k, 1)
        assert osc.osc_tuning_get(k) == 1
        osc.osc_tuning_set(k, -5)
        assert osc.osc_tuning_get(k) == -1
    assert lib.osc_tuning_set(99, 1) == -4 and lib.osc_tuning_get(99) == -1


def test_no_entry_point_reads_the_environment():
    for f in os.listdir(os.path.join(ROOT, "paper_2604_12782_amd", "csrc")):
        if f.endswith((".hip", ".h")):
            assert "getenv" not in open(os.path.join(ROOT, "paper_2604_12782_amd", "csrc", f)).read(), f


def test_table_to_index_g_host(lib):
    t = np.array([[63, -1], [0, 40], [-1, -1]], np.int16)
    assert osc.osc_table_to_index_g(t, 64).tolist() == [63, 64, 104]
    assert osc.osc_table_to_index_g(np.array([[15, 0], [-1, 3]], np.int16), 16).tolist() == [0, 15, 19]
    assert osc.osc_table_to_index_g(t[:, :1] % 32, 32).tolist() == osc.osc_table_to_index(t[:, :1] % 32).tolist()
    for bad, G in (([[64]], 64), ([[16]], 16), ([[3, 3]], 64), ([[1]], 48), ([[1]], 0)):
        with pytest.raises(osc.OscError):
            osc.osc_table_to_index_g(np.array(bad, np.int16), G)


def test_table_to_index_host(lib):
    t = np.array([[5, -1], [-1, -1], [31, 0], [-1, 7]], np.int16)
    assert osc.osc_table_to_index(t).tolist() == [5, 64, 95, 96 + 7]
    assert osc.osc_table_to_index(np.full((4, 1), -1, np.int16)).tolist() == []
    for bad in ([[32]], [[-2]], [[4, 4]]):
        with pytest.raises(osc.OscError) as e:
            osc.osc_table_to_index(np.array(bad, np.int16))
        assert e.value.code == -3


def test_packed_sizes(lib):
    # sections: codes N*K/2, scales, W_L N*round_up(K_o,64)*2, 256 zero bytes; each 256-byte aligned
    assert osc.osc_packed_weight_bytes(4096, 4096, 256) == 4096 * 2048 + 4096 * 128 + 4096 * 256 * 2 + 256
    assert osc.osc_packed_weight_bytes(256, 256, 8) == 256 * 128 + 256 * 8 + 256 * 64 * 2 + 256
    assert osc.osc_packed_weight_bytes(3, 32, 0) == 256 + 256 + 256
    # row-block-major scales: [ceil(M/32)][ceil(K/128)][32][4]
    assert osc.osc_act_scale_bytes(8192, 4096) == 8192 * 128
    assert osc.osc_act_scale_bytes(33, 96) == 2 * 1 * 128
    assert osc.osc_packed_weight_bytes(16, 33, 0) == 0  # K % 32 != 0
    assert osc.osc_packed_weight_fp8_bytes(4096, 12288) == 4096 * 12288 + 4096 * 4 + 256


FAKE = 0x10000  # a non-null, suitably aligned "device pointer" that is never dereferenced


def test_bad_arguments_are_rejected_on_the_host(lib):
    q = lib.osc_quantize_act
    # null pointers
    assert q(None, 4, 64, 64, None, 0, 0, FAKE, FAKE, None, 0, None) == -1
    assert "null" in osc.osc_last_error()
    assert q(FAKE, 4, 64, 64, None, 2, 0, FAKE, FAKE, FAKE, 8, None) == -1  # K_o > 0 without oidx
    # shapes
    assert q(FAKE, 4, 48, 48, None, 0, 0, FAKE, FAKE, None, 0, None) == -2  # K % 32
    assert q(FAKE, 4, 64, 32, None, 0, 0, FAKE, FAKE, None, 0, None) == -2  # ldx < K
    assert q(FAKE, -1, 64, 64, None, 0, 0, FAKE, FAKE, None, 0, None) == -2
    assert q(FAKE, 4, 64, 64, FAKE, 9, 0, FAKE, FAKE, FAKE, 8, None) == -2  # ldb < K_o
    # unsupported: format enum, alignment
    assert q(FAKE, 4, 64, 64, None, 0, 7, FAKE, FAKE, None, 0, None) == -4
    assert q(FAKE + 2, 4, 64, 64, None, 0, 0, FAKE, FAKE, None, 0, None) == -4
    assert q(FAKE, 4, 64, 68, None, 0, 0, FAKE, FAKE, None, 0, None) == -4  # ldx % 8
    assert q(FAKE, 4, 64, 64, FAKE, 2, 0, FAKE, FAKE, FAKE, 12, None) == -4  # ldb % 8
    # empty problems are fine and touch nothing
    assert q(None, 0, 64, 64, None, 0, 0, None, None, None, 0, None) == 0
    g = lib.osc_dual_gemm
    assert g(None, None, None, 0, None, 0, 64, 64, 0, None, 0, 64, None) == 0
    assert g(FAKE, FAKE, None, 0, FAKE, 4, 64, 48, 0, FAKE, 0, 64, None) == -2  # K % 32
    assert g(FAKE, FAKE, None, 0, FAKE, 4, 64, 64, 0, FAKE, 0, 32, None) == -2  # ldy < N
    assert g(FAKE, FAKE, None, 0, FAKE, 4, 64, 64, 0, FAKE, 5, 64, None) == -4  # y_dtype
    assert g(FAKE, FAKE, None, 0, None, 4, 64, 64, 0, FAKE, 0, 64, None) == -1  # Wpack null
    assert g(FAKE, FAKE, None, 0, FAKE, 4, 64, 64, 8, FAKE, 0, 64, None) == -2  # K_o without ldb
    f = lib.osc_fp8_gemm
    assert f(FAKE, FAKE, FAKE, 4, 64, 40, None, 0, FAKE, 0, 64, None) == -2  # K % 16
    assert f(FAKE, None, FAKE, 4, 64, 64, None, 0, FAKE, 0, 64, None) == -1
    gg = lib.osc_grouped_dual_gemm
    assert gg(FAKE, FAKE, None, 0, None, None, 2, 8, FAKE, 64, 64, 0, FAKE, 0, 64, None) == -1  # offsets null
    assert gg(FAKE, FAKE, None, 0, None, FAKE, -1, 8, FAKE, 64, 64, 0, FAKE, 0, 64, None) == -2
    p = lib.osc_pack_weight
    assert p(FAKE, 4, 40, 40, None, 0, FAKE, None) == -2
    assert p(None, 4, 64, 64, None, 0, FAKE, None) == -1
    assert p(FAKE, 4, 64, 64, None, 0, FAKE + 16, None) == -4  # Wpack alignment
    m8 = lib.osc_mxfp8_gemm
    assert m8(FAKE, FAKE, FAKE, 4, 64, 96, None, 0, FAKE, 0, 64, None) == -4  # K % 128
    assert m8(FAKE, None, FAKE, 4, 64, 128, None, 0, FAKE, 0, 64, None) == -1
    assert q(FAKE, 4, 48, 48, None, 0, 2, FAKE, FAKE, None, 0, None) == -2  # MXFP8 quantiser, K % 32
    from paper_2604_12782_amd import probe
    pr = probe.lib().osc_probe_mfma_fp4
    fl = C.c_double(0.0)
    assert pr(0, 4, FAKE, C.addressof(fl), None) == -2 and pr(4, 4, None, C.addressof(fl), None) == -1
    ps = probe.lib().osc_probe_stream
    assert ps(None, FAKE, 32768, 0, 4, None) == -1 and ps(FAKE, FAKE, 1000, 0, 4, None) == -2
    assert ps(FAKE, FAKE, 32768, 3, 4, None) == -2 and ps(FAKE, FAKE + 8, 32768, 4, 4, None) == -4
    fq = lib.osc_rmsnorm_quantize_act
    assert fq(FAKE, None, 1e-6, 4, 64, 64, None, 0, FAKE, FAKE, None, 0, None, None) == -1     # gamma
    assert fq(FAKE, FAKE, -1.0, 4, 64, 64, None, 0, FAKE, FAKE, None, 0, None, None) == -2     # eps < 0
    assert fq(FAKE, FAKE, 1e-6, 4, 48, 48, None, 0, FAKE, FAKE, None, 0, None, None) == -2     # K % 32
    assert fq(FAKE, FAKE + 2, 1e-6, 4, 64, 64, None, 0, FAKE, FAKE, None, 0, None, None) == -4
    assert fq(None, None, 1e-6, 0, 64, 64, None, 0, None, None, None, 0, None, None) == 0
    sw = lib.osc_swiglu_quantize_act
    assert sw(FAKE, None, 4, 64, 64, 64, FAKE, FAKE, None, None) == -1
    assert sw(FAKE, FAKE, 4, 64, 64, 32, FAKE, FAKE, None, None) == -2   # ldu < K
    assert sw(FAKE, FAKE, 4, 64, 68, 64, FAKE, FAKE, None, None) == -4   # ldg % 8
    assert sw(None, None, 0, 64, 64, 64, None, None, None, None) == 0
    s8 = lib.osc_swiglu_quantize_act_fp8
    assert s8(FAKE, None, 4, 64, 64, 64, FAKE, FAKE, None, None) == -1
    assert s8(FAKE, FAKE, 4, 64, 64, 32, FAKE, FAKE, None, None) == -2   # ldu < K
    assert s8(FAKE, FAKE, 4, 60, 64, 64, FAKE, FAKE, None, None) == -2   # K % 8
    assert s8(FAKE, FAKE, 4, 64, 68, 64, FAKE, FAKE, None, None) == -4   # ldg % 8
    assert s8(FAKE, FAKE, 4, 32768, 32768, 32768, FAKE, FAKE, None, None) == -4   # K above the kernel's limit
    assert s8(None, None, 0, 64, 64, 64, None, None, None, None) == 0
    dq = lib.osc_quantize_act_dynamic
    assert dq(FAKE, 4, 64, 64, FAKE, FAKE, FAKE, 32, None, None) == -2   # ldb < K
    assert dq(FAKE, 4, 48, 48, FAKE, FAKE, FAKE, 48, None, None) == -2   # K % 32
    assert dq(FAKE, 4, 64, 64, FAKE, FAKE, None, 64, None, None) == -1
    assert dq(FAKE, 4, 64, 64, FAKE, FAKE, FAKE, 64, FAKE + 1, None) == -4
    assert dq(None, 0, 64, 64, None, None, None, 64, None, None) == 0
    # offline profiling
    a = lib.osc_profile_abs_sum
    assert a(None, 4, 64, 64, FAKE, None) == -1 and a(FAKE, 4, 64, 64, None, None) == -1
    assert a(FAKE, 4, 60, 64, FAKE, None) == -2 and a(FAKE, 4, 64, 32, FAKE, None) == -2
    assert a(FAKE + 2, 4, 64, 64, FAKE, None) == -4
    assert a(None, 0, 64, 64, FAKE, None) == 0
    th = lib.osc_profile_threshold
    assert th(FAKE, 0, 5.0, FAKE, None) == -2 and th(None, 8, 5.0, FAKE, None) == -1
    h = lib.osc_profile_hist
    assert h(FAKE, 4, 64, 64, 8, FAKE, FAKE, None) == -4     # group size
    assert h(FAKE, 4, 96, 96, 64, FAKE, FAKE, None) == -2    # H % G
    assert h(FAKE, 4, 64, 64, 32, None, FAKE, None) == -1
    assert h(None, 0, 64, 64, 32, None, None, None) == 0
    t = lib.osc_profile_table
    assert t(None, 4, 32, 1, FAKE, None, None, None, None, None) == -1
    assert t(FAKE, 4, 65, 1, FAKE, None, None, None, None, None) == -4
    assert t(FAKE, -1, 32, 1, FAKE, None, None, None, None, None) == -2
    assert t(None, 0, 32, 1, None, None, None, None, None, None) == 0


def test_binding_refuses_to_run_without_the_library(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", "/nonexistent/libosc.so")
    with pytest.raises(OSError):
        binding.lib()


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: the benchmark says so and exits before touching a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)


def test_profile_calibrate_arguments(lib):
    f = lib.osc_profile_calibrate
    ok = (FAKE, 8, 64, 64, 32, 5.0, 1, FAKE, None, None, None, None, None, FAKE, 256 + 4 * 64, None)

    def call(**kw):
        names = ["X", "S", "H", "ldx", "G", "alpha", "R", "table", "n_total", "n_hit", "density", "cbar", "T", "ws", "wsb", "st"]
        a = dict(zip(names, ok))
        a.update(kw)
        return f(*[a[n] for n in names])
    assert lib.osc_profile_workspace_bytes(64) == 256 + 4 * 64 and lib.osc_profile_workspace_bytes(-1) == 0
    assert call(wsb=256 + 4 * 64 - 1) == -5                 # workspace too small
    assert call(ws=None) == -1 and call(table=None) == -1 and call(X=None) == -1
    assert call(ws=FAKE + 64) == -4                          # workspace alignment
    assert call(G=48) == -4 and call(H=72, ldx=72) == -2     # group size; H % G
    assert call(S=0) == -2 and call(R=-1) == -2 and call(ldx=32) == -2


def test_g16_arguments(lib):
    q = lib.osc_quantize_act_g16
    assert q(FAKE, 4, 96, 96, None, 0, 0, 1.0, FAKE, FAKE, None, 0, None) == -2      # K % 64
    assert q(FAKE, 4, 128, 128, None, 0, 7, 1.0, FAKE, FAKE, None, 0, None) == -4    # format
    assert q(FAKE, 4, 128, 128, None, 0, 1, 0.0, FAKE, FAKE, None, 0, None) == -2    # NVFP4 tensor scale
    assert q(None, 4, 128, 128, None, 0, 0, 1.0, FAKE, FAKE, None, 0, None) == -1
    assert q(None, 0, 128, 128, None, 0, 0, 1.0, None, None, None, 0, None) == 0
    g = lib.osc_dual_gemm_g16
    assert g(FAKE, FAKE, 1.0, None, 0, FAKE, 1.0, 4, 64, 128, 0, 0, FAKE, 0, 64, None) == -4   # K % 256
    assert g(FAKE, FAKE, 1.0, None, 0, FAKE, 1.0, 4, 64, 256, 0, 0, FAKE, 0, 32, None) == -2   # ldy < N
    assert g(FAKE, FAKE, 1.0, None, 0, FAKE, 1.0, 4, 64, 256, 0, 0, None, 0, 64, None) == -1
    assert g(FAKE, FAKE, 1.0, FAKE, 40, FAKE, 1.0, 4, 64, 256, 16, 0, FAKE, 0, 64, None) == -4  # ldb % 64
    assert lib.osc_packed_weight_g16_bytes(64, 256, 16) > 64 * 128 + 64 * 16 + 64 * 64 * 2
    assert lib.osc_packed_weight_g16_bytes(64, 100, 0) == 0
