"""GPU parity of the 4-bit formats with one scale per 16 channels (E8M0 per 16; NVFP4) against the CPU
oracle: codes, scale bytes, gathered sub-tensor and packed weights bit for bit; the dual-path GEMM
within 1e-3 * max|Y| on the same quantised operands."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from test_gpu_parity import check_close, dev, host, osc  # noqa: F401  (osc is a fixture)

pytestmark = pytest.mark.gpu

FORMATS = [(0, 1.0, 1.0), (1, 1.0 / 64, 1.0 / 4096), (1, 0.0123, 0.00071)]


def quant_both16(osc, X, oidx, fmt, ts, ldb=None):
    K_o = len(oidx)
    if ldb is None:
        ldb = (K_o + 63) // 64 * 64
    Xq, Xs, B = osc.osc_quantize_act_g16(dev(X), dev(oidx.astype(np.int32)) if K_o else None, fmt, ts, ldb=ldb)
    rq, rs, rb = oracle.quantize_fp4_g16(X, oidx if K_o else None, ldb=ldb, fmt=fmt, tensor_scale=ts)
    assert np.array_equal(host(Xs), rs), "scale bytes differ"
    assert np.array_equal(host(Xq), rq), "E2M1 codes differ"
    if ldb:
        assert np.array_equal(host(B), rb), "gathered sub-tensor differs"
    return (Xq, Xs, B), (rq, rs, rb)


@pytest.mark.parametrize("fmt,xts,wts", FORMATS)
@pytest.mark.parametrize("M,K,r", [(1, 64, 1), (7, 256, 2), (33, 1024, 1), (130, 4096, 2), (64, 1088, 0), (5, 12288, 4)])
def test_quantiser_bit_exact(osc, fmt, xts, wts, M, K, r):
    X, table = wl.activations_persistent(9100 + M, M, K, r) if r else (wl.activations_diffuse(9100 + M, M, K, p=0.02), None)
    oidx = oracle.table_to_index(table) if r else np.zeros(0, np.int32)
    quant_both16(osc, X, oidx, fmt, xts)


@pytest.mark.parametrize("fmt,xts,wts", FORMATS)
def test_quantiser_rough_values(osc, fmt, xts, wts):
    """zero blocks, tiny blocks whose scale rounds to zero, bf16 subnormals, huge values, signed zeros"""
    gen = wl.rng(9200)
    M, K = 16, 512
    x = gen.standard_normal((M, K)).astype(np.float32)
    x[0, :] = 0.0
    x[1, :64] = 2.0 ** -30
    x[2, 64:128] *= 2.0 ** 60
    x[3, ::2] = -0.0
    X = wl.to_bf16_bits(x)
    X[4, :32] = np.arange(32, dtype=np.uint16)            # positive subnormals and zero
    X[5, :32] = 0x8000 | np.arange(32, dtype=np.uint16)   # negative ones
    tab = wl.planted_table(wl.rng(9201), K, 1)
    quant_both16(osc, X, oracle.table_to_index(tab), fmt, xts)
    quant_both16(osc, X, np.zeros(0, np.int32), fmt, xts)


@pytest.mark.parametrize("fmt,xts,wts", FORMATS)
@pytest.mark.parametrize("M,N,K,r", [(1, 64, 256, 1), (16, 96, 512, 2), (40, 200, 1024, 2), (64, 1000, 256, 0),
                                      (100, 64, 768, 4), (8, 4096, 4096, 2)])
def test_dual_gemm_g16(osc, fmt, xts, wts, M, N, K, r):
    X, table = wl.activations_persistent(9300 + M, M, K, r) if r else (wl.activations_diffuse(9300 + M, M, K), None)
    W = wl.weights(9400 + N, N, K)
    oidx = oracle.table_to_index(table) if r else np.zeros(0, np.int32)
    K_o = len(oidx)
    (Xq, Xs, B), (rq, rs, rb) = quant_both16(osc, X, oidx, fmt, xts)
    Wp = osc.osc_pack_weight_g16(dev(W), dev(oidx) if K_o else None, fmt, wts)
    uq, us, ul = osc.osc_unpack_weight_g16(Wp, N, K, K_o)
    wq, ws, _ = oracle.quantize_fp4_g16(W, None, fmt=fmt, tensor_scale=wts)
    wlr = oracle.gather_wl(W, oidx) if K_o else None
    assert np.array_equal(host(uq), wq) and np.array_equal(host(us), ws)
    if K_o:
        assert np.array_equal(host(ul), wlr)
    ref = oracle.dual_gemm_g16(rq, rs, rb if K_o else None, wq, ws, wlr, fmt, xts, wts)
    for ydt, bf in ((osc.OSC_DT_F32, False), (osc.OSC_DT_BF16, True)):
        Y = osc.osc_dual_gemm_g16(Xq, Xs, B, Wp, N, K, K_o, fmt, xts, wts, ydt)
        Y2 = osc.osc_dual_gemm_g16(Xq, Xs, B, Wp, N, K, K_o, fmt, xts, wts, ydt)
        assert torch.equal(Y, Y2), "not run-to-run deterministic"
        check_close(host(Y.float()), ref, f"fmt {fmt} {M}x{N}x{K} r={r} bf16={bf}", bf16_out=bf)


@pytest.mark.parametrize("fmt,xts,wts", FORMATS[:2])
def test_decode_shape_of_the_density_sweep(osc, fmt, xts, wts):
    """the weight-bound shape of the benchmark's Table-2 rows: 64 tokens, 4096 -> 12288, one protected
    channel per 16; sampled output columns against the oracle"""
    M, N, K = 64, 12288, 4096
    tab = wl.rng(9500).integers(0, 16, (K // 16, 1)).astype(np.int16)
    oidx = oracle.table_to_index(tab, 16)
    X = wl.activations_persistent(9501, M, K, 0)[0]
    W = wl.weights(9502, N, K)
    (Xq, Xs, B), (rq, rs, rb) = quant_both16(osc, X, oidx, fmt, xts)
    Wp = osc.osc_pack_weight_g16(dev(W), dev(oidx), fmt, wts)
    Y = host(osc.osc_dual_gemm_g16(Xq, Xs, B, Wp, N, K, len(oidx), fmt, xts, wts, osc.OSC_DT_BF16).float())
    cols = np.unique(np.concatenate([[0, 31, 32, N - 1], wl.rng(9503).integers(0, N, 300)]))
    wq, ws, _ = oracle.quantize_fp4_g16(W[cols], None, fmt=fmt, tensor_scale=wts)
    ref = oracle.dual_gemm_g16(rq, rs, rb, wq, ws, oracle.gather_wl(W, oidx)[:, cols], fmt, xts, wts)
    check_close(Y[:, cols], ref, f"fmt {fmt} decode shape", bf16_out=True)
    assert np.isfinite(Y).all()
