"""GPU parity on seeded random shapes: the launcher's own kernel choice on sizes nobody picked by hand.

Forty shapes per case, drawn from a fixed seed so that a failure names its shape: M, N around and across
the tile borders (32, 64, 128, 256), K any multiple of 32 (row pitches that are and are not whole 64- and
128-byte lines, so every GEMM kernel family is reached), 0 to 4 protected channels per group.  The
quantiser outputs must match the oracle bit for bit, the GEMM outputs within the GEMM tolerance."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from test_gpu_parity import check_close, dev, host, pack_both, quant_both

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def osc():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2604_12782_amd as m
    m.lib()
    return m


def draw_shapes(seed, n):
    g = wl.rng(seed)
    borders = np.array([1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 383, 511, 512, 513, 700])
    out = []
    for _ in range(n):
        M = int(g.choice(borders)) if g.random() < 0.6 else int(g.integers(1, 900))
        N = int(g.choice(borders)) if g.random() < 0.6 else int(g.integers(1, 900))
        # K: mostly multiples of 256 (whole 128-byte lines of codes), some of 128, some of 32
        u = g.random()
        K = int(g.integers(1, 9)) * 256 if u < 0.5 else int(g.integers(1, 17)) * 128 if u < 0.8 else int(g.integers(1, 40)) * 32
        r = int(g.choice([0, 1, 2, 4]))
        out.append((M, N, K, r))
    return out


SHAPES = draw_shapes(9001, 40)


@pytest.mark.parametrize("M,N,K,r", SHAPES)
def test_dual_path_layer_random_shape(osc, M, N, K, r):
    X, table = wl.activations_persistent(9100 + M + K, M, K, r) if r else (wl.activations_diffuse(9100 + M + K, M, K), None)
    W = wl.weights(9200 + N + K, N, K)
    oidx = oracle.table_to_index(table) if r else np.zeros(0, np.int32)
    (Xq, Xs, B), (rq, rs, rb) = quant_both(osc, X, oidx)
    Wp, (wq, ws, wlr) = pack_both(osc, W, oidx)
    ref = oracle.dual_gemm(rq, rs, rb if r else None, wq, ws, wlr)
    for ydt, bf in ((osc.OSC_DT_F32, False), (osc.OSC_DT_BF16, True)):
        Y = osc.osc_dual_gemm(Xq, Xs, B, Wp, N, K, len(oidx), ydt)
        check_close(host(Y.float()), ref, f"dual {M}x{N}x{K} r={r} bf16={bf}", bf)


@pytest.mark.parametrize("M,N,K,r", SHAPES[:24])
def test_fp8_layer_random_shape(osc, M, N, K, r):
    K8 = max(K // 4 // 16 * 16, 16) if K % 128 else K  # 8-bit rows: any multiple of 16 (the weight pack asks for it)
    X = wl.activations_diffuse(9300 + M + K8, M, K8)
    W = wl.weights(9400 + N + K8, N, K8)
    X8, xs = osc.osc_quantize_act(dev(X), None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    r8, rs = oracle.quantize_fp8_rows(X)
    assert np.array_equal(host(X8), r8) and np.array_equal(host(xs).view(np.uint32), rs.view(np.uint32))
    w8, ws = oracle.quantize_fp8_rows(W)
    Y = osc.osc_fp8_gemm(X8, xs, osc.osc_pack_weight_fp8(dev(W)), N, K8)
    check_close(host(Y.float()), oracle.fp8_gemm(r8, rs, w8, ws), f"fp8 {M}x{N}x{K8}")
    if K8 % 128 == 0:
        Xm, Xms = osc.osc_quantize_act(dev(X), None, osc.OSC_FMT_MXFP8)
        q, s = oracle.quantize_mxfp8(X)
        assert np.array_equal(host(Xm), q) and np.array_equal(host(osc.osc_unpack_act_scales(Xms, M, K8)), s)
        wq, wsc = oracle.quantize_mxfp8(W)
        Ym = osc.osc_mxfp8_gemm(Xm, Xms, osc.osc_pack_weight_mxfp8(dev(W)), N, K8)
        check_close(host(Ym.float()), oracle.mxfp8_gemm(q, s, wq, wsc), f"mxfp8 {M}x{N}x{K8}")
