"""GPU parity of the "Dynamic" protection control (Section 4.2; Table 3, note 3): the run-time
quantiser bit for bit against the oracle, and the linear layer built from it (Path B over all K
channels) within the GEMM tolerance."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from workloads import to_bf16_bits

pytestmark = pytest.mark.gpu
TOL = 1e-3


@pytest.fixture(scope="module")
def osc():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2604_12782_amd as m
    m.lib()
    return m


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def both(osc, X, ldb=None):
    Xq, Xs, Bd, idx = osc.osc_quantize_act_dynamic(dev(X), ldb=ldb)
    rq, rs, rb, ri = oracle.quantize_mxfp4_dynamic(X, ldb=ldb)
    M, K = X.shape
    assert np.array_equal(idx.cpu().numpy(), ri), "positions differ"
    assert np.array_equal(Bd.cpu().numpy(), rb), "backed-up values differ"
    assert np.array_equal(osc.osc_unpack_act_scales(Xs, M, K).cpu().numpy(), rs), "scales differ"
    assert np.array_equal(Xq.cpu().numpy(), rq), "codes differ"
    return (Xq, Xs, Bd), (rq, rs, rb)


@pytest.mark.parametrize("M,K", [(1, 32), (3, 96), (33, 1056), (70, 4096), (257, 2080), (16, 12288)])
def test_quantiser_bit_exact(osc, M, K):
    both(osc, wl.activations_diffuse(800 + M, M, K, p=0.02))
    both(osc, wl.activations_persistent(900 + M, M, K, 2, jitter=0.5)[0])


def test_quantiser_edge_values_and_padding(osc):
    x = np.zeros((8, 128), np.float32)
    x[0, :32] = 1.0
    x[0, 32 + 7] = -100.0
    x[1, 5], x[1, 9] = 3.0, -3.0
    x[2, 31], x[2, 0] = 2.0, -2.0
    x[3, :] = 1e-39
    x[4, 64:96] = np.arange(32) - 15.5
    x[5, 96 + 31] = 3.3e38
    X = to_bf16_bits(x)
    X[6, :] = 0x8000
    X[7, ::2] = 0x8000
    both(osc, X)
    both(osc, X, ldb=192)
    Xq, Xs, Bd, idx = osc.osc_quantize_act_dynamic(dev(X), want_idx=False)
    assert idx is None
    assert np.array_equal(Bd.cpu().numpy(), oracle.quantize_mxfp4_dynamic(X)[2])


def test_dynamic_linear_layer(osc):
    """Y = (Q_X (x) Q_W) S + Bd W^T with Bd dense: the existing dual GEMM with every channel listed."""
    M, N, K = 200, 384, 1024
    X = wl.activations_diffuse(1001, M, K, p=0.02)
    W = wl.weights(1002, N, K)
    (Xq, Xs, Bd), (rq, rs, rb) = both(osc, X)
    oidx = np.arange(K, dtype=np.int32)
    Wp = osc.osc_pack_weight(dev(W), dev(oidx))
    Y = osc.osc_dual_gemm(Xq, Xs, Bd, Wp, N, K, K)
    wq, ws, _ = oracle.quantize_mxfp4_osc(W)
    ref = oracle.dual_gemm(rq, rs, rb, wq, ws, oracle.gather_wl(W, oidx))
    err = np.abs(Y.cpu().numpy().astype(np.float64) - ref).max()
    assert err <= TOL * np.abs(ref).max(), err
    # the protected maxima are carried exactly: the dynamic layer is closer to the unquantised product
    # than plain MXFP4 without protection
    exact = wl.from_bf16_bits(X).astype(np.float64) @ wl.from_bf16_bits(W).astype(np.float64).T
    q0, s0, b0 = oracle.quantize_mxfp4_osc(X)
    plain = oracle.dual_gemm(q0, s0, b0, wq, ws, oracle.gather_wl(W, np.zeros(0, np.int32)))
    assert np.square(ref - exact).sum() < 0.5 * np.square(plain - exact).sum()
