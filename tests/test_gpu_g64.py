"""GPU parity for scale groups of 64 channels (Section 3.1: G in {16, 32, 64}; Table 2, row
G = 64): quantiser, weight packing and the dual-path GEMM on operands quantised that way,
through the C ABI against the CPU oracle.  Codes, scales and B bit for bit; GEMM within
1e-3 * max|Y_oracle|."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from test_gpu_parity import check_close, dev, host, osc  # noqa: F401

pytestmark = pytest.mark.gpu


def quant_both_g64(osc, X, oidx, ldb=None):
    K_o = len(oidx)
    if ldb is None:
        ldb = (K_o + 63) // 64 * 64
    d_oidx = dev(oidx.astype(np.int32)) if K_o else None
    Xq, Xs, B = osc.osc_quantize_act(dev(X), d_oidx, osc.OSC_FMT_MXFP4_OSC_G64, ldb=ldb)
    rq, rs, rb = oracle.quantize_mxfp4_osc(X, oidx, ldb=ldb, G=64)
    torch.cuda.synchronize()
    assert np.array_equal(host(osc.osc_unpack_act_scales(Xs, *X.shape)), rs), "E8M0 scales differ"
    assert np.array_equal(host(Xq), rq), "E2M1 codes differ"
    if ldb:
        assert np.array_equal(host(B), rb), "gathered sub-tensor differs"
    return (Xq, Xs, B), (rq, rs, rb)


def test_table_to_index_g(osc):
    for G in (16, 32, 64):
        tab = wl.planted_table(wl.rng(40 + G), 1024, 2, group=G)
        assert np.array_equal(osc.osc_table_to_index_g(tab, G), oracle.table_to_index(tab, G=G))
    with pytest.raises(osc.OscError):
        osc.osc_table_to_index_g(np.array([[16]], np.int16), 16)
    with pytest.raises(osc.OscError):
        osc.osc_table_to_index_g(np.array([[1]], np.int16), 48)


@pytest.mark.parametrize("M,K,r", [(70, 256, 1), (33, 4096, 2), (5, 1088, 1), (130, 64, 1), (64, 8192, 0), (1, 1024, 3)])
def test_quant_g64(osc, M, K, r):
    X, table = wl.activations_persistent(6400 + M + K, M, K, r, group=64)
    oidx = oracle.table_to_index(table, G=64) if r else np.zeros(0, np.int32)
    assert len(oidx) == r * K // 64
    quant_both_g64(osc, X, oidx)
    # the two scale groupings differ on this data (else the test would not tell them apart)
    _, rs32, _ = oracle.quantize_mxfp4_osc(X, oidx)
    _, rs64, _ = oracle.quantize_mxfp4_osc(X, oidx, G=64)
    assert not np.array_equal(rs32, rs64)


def test_quant_g64_rough_values(osc):
    gen = wl.rng(6464)
    x = gen.standard_normal((40, 640)).astype(np.float32) * np.exp(gen.uniform(-40, 40, (40, 640)))
    x[0] = 0
    x[1, 64:96] = 0
    x[2, :64] = 1e-39
    X = wl.to_bf16_bits(x)
    oidx = oracle.table_to_index(wl.planted_table(gen, 640, 2, group=64), G=64)
    quant_both_g64(osc, X, oidx, ldb=32)


def test_quant_g64_shape_errors(osc):
    X = dev(np.zeros((4, 96), np.uint16))
    with pytest.raises(osc.OscError):
        osc.osc_quantize_act(X, None, osc.OSC_FMT_MXFP4_OSC_G64)
    W = dev(np.zeros((32, 96), np.uint16))
    with pytest.raises(osc.OscError):
        osc.osc_pack_weight_g(W, None, 64)
    with pytest.raises(osc.OscError):
        osc.osc_pack_weight_g(dev(np.zeros((32, 128), np.uint16)), None, 16)


@pytest.mark.parametrize("M,N,K,r", [(96, 160, 512, 1), (300, 256, 1024, 2), (17, 64, 128, 0)])
def test_pack_and_dual_gemm_g64(osc, M, N, K, r):
    X, table = wl.activations_persistent(7400 + M, M, K, r, group=64)
    W = wl.weights(7500 + N, N, K)
    oidx = oracle.table_to_index(table, G=64) if r else np.zeros(0, np.int32)
    K_o = len(oidx)
    d_oidx = dev(oidx) if K_o else None
    Wp = osc.osc_pack_weight_g(dev(W), d_oidx, 64)
    Wq, Ws, WL = osc.osc_unpack_weight(Wp, N, K, K_o)
    wq, ws, _ = oracle.quantize_mxfp4_osc(W, G=64)
    wl_ref = oracle.gather_wl(W, oidx) if K_o else None
    torch.cuda.synchronize()
    assert np.array_equal(host(Wq), wq) and np.array_equal(host(Ws), ws)
    if K_o:
        assert np.array_equal(host(WL), wl_ref)
    (Xq, Xs, B), (rq, rs, rb) = quant_both_g64(osc, X, oidx)
    Y_ref = oracle.dual_gemm(rq, rs, rb[:, :K_o] if K_o else None, wq, ws, wl_ref)
    Y = osc.osc_dual_gemm(Xq, Xs, B, Wp, N, K, K_o, osc.OSC_DT_F32)
    check_close(host(Y), Y_ref, f"g64 dual gemm {M}x{N}x{K} r={r}")
    Yb = osc.osc_dual_gemm(Xq, Xs, B, Wp, N, K, K_o, osc.OSC_DT_BF16)
    check_close(host(Yb.float()), Y_ref, "g64 dual gemm bf16 out", bf16_out=True)


def test_g64_attention_m8192_full_size():
    """The bench workload's shape with scale groups of 64: quantiser and weight packing compared in
    full, the GEMM on a sample of complete output rows (K_o = r*K/64 = 128)."""
    import paper_2604_12782_amd as m
    from test_gpu_fullsize import dual_sampled, sample_rows
    M, K, N = 8192, 4096, 4096
    X, table = wl.activations_persistent(2064, M, K, 2, group=64)
    oidx = oracle.table_to_index(table, G=64)
    assert len(oidx) == 128
    qd, qr = quant_both_g64(m, X, oidx)
    W = wl.weights(2164, N, K)
    Wp = m.osc_pack_weight_g(dev(W), dev(oidx), 64)
    Wq, Ws, WL = m.osc_unpack_weight(Wp, N, K, 128)
    wq, ws, _ = oracle.quantize_mxfp4_osc(W, G=64)
    wl_ref = oracle.gather_wl(W, oidx)
    assert np.array_equal(host(Wq), wq) and np.array_equal(host(Ws), ws) and np.array_equal(host(WL), wl_ref)
    dual_sampled(m, qd, qr, Wp, (wq, ws, wl_ref), N, K, 128, sample_rows(64, M, 32), m.OSC_DT_BF16, "g64 cfg2 bf16")


def test_profile_to_quantiser_pipeline_g64(osc):
    """The offline chain at G = 64, all on the device side: threshold (Eq. 1), per-token group
    argmax counts, table (Alg. 1), then the table through osc_table_to_index_g into the G = 64
    quantiser.  The planted table comes back, and the quantiser's gathered sub-tensor holds exactly
    the planted channels."""
    S, H, r = 600, 1024, 1
    X, planted = wl.activations_persistent(6464, S, H, r, group=64)
    dX = dev(X.view(np.int16)).view(torch.bfloat16)
    T = osc.osc_profile_threshold(osc.osc_profile_abs_sum(dX), S * H, 5.0)
    hist = osc.osc_profile_hist(dX, T, 64)
    table, n_total, n_hit, density, cbar = osc.osc_profile_table(hist, 1)
    torch.cuda.synchronize()
    assert np.array_equal(table.cpu().numpy(), planted)
    assert cbar.item() > 0.95
    # the oracle's profile of the same data agrees
    rt, _, _, _, _ = oracle.profile_table(oracle.profile_hist(X, oracle.profile_threshold(X, 5.0), G=64), 1)
    assert np.array_equal(rt, planted)
    oidx = osc.osc_table_to_index_g(table.cpu().numpy(), 64)
    assert np.array_equal(oidx, oracle.table_to_index(planted, G=64))
    (Xq, Xs, B), _ = quant_both_g64(osc, X, oidx)
    assert np.array_equal(host(B)[:, :len(oidx)], X[:, oidx])
