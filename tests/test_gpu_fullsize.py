"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration that bench.py times.

The quantisers' outputs are compared with the oracle in full (bit for bit).  The GEMMs run on the
whole problem on the GPU; the oracle recomputes a seeded sample of complete output rows (all N)
from the same quantised operands, chosen to hit the first and last tile, tile borders and the
interior.  Criterion as everywhere: max|Y_gpu - Y_oracle| <= 1e-3 * max|Y_oracle| (+ the bf16
rounding of the output itself when Y is bf16).
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from test_gpu_parity import check_close, dev, host, osc  # noqa: F401  (osc is a fixture)

pytestmark = pytest.mark.gpu


def sample_rows(seed, M, n):
    """First/last rows, both sides of the 128- and 256-row tile borders, and random interior rows."""
    fixed = [0, 1, 31, 32, 127, 128, 255, 256, M - 257, M - 256, M - 129, M - 128, M - 2, M - 1]
    fixed = [m for m in fixed if 0 <= m < M]
    if M <= n:
        return np.arange(M)
    extra = wl.rng(seed).integers(0, M, size=max(n - len(fixed), 0)).tolist()
    return np.unique(np.array(fixed + extra, np.int64))


def quant_full(osc, X, oidx):
    """MXFP4 quantiser on the whole tensor, compared in full."""
    K_o = len(oidx)
    d_oidx = dev(oidx.astype(np.int32)) if K_o else None
    Xq, Xs, B = osc.osc_quantize_act(dev(X), d_oidx, osc.OSC_FMT_MXFP4_OSC)
    ldb = 0 if B is None else B.shape[1]
    rq, rs, rb = oracle.quantize_mxfp4_osc(X, oidx, ldb=ldb)
    assert np.array_equal(host(osc.osc_unpack_act_scales(Xs, *X.shape)), rs), "E8M0 scales differ"
    assert np.array_equal(host(Xq), rq), "E2M1 codes differ"
    if K_o:
        assert np.array_equal(host(B), rb), "gathered sub-tensor differs"
    return (Xq, Xs, B), (rq, rs, rb)


def pack_full(osc, W, oidx):
    K_o = len(oidx)
    N, K = W.shape
    d_oidx = dev(oidx.astype(np.int32)) if K_o else None
    Wp = osc.osc_pack_weight(dev(W), d_oidx)
    Wq, Ws, WL = osc.osc_unpack_weight(Wp, N, K, K_o)
    rq, rs, _ = oracle.quantize_mxfp4_osc(W)
    rl = oracle.gather_wl(W, oidx) if K_o else None
    assert np.array_equal(host(Wq), rq) and np.array_equal(host(Ws), rs), "weight codes/scales differ"
    if K_o:
        assert np.array_equal(host(WL), rl), "W_L differs"
    return Wp, (rq, rs, rl)


def dual_sampled(osc, q_dev, q_ref, Wp, w_ref, N, K, K_o, rows, y_dtype, what):
    Xq, Xs, B = q_dev
    rq, rs, rb = q_ref
    Y = osc.osc_dual_gemm(Xq, Xs, B, Wp, N, K, K_o, y_dtype)
    Y2 = osc.osc_dual_gemm(Xq, Xs, B, Wp, N, K, K_o, y_dtype)
    assert torch.equal(Y, Y2), what + ": not run-to-run deterministic"
    assert bool(torch.isfinite(Y.float()).all()), what + ": non-finite output"
    ref = oracle.dual_gemm(rq[rows], rs[rows], rb[rows] if K_o else None, *w_ref)
    got = host(Y[torch.from_numpy(rows).cuda()].float())
    check_close(got, ref, what, bf16_out=y_dtype == osc.OSC_DT_BF16)


# ---- configs[1]: Qwen3-8B attention projections (the bench workload) ---------------------------


def test_config2_attention_m8192(osc):
    M, K = 8192, 4096
    X, table = wl.activations_persistent(2001, M, K, 2)
    oidx = oracle.table_to_index(table)
    assert len(oidx) == 256
    qd, qr = quant_full(osc, X, oidx)
    rows = sample_rows(1, M, 40)
    for i, N in enumerate((4096, 1024)):
        W = wl.weights(2100 + i, N, K)
        Wp, wr = pack_full(osc, W, oidx)
        dual_sampled(osc, qd, qr, Wp, wr, N, K, 256, rows, osc.OSC_DT_BF16, f"cfg2 N={N} bf16")
        if N == 4096:
            dual_sampled(osc, qd, qr, Wp, wr, N, K, 256, rows[:16], osc.OSC_DT_F32, f"cfg2 N={N} f32")


def test_persistent_kernel_with_ragged_row_tail(osc):
    """M is not a multiple of the 256-row tile: the whole tiles and the tail rows go to different
    kernels; rows on both sides of the seam and the last rows are checked."""
    M, K, N = 8192 + 100, 4096, 4096
    X, table = wl.activations_persistent(2001, M, K, 2)
    oidx = oracle.table_to_index(table)
    qd, qr = quant_full(osc, X, oidx)
    W = wl.weights(2100, N, K)
    Wp, wr = pack_full(osc, W, oidx)
    rows = np.array([0, 255, 256, 4095, 8190, 8191, 8192, 8193, 8255, 8256, 8290, 8291], np.int64)
    dual_sampled(osc, qd, qr, Wp, wr, N, K, 256, rows, osc.OSC_DT_BF16, "ragged tail bf16")
    dual_sampled(osc, qd, qr, Wp, wr, N, K, 256, rows, osc.OSC_DT_F32, "ragged tail f32")


@pytest.mark.parametrize("M", [1, 16, 128, 2048])
def test_config2_attention_small_m(osc, M):
    K = 4096
    X, table = wl.activations_persistent(2001, M, K, 2)
    oidx = oracle.table_to_index(table)
    qd, qr = quant_full(osc, X, oidx)
    rows = sample_rows(2, M, 24)
    for i, N in enumerate((4096, 1024)):
        W = wl.weights(2100 + i, N, K)
        Wp, wr = pack_full(osc, W, oidx)
        dual_sampled(osc, qd, qr, Wp, wr, N, K, 256, rows, osc.OSC_DT_BF16, f"cfg2 M={M} N={N}")


# ---- configs[2]: Qwen3-8B FFN --------------------------------------------------------------------


def test_config3_ffn_w1w3_dual(osc):
    M, K, N = 8192, 4096, 24576
    X, table = wl.activations_persistent(3001, M, K, 2)
    oidx = oracle.table_to_index(table)
    qd, qr = quant_full(osc, X, oidx)
    W = wl.weights(3002, N, K)
    Wp, wr = pack_full(osc, W, oidx)
    del W
    dual_sampled(osc, qd, qr, Wp, wr, N, K, 256, sample_rows(3, M, 12), osc.OSC_DT_BF16, "cfg3 W1|W3")


def test_config3_ffn_w2_fp8(osc):
    M, K, N = 8192, 12288, 4096
    X = wl.activations_diffuse(3003, M, K)
    W = wl.weights(3004, N, K)
    X8, xs = osc.osc_quantize_act(dev(X), None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    r8, rs = oracle.quantize_fp8_rows(X)
    assert np.array_equal(host(xs).view(np.uint32), rs.view(np.uint32)), "fp8 scales differ"
    assert np.array_equal(host(X8), r8), "e4m3 codes differ"
    Wp = osc.osc_pack_weight_fp8(dev(W))
    w8, wsc = oracle.quantize_fp8_rows(W)
    u8, us = osc.osc_unpack_weight_fp8(Wp, N, K)
    assert np.array_equal(host(u8), w8) and np.array_equal(host(us).view(np.uint32), wsc.view(np.uint32))
    Y = osc.osc_fp8_gemm(X8, xs, Wp, N, K, y_dtype=osc.OSC_DT_BF16)
    rows = sample_rows(4, M, 16)
    ref = oracle.fp8_gemm(r8[rows], rs[rows], w8, wsc)
    check_close(host(Y[torch.from_numpy(rows).cuda()].float()), ref, "cfg3 W2 fp8", bf16_out=True)


def test_config3_ffn_w2_mxfp8(osc):
    """The same W_2 shape through the MXFP8 form of the fallback (Section 4.1, implementation details)."""
    M, K, N = 8192, 12288, 4096
    X = wl.activations_diffuse(3003, M, K)
    W = wl.weights(3004, N, K)
    X8, Xs = osc.osc_quantize_act(dev(X), None, osc.OSC_FMT_MXFP8)
    r8, rs = oracle.quantize_mxfp8(X)
    assert np.array_equal(host(osc.osc_unpack_act_scales(Xs, M, K)), rs), "mxfp8 scales differ"
    assert np.array_equal(host(X8), r8), "e4m3 codes differ"
    Wp = osc.osc_pack_weight_mxfp8(dev(W))
    w8, wsc = oracle.quantize_mxfp8(W)
    u8, us = osc.osc_unpack_weight_mxfp8(Wp, N, K)
    assert np.array_equal(host(u8), w8) and np.array_equal(host(us), wsc)
    Y = osc.osc_mxfp8_gemm(X8, Xs, Wp, N, K, y_dtype=osc.OSC_DT_BF16)
    rows = sample_rows(4, M, 16)
    ref = oracle.mxfp8_gemm(r8[rows], rs[rows], w8, wsc)
    check_close(host(Y[torch.from_numpy(rows).cuda()].float()), ref, "cfg3 W2 mxfp8", bf16_out=True)


# ---- configs[3]: Qwen3-30B-A3B MoE layer ---------------------------------------------------------


def test_config4_moe_grouped(osc):
    tokens, K, E, topk, N = 4096, 2048, 128, 8, 1536
    X, table = wl.activations_persistent(4001, tokens, K, 2)
    oidx = oracle.table_to_index(table)
    K_o = len(oidx)
    assert K_o == 128
    qd, (rq, rs, rb) = quant_full(osc, X, oidx)
    off, row_map = wl.moe_routing(4002, tokens, E, topk)
    T = int(off[-1])
    assert T == tokens * topk
    checked = [0, 1, 63, 64, 127]
    stride = osc.osc_packed_weight_bytes(N, K, K_o)
    Wp = torch.empty(E * stride, dtype=torch.uint8, device="cuda")
    d_oidx = dev(oidx)
    wref = {}
    for e in range(E):
        W = wl.weights(4100 + e, N, K)
        osc.osc_pack_weight(dev(W), d_oidx, out=Wp[e * stride:(e + 1) * stride])
        if e in checked:
            q, s, _ = oracle.quantize_mxfp4_osc(W)
            wref[e] = (q, s, oracle.gather_wl(W, oidx))
    Y = osc.osc_grouped_dual_gemm(*qd, dev(row_map), dev(off), T, Wp, N, K, K_o, osc.OSC_DT_BF16)
    assert bool(torch.isfinite(Y.float()).all())
    Yh = host(Y.float())
    for e in checked:
        lo, hi = int(off[e]), int(off[e + 1])
        assert hi > lo
        ts = np.unique(np.concatenate([[lo, hi - 1], wl.rng(e).integers(lo, hi, size=22)]))
        src = row_map[ts]
        ref = oracle.dual_gemm(rq[src], rs[src], rb[src], *wref[e])
        check_close(Yh[ts], ref, f"cfg4 expert {e}", bf16_out=True)

    # W2 of the experts: grouped FP8, rows already sorted by expert
    K2, N2 = 768, 2048
    X2 = wl.activations_diffuse(4003, T, K2)
    X8, xs = osc.osc_quantize_act(dev(X2), None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    r8, r8s = oracle.quantize_fp8_rows(X2)
    assert np.array_equal(host(X8), r8) and np.array_equal(host(xs).view(np.uint32), r8s.view(np.uint32))
    stride8 = osc.osc_packed_weight_fp8_bytes(N2, K2)
    Wp8 = torch.empty(E * stride8, dtype=torch.uint8, device="cuda")
    w8ref = {}
    for e in range(E):
        W = wl.weights(4300 + e, N2, K2)
        osc.osc_pack_weight_fp8(dev(W), out=Wp8[e * stride8:(e + 1) * stride8])
        if e in checked:
            w8ref[e] = oracle.quantize_fp8_rows(W)
    Y8 = osc.osc_fp8_gemm(X8, xs, Wp8, N2, K2, expert_offsets=dev(off), y_dtype=osc.OSC_DT_BF16)
    Y8h = host(Y8.float())
    for e in checked:
        lo, hi = int(off[e]), int(off[e + 1])
        ts = np.unique(np.concatenate([[lo, hi - 1], wl.rng(100 + e).integers(lo, hi, size=22)]))
        ref = oracle.fp8_gemm(r8[ts], r8s[ts], *w8ref[e])
        check_close(Y8h[ts], ref, f"cfg4 fp8 expert {e}", bf16_out=True)

    # the same W2 inputs in MXFP8 (Section 4.1), grouped
    Xm, Xms = osc.osc_quantize_act(dev(X2), None, osc.OSC_FMT_MXFP8)
    mq, ms_ = oracle.quantize_mxfp8(X2)
    assert np.array_equal(host(Xm), mq)
    stridem = osc.osc_packed_weight_mxfp8_bytes(N2, K2)
    Wpm = torch.empty(E * stridem, dtype=torch.uint8, device="cuda")
    wmref = {}
    for e in range(E):
        W = wl.weights(4300 + e, N2, K2)
        osc.osc_pack_weight_mxfp8(dev(W), out=Wpm[e * stridem:(e + 1) * stridem])
        if e in checked:
            wmref[e] = oracle.quantize_mxfp8(W)
    Ym = osc.osc_mxfp8_gemm(Xm, Xms, Wpm, N2, K2, expert_offsets=dev(off), y_dtype=osc.OSC_DT_BF16)
    Ymh = host(Ym.float())
    for e in checked:
        lo, hi = int(off[e]), int(off[e + 1])
        ts = np.unique(np.concatenate([[lo, hi - 1], wl.rng(200 + e).integers(lo, hi, size=22)]))
        ref = oracle.mxfp8_gemm(mq[ts], ms_[ts], *wmref[e])
        check_close(Ymh[ts], ref, f"cfg4 mxfp8 expert {e}", bf16_out=True)


# ---- configs[4]: Table-2 style sweep -------------------------------------------------------------


@pytest.mark.parametrize("r", [0, 1, 2, 4])
def test_config5_sweep(osc, r):
    N, K = 12288, 4096
    W = wl.weights(5101, N, K)
    wq, wsc, _ = oracle.quantize_mxfp4_osc(W)
    dW = dev(W)
    for M in (1, 8, 32, 64, 512, 4096):
        X, table = wl.activations_persistent(5001 + r, M, K, r, factor=64.0)
        oidx = oracle.table_to_index(table) if r else np.zeros(0, np.int32)
        assert len(oidx) == 128 * r
        qd, qr = quant_full(osc, X, oidx)
        Wp = osc.osc_pack_weight(dW, dev(oidx) if r else None)
        wr = (wq, wsc, oracle.gather_wl(W, oidx) if r else None)
        rows = sample_rows(5 + M, M, 8)
        dual_sampled(osc, qd, qr, Wp, wr, N, K, len(oidx), rows, osc.OSC_DT_BF16, f"cfg5 M={M} r={r}")


# ---- offline profiling at the headline shape (Section 2; Alg. 1) --------------------------------
def test_profile_config1_shape(osc):
    M, K = 8192, 4096
    X, planted = wl.activations_persistent(6001, M, K, 2, jitter=0.3)
    Xd = dev(X)
    acc = osc.osc_profile_abs_sum(Xd)
    T = osc.osc_profile_threshold(acc, M * K, 5.0)
    ref_T = oracle.profile_threshold(X, 5.0)
    assert abs(T.item() - ref_T) <= 1e-6 * ref_T
    for G in (16, 32, 64):
        hist = osc.osc_profile_hist(Xd, T, G)
        assert np.array_equal(host(hist).view(np.uint32), oracle.profile_hist(X, T.item(), G)), G
    hist = osc.osc_profile_hist(Xd, T, 32)
    table = osc.osc_profile_table(hist, 2)[0]
    ref_table = oracle.profile_table(oracle.profile_hist(X, T.item(), 32), 2)[0]
    assert np.array_equal(host(table), ref_table)
    assert np.array_equal(np.sort(host(table), axis=1), np.sort(planted, axis=1))


# ---- producer fusion at the headline shape ------------------------------------------------------
def test_fused_rmsnorm_quant_config1_shape(osc):
    M, K = 8192, 4096
    X, table = wl.activations_persistent(6101, M, K, 2, jitter=0.2)
    gamma = wl.to_bf16_bits((1.0 + 0.2 * wl.rng(6102).standard_normal(K)).astype(np.float32))
    oidx = oracle.table_to_index(table)
    Xq, Xs, B, Xn = osc.osc_rmsnorm_quantize_act(dev(X), dev(gamma), 1e-6, dev(oidx.astype(np.int32)), want_norm=True)
    y = oracle.rmsnorm(X, gamma, 1e-6)
    rq, rs, rb = oracle.quantize_mxfp4_osc(y, oidx, ldb=B.shape[1])
    assert np.array_equal(host(Xn), y)
    assert np.array_equal(host(osc.osc_unpack_act_scales(Xs, M, K)), rs)
    assert np.array_equal(host(Xq), rq) and np.array_equal(host(B), rb)


def test_fused_swiglu_quant_ffn_width(osc):
    """Both SwiGLU fusions at the FFN width of configs[2] (K = 12288), gate and up as the two halves
    of one buffer, compared in full."""
    M, K = 2048, 12288
    gen = wl.rng(3300)
    G = wl.to_bf16_bits((gen.standard_normal((M, K)) * 2.5).astype(np.float32))
    U = wl.activations_diffuse(3301, M, K, p=0.005)
    both = dev(np.concatenate([G, U], axis=1))
    y = oracle.swiglu(G, U)
    Xq, Xs, Yn = osc.osc_swiglu_quantize_act(both[:, :K], both[:, K:], want_y=True)
    rq, rs = oracle.quantize_mxfp8(y)
    assert np.array_equal(host(Yn), y) and np.array_equal(host(Xq), rq)
    assert np.array_equal(host(osc.osc_unpack_act_scales(Xs, M, K)), rs)
    X8, xs, _ = osc.osc_swiglu_quantize_act_fp8(both[:, :K], both[:, K:])
    r8, rsc = oracle.quantize_fp8_rows(y)
    assert np.array_equal(host(X8), r8) and np.array_equal(host(xs).view(np.uint32), rsc.view(np.uint32))
