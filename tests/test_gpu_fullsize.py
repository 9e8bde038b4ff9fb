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


def sample_rows(seed, M, n, band=256):
    """First/last rows, both sides of the 128- and 256-row tile borders, one seeded row out of every
    band of `band` rows (every m-tile of every kernel is touched), and n more seeded rows anywhere."""
    if M <= n:
        return np.arange(M)
    fixed = [0, 1, 31, 32, 127, 128, 255, 256, M - 257, M - 256, M - 129, M - 128, M - 2, M - 1]
    fixed = [m for m in fixed if 0 <= m < M]
    g = wl.rng(seed)
    per_band = [int(b + g.integers(0, min(band, M - b))) for b in range(0, M, band)]
    extra = g.integers(0, M, size=n).tolist()
    return np.unique(np.array(fixed + per_band + extra, np.int64))


def tile_points(seed, M, N, bm=256, bn=256, cols=32):
    """One seeded (row, first column of a block of `cols` columns) inside every bm x bn output tile."""
    g = wl.rng(seed)
    pts = []
    for m0 in range(0, M, bm):
        for n0 in range(0, N, bn):
            m = m0 + int(g.integers(0, min(bm, M - m0)))
            w = min(bn, N - n0)
            c = n0 + (int(g.integers(0, w - cols + 1)) if w > cols else 0)
            pts.append((m, c, min(cols, N - c)))
    return pts


def check_tiles(Yh, pts, ref_fn, scale, what, bf16_out=True):
    """Yh: the whole GPU output on the host (float64-convertible); ref_fn(m, c, w) -> oracle values
    of row m, columns c .. c+w-1.  Every point against the oracle with the tolerance scaled by
    `scale` (max|Y_ref| over the sampled full rows)."""
    for m, c, w in pts:
        check_close(Yh[m:m + 1, c:c + w], ref_fn(m, c, w), f"{what} tile point ({m},{c})", bf16_out, scale=scale)


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


def dual_sampled(osc, q_dev, q_ref, Wp, w_ref, N, K, K_o, rows, y_dtype, what, tiles_seed=None):
    """Whole problem on the GPU (twice: run-to-run identical); the oracle recomputes the complete
    rows `rows` and, with tiles_seed, one seeded block of 32 columns of one seeded row inside every
    256 x 256 output tile (the oracle gets that row and those 32 weight rows only)."""
    Xq, Xs, B = q_dev
    rq, rs, rb = q_ref
    wq, ws, wlr = w_ref
    Y = osc.osc_dual_gemm(Xq, Xs, B, Wp, N, K, K_o, y_dtype)
    Y2 = osc.osc_dual_gemm(Xq, Xs, B, Wp, N, K, K_o, y_dtype)
    assert torch.equal(Y, Y2), what + ": not run-to-run deterministic"
    assert bool(torch.isfinite(Y.float()).all()), what + ": non-finite output"
    bf = y_dtype == osc.OSC_DT_BF16
    ref = oracle.dual_gemm(rq[rows], rs[rows], rb[rows] if K_o else None, *w_ref)
    got = host(Y[torch.from_numpy(rows).cuda()].float())
    check_close(got, ref, what, bf16_out=bf)
    if tiles_seed is not None:
        Yh = host(Y.float())

        def one(m, c, w):
            return oracle.dual_gemm(rq[m:m + 1], rs[m:m + 1], rb[m:m + 1] if K_o else None, wq[c:c + w], ws[c:c + w],
                                    wlr[:, c:c + w] if K_o else None)
        check_tiles(Yh, tile_points(tiles_seed, Y.shape[0], N), one, np.abs(ref).max(), what, bf)
    return Y


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
        dual_sampled(osc, qd, qr, Wp, wr, N, K, 256, rows, osc.OSC_DT_BF16, f"cfg2 N={N} bf16", tiles_seed=11 + i)
        if N == 4096:
            dual_sampled(osc, qd, qr, Wp, wr, N, K, 256, rows[:16], osc.OSC_DT_F32, f"cfg2 N={N} f32")


def test_config2_attention_m8192_fp8_comparison_leg(osc):
    """The FP8 W8A8 step the bench compares against, at the bench's sizes and through the launcher's own choice
    (N = 4096: the persistent kernel; N = 1024: the DMA kernel): the persistent-channel activations of the
    workload, sampled rows in full and a point inside every 256 x 256 tile."""
    M, K = 8192, 4096
    X, _ = wl.activations_persistent(2001, M, K, 2)
    X8, xs = osc.osc_quantize_act(dev(X), None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    r8, rs = oracle.quantize_fp8_rows(X)
    assert np.array_equal(host(X8), r8) and np.array_equal(host(xs).view(np.uint32), rs.view(np.uint32))
    rows = sample_rows(5, M, 24)
    for i, N in enumerate((4096, 1024)):
        W = wl.weights(2100 + i, N, K)
        Wp = osc.osc_pack_weight_fp8(dev(W))
        w8, wsc = oracle.quantize_fp8_rows(W)
        Y = osc.osc_fp8_gemm(X8, xs, Wp, N, K, y_dtype=osc.OSC_DT_BF16)
        assert torch.equal(Y, osc.osc_fp8_gemm(X8, xs, Wp, N, K, y_dtype=osc.OSC_DT_BF16)), "not run-to-run deterministic"
        ref = oracle.fp8_gemm(r8[rows], rs[rows], w8, wsc)
        check_close(host(Y[torch.from_numpy(rows).cuda()].float()), ref, f"cfg2 fp8 N={N}", bf16_out=True)
        check_tiles(host(Y.float()), tile_points(41 + i, M, N),
                    lambda m, c, w: oracle.fp8_gemm(r8[m:m + 1], rs[m:m + 1], w8[c:c + w], wsc[c:c + w]),
                    np.abs(ref).max(), f"cfg2 fp8 N={N}")


def test_config2_q_projection_whole_output(osc, capsys):
    """The bench's dominant launch (M = 8192, N = K = 4096, K_o = 256, bf16 out), every one of its
    33.5 million outputs against the oracle.  The oracle needs a few minutes on the host cores, so it
    runs in slabs of rows and a progress line per slab goes to the real stdout."""
    M, K, N = 8192, 4096, 4096
    X, table = wl.activations_persistent(2001, M, K, 2)
    oidx = oracle.table_to_index(table)
    qd, (rq, rs, rb) = quant_full(osc, X, oidx)
    W = wl.weights(2100, N, K)
    Wp, w_ref = pack_full(osc, W, oidx)
    Yh = host(osc.osc_dual_gemm(*qd, Wp, N, K, 256, osc.OSC_DT_BF16).float())
    slab = 512
    scale = None
    for m0 in range(0, M, slab):
        ref = oracle.dual_gemm(rq[m0:m0 + slab], rs[m0:m0 + slab], rb[m0:m0 + slab], *w_ref)
        scale = np.abs(ref).max() if scale is None else scale  # the first slab's maximum: a lower bound of max|Y|
        check_close(Yh[m0:m0 + slab], ref, f"whole Y rows {m0}..", bf16_out=True, scale=scale)
        with capsys.disabled():
            print(f"[whole-Y] rows {m0 + slab}/{M} ok", flush=True)


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
        dual_sampled(osc, qd, qr, Wp, wr, N, K, 256, rows, osc.OSC_DT_BF16, f"cfg2 M={M} N={N}", tiles_seed=20 + i)


# ---- configs[2]: Qwen3-8B FFN --------------------------------------------------------------------


def test_config3_ffn_w1w3_dual(osc):
    M, K, N = 8192, 4096, 24576
    X, table = wl.activations_persistent(3001, M, K, 2)
    oidx = oracle.table_to_index(table)
    qd, qr = quant_full(osc, X, oidx)
    W = wl.weights(3002, N, K)
    Wp, wr = pack_full(osc, W, oidx)
    del W
    dual_sampled(osc, qd, qr, Wp, wr, N, K, 256, sample_rows(3, M, 12), osc.OSC_DT_BF16, "cfg3 W1|W3", tiles_seed=30)


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
    check_tiles(host(Y.float()), tile_points(31, M, N),
                lambda m, c, w: oracle.fp8_gemm(r8[m:m + 1], rs[m:m + 1], w8[c:c + w], wsc[c:c + w]),
                np.abs(ref).max(), "cfg3 W2 fp8")


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
    check_tiles(host(Y.float()), tile_points(32, M, N),
                lambda m, c, w: oracle.mxfp8_gemm(r8[m:m + 1], rs[m:m + 1], w8[c:c + w], wsc[c:c + w]),
                np.abs(ref).max(), "cfg3 W2 mxfp8")


# ---- configs[3]: Qwen3-30B-A3B MoE layer ---------------------------------------------------------


def expert_rows(off, e, heavy, seed):
    """Routed rows of expert e to check: first, last and one seeded interior row; 22 more for the
    experts in `heavy`."""
    lo, hi = int(off[e]), int(off[e + 1])
    if hi <= lo:
        return np.zeros(0, np.int64)
    g = wl.rng(seed + e)
    more = g.integers(lo, hi, size=22 if e in heavy else 1)
    return np.unique(np.concatenate([[lo, hi - 1], more])).astype(np.int64)


def test_config4_moe_grouped(osc):
    """Every one of the 128 experts is checked (first, last and an interior routed row, all N
    columns; five experts on 24 rows), for the grouped dual path with its row map and for the
    grouped FP8 and MXFP8 forms of W_2."""
    tokens, K, E, topk, N = 4096, 2048, 128, 8, 1536
    X, table = wl.activations_persistent(4001, tokens, K, 2)
    oidx = oracle.table_to_index(table)
    K_o = len(oidx)
    assert K_o == 128
    qd, (rq, rs, rb) = quant_full(osc, X, oidx)
    off, row_map = wl.moe_routing(4002, tokens, E, topk)
    T = int(off[-1])
    assert T == tokens * topk
    heavy = [0, 1, 63, 64, 127]
    stride = osc.osc_packed_weight_bytes(N, K, K_o)
    Wp = torch.empty(E * stride, dtype=torch.uint8, device="cuda")
    d_oidx = dev(oidx)
    for e in range(E):
        osc.osc_pack_weight(dev(wl.weights(4100 + e, N, K)), d_oidx, out=Wp[e * stride:(e + 1) * stride])
    Y = osc.osc_grouped_dual_gemm(*qd, dev(row_map), dev(off), T, Wp, N, K, K_o, osc.OSC_DT_BF16)
    assert bool(torch.isfinite(Y.float()).all())
    Yh = host(Y.float())
    covered = 0
    for e in range(E):
        ts = expert_rows(off, e, heavy, 0)
        if len(ts) == 0:
            continue
        W = wl.weights(4100 + e, N, K)
        q, s_, _ = oracle.quantize_mxfp4_osc(W)
        src = row_map[ts]
        ref = oracle.dual_gemm(rq[src], rs[src], rb[src], q, s_, oracle.gather_wl(W, oidx))
        check_close(Yh[ts], ref, f"cfg4 expert {e}", bf16_out=True)
        covered += 1
    assert covered == E, "an expert without rows: the routing recipe changed"
    del Y, Yh

    # W2 of the experts: grouped FP8, rows already sorted by expert
    K2, N2 = 768, 2048
    X2 = wl.activations_diffuse(4003, T, K2)
    X8, xs = osc.osc_quantize_act(dev(X2), None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    r8, r8s = oracle.quantize_fp8_rows(X2)
    assert np.array_equal(host(X8), r8) and np.array_equal(host(xs).view(np.uint32), r8s.view(np.uint32))
    stride8 = osc.osc_packed_weight_fp8_bytes(N2, K2)
    Wp8 = torch.empty(E * stride8, dtype=torch.uint8, device="cuda")
    for e in range(E):
        osc.osc_pack_weight_fp8(dev(wl.weights(4300 + e, N2, K2)), out=Wp8[e * stride8:(e + 1) * stride8])
    Y8 = osc.osc_fp8_gemm(X8, xs, Wp8, N2, K2, expert_offsets=dev(off), y_dtype=osc.OSC_DT_BF16)
    Y8h = host(Y8.float())
    for e in range(E):
        ts = expert_rows(off, e, heavy, 100)
        ref = oracle.fp8_gemm(r8[ts], r8s[ts], *oracle.quantize_fp8_rows(wl.weights(4300 + e, N2, K2)))
        check_close(Y8h[ts], ref, f"cfg4 fp8 expert {e}", bf16_out=True)
    del Y8, Y8h

    # the same W2 inputs in MXFP8 (Section 4.1), grouped
    Xm, Xms = osc.osc_quantize_act(dev(X2), None, osc.OSC_FMT_MXFP8)
    mq, ms_ = oracle.quantize_mxfp8(X2)
    assert np.array_equal(host(Xm), mq)
    stridem = osc.osc_packed_weight_mxfp8_bytes(N2, K2)
    Wpm = torch.empty(E * stridem, dtype=torch.uint8, device="cuda")
    for e in range(E):
        osc.osc_pack_weight_mxfp8(dev(wl.weights(4300 + e, N2, K2)), out=Wpm[e * stridem:(e + 1) * stridem])
    Ym = osc.osc_mxfp8_gemm(Xm, Xms, Wpm, N2, K2, expert_offsets=dev(off), y_dtype=osc.OSC_DT_BF16)
    Ymh = host(Ym.float())
    for e in range(E):
        ts = expert_rows(off, e, heavy, 200)
        ref = oracle.mxfp8_gemm(mq[ts], ms_[ts], *oracle.quantize_mxfp8(wl.weights(4300 + e, N2, K2)))
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
        dual_sampled(osc, qd, qr, Wp, wr, N, K, len(oidx), rows, osc.OSC_DT_BF16, f"cfg5 M={M} r={r}", tiles_seed=50 + r)


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


# ---- the fused producers against the oracle's plain double-precision forms ------------------------
def _bf16_steps(a_bits, b_bits):
    def key(b):
        b = b.astype(np.int32)
        return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)
    return np.abs(key(a_bits) - key(b_bits))


def test_fused_rmsnorm_against_plain_rmsnorm(osc):
    """The kernel's normalised rows against the textbook RMSNorm of the oracle (double precision,
    libm sqrt; no fixed-point sum, no recipe shared with the kernel): within one bf16 step of the
    singly rounded form everywhere, and identical to the form that rounds where bf16 modules round in
    at least 99.9 % of the 33.5 million values."""
    M, K = 8192, 4096
    X, table = wl.activations_persistent(6101, M, K, 2, jitter=0.2)
    gamma = wl.to_bf16_bits((1.0 + 0.2 * wl.rng(6102).standard_normal(K)).astype(np.float32))
    oidx = oracle.table_to_index(table)
    Xn = host(osc.osc_rmsnorm_quantize_act(dev(X), dev(gamma), 1e-6, dev(oidx.astype(np.int32)), want_norm=True)[3])
    assert _bf16_steps(Xn, oracle.rmsnorm_plain(X, gamma, 1e-6)).max() <= 1
    d = _bf16_steps(Xn, oracle.rmsnorm_plain(X, gamma, 1e-6, mid_round=True))
    assert d.max() <= 2 and (d == 0).mean() >= 0.999
    ones = wl.to_bf16_bits(np.ones(K, np.float32))
    X1 = host(osc.osc_rmsnorm_quantize_act(dev(X), dev(ones), 1e-6, dev(oidx.astype(np.int32)), want_norm=True)[3])
    d1 = _bf16_steps(X1, oracle.rmsnorm_plain(X, ones, 1e-6))
    assert d1.max() <= 1 and (d1 == 0).mean() >= 0.999


def test_fused_swiglu_against_plain_swiglu(osc):
    """Both SwiGLU fusions' y against the textbook form (libm exp in double)."""
    M, K = 2048, 12288
    gen = wl.rng(3300)
    G = wl.to_bf16_bits((gen.standard_normal((M, K)) * 2.5).astype(np.float32))
    U = wl.activations_diffuse(3301, M, K, p=0.005)
    both = dev(np.concatenate([G, U], axis=1))
    plain1 = oracle.swiglu_plain(G, U)
    plain2 = oracle.swiglu_plain(G, U, mid_round=True)
    for name, fn in (("mxfp8", osc.osc_swiglu_quantize_act), ("fp8", osc.osc_swiglu_quantize_act_fp8)):
        Yn = host(fn(both[:, :K], both[:, K:], want_y=True)[2])
        assert _bf16_steps(Yn, plain1).max() <= 1, name
        d = _bf16_steps(Yn, plain2)
        assert d.max() <= 1 and (d == 0).mean() >= 0.999, name
