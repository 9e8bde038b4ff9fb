"""Every GEMM kernel template on shapes it would not be chosen for: the launcher's tuning knobs
(include/osc_tuning.h) force the tile size and the kernel, the results must still meet the GEMM tolerance.  Also outputs
written into wider buffers (ldy > N) and through the unaligned bf16 store path."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl

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


def close(Y, ref, what, bf16=False):
    Y = Y.float().cpu().numpy().astype(np.float64)
    slack = TOL * np.abs(ref).max() + (2.0 ** -8 * np.abs(ref) if bf16 else 0.0)
    assert np.isfinite(Y).all() and (np.abs(Y - ref) <= slack).all(), what


# tile rows / 64, kernel id: 0 staged, 1 DMA (eight wavefronts at 256 rows), 2 persistent, 3 skinny,
# 4 ring (wavefront groups in anti-phase), 5 ring (in phase)
FORCED = ["4,1", "2,1", "1,1", "1,0", "2,0", "4,2", "2,2", "4,4", "4,5"]


@pytest.mark.parametrize("cfg", FORCED)
@pytest.mark.parametrize("M,N,K,r", [(300, 200, 1024, 2), (513, 520, 512, 1), (256, 512, 768, 0), (70, 1000, 256, 4)])
def test_dual_forced(osc, tuning, cfg, M, N, K, r):
    tuning.gemm(cfg)
    X, table = wl.activations_persistent(7000 + M, M, K, r)
    W = wl.weights(7100 + N, N, K)
    oidx = oracle.table_to_index(table) if r else np.zeros(0, np.int32)
    d_oidx = dev(oidx) if r else None
    Xq, Xs, B = osc.osc_quantize_act(dev(X), d_oidx)
    Wp = osc.osc_pack_weight(dev(W), d_oidx)
    rq, rs, rb = oracle.quantize_mxfp4_osc(X, oidx, ldb=B.shape[1] if B is not None else 0)
    wq, ws, _ = oracle.quantize_mxfp4_osc(W)
    ref = oracle.dual_gemm(rq, rs, rb if r else None, wq, ws, oracle.gather_wl(W, oidx))
    for ydt, bf in ((osc.OSC_DT_F32, False), (osc.OSC_DT_BF16, True)):
        Y = osc.osc_dual_gemm(Xq, Xs, B, Wp, N, K, len(oidx), ydt)
        close(Y, ref, f"{cfg} {M}x{N}x{K} r={r} bf16={bf}", bf)


@pytest.mark.parametrize("M,N,K,r", [(300, 200, 1024, 2), (200, 300, 1280, 2), (64, 128, 2048, 1), (130, 260, 4096, 4),
                                     (513, 520, 1024, 0), (1, 40, 2304, 3), (2048, 1024, 4096, 2)])
@pytest.mark.parametrize("tile", ["1,1", "2,1"])
def test_dual_small_tiles_with_k_split(osc, tuning, tile, M, N, K, r):
    """64 x 128 and 128 x 128 tiles with the reduction axis split over two groups of wavefronts (forced on:
    the launcher itself takes it only when the launch has at most one tile per CU): even and odd numbers
    of stages, a branch of one to eight stages, ragged tiles in both directions."""
    tuning.gemm(tile)
    tuning.gemm_ksplit(1)
    X, table = wl.activations_persistent(7060 + M, M, K, r) if r else (wl.activations_diffuse(7060 + M, M, K), None)
    W = wl.weights(7160 + N, N, K)
    oidx = oracle.table_to_index(table) if r else np.zeros(0, np.int32)
    d_oidx = dev(oidx) if r else None
    Xq, Xs, B = osc.osc_quantize_act(dev(X), d_oidx)
    Wp = osc.osc_pack_weight(dev(W), d_oidx)
    rows = np.arange(M) if M <= 600 else np.unique(np.concatenate([np.arange(0, M, 61), [63, 64, M - 1]]))
    rq, rs, rb = oracle.quantize_mxfp4_osc(X[rows], oidx, ldb=B.shape[1] if B is not None else 0)
    wq, ws, _ = oracle.quantize_mxfp4_osc(W)
    ref = oracle.dual_gemm(rq, rs, rb if r else None, wq, ws, oracle.gather_wl(W, oidx))
    sel = torch.from_numpy(rows).cuda()
    for ydt, bf in ((osc.OSC_DT_F32, False), (osc.OSC_DT_BF16, True)):
        Y = osc.osc_dual_gemm(Xq, Xs, B, Wp, N, K, len(oidx), ydt)
        close(Y[sel], ref, f"k split {M}x{N}x{K} r={r} bf16={bf}", bf)
    # the same launch without the split gives the same numbers up to the order of two partial sums
    tuning.gemm_ksplit(0)
    Y0 = osc.osc_dual_gemm(Xq, Xs, B, Wp, N, K, len(oidx), osc.OSC_DT_F32)
    tuning.gemm_ksplit(1)
    Y1 = osc.osc_dual_gemm(Xq, Xs, B, Wp, N, K, len(oidx), osc.OSC_DT_F32)
    assert float((Y0 - Y1).abs().max()) <= 1e-5 * float(Y0.abs().max())


@pytest.mark.parametrize("M,N,K", [(300, 200, 1024), (200, 300, 640), (64, 128, 2048), (513, 520, 896), (2048, 1024, 4096)])
@pytest.mark.parametrize("tile", ["1,1", "2,1"])
def test_fp8_small_tiles_with_k_split(osc, tuning, tile, M, N, K):
    """The per-token FP8 GEMM on 64 x 128 and 128 x 128 tiles with the K split forced on: even and odd stage counts."""
    tuning.gemm(tile)
    tuning.gemm_ksplit(1)
    X = wl.activations_diffuse(7250 + M, M, K)
    W = wl.weights(7251 + N, N, K)
    X8, xs = osc.osc_quantize_act(dev(X), None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    rows = np.arange(M) if M <= 600 else np.unique(np.concatenate([np.arange(0, M, 61), [63, 64, M - 1]]))
    r8, rs = oracle.quantize_fp8_rows(X[rows])
    w8, ws = oracle.quantize_fp8_rows(W)
    sel = torch.from_numpy(rows).cuda()
    for ydt, bf in ((osc.OSC_DT_F32, False), (osc.OSC_DT_BF16, True)):
        Y = osc.osc_fp8_gemm(X8, xs, osc.osc_pack_weight_fp8(dev(W)), N, K, y_dtype=ydt)
        close(Y[sel], oracle.fp8_gemm(r8, rs, w8, ws), f"fp8 k split {M}x{N}x{K} bf16={bf}", bf)


@pytest.mark.parametrize("M,N,K", [(256, 512, 768), (300, 256, 384), (4392, 4096, 384), (2560, 7168, 640)])
def test_fp8_persistent_pipeline(osc, tuning, M, N, K):
    """The per-token FP8 GEMM (and, below, the MXFP8 GEMM) on the persistent kernel (forced; the launcher takes it from 257 tiles of 256 x 256 on):
    one tile, a ragged tail of rows (handled by a second launch), more tiles than workgroups (so that a workgroup
    walks several tiles and both copies of the tile scales in LDS are used), three (the minimum) and five stages."""
    tuning.gemm("4,2")
    X = wl.activations_diffuse(7300 + M, M, K)
    W = wl.weights(7301 + N, N, K)
    X8, xs = osc.osc_quantize_act(dev(X), None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    rows = np.arange(M) if M <= 600 else np.unique(np.concatenate([np.arange(0, M, 37), [255, 256, 257, M - 41, M - 1]]))
    r8, rs = oracle.quantize_fp8_rows(X[rows])
    w8, ws = oracle.quantize_fp8_rows(W)
    ref = oracle.fp8_gemm(r8, rs, w8, ws)
    sel = torch.from_numpy(rows).cuda()
    Wp = osc.osc_pack_weight_fp8(dev(W))
    for ydt, bf in ((osc.OSC_DT_F32, False), (osc.OSC_DT_BF16, True)):
        Y = osc.osc_fp8_gemm(X8, xs, Wp, N, K, y_dtype=ydt)
        close(Y[sel], ref, f"fp8 persistent {M}x{N}x{K} bf16={bf}", bf)
    if M <= 600:
        # wide, shifted and odd output views: the 16-byte, 8-byte and element store paths of the epilogue
        for dt, ydt, bf in ((torch.float32, osc.OSC_DT_F32, False), (torch.bfloat16, osc.OSC_DT_BF16, True)):
            for width, col0 in ((N + 64, 0), (N + 64, 4), (N + 7, 3)):
                wide = torch.full((M, width), 7.0, dtype=dt, device="cuda")
                view = wide[:, col0:col0 + N]
                osc.osc_fp8_gemm(X8, xs, Wp, N, K, y_dtype=ydt, out=view)
                close(view, ref, f"fp8 persistent ldy={width} col0={col0} bf16={bf}", bf)
                assert (torch.cat([wide[:, :col0], wide[:, col0 + N:]], dim=1) == 7.0).all(), "wrote outside the output view"
    # every element against the DMA kernel (same products, same order inside a stage)
    Y2 = osc.osc_fp8_gemm(X8, xs, Wp, N, K)
    tuning.gemm("4,1")
    Y1 = osc.osc_fp8_gemm(X8, xs, Wp, N, K)
    assert float((Y1 - Y2).abs().max()) <= 1e-5 * float(Y1.abs().max())
    # the MXFP8 form of the same kernel: block scales travel with the stages
    tuning.gemm("4,2")
    Xm, Xms = osc.osc_quantize_act(dev(X), None, osc.OSC_FMT_MXFP8)
    q, sc = oracle.quantize_mxfp8(X[rows])
    wq, wsc = oracle.quantize_mxfp8(W)
    refm = oracle.mxfp8_gemm(q, sc, wq, wsc)
    Wm = osc.osc_pack_weight_mxfp8(dev(W))
    for ydt, bf in ((osc.OSC_DT_F32, False), (osc.OSC_DT_BF16, True)):
        Ym = osc.osc_mxfp8_gemm(Xm, Xms, Wm, N, K, y_dtype=ydt)
        close(Ym[sel], refm, f"mxfp8 persistent {M}x{N}x{K} bf16={bf}", bf)
    Y2 = osc.osc_mxfp8_gemm(Xm, Xms, Wm, N, K)
    tuning.gemm("4,1")
    Y1 = osc.osc_mxfp8_gemm(Xm, Xms, Wm, N, K)
    assert float((Y1 - Y2).abs().max()) <= 1e-5 * float(Y1.abs().max())


@pytest.mark.parametrize("cfg", ["4,1", "2,1", "1,1", "1,0", "2,0"])
def test_fp8_and_mxfp8_forced(osc, tuning, cfg):
    tuning.gemm(cfg)
    M, N, K = 300, 264, 768
    X = wl.activations_diffuse(7200, M, K)
    W = wl.weights(7201, N, K)
    X8, xs = osc.osc_quantize_act(dev(X), None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    r8, rs = oracle.quantize_fp8_rows(X)
    w8, ws = oracle.quantize_fp8_rows(W)
    close(osc.osc_fp8_gemm(X8, xs, osc.osc_pack_weight_fp8(dev(W)), N, K), oracle.fp8_gemm(r8, rs, w8, ws), "fp8 " + cfg)
    if cfg.endswith(",1"):  # the MXFP8 GEMM exists in the DMA (and skinny) kernels only
        Xm, Xms = osc.osc_quantize_act(dev(X), None, osc.OSC_FMT_MXFP8)
        q, s = oracle.quantize_mxfp8(X)
        wq, wsc = oracle.quantize_mxfp8(W)
        Y = osc.osc_mxfp8_gemm(Xm, Xms, osc.osc_pack_weight_mxfp8(dev(W)), N, K)
        close(Y, oracle.mxfp8_gemm(q, s, wq, wsc), "mxfp8 " + cfg)


@pytest.mark.parametrize("cfg", [None, "4,1", "1,1", "1,0"])
def test_output_into_wider_and_odd_buffers(osc, tuning, cfg):
    if cfg:
        tuning.gemm(cfg)
    M, N, K = 200, 320, 512
    X, table = wl.activations_persistent(7300, M, K, 2)
    W = wl.weights(7301, N, K)
    oidx = oracle.table_to_index(table)
    Xq, Xs, B = osc.osc_quantize_act(dev(X), dev(oidx))
    Wp = osc.osc_pack_weight(dev(W), dev(oidx))
    rq, rs, rb = oracle.quantize_mxfp4_osc(X, oidx, ldb=B.shape[1])
    wq, ws, _ = oracle.quantize_mxfp4_osc(W)
    ref = oracle.dual_gemm(rq, rs, rb, wq, ws, oracle.gather_wl(W, oidx))
    for dt, ydt, bf in ((torch.float32, osc.OSC_DT_F32, False), (torch.bfloat16, osc.OSC_DT_BF16, True)):
        # aligned wide buffer (16-byte stores); first column 4 elements in (8-byte stores for bf16);
        # odd stride and odd first column (element stores)
        for width, col0 in ((N + 64, 0), (N + 64, 4), (N + 7, 3)):
            wide = torch.full((M, width), 7.0, dtype=dt, device="cuda")
            view = wide[:, col0:col0 + N]
            osc.osc_dual_gemm(Xq, Xs, B, Wp, N, K, len(oidx), ydt, out=view)
            close(view, ref, f"ldy={width} col0={col0} bf16={bf}", bf)
            rest = torch.cat([wide[:, :col0], wide[:, col0 + N:]], dim=1)
            assert (rest == 7.0).all(), "wrote outside the output view"


@pytest.mark.parametrize("cfg", ["4,1", "2,1", "1,1"])
def test_grouped_with_skewed_experts(osc, tuning, cfg):
    """Experts of 0, 1, 63 ... 700 rows, sizes on both sides of every tile border, through the
    256-row tiles with their 64-row remainder pass (4,1) and the smaller tiles: dual path with a row
    map, per-token FP8 and MXFP8."""
    tuning.gemm(cfg)
    sizes = [0, 1, 63, 64, 65, 127, 128, 129, 255, 256, 257, 383, 384, 385, 700, 0, 130]
    E = len(sizes)
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    T = int(off[-1])
    tokens, K, N, r = 900, 512, 256, 2
    X, table = wl.activations_persistent(7500, tokens, K, r)
    oidx = oracle.table_to_index(table)
    row_map = wl.rng(7501).integers(0, tokens, T).astype(np.int32)
    Xq, Xs, B = osc.osc_quantize_act(dev(X), dev(oidx))
    rq, rs, rb = oracle.quantize_mxfp4_osc(X, oidx, ldb=B.shape[1])
    stride = osc.osc_packed_weight_bytes(N, K, len(oidx))
    Wp = torch.empty(E * stride, dtype=torch.uint8, device="cuda")
    wq, wsc, wlr = [], [], []
    for e in range(E):
        W = wl.weights(7510 + e, N, K)
        osc.osc_pack_weight(dev(W), dev(oidx), out=Wp[e * stride:(e + 1) * stride])
        a, b, _ = oracle.quantize_mxfp4_osc(W)
        wq.append(a), wsc.append(b), wlr.append(oracle.gather_wl(W, oidx))
    ref = oracle.grouped_dual_gemm(rq, rs, rb, row_map, off, np.stack(wq), np.stack(wsc), np.stack(wlr))
    for ydt, bf in ((osc.OSC_DT_F32, False), (osc.OSC_DT_BF16, True)):
        Y = osc.osc_grouped_dual_gemm(Xq, Xs, B, dev(row_map), dev(off), T, Wp, N, K, len(oidx), ydt)
        close(Y, ref, f"grouped dual {cfg} bf16={bf}", bf)
    # 8-bit forms: rows in expert order (no row map in these entry points)
    K2 = 384
    X2 = wl.activations_diffuse(7502, T, K2)
    X8, xs = osc.osc_quantize_act(dev(X2), None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    Xm, Xms = osc.osc_quantize_act(dev(X2), None, osc.OSC_FMT_MXFP8)
    r8, r8s = oracle.quantize_fp8_rows(X2)
    m8, m8s = oracle.quantize_mxfp8(X2)
    s8, sm = osc.osc_packed_weight_fp8_bytes(N, K2), osc.osc_packed_weight_mxfp8_bytes(N, K2)
    Wp8 = torch.empty(E * s8, dtype=torch.uint8, device="cuda")
    Wpm = torch.empty(E * sm, dtype=torch.uint8, device="cuda")
    w8, w8s = [], []
    refm = np.zeros((T, N))
    for e in range(E):
        W = wl.weights(7530 + e, N, K2)
        osc.osc_pack_weight_fp8(dev(W), out=Wp8[e * s8:(e + 1) * s8])
        osc.osc_pack_weight_mxfp8(dev(W), out=Wpm[e * sm:(e + 1) * sm])
        a, b = oracle.quantize_fp8_rows(W)
        w8.append(a), w8s.append(b)
        if off[e + 1] > off[e]:
            refm[off[e]:off[e + 1]] = oracle.mxfp8_gemm(m8[off[e]:off[e + 1]], m8s[off[e]:off[e + 1]], *oracle.quantize_mxfp8(W))
    ref8 = oracle.grouped_fp8_gemm(r8, r8s, off, np.stack(w8), np.stack(w8s))
    close(osc.osc_fp8_gemm(X8, xs, Wp8, N, K2, expert_offsets=dev(off), y_dtype=osc.OSC_DT_BF16), ref8, "grouped fp8 " + cfg, True)
    close(osc.osc_mxfp8_gemm(Xm, Xms, Wpm, N, K2, expert_offsets=dev(off), y_dtype=osc.OSC_DT_BF16), refm, "grouped mxfp8 " + cfg, True)


def test_wide_128x256_tiles_ragged(osc):
    """4100 x 2000: the launcher's own choice here is 128x256 tiles on eight wavefronts, with a ragged
    last tile in both directions; a row of every fourth m-tile and the borders against the oracle."""
    M, N, K, r = 4100, 2000, 512, 2
    X, table = wl.activations_persistent(7600, M, K, r)
    W = wl.weights(7601, N, K)
    oidx = oracle.table_to_index(table)
    rows = np.unique(np.concatenate([np.arange(0, 32, 4) * 128 + 5, [0, 127, 128, 4095, 4096, 4099]]))
    Xq, Xs, B = osc.osc_quantize_act(dev(X), dev(oidx))
    Wp = osc.osc_pack_weight(dev(W), dev(oidx))
    rq, rs, rb = oracle.quantize_mxfp4_osc(X[rows], oidx, ldb=B.shape[1])
    wq, ws, _ = oracle.quantize_mxfp4_osc(W)
    ref = oracle.dual_gemm(rq, rs, rb, wq, ws, oracle.gather_wl(W, oidx))
    sel = torch.from_numpy(rows).cuda()
    for ydt, bf in ((osc.OSC_DT_BF16, True), (osc.OSC_DT_F32, False)):
        Y = osc.osc_dual_gemm(Xq, Xs, B, Wp, N, K, len(oidx), ydt)
        close(Y[sel], ref, f"128x256 tiles bf16={bf}", bf)
