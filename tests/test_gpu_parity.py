"""GPU parity: the HIP path through the C ABI against the CPU oracle, same seeded inputs.

Quantised codes, scales and gathered sub-tensors must match bit for bit; GEMM outputs must
satisfy max|Y_gpu - Y_oracle| <= 1e-3 * max|Y_oracle| on the same quantised operands.
"""
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
    m.lib()  # fails loudly when libosc.so is missing
    return m


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.cpu().numpy()


def check_close(Y_gpu, Y_ref, what="", bf16_out=False, scale=None):
    """max|Y_gpu - Y_ref| <= 1e-3 * max|Y_ref| on the fp32 result.  A bf16 output adds its own
    rounding: half a unit in the last place of 8 significant bits, at most 2^-8 of the value.
    `scale` stands in for max|Y_ref| when Y_ref is a small sample of a larger output (pass the
    maximum over a bigger sample of the same output: never more than the true maximum)."""
    Y_gpu = np.asarray(Y_gpu, np.float64)
    ref = np.abs(Y_ref).max() if scale is None else float(scale)
    assert np.isfinite(Y_gpu).all(), what
    slack = TOL * ref + (2.0 ** -8 * np.abs(Y_ref) if bf16_out else 0.0)
    excess = np.abs(Y_gpu - Y_ref) - slack
    assert excess.max() <= 0, f"{what}: max err {np.abs(Y_gpu - Y_ref).max():.3e} vs {TOL}*{ref:.3e}"


def quant_both(osc, X, oidx, ldb=None):
    """Runs both quantisers, asserts bit equality, returns (device outputs, host oracle outputs)."""
    K_o = len(oidx)
    if ldb is None:
        ldb = (K_o + 63) // 64 * 64
    d_oidx = dev(oidx.astype(np.int32)) if K_o else None
    Xq, Xs, B = osc.osc_quantize_act(dev(X), d_oidx, osc.OSC_FMT_MXFP4_OSC, ldb=ldb)
    rq, rs, rb = oracle.quantize_mxfp4_osc(X, oidx, ldb=ldb)
    torch.cuda.synchronize()
    assert np.array_equal(host(osc.osc_unpack_act_scales(Xs, *X.shape)), rs), "E8M0 scales differ"
    assert np.array_equal(host(Xq), rq), "E2M1 codes differ"
    if ldb:
        assert np.array_equal(host(B), rb), "gathered sub-tensor differs"
    return (Xq, Xs, B), (rq, rs, rb)


def pack_both(osc, W, oidx):
    K_o = len(oidx)
    N, K = W.shape
    d_oidx = dev(oidx.astype(np.int32)) if K_o else None
    Wp = osc.osc_pack_weight(dev(W), d_oidx)
    Wq, Ws, WL = osc.osc_unpack_weight(Wp, N, K, K_o)
    rq, rs, _ = oracle.quantize_mxfp4_osc(W)
    rl = oracle.gather_wl(W, oidx) if K_o else None
    torch.cuda.synchronize()
    assert np.array_equal(host(Wq), rq) and np.array_equal(host(Ws), rs)
    if K_o:
        assert np.array_equal(host(WL), rl)
    return Wp, (rq, rs, rl)


# ---- quantiser ----------------------------------------------------------------------------


def test_quant_config1(osc):
    c = wl.config1_tiny()
    quant_both(osc, c["X"], oracle.table_to_index(c["table"]))
    quant_both(osc, c["X"], np.zeros(0, np.int32))


@pytest.mark.parametrize("M,K,r", [(1, 4096, 2), (37, 4096, 2), (300, 4096, 4), (64, 2048, 2),
                                   (5, 96, 1), (9, 32, 1), (3, 12288, 1), (2500, 256, 0),
                                   (130, 8192, 3)])
def test_quant_shapes(osc, M, K, r):
    X, table = wl.activations_persistent(100 + M + K + r, M, K, r)
    oidx = oracle.table_to_index(table)
    quant_both(osc, X, oidx)
    if r:
        quant_both(osc, X, oidx, ldb=len(oidx) + (-len(oidx)) % 8 + 8)  # odd padding width


def test_quant_partial_table_and_full_table(osc):
    X, table = wl.activations_persistent(7, 33, 512, 3)
    table[::3] = -1  # some groups bypass suppression
    table[1, 1:] = -1
    quant_both(osc, X, oracle.table_to_index(table))
    quant_both(osc, X, np.arange(512, dtype=np.int32))  # every channel protected


def test_quant_edge_values(osc):
    gen = wl.rng(99)
    x = gen.standard_normal((64, 256)).astype(np.float32) * np.exp(gen.uniform(-60, 60, (64, 256))).astype(np.float32)
    x = np.clip(x, -3e38, 3e38)
    x[0, :32] = 0.0
    x[1, :32] = -0.0
    x[2, :32] = 1e-38  # bf16 subnormals
    x[3, :64] = np.tile([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 7.0], 8)  # exact ties at scale 1
    x[3, 0] = 6.0
    x[4, :32] = -x[3, :32]
    x[5, 32:64] = 3.3e38
    bits = wl.to_bf16_bits(x)
    # every finite bf16 pattern once, in random group company
    allpat = np.arange(65536, dtype=np.uint32)
    allpat = allpat[((allpat >> 7) & 0xFF) != 0xFF].astype(np.uint16)
    gen.shuffle(allpat)
    allpat = np.concatenate([allpat, allpat[: (-len(allpat)) % 256]]).reshape(-1, 256)
    bits = np.concatenate([bits, allpat])
    tab = wl.planted_table(gen, 256, 2)
    quant_both(osc, bits, oracle.table_to_index(tab))
    quant_both(osc, bits, np.zeros(0, np.int32))


def test_quant_strided_input(osc):
    X, table = wl.activations_persistent(21, 50, 256, 1)
    oidx = oracle.table_to_index(table)
    big = torch.zeros((50, 256 + 64), dtype=torch.uint16, device="cuda")
    big[:, :256] = dev(X)
    Xq, Xs, B = osc.osc_quantize_act(big[:, :256], dev(oidx), osc.OSC_FMT_MXFP4_OSC)
    rq, rs, rb = oracle.quantize_mxfp4_osc(X, oidx, ldb=64)
    assert np.array_equal(host(Xq), rq) and np.array_equal(host(B), rb)
    assert np.array_equal(host(osc.osc_unpack_act_scales(Xs, 50, 256)), rs)


@pytest.mark.parametrize("M,K", [(1, 768), (33, 768), (64, 12288), (7, 4096), (5, 8), (300, 2048)])
def test_quant_fp8(osc, M, K):
    X = wl.activations_diffuse(300 + M + K, M, K)
    X[0, : min(K, 16)] = 0
    if M > 2:
        X[2] = 0  # all-zero row
    X8, xs = osc.osc_quantize_act(dev(X), None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    r8, rs = oracle.quantize_fp8_rows(X)
    assert np.array_equal(host(xs).view(np.uint32), rs.view(np.uint32)), "scales differ"
    assert np.array_equal(host(X8), r8), "e4m3 codes differ"


# ---- weights ------------------------------------------------------------------------------


def test_pack_weight_roundtrip(osc):
    for N, K, r in ((256, 256, 1), (40, 4096, 2), (130, 96, 0), (64, 2048, 4)):
        W = wl.weights(500 + N, N, K)
        tab = wl.planted_table(wl.rng(N), K, r)
        pack_both(osc, W, oracle.table_to_index(tab))
    W = wl.weights(77, 48, 768)
    Wp = osc.osc_pack_weight_fp8(dev(W))
    W8, ws = osc.osc_unpack_weight_fp8(Wp, 48, 768)
    r8, rs = oracle.quantize_fp8_rows(W)
    assert np.array_equal(host(W8), r8) and np.array_equal(host(ws).view(np.uint32), rs.view(np.uint32))


# ---- GEMMs --------------------------------------------------------------------------------


def run_dual(osc, X, W, oidx, y_dtype=None):
    y_dtype = osc.OSC_DT_F32 if y_dtype is None else y_dtype
    (Xq, Xs, B), (rq, rs, rb) = quant_both(osc, X, oidx)
    Wp, (wq, wsc, wlr) = pack_both(osc, W, oidx)
    N, K = W.shape
    Y = osc.osc_dual_gemm(Xq, Xs, B, Wp, N, K, len(oidx), y_dtype)
    Y2 = osc.osc_dual_gemm(Xq, Xs, B, Wp, N, K, len(oidx), y_dtype)
    ref = oracle.dual_gemm(rq, rs, rb if len(oidx) else None, wq, wsc, wlr)
    torch.cuda.synchronize()
    assert torch.equal(Y, Y2), "not run-to-run deterministic"
    check_close(host(Y.float()), ref, f"dual gemm {X.shape}x{W.shape} K_o={len(oidx)}",
                bf16_out=y_dtype == osc.OSC_DT_BF16)
    return Y, ref


def test_dual_gemm_config1(osc):
    c = wl.config1_tiny()
    oidx = oracle.table_to_index(c["table"])
    Y, ref = run_dual(osc, c["X"], c["W"], oidx)
    assert Y.dtype == torch.float32 and Y.shape == (16, 256)
    run_dual(osc, c["X"], c["W"], np.zeros(0, np.int32))  # empty table: pure W4A4
    Yb, _ = run_dual(osc, c["X"], c["W"], oidx, osc.OSC_DT_BF16)
    assert Yb.dtype == torch.bfloat16


def test_dual_gemm_all_channels_is_bf16_gemm(osc):
    c = wl.config1_tiny()
    allc = np.arange(256, dtype=np.int32)
    Y, ref = run_dual(osc, c["X"], c["W"], allc)
    exact = wl.from_bf16_bits(c["X"]).astype(np.float64) @ wl.from_bf16_bits(c["W"]).astype(np.float64).T
    check_close(host(Y), exact, "all-channel table vs bf16 GEMM")


@pytest.mark.parametrize("M,N,K,r", [(1, 256, 4096, 2), (16, 1024, 4096, 2), (128, 512, 4096, 2),
                                     (200, 384, 2048, 1), (129, 130, 256, 1), (70, 1000, 96, 1),
                                     (257, 136, 4096, 4), (64, 128, 512, 0), (300, 300, 1536, 3),
                                     (40, 200, 512, 2), (33, 96, 256, 1), (64, 72, 768, 4), (5, 40, 256, 0)])
def test_dual_gemm_shapes(osc, M, N, K, r):
    X, table = wl.activations_persistent(1000 + M + N, M, K, r)
    W = wl.weights(2000 + N + K, N, K)
    run_dual(osc, X, W, oracle.table_to_index(table))


@pytest.mark.parametrize("M,N,K", [(1, 256, 768), (33, 130, 768), (128, 512, 12288), (200, 96, 48),
                                   (64, 2048, 768)])
def test_fp8_gemm_shapes(osc, M, N, K):
    X = wl.activations_diffuse(3000 + M + K, M, K)
    W = wl.weights(3001 + N, N, K)
    X8, xs = osc.osc_quantize_act(dev(X), None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    Wp = osc.osc_pack_weight_fp8(dev(W))
    Y = osc.osc_fp8_gemm(X8, xs, Wp, N, K)
    r8, rs = oracle.quantize_fp8_rows(X)
    w8, wsc = oracle.quantize_fp8_rows(W)
    assert np.array_equal(host(X8), r8)
    check_close(host(Y), oracle.fp8_gemm(r8, rs, w8, wsc), f"fp8 gemm {M}x{N}x{K}")


def test_grouped_dual_and_fp8(osc):
    E, N, K, tokens, topk, r = 6, 192, 512, 150, 2, 2
    X, table = wl.activations_persistent(41, tokens, K, r)
    oidx = oracle.table_to_index(table)
    (Xq, Xs, B), (rq, rs, rb) = quant_both(osc, X, oidx)
    off, row_map = wl.moe_routing(42, tokens, E, topk)
    off[3:] += 0  # (kept as drawn)
    T = int(off[-1])
    stride = osc.osc_packed_weight_bytes(N, K, len(oidx))
    Wp = torch.empty(E * stride, dtype=torch.uint8, device="cuda")
    wq, wsc, wlr = [], [], []
    for e in range(E):
        W = wl.weights(50 + e, N, K)
        osc.osc_pack_weight(dev(W), dev(oidx), out=Wp[e * stride:(e + 1) * stride])
        q, s, _ = oracle.quantize_mxfp4_osc(W)
        wq.append(q), wsc.append(s), wlr.append(oracle.gather_wl(W, oidx))
    Y = osc.osc_grouped_dual_gemm(Xq, Xs, B, dev(row_map), dev(off), T, Wp, N, K, len(oidx))
    ref = oracle.grouped_dual_gemm(rq, rs, rb, row_map, off, np.stack(wq), np.stack(wsc), np.stack(wlr))
    check_close(host(Y), ref, "grouped dual gemm")
    # an expert with no rows and an identity row_map
    off2 = np.array([0, 10, 10, 75, 150], np.int32)
    Y2 = osc.osc_grouped_dual_gemm(Xq, Xs, B, None, dev(off2), 150, Wp, N, K, len(oidx))
    ref2 = oracle.grouped_dual_gemm(rq, rs, rb, None, off2, np.stack(wq[:4]), np.stack(wsc[:4]), np.stack(wlr[:4]))
    check_close(host(Y2), ref2, "grouped dual gemm, identity map")
    # grouped FP8 (W2 of the experts)
    K2, N2 = 192, 256
    X2 = wl.activations_diffuse(43, T, K2)
    X8, xs = osc.osc_quantize_act(dev(X2), None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    stride8 = osc.osc_packed_weight_fp8_bytes(N2, K2)
    Wp8 = torch.empty(E * stride8, dtype=torch.uint8, device="cuda")
    w8, w8s = [], []
    for e in range(E):
        W = wl.weights(60 + e, N2, K2)
        osc.osc_pack_weight_fp8(dev(W), out=Wp8[e * stride8:(e + 1) * stride8])
        a, b = oracle.quantize_fp8_rows(W)
        w8.append(a), w8s.append(b)
    Y8 = osc.osc_fp8_gemm(X8, xs, Wp8, N2, K2, expert_offsets=dev(off))
    r8, r8s = oracle.quantize_fp8_rows(X2)
    ref8 = oracle.grouped_fp8_gemm(r8, r8s, off, np.stack(w8), np.stack(w8s))
    check_close(host(Y8), ref8, "grouped fp8 gemm")


def test_empty_problems_are_noops(osc):
    X = torch.zeros((0, 256), dtype=torch.uint16, device="cuda")
    Xq, Xs, B = osc.osc_quantize_act(X, None, osc.OSC_FMT_MXFP4_OSC)
    assert Xq.shape == (0, 128)
    Wp = osc.osc_pack_weight(dev(wl.weights(1, 64, 256)), None)
    Y = osc.osc_dual_gemm(Xq, Xs, None, Wp, 64, 256, 0)
    assert Y.shape == (0, 64)


# ---- MXFP8 form of the fallback -----------------------------------------------------------------


@pytest.mark.parametrize("M,K", [(1, 128), (33, 768), (64, 12288), (7, 4096), (300, 2048), (130, 96)])
def test_quant_mxfp8(osc, M, K):
    X = wl.activations_diffuse(700 + M + K, M, K)
    X[0, : min(K, 32)] = 0
    if M > 2:
        X[2] = 0x8000  # a row of negative zeros
    X8, Xs = osc.osc_quantize_act(dev(X), None, osc.OSC_FMT_MXFP8)
    r8, rs = oracle.quantize_mxfp8(X)
    assert np.array_equal(host(osc.osc_unpack_act_scales(Xs, M, K)), rs), "E8M0 scales differ"
    assert np.array_equal(host(X8), r8), "e4m3 codes differ"


def test_quant_mxfp8_edge_values(osc):
    gen = wl.rng(98)
    x = gen.standard_normal((64, 256)).astype(np.float32) * np.exp(gen.uniform(-60, 60, (64, 256))).astype(np.float32)
    x = np.clip(x, -3e38, 3e38)
    x[1, :32] = 1e-38  # bf16 subnormals
    x[2, :8] = [31.5, 28, 27, 26, 25, -27, 0.001, 2 ** -14]  # saturation and exact ties
    x[3, 32:64] = 3.3e38
    bits = wl.to_bf16_bits(x)
    allpat = np.arange(65536, dtype=np.uint32)
    allpat = allpat[((allpat >> 7) & 0xFF) != 0xFF].astype(np.uint16)  # every finite bf16 pattern
    gen.shuffle(allpat)
    allpat = np.concatenate([allpat, allpat[: (-len(allpat)) % 256]]).reshape(-1, 256)
    bits = np.concatenate([bits, allpat])
    X8, Xs = osc.osc_quantize_act(dev(bits), None, osc.OSC_FMT_MXFP8)
    r8, rs = oracle.quantize_mxfp8(bits)
    assert np.array_equal(host(osc.osc_unpack_act_scales(Xs, *bits.shape)), rs)
    assert np.array_equal(host(X8), r8)


@pytest.mark.parametrize("M,N,K", [(1, 256, 768), (33, 130, 768), (64, 2048, 768), (128, 512, 12288),
                                   (200, 96, 128), (300, 300, 1536), (257, 136, 4096)])
def test_mxfp8_gemm_shapes(osc, M, N, K):
    X = wl.activations_diffuse(3100 + M + K, M, K)
    W = wl.weights(3101 + N, N, K)
    X8, Xs = osc.osc_quantize_act(dev(X), None, osc.OSC_FMT_MXFP8)
    Wp = osc.osc_pack_weight_mxfp8(dev(W))
    W8, Ws = osc.osc_unpack_weight_mxfp8(Wp, N, K)
    r8, rs = oracle.quantize_mxfp8(X)
    w8, wsc = oracle.quantize_mxfp8(W)
    assert np.array_equal(host(X8), r8) and np.array_equal(host(W8), w8) and np.array_equal(host(Ws), wsc)
    Y = osc.osc_mxfp8_gemm(X8, Xs, Wp, N, K)
    Y2 = osc.osc_mxfp8_gemm(X8, Xs, Wp, N, K)
    assert torch.equal(Y, Y2)
    check_close(host(Y), oracle.mxfp8_gemm(r8, rs, w8, wsc), f"mxfp8 gemm {M}x{N}x{K}")


def test_mxfp8_grouped(osc):
    E, N, K, T = 5, 256, 384, 700
    off = np.array([0, 150, 150, 400, 690, 700], np.int32)
    X = wl.activations_diffuse(45, T, K)
    X8, Xs = osc.osc_quantize_act(dev(X), None, osc.OSC_FMT_MXFP8)
    r8, rs = oracle.quantize_mxfp8(X)
    stride = osc.osc_packed_weight_mxfp8_bytes(N, K)
    Wp = torch.empty(E * stride, dtype=torch.uint8, device="cuda")
    ref = np.zeros((T, N))
    for e in range(E):
        W = wl.weights(70 + e, N, K)
        osc.osc_pack_weight_mxfp8(dev(W), out=Wp[e * stride:(e + 1) * stride])
        w8, wsc = oracle.quantize_mxfp8(W)
        lo, hi = off[e], off[e + 1]
        if hi > lo:
            ref[lo:hi] = oracle.mxfp8_gemm(r8[lo:hi], rs[lo:hi], w8, wsc)
    Y = osc.osc_mxfp8_gemm(X8, Xs, Wp, N, K, expert_offsets=dev(off))
    check_close(host(Y), ref, "grouped mxfp8 gemm")


# ---- largest supported row length ---------------------------------------------------------------


@pytest.mark.parametrize("r", [0, 1])
def test_quant_longest_rows(osc, r):
    """K = 65536 is the quantiser's limit (with a table the masks of a row take 128 KB of LDS)."""
    M, K = 5, 65536
    X, table = wl.activations_persistent(900 + r, M, K, r)
    oidx = oracle.table_to_index(table)
    assert len(oidx) == r * K // 32
    quant_both(osc, X, oidx)
    with pytest.raises(osc.OscError):
        osc.osc_quantize_act(dev(np.zeros((2, 65536 + 32), np.uint16)), None)


def test_dual_gemm_long_k(osc):
    """256 stages in one tile: M = 40 rows (the skinny kernel) and 200 rows (the DMA kernel)."""
    N, K = 96, 32768
    W = wl.weights(911, N, K)
    for M in (40, 200):
        X, table = wl.activations_persistent(910 + M, M, K, 1)
        run_dual(osc, X, W, oracle.table_to_index(table))


def test_raw_scale_layout_against_the_header_formula(osc):
    """The row-block-major E8M0 layout as include/osc.h states it, read from the raw bytes with
    numpy indexing (no unpack kernel of the library involved): the scale of (row m, group g) is byte
    ((m/32)*ceil(K/128) + g/4)*128 + (m%32)*4 + g%4; bytes of groups >= K/32 are zero."""
    for M, K, r in ((70, 96, 1), (33, 4096, 2), (256, 160, 0), (5, 32, 1)):
        X, table = wl.activations_persistent(8800 + M, M, K, r)
        oidx = oracle.table_to_index(table) if r else np.zeros(0, np.int32)
        Xq, Xs, B = osc.osc_quantize_act(dev(X), dev(oidx) if r else None)
        raw = host(Xs)
        assert raw.size == osc.osc_act_scale_bytes(M, K)
        _, rs, _ = oracle.quantize_mxfp4_osc(X, oidx, ldb=0 if B is None else B.shape[1])
        Kg, nb = K // 32, (K // 32 + 3) // 4
        m, g = np.meshgrid(np.arange(M), np.arange(nb * 4), indexing="ij")
        at = ((m // 32) * nb + g // 4) * 128 + (m % 32) * 4 + g % 4
        got = raw[at]
        assert np.array_equal(got[:, :Kg], rs), (M, K)
        assert (got[:, Kg:] == 0).all(), "bytes of groups past K/32 must be zero"
        # the same for the 8-bit micro-scaling quantiser
        X8, X8s = osc.osc_quantize_act(dev(X), None, osc.OSC_FMT_MXFP8)
        _, r8s = oracle.quantize_mxfp8(X)
        got8 = host(X8s)[at]
        assert np.array_equal(got8[:, :Kg], r8s) and (got8[:, Kg:] == 0).all(), (M, K, "mxfp8")
