"""Pins for the oracle's dual-path GEMM (Eq. dual-path), FP8 GEMM and grouped forms -- CPU only.

The independent side of each comparison is numpy/torch: dequantise with the
OCP value tables and call a library matmul in float64, or use an algebraic
invariant of the method.
"""
import os

import numpy as np
import torch

import oracle
import workloads as wl
from workloads import from_bf16_bits, to_bf16_bits
from test_oracle_quant import dequant, _gold


def bf(b):
    return from_bf16_bits(b).astype(np.float64)


def prep(c):
    oidx = oracle.table_to_index(c["table"])
    Xq, Xs, B = oracle.quantize_mxfp4_osc(c["X"], oidx)
    Wq, Ws, _ = oracle.quantize_mxfp4_osc(c["W"])
    WL = oracle.gather_wl(c["W"], oidx)
    return oidx, Xq, Xs, B, Wq, Ws, WL


def test_hand_worked_dot():
    g = _gold("mxfp4_group_example.txt")
    x = np.zeros(32, np.float32)
    x[:11] = [float(v) for v in g["x"]]
    X = to_bf16_bits(x).reshape(1, 32)
    W = to_bf16_bits(np.ones((1, 32), np.float32))
    Wq, Ws, _ = oracle.quantize_mxfp4_osc(W)
    assert Ws[0, 0] == 125 and np.all(Wq == 0x66)
    oidx = np.array([3], np.int32)
    Xq, Xs, B = oracle.quantize_mxfp4_osc(X, oidx)
    Y = oracle.dual_gemm(Xq, Xs, B, Wq, Ws, oracle.gather_wl(W, oidx))
    assert Y[0, 0] == float(g["y_osc"][0])
    Xq0, Xs0, _ = oracle.quantize_mxfp4_osc(X)
    assert oracle.dual_gemm(Xq0, Xs0, None, Wq, Ws, None)[0, 0] == float(g["y_plain"][0])
    assert float((bf(X) @ bf(W).T)[0, 0]) == float(g["y_exact"][0])


def test_dual_gemm_vs_numpy_matmul_config1():
    c = wl.config1_tiny()
    oidx, Xq, Xs, B, Wq, Ws, WL = prep(c)
    Y = oracle.dual_gemm(Xq, Xs, B, Wq, Ws, WL)
    want = dequant(Xq, Xs) @ dequant(Wq, Ws).T + bf(B[:, :8]) @ bf(WL)
    assert np.allclose(Y, want, rtol=1e-12, atol=1e-12 * np.abs(want).max())
    # transposed-operand / wrong-index mistakes would show here: N != K != M
    W2 = wl.weights(77, 40, 256)
    Wq2, Ws2, _ = oracle.quantize_mxfp4_osc(W2)
    WL2 = oracle.gather_wl(W2, oidx)
    Y2 = oracle.dual_gemm(Xq, Xs, B, Wq2, Ws2, WL2)
    want2 = dequant(Xq, Xs) @ dequant(Wq2, Ws2).T + bf(B[:, :8]) @ bf(WL2)
    assert Y2.shape == (16, 40) and np.allclose(Y2, want2, rtol=1e-12, atol=1e-14)


def test_empty_table_is_pure_w4a4_and_full_table_is_bf16_gemm():
    c = wl.config1_tiny()
    Wq, Ws, _ = oracle.quantize_mxfp4_osc(c["W"])
    Xq0, Xs0, _ = oracle.quantize_mxfp4_osc(c["X"])
    Y0 = oracle.dual_gemm(Xq0, Xs0, None, Wq, Ws, None)
    assert np.allclose(Y0, dequant(Xq0, Xs0) @ dequant(Wq, Ws).T, rtol=1e-12, atol=1e-14)
    # every channel protected: the 4-bit path is all zeros and Y is the bf16 GEMM
    allc = np.arange(256, dtype=np.int32)
    Xq, Xs, B = oracle.quantize_mxfp4_osc(c["X"], allc)
    Y = oracle.dual_gemm(Xq, Xs, B, Wq, Ws, oracle.gather_wl(c["W"], allc))
    exact = bf(c["X"]) @ bf(c["W"]).T
    assert np.allclose(Y, exact, rtol=1e-12, atol=1e-14)


def test_osc_beats_direct_mxfp4_on_planted_outliers():
    c = wl.config1_tiny()
    oidx, Xq, Xs, B, Wq, Ws, WL = prep(c)
    exact = bf(c["X"]) @ bf(c["W"]).T
    Y = oracle.dual_gemm(Xq, Xs, B, Wq, Ws, WL)
    Xq0, Xs0, _ = oracle.quantize_mxfp4_osc(c["X"])
    Y0 = oracle.dual_gemm(Xq0, Xs0, None, Wq, Ws, None)
    assert np.linalg.norm(Y - exact) < 0.5 * np.linalg.norm(Y0 - exact)


def test_protected_weight_column_matters_only_through_wl():
    c = wl.config1_tiny()
    oidx, Xq, Xs, B, Wq, Ws, WL = prep(c)
    Y = oracle.dual_gemm(Xq, Xs, B, Wq, Ws, WL)
    # scramble the 4-bit codes of W at the protected channels: Path A multiplies them by code 0
    Wq2 = Wq.copy()
    for ch in oidx:
        Wq2[:, ch // 2] ^= np.uint8(0x7 << (4 * (int(ch) & 1)))
    assert np.array_equal(oracle.dual_gemm(Xq, Xs, B, Wq2, Ws, WL), Y)
    # and Y is linear in B
    Bz = np.zeros_like(B)
    Ya = oracle.dual_gemm(Xq, Xs, Bz, Wq, Ws, WL)
    assert np.allclose(Y - Ya, bf(B[:, :8]) @ bf(WL), rtol=1e-9, atol=1e-12)


def test_group_preserving_permutation_equivariance():
    c = wl.config1_tiny()
    gen = wl.rng(123)
    gperm = gen.permutation(8)
    perm = np.concatenate([32 * g + gen.permutation(32) for g in gperm])
    X2, W2 = c["X"][:, perm], c["W"][:, perm]
    inv = np.argsort(perm)
    oidx = oracle.table_to_index(c["table"])
    oidx2 = np.sort(inv[oidx]).astype(np.int32)  # where the protected channels went
    _, Xq, Xs, B, Wq, Ws, WL = prep(c)
    Y = oracle.dual_gemm(Xq, Xs, B, Wq, Ws, WL)
    Xq2, Xs2, B2 = oracle.quantize_mxfp4_osc(X2, oidx2)
    Wq2, Ws2, _ = oracle.quantize_mxfp4_osc(W2)
    Y2 = oracle.dual_gemm(Xq2, Xs2, B2, Wq2, Ws2, oracle.gather_wl(W2, oidx2))
    assert np.array_equal(Xs2, Xs[:, gperm])
    assert np.allclose(Y2, Y, rtol=1e-12, atol=1e-14)


def test_paper_form_buffer_with_zero_columns_gives_same_y():
    """Alg. 2 keeps one column of B per group (zero where the table holds -1); the compact form
    used here drops those columns.  Both give the same Y."""
    c = wl.config1_tiny()
    tab = c["table"].copy()
    tab[[1, 4, 6]] = -1
    oidx = oracle.table_to_index(tab)
    assert len(oidx) == 5
    Xq, Xs, B = oracle.quantize_mxfp4_osc(c["X"], oidx)
    Wq, Ws, _ = oracle.quantize_mxfp4_osc(c["W"])
    Y = oracle.dual_gemm(Xq, Xs, B, Wq, Ws, oracle.gather_wl(c["W"], oidx))
    Bp = np.zeros((16, 8), np.uint16)
    WLp = wl.weights(5, 8, 256)  # arbitrary rows where the group has no entry
    k = 0
    for g in range(8):
        if tab[g, 0] >= 0:
            Bp[:, g] = B[:, k]
            WLp[g] = c["W"][:, 32 * g + tab[g, 0]]
            k += 1
    Yp = oracle.dual_gemm(Xq, Xs, Bp, Wq, Ws, WLp)
    assert np.allclose(Yp, Y, rtol=1e-12, atol=1e-14)


def test_fp8_gemm_vs_torch_decode_matmul():
    X = wl.activations_diffuse(31, 9, 96)
    W = wl.weights(32, 14, 96)
    X8, xs = oracle.quantize_fp8_rows(X)
    W8, ws = oracle.quantize_fp8_rows(W)
    Y = oracle.fp8_gemm(X8, xs, W8, ws)
    dx = torch.from_numpy(X8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    dw = torch.from_numpy(W8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    want = (dx @ dw.T) * xs.astype(np.float64)[:, None] * ws.astype(np.float64)[None, :]
    assert Y.shape == (9, 14) and np.allclose(Y, want, rtol=1e-12, atol=1e-14)
    exact = bf(X) @ bf(W).T
    assert np.abs(Y - exact).max() < 0.05 * np.abs(exact).max()


def test_grouped_forms_equal_per_expert_calls():
    E, N, K, tokens, topk = 5, 24, 64, 12, 2
    X, table = wl.activations_persistent(41, tokens, K, 1)
    oidx = oracle.table_to_index(table)
    Xq, Xs, B = oracle.quantize_mxfp4_osc(X, oidx)
    off, row_map = wl.moe_routing(42, tokens, E, topk)
    assert off[-1] == tokens * topk and sorted(row_map.tolist()) == sorted(list(range(tokens)) * 2)
    Wq, Ws, WL = [], [], []
    for e in range(E):
        W = wl.weights(50 + e, N, K)
        q, s, _ = oracle.quantize_mxfp4_osc(W)
        Wq.append(q), Ws.append(s), WL.append(oracle.gather_wl(W, oidx))
    Wq, Ws, WL = np.stack(Wq), np.stack(Ws), np.stack(WL)
    Y = oracle.grouped_dual_gemm(Xq, Xs, B, row_map, off, Wq, Ws, WL)
    for e in range(E):
        rows = row_map[off[e]:off[e + 1]]
        want = oracle.dual_gemm(Xq[rows], Xs[rows], B[rows], Wq[e], Ws[e], WL[e])
        assert np.array_equal(Y[off[e]:off[e + 1]], want)
    # grouped FP8
    T = int(off[-1])
    X2 = wl.activations_diffuse(43, T, 96)
    X8, xs = oracle.quantize_fp8_rows(X2)
    W8, ws = zip(*[oracle.quantize_fp8_rows(wl.weights(60 + e, N, 96)) for e in range(E)])
    W8, ws = np.stack(W8), np.stack(ws)
    Y8 = oracle.grouped_fp8_gemm(X8, xs, off, W8, ws)
    for e in range(E):
        sl = slice(off[e], off[e + 1])
        assert np.array_equal(Y8[sl], oracle.fp8_gemm(X8[sl], xs[sl], W8[e], ws[e]))


def test_moe_routing_lists():
    off, row_map = wl.moe_routing(4001, 64, 16, 4)
    assert off[0] == 0 and off[-1] == 256 and np.all(np.diff(off) >= 0)
    for e in range(16):
        seg = row_map[off[e]:off[e + 1]]
        assert np.all(np.diff(seg) > 0)  # each token at most once per expert, ascending
    assert np.array_equal(np.bincount(row_map, minlength=64), np.full(64, 4))
