"""Pins for the oracle's MXFP8 quantiser and GEMM (the 8-bit micro-scaling form of the W_2
fallback: Section 3.4, Section 4.1 implementation details) -- CPU only.

Nothing here calls the function under test to produce its own expectation: hand-worked groups
(golden file), the closed-form scale rule on bit patterns, a brute-force nearest-value search over
the E4M3 value table as decoded by torch, invariants under power-of-two scaling, and numpy's
matmul on dequantised operands.
"""
import os

import numpy as np
import torch

import oracle
import workloads as wl
from workloads import from_bf16_bits, to_bf16_bits

GOLD = os.path.join(os.path.dirname(__file__), "golden")

# all 256 E4M3 codes decoded by torch (OCP e4m3fn); 0x7F / 0xFF are NaN
E4M3 = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
FINITE = np.array([c for c in range(128) if c != 0x7F])  # non-negative finite codes, ascending values


def test_hand_worked_groups():
    n = 0
    for line in open(os.path.join(GOLD, "mxfp8_group_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        t = line.split()
        scale_code = int(t[1])
        vals, exp = t[2::2], [int(v, 16) for v in t[3::2]]
        x = np.zeros((1, 32), np.float32)
        x[0, :len(vals)] = [float(v) for v in vals]
        bits = to_bf16_bits(x)
        for i, v in enumerate(vals):
            if v == "-0":
                bits[0, i] = 0x8000
        q, s = oracle.quantize_mxfp8(bits)
        assert int(s[0, 0]) == scale_code, t[0]
        assert [int(c) for c in q[0, :len(vals)]] == exp, t[0]
        n += 1
    assert n == 4


def test_scale_rule_all_bf16_patterns():
    """E8M0 code = max(E - 8, 0) with E the biased exponent field of the largest magnitude
    (bf16 subnormals have E = 0), checked for every non-negative finite bf16 pattern."""
    pats = np.arange(0x7F80, dtype=np.uint16)
    vals = from_bf16_bits(pats).astype(np.float64)
    for p, v in zip(pats[::7], vals[::7]):  # every 7th pattern: 4 660 cases, all binades
        assert oracle.e8m0_code_for_amax_e4m3(v) == max(int(p >> 7) - 8, 0), hex(p)
    # and through the quantiser, the group's scale follows its largest element
    gen = wl.rng(5)
    x = gen.standard_normal((64, 32)).astype(np.float32) * np.exp(gen.uniform(-80, 80, (64, 1))).astype(np.float32)
    bits = to_bf16_bits(np.clip(x, -3e38, 3e38))
    _, s = oracle.quantize_mxfp8(bits)
    E = ((bits & 0x7FFF).max(axis=1) >> 7).astype(int)
    assert np.array_equal(s[:, 0].astype(int), np.maximum(E - 8, 0))


def _brute(bits, q, s):
    """Every element is a nearest E4M3 value of x / 2^e (ties to the even code), saturating."""
    x = from_bf16_bits(bits).astype(np.float64)
    M, K = x.shape
    grid = E4M3[FINITE]
    for m in range(M):
        for g in range(K // 32):
            seg = x[m, 32 * g:32 * g + 32]
            v = np.abs(seg) / 2.0 ** (int(s[m, g]) - 127)
            codes = q[m, 32 * g:32 * g + 32]
            assert np.array_equal(codes >> 7, (bits[m, 32 * g:32 * g + 32] >> 15).astype(np.uint8))
            got = grid[np.searchsorted(FINITE, codes & 0x7F)]
            assert np.array_equal(FINITE[np.searchsorted(FINITE, codes & 0x7F)], codes & 0x7F)  # never NaN codes
            vc = np.minimum(v, 448.0)  # saturation
            dist = np.abs(vc[:, None] - grid[None, :])
            assert np.all(np.abs(vc - got) == dist.min(axis=1))
            tie = (dist == dist.min(axis=1, keepdims=True)).sum(axis=1) == 2
            assert np.all((codes[tie] & 1) == 0)


def test_bruteforce_nearest():
    X = wl.activations_diffuse(3003, 24, 256)
    q, s = oracle.quantize_mxfp8(X)
    _brute(X, q, s)
    # rough values: wide exponent range, exact ties, saturating elements, zeros, subnormals
    gen = wl.rng(11)
    x = gen.standard_normal((16, 128)).astype(np.float32) * np.exp(gen.uniform(-40, 40, (16, 128))).astype(np.float32)
    x[0, :32] = 0.0
    x[1, :32] = 1e-38
    x[2, :8] = [31.5, 28, 27, 26, 25, -27, 0.001, 2 ** -14]
    bits = to_bf16_bits(np.clip(x, -3e38, 3e38))
    q, s = oracle.quantize_mxfp8(bits)
    _brute(bits, q, s)


def test_power_of_two_scaling_moves_only_the_scales():
    X = wl.activations_diffuse(77, 8, 128)
    q0, s0 = oracle.quantize_mxfp8(X)
    for k in (-9, 3, 20):
        Xk = to_bf16_bits(from_bf16_bits(X) * np.float32(2.0 ** k))
        qk, sk = oracle.quantize_mxfp8(Xk)
        assert np.array_equal(qk, q0)
        assert np.array_equal(sk.astype(int), s0.astype(int) + k)


def test_error_bound_and_better_than_mxfp4():
    X = wl.activations_diffuse(78, 32, 512)
    x = from_bf16_bits(X).astype(np.float64)
    q, s = oracle.quantize_mxfp8(X)
    deq = E4M3[q] * np.repeat(2.0 ** (s.astype(int) - 127), 32, axis=1)
    err = np.abs(deq - x)
    scale = np.repeat(2.0 ** (s.astype(int) - 127), 32, axis=1)
    v = np.abs(x) / scale
    # 3 mantissa bits: half an ulp is at most 2^-4 of the value; below the block's normal range the
    # step is 2^-9 (half of it: 2^-10); a scaled value above 464 would round to 480 or more and
    # saturates to 448 instead, at most (512 - 448) / 464 < 14 % away
    assert (err[v <= 464] <= (v[v <= 464] * 2.0 ** -4 + 2.0 ** -10) * scale[v <= 464]).all()
    assert (v < 512).all()
    assert (err[v > 464] <= 0.14 * np.abs(x)[v > 464]).all() and (q[v > 464] & 0x7F == 0x7E).all()
    q4, s4, _ = oracle.quantize_mxfp4_osc(X)
    e2m1 = np.array([0, .5, 1, 1.5, 2, 3, 4, 6, -0., -.5, -1, -1.5, -2, -3, -4, -6])
    codes4 = np.stack([q4 & 15, q4 >> 4], axis=-1).reshape(q4.shape[0], -1)
    deq4 = e2m1[codes4] * np.repeat(2.0 ** (s4.astype(int) - 127), 32, axis=1)
    # two more mantissa bits: the squared error drops by about 16 (measured here against E2M1 blocks)
    assert np.square(deq - x).sum() < 0.15 * np.square(deq4 - x).sum()


def test_gemm_vs_numpy_on_dequantised_operands():
    X = wl.activations_diffuse(79, 9, 256)
    W = wl.weights(80, 13, 256)
    xq, xs = oracle.quantize_mxfp8(X)
    wq, ws = oracle.quantize_mxfp8(W)
    Y = oracle.mxfp8_gemm(xq, xs, wq, ws)
    dx = E4M3[xq] * np.repeat(2.0 ** (xs.astype(int) - 127), 32, axis=1)
    dw = E4M3[wq] * np.repeat(2.0 ** (ws.astype(int) - 127), 32, axis=1)
    ref = dx @ dw.T
    assert np.allclose(Y, ref, rtol=1e-12, atol=1e-300)
    # and it approximates the unquantised product
    exact = from_bf16_bits(X).astype(np.float64) @ from_bf16_bits(W).astype(np.float64).T
    assert np.abs(Y - exact).max() < 0.05 * np.abs(exact).max()


def test_nonfinite_rejected():
    X = to_bf16_bits(np.ones((2, 32), np.float32))
    X[1, 3] = 0x7F80
    try:
        oracle.quantize_mxfp8(X)
    except oracle.OracleError:
        return
    raise AssertionError("a non-finite input must be refused")
