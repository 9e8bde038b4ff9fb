"""Pins for the oracle's OSC-enhanced MXFP4 quantiser (Alg. 2) -- CPU only."""
import os

import numpy as np
import torch

import oracle
import workloads as wl
from workloads import from_bf16_bits, to_bf16_bits

GOLD = os.path.join(os.path.dirname(__file__), "golden")
E2M1 = np.array([0, .5, 1, 1.5, 2, 3, 4, 6, -0., -.5, -1, -1.5, -2, -3, -4, -6])  # OCP table


def _gold(name):
    rows = {}
    for line in open(os.path.join(GOLD, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            k, *v = line.split()
            rows[k] = v
    return rows


def unpack_codes(Xq):
    out = np.empty((Xq.shape[0], Xq.shape[1] * 2), np.uint8)
    out[:, 0::2] = Xq & 15
    out[:, 1::2] = Xq >> 4
    return out


def dequant(Xq, Xs):
    c = unpack_codes(Xq)
    s = np.ldexp(1.0, Xs.astype(np.int64) - 127)
    return E2M1[c] * np.repeat(s, 32, axis=1)


def test_hand_worked_group():
    g = _gold("mxfp4_group_example.txt")
    x = np.zeros(32, np.float32)
    x[:11] = [float(v) for v in g["x"]]
    bits = to_bf16_bits(x).reshape(1, 32)
    assert np.array_equal(from_bf16_bits(bits)[0], x)  # representable
    # no suppression
    Xq, Xs, B = oracle.quantize_mxfp4_osc(bits)
    assert Xs[0, 0] == int(g["plain_scale"][0]) and B.shape == (1, 0)
    assert unpack_codes(Xq)[0, :11].tolist() == [int(c, 16) for c in g["plain_codes"]]
    assert not unpack_codes(Xq)[0, 11:].any()
    # table entry 3
    oidx = oracle.table_to_index(np.array([[3]], np.int16))
    assert oidx.tolist() == [3]
    Xq, Xs, B = oracle.quantize_mxfp4_osc(bits, oidx)
    assert Xs[0, 0] == int(g["osc_scale"][0])
    assert B.shape == (1, 32) and B[0, 0] == int(g["osc_b_bits"][0], 16) and not B[0, 1:].any()
    assert unpack_codes(Xq)[0, :11].tolist() == [int(c, 16) for c in g["osc_codes"]]
    assert Xq[0, :6].tolist() == [int(c, 16) for c in g["osc_bytes"]] and not Xq[0, 6:].any()
    deq = dequant(Xq, Xs)[0, :11]
    want = np.array([float(v) for v in g["osc_dequant"]])
    assert np.array_equal(deq, want) and np.array_equal(np.signbit(deq), np.signbit(want))


def test_saturation_examples():
    for amax, code, deq in ((7.5, 127, 6.0), (3.75, 126, 3.0)):
        x = np.zeros(32, np.float32)
        x[5] = -amax
        Xq, Xs, _ = oracle.quantize_mxfp4_osc(to_bf16_bits(x).reshape(1, 32))
        assert Xs[0, 0] == code and unpack_codes(Xq)[0, 5] == 0xF
        assert dequant(Xq, Xs)[0, 5] == -deq


def test_table_to_index():
    t = np.array([[5, -1], [-1, -1], [31, 0], [-1, 7]], np.int16)
    assert oracle.table_to_index(t).tolist() == [5, 64, 95, 96 + 7]
    assert oracle.table_to_index(np.full((3, 1), -1, np.int16)).tolist() == []
    for bad in ([[32]], [[-2]], [[4, 4]]):
        try:
            oracle.table_to_index(np.array(bad, np.int16))
            assert False
        except oracle.OracleError:
            pass
    # agrees with the workload module's own bookkeeping
    gen = wl.rng(3)
    tab = wl.planted_table(gen, 256, 4)
    assert np.array_equal(oracle.table_to_index(tab), wl.table_channels(tab))


def _brute_check(bits, oidx, Xq, Xs, B):
    """Definition-level check with no oracle code: per group, the scale is floor(log2 amax')-2
    and every element's dequantised value is a nearest point of the scaled E2M1 grid."""
    x = from_bf16_bits(bits).astype(np.float64)
    M, K = x.shape
    xz = x.copy()
    xz[:, oidx] = 0.0
    assert np.array_equal(B[:, :len(oidx)], bits[:, oidx])  # bit copy
    assert not B[:, len(oidx):].any()
    codes = unpack_codes(Xq)
    sign_in = (bits >> 15).astype(bool)
    sign_in[:, oidx] = False  # a removed element is written as +0
    assert np.array_equal(codes >> 3, sign_in.astype(np.uint8))
    grid = E2M1[:8]
    for m in range(M):
        for g in range(K // 32):
            seg = np.abs(xz[m, 32 * g:32 * g + 32])
            amax = seg.max()
            e = -127 if amax == 0 else min(max(int(np.floor(np.log2(amax))) - 2, -127), 127)
            assert Xs[m, g] == e + 127
            v = seg / 2.0 ** e
            got = grid[codes[m, 32 * g:32 * g + 32] & 7]
            dist = np.abs(v[:, None] - grid[None, :])
            assert np.all(np.abs(v - got) == dist.min(axis=1))
            # where two grid points are equally near, the chosen code is even
            tie = (dist == dist.min(axis=1, keepdims=True)).sum(axis=1) == 2
            assert np.all((codes[m, 32 * g:32 * g + 32][tie] & 1) == 0)


def test_bruteforce_nearest_on_config1():
    c = wl.config1_tiny()
    oidx = oracle.table_to_index(c["table"])
    assert len(oidx) == 8
    Xq, Xs, B = oracle.quantize_mxfp4_osc(c["X"], oidx)
    _brute_check(c["X"], oidx, Xq, Xs, B)
    Xq0, Xs0, B0 = oracle.quantize_mxfp4_osc(c["X"])
    _brute_check(c["X"], np.zeros(0, np.int64), Xq0, Xs0, B0)
    # removing an element never widens a scale; removing the x64 channel (an N(0,1) draw times
    # 64, so not always the group's largest) tightens it by several binades on average
    drop = Xs0.astype(int) - Xs.astype(int)
    assert drop.min() >= 0 and drop.max() <= 9 and drop.mean() > 3


def test_bruteforce_nearest_on_rough_values():
    gen = wl.rng(17)
    x = gen.standard_normal((12, 128)).astype(np.float32) * np.exp(gen.uniform(-30, 30, (12, 128)))
    x[0, :32] = 0  # all-zero group
    x[1, 32:64] = 1e-38  # bf16-subnormal group -> scale code 0, codes still decided
    x[2, 5] = -0.0
    bits = to_bf16_bits(x)
    tab = wl.planted_table(gen, 128, 2)
    oidx = oracle.table_to_index(tab)
    Xq, Xs, B = oracle.quantize_mxfp4_osc(bits, oidx)
    _brute_check(bits, oidx, Xq, Xs, B)
    assert Xs[0, 0] == 0 and Xs[1, 1] == 0 and (unpack_codes(Xq)[1, 32:64] & 7).any()


def test_exact_64x_drops_scale_by_6():
    gen = wl.rng(5)
    x = gen.standard_normal((4, 64)).astype(np.float32)
    bits = to_bf16_bits(x)
    x = from_bf16_bits(bits).copy()
    for m in range(4):
        for g in range(2):
            seg = x[m, 32 * g:32 * g + 32]
            seg[7] = 0
            seg[7] = 64 * np.abs(seg).max()  # exactly 6 binades above the rest
    bits = to_bf16_bits(x)
    _, Xs0, _ = oracle.quantize_mxfp4_osc(bits)
    _, Xs1, _ = oracle.quantize_mxfp4_osc(bits, np.array([7, 39], np.int32))
    assert np.all(Xs0.astype(int) - Xs1.astype(int) == 6)


def test_scale_and_codes_independent_of_protected_value():
    c = wl.config1_tiny()
    oidx = oracle.table_to_index(c["table"])
    Xq, Xs, B = oracle.quantize_mxfp4_osc(c["X"], oidx)
    X2 = c["X"].copy()
    X2[:, oidx] = to_bf16_bits(np.float32([-12345.0]))[0]
    Xq2, Xs2, B2 = oracle.quantize_mxfp4_osc(X2, oidx)
    assert np.array_equal(Xq, Xq2) and np.array_equal(Xs, Xs2)
    assert np.all(B2[:, :8] == X2[:, oidx])
    # groups flagged -1 are plain MXFP4: drop half the table and compare those groups
    half = oidx[::2]
    Xq3, Xs3, _ = oracle.quantize_mxfp4_osc(c["X"], half)
    Xq0, Xs0, _ = oracle.quantize_mxfp4_osc(c["X"])
    for g in range(8):
        ref_q, ref_s = (Xq, Xs) if g % 2 == 0 else (Xq0, Xs0)
        assert np.array_equal(Xq3[:, 16 * g:16 * g + 16], ref_q[:, 16 * g:16 * g + 16])
        assert np.array_equal(Xs3[:, g], ref_s[:, g])


def test_ldb_padding_and_all_channels():
    c = wl.config1_tiny()
    oidx = oracle.table_to_index(c["table"])
    _, _, B = oracle.quantize_mxfp4_osc(c["X"], oidx, ldb=40)
    assert B.shape == (16, 40) and not B[:, 8:].any()
    allc = np.arange(256, dtype=np.int32)
    Xq, Xs, B = oracle.quantize_mxfp4_osc(c["X"], allc)
    assert not Xq.any() and not Xs.any() and np.array_equal(B, c["X"])


def test_weight_quantisation_is_plain_mxfp4_rows():
    W = wl.weights(9, 24, 96)
    Wq, Ws, _ = oracle.quantize_mxfp4_osc(W)
    _brute_check(W, np.zeros(0, np.int64), Wq, Ws, np.zeros((24, 0), np.uint16))
    WL = oracle.gather_wl(W, np.array([3, 40, 95], np.int32))
    assert WL.shape == (3, 24) and np.array_equal(WL, W[:, [3, 40, 95]].T)
