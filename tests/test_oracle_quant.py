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


def _brute_check(bits, oidx, Xq, Xs, B, G=32):
    """Definition-level check with no oracle code: per scale group of G channels, the scale is
    floor(log2 amax')-2 (written to every stored block of 32 that the group covers) and every
    element's dequantised value is a nearest point of the scaled E2M1 grid."""
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
        for g in range(K // G):
            seg = np.abs(xz[m, G * g:G * g + G])
            amax = seg.max()
            e = -127 if amax == 0 else min(max(int(np.floor(np.log2(amax))) - 2, -127), 127)
            assert np.all(Xs[m, g * (G // 32):(g + 1) * (G // 32)] == e + 127)
            v = seg / 2.0 ** e
            got = grid[codes[m, G * g:G * g + G] & 7]
            dist = np.abs(v[:, None] - grid[None, :])
            assert np.all(np.abs(v - got) == dist.min(axis=1))
            # where two grid points are equally near, the chosen code is even
            tie = (dist == dist.min(axis=1, keepdims=True)).sum(axis=1) == 2
            assert np.all((codes[m, G * g:G * g + G][tie] & 1) == 0)


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


# ---- scale groups of 64 channels (Table 2's G = 64 row) ---------------------------------------


def test_g64_table_to_index():
    t = np.array([[63, -1], [0, 40], [-1, -1]], np.int16)
    assert oracle.table_to_index(t, G=64).tolist() == [63, 64, 104]
    for bad in ([[64]], [[-2]], [[40, 40]]):
        try:
            oracle.table_to_index(np.array(bad, np.int16), G=64)
            assert False
        except oracle.OracleError:
            pass
    tab = wl.planted_table(wl.rng(3), 512, 3, group=64)
    assert tab.shape == (8, 3) and tab.max() > 31
    assert np.array_equal(oracle.table_to_index(tab, G=64), wl.table_channels(tab, group=64))


def test_g64_hand_worked_group():
    # first half: amax 5 -> shared exponent floor(log2 5) - 2 = 0 (code 127) for all 64 channels.
    # second half on that grid (step 0.5 below 2): 0.75 lies half-way between 0.5 and 1 and goes
    # to 1 (code 2, mantissa bit 0); 0.25 half-way between 0 and 0.5 goes to 0; 0.375 is nearer
    # 0.5 (code 1); -1.5 is a grid point (code 0xB); 5 itself, half-way between 4 and 6, goes to 4
    # (code 6).  With blocks of 32 the second half takes exponent floor(log2 1.5) - 2 = -2, a grid
    # of step 0.125, and keeps all four values exactly.
    x = np.zeros(64, np.float32)
    x[3], x[32], x[33], x[34], x[35] = 5.0, 0.75, 0.25, 0.375, -1.5
    bits = to_bf16_bits(x).reshape(1, 64)
    assert np.array_equal(from_bf16_bits(bits)[0], x)
    Xq, Xs, _ = oracle.quantize_mxfp4_osc(bits, G=64)
    assert Xs.tolist() == [[127, 127]]
    c = unpack_codes(Xq)[0]
    assert c[3] == 6 and c[32:36].tolist() == [2, 0, 1, 0xB] and c.astype(bool).sum() == 4
    Xq, Xs, _ = oracle.quantize_mxfp4_osc(bits)
    assert Xs.tolist() == [[127, 125]]
    assert np.array_equal(dequant(Xq, Xs)[0, 32:], x[32:].astype(np.float64))
    # protecting channel 3 leaves amax 1.5 for the whole group: exponent -2, everything exact
    oidx = oracle.table_to_index(np.array([[3]], np.int16), G=64)
    Xq, Xs, B = oracle.quantize_mxfp4_osc(bits, oidx, G=64)
    assert Xs.tolist() == [[125, 125]] and B[0, 0] == bits[0, 3]
    want = x.astype(np.float64)
    want[3] = 0
    assert np.array_equal(dequant(Xq, Xs)[0], want)


def test_g64_bruteforce_and_relation_to_blocks_of_32():
    gen = wl.rng(23)
    x = gen.standard_normal((10, 256)).astype(np.float32) * np.exp(gen.uniform(-8, 8, (10, 256)))
    x[0, :64] = 0
    x[1, 64:96] = 0  # half of a group empty
    bits = to_bf16_bits(x)
    tab = wl.planted_table(gen, 256, 2, group=64)
    oidx = oracle.table_to_index(tab, G=64)
    assert len(oidx) == 8
    Xq, Xs, B = oracle.quantize_mxfp4_osc(bits, oidx, G=64)
    _brute_check(bits, oidx, Xq, Xs, B, G=64)
    # against the same call with blocks of 32: a group's code is the larger of its two block
    # codes, and the block that owns that code keeps its element codes
    Xq32, Xs32, B32 = oracle.quantize_mxfp4_osc(bits, oidx)
    assert np.array_equal(B, B32)
    pair = Xs32.reshape(10, -1, 2)
    assert np.array_equal(Xs.reshape(10, -1, 2), np.repeat(pair.max(axis=2, keepdims=True), 2, axis=2))
    same = np.repeat(Xs == Xs32, 16, axis=1)
    assert np.array_equal(Xq[same], Xq32[same]) and same.mean() > 0.5 and not same.all()
    assert Xs[0, 0] == 0 and Xs[1, 2] == Xs[1, 3] == Xs32[1, 3] and Xs32[1, 2] == 0


def test_g64_needs_whole_groups():
    try:
        oracle.quantize_mxfp4_osc(np.zeros((1, 96), np.uint16), G=64)
        assert False
    except oracle.OracleError:
        pass


def test_g64_operands_through_the_dual_gemm():
    """Operands quantised in groups of 64 go through the unchanged GEMM definition: the result is
    the plain matrix product of the dequantised operands plus the bypass product."""
    gen = wl.rng(29)
    M, N, K = 5, 7, 192
    X = to_bf16_bits(gen.standard_normal((M, K)).astype(np.float32) * 3)
    W = to_bf16_bits(gen.standard_normal((N, K)).astype(np.float32) * 0.05)
    oidx = oracle.table_to_index(wl.planted_table(gen, K, 1, group=64), G=64)
    assert len(oidx) == 3
    Xq, Xs, B = oracle.quantize_mxfp4_osc(X, oidx, G=64)
    Wq, Ws, _ = oracle.quantize_mxfp4_osc(W, G=64)
    WL = oracle.gather_wl(W, oidx)
    Y = oracle.dual_gemm(Xq, Xs, B[:, :3], Wq, Ws, WL)
    want = dequant(Xq, Xs) @ dequant(Wq, Ws).T + \
        from_bf16_bits(B[:, :3]).astype(np.float64) @ from_bf16_bits(W)[:, oidx].astype(np.float64).T
    assert np.allclose(Y, want, rtol=1e-13, atol=1e-13)
