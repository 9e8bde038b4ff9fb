"""Pins for the oracle's "Dynamic" protection quantiser (Section 4.2; Table 3, note 3) -- CPU only.

The dynamic scheme is the static one with a table that changes from token to token, so every row
is checked against the already pinned static quantiser fed with that row's own table, the table
coming from numpy's argmax (first maximum).  Plus closed cases and invariants.
"""
import numpy as np

import oracle
import workloads as wl
from workloads import from_bf16_bits, to_bf16_bits


def _rowwise_static(X):
    M, K = X.shape
    a = np.abs(from_bf16_bits(X).astype(np.float64)).reshape(M, K // 32, 32)
    j = a.argmax(axis=2)
    q = np.empty((M, K // 2), np.uint8)
    s = np.empty((M, K // 32), np.uint8)
    Bd = np.zeros((M, K), np.uint16)
    for m in range(M):
        oidx = (np.arange(K // 32) * 32 + j[m]).astype(np.int32)
        qm, sm, bm = oracle.quantize_mxfp4_osc(X[m:m + 1], oidx, ldb=K // 32)
        q[m], s[m] = qm[0], sm[0]
        Bd[m, oidx] = bm[0]
    return q, s, Bd, j.astype(np.uint8)


def test_rows_equal_static_quantiser_with_their_own_table():
    for X in (wl.activations_diffuse(71, 40, 512, p=0.02), wl.activations_persistent(72, 40, 512, 1, jitter=0.5)[0]):
        q, s, Bd, idx = oracle.quantize_mxfp4_dynamic(X)
        rq, rs, rB, rj = _rowwise_static(X)
        assert np.array_equal(idx, rj)
        assert np.array_equal(Bd, rB)
        assert np.array_equal(s, rs)
        assert np.array_equal(q, rq)


def test_closed_cases():
    x = np.zeros((3, 64), np.float32)
    x[0, :32] = 1.0            # all equal: position 0 is protected, the rest quantise with amax 1
    x[0, 32 + 7] = -100.0      # a lone outlier: protected, the group left behind is all zero
    x[1, 5], x[1, 9] = 3.0, -3.0   # equal magnitudes: the lower position
    x[2, :] = 0.0
    X = to_bf16_bits(x)
    X[2, 40] = 0x8000          # -0 among zeros: magnitude 0, position 0 wins
    q, s, Bd, idx = oracle.quantize_mxfp4_dynamic(X)
    assert idx[0, 0] == 0 and idx[0, 1] == 7 and idx[1, 0] == 5 and idx[2, 1] == 0
    assert from_bf16_bits(Bd[0, :1])[0] == 1.0 and from_bf16_bits(Bd[0, 39:40])[0] == -100.0
    assert (np.count_nonzero(Bd, axis=1) <= 2).all()
    # group 0 of row 0: element 0 removed (code 0), the others are 1.0 with scale 2^-2 -> E2M1 4.0 = code 6
    assert s[0, 0] == 125 and q[0, 0] == 0x60 and (q[0, 1:16] == 0x66).all()
    # group 1 of row 0: nothing left -> scale code 0 and zero codes
    assert s[0, 1] == 0 and (q[0, 16:32] == 0).all()
    # row 1: position 9 stays and sets the scale (3 -> exponent 1 - 2 = -1 -> 3 / 0.5 = 6 = code 7, negative: 0xF)
    assert s[1, 0] == 126 and q[1, 4] == 0xF0 and q[1, 2] == 0x00


def test_invariants():
    X = wl.activations_diffuse(73, 16, 256, p=0.05)
    q, s, Bd, idx = oracle.quantize_mxfp4_dynamic(X)
    x = from_bf16_bits(X).astype(np.float64)
    # exactly one protected position per group; it holds the group's largest magnitude
    nz = (Bd.reshape(16, 8, 32) != 0).sum(axis=2)
    assert (nz <= 1).all()
    amax = np.abs(x).reshape(16, 8, 32).max(axis=2)
    got = np.abs(from_bf16_bits(Bd).astype(np.float64)).reshape(16, 8, 32).max(axis=2)
    assert np.array_equal(got, amax)
    # dequantised base + protected values reproduces X to within the MXFP4 step of what is left
    e2m1 = np.array([0, .5, 1, 1.5, 2, 3, 4, 6, -0., -.5, -1, -1.5, -2, -3, -4, -6])
    codes = np.stack([q & 15, q >> 4], axis=-1).reshape(16, -1)
    deq = e2m1[codes] * np.repeat(2.0 ** (s.astype(int) - 127), 32, axis=1) + from_bf16_bits(Bd)
    rest = x.copy().reshape(16, 8, 32)
    np.put_along_axis(rest, idx[..., None].astype(np.int64), 0.0, axis=2)
    second = np.abs(rest).max(axis=2)
    assert (np.abs(deq - x).reshape(16, 8, 32).max(axis=2) <= 0.25 * second + 1e-30).all()
    # protecting the maximum can only lower the scale
    _, s0, _ = oracle.quantize_mxfp4_osc(X)
    assert (s <= s0).all() and (s < s0).any()
    # a wider Bd keeps its padding at +0
    _, _, Bw, _ = oracle.quantize_mxfp4_dynamic(X, ldb=320)
    assert np.array_equal(Bw[:, :256], Bd) and (Bw[:, 256:] == 0).all()
