"""Pins for the oracle's number formats (E2M1, E8M0, E4M3) -- CPU only.

Each check compares the oracle with something it does not contain: the OCP
value tables (golden files), closed forms evaluated on bit patterns, torch's
own float8 codec, or brute-force nearest-value search.
"""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from workloads import from_bf16_bits

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _gold(name):
    rows = {}
    for line in open(os.path.join(GOLD, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            k, *v = line.split()
            rows[k] = v
    return rows


def test_e2m1_decode_table():
    gold = _gold("e2m1_decode.txt")
    assert len(gold) == 16
    for code, (val,) in gold.items():
        got = oracle.e2m1_decode(int(code, 16))
        assert got == float(val) and math.copysign(1, got) == math.copysign(1, float(val))


# Decision thresholds of round-to-nearest-even onto {0,.5,1,1.5,2,3,4,6}: each
# midpoint goes to the neighbour with mantissa bit 0 (codes 0,2,4,6).
_MIDS = [(0.25, 0), (0.75, 2), (1.25, 2), (1.75, 4), (2.5, 4), (3.5, 6), (5.0, 6)]


def _e2m1_by_thresholds(a):
    code = 0
    for c, (mid, even_code) in enumerate(_MIDS):
        if a > mid or (a == mid and even_code == c + 1):
            code = c + 1
    return code


def test_e2m1_encode_ties_and_grid():
    for mid, even_code in _MIDS:
        assert oracle.e2m1_encode(mid) == even_code
        assert oracle.e2m1_encode(-mid) == even_code | 8
        assert oracle.e2m1_encode(np.nextafter(mid, 0)) == _e2m1_by_thresholds(np.nextafter(mid, 0))
        assert oracle.e2m1_encode(np.nextafter(mid, 9)) == _e2m1_by_thresholds(np.nextafter(mid, 9))
    for a in np.arange(0, 9, 1 / 64):
        assert oracle.e2m1_encode(a) == _e2m1_by_thresholds(a), a
        assert oracle.e2m1_encode(-a, True) == _e2m1_by_thresholds(a) | 8
    # saturation: 7.0 would tie with a non-existent 8; everything above 6 is 6
    for a in (6.0, 6.5, 7.0, 7.5, 7.999, 100.0, 2.0 ** 60, 1.7e38, 1e300):
        assert oracle.e2m1_encode(a) == 7
    # the sign bit follows the input even when the magnitude rounds to zero
    assert oracle.e2m1_encode(-0.0, True) == 8
    assert oracle.e2m1_encode(-0.2, True) == 8
    # round trip of all 16 codes
    for c in range(16):
        assert oracle.e2m1_encode(oracle.e2m1_decode(c), c >= 8) == c


def test_e8m0_rule_all_bf16_patterns():
    """code == max(E - 2, 0) with E the bf16 exponent field == floor(log2)-2+127 in fp64."""
    bits = np.arange(0, 0x7F80, dtype=np.uint16)  # every non-negative finite bf16
    vals = from_bf16_bits(bits).astype(np.float64)
    for b, v in zip(bits.tolist(), vals.tolist()):
        E = b >> 7
        want_int = max(E - 2, 0)
        got = oracle.e8m0_code_for_amax(v)
        assert got == want_int, (hex(b), v)
        if v > 0:
            assert got == min(max(math.floor(math.log2(v)) - 2, -127), 127) + 127
    # hand examples: 96 -> 131, 2.5 -> 126, 7.5 -> 127, 3.75 -> 126, 1.0 -> 125
    for amax, code in ((96.0, 131), (2.5, 126), (7.5, 127), (3.75, 126), (1.0, 125), (160.0, 132)):
        assert oracle.e8m0_code_for_amax(amax) == code


def test_e4m3_decode_matches_torch():
    codes = torch.arange(256, dtype=torch.uint8)
    want = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    for c in range(256):
        got = oracle.e4m3_decode(c)
        if math.isnan(want[c]):
            assert math.isnan(got) and c in (0x7F, 0xFF)
        else:
            assert got == want[c] and math.copysign(1, got) == math.copysign(1, want[c])
    assert oracle.e4m3_decode(0x7E) == 448.0 and oracle.e4m3_decode(0x01) == 2.0 ** -9


def test_e4m3_encode_matches_torch_and_bruteforce():
    gen = np.random.Generator(np.random.PCG64(7))
    xs = np.concatenate([
        gen.standard_normal(20000).astype(np.float32) * 100,
        gen.standard_normal(20000).astype(np.float32),
        gen.standard_normal(20000).astype(np.float32) * 2.0 ** -8,
        np.float32(np.arange(-464, 465, 0.5)),
    ])
    xs = xs[np.abs(xs) <= 464.0]
    want = torch.from_numpy(xs).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.e4m3_encode(v) for v in xs], np.uint8)
    assert np.array_equal(got, want)
    # brute force: nearest of the 127 finite magnitudes, ties to the even code
    mags = np.array([oracle.e4m3_decode(c) for c in range(127)])
    for v in xs[:4000]:
        d = np.abs(mags - abs(float(v)))
        best = np.flatnonzero(d == d.min())
        c = best[0] if len(best) == 1 else [b for b in best if b % 2 == 0][0]
        assert oracle.e4m3_encode(v) == (c | (0x80 if np.signbit(v) else 0))
    # saturation and round trip
    for v in (449.0, 464.0, 465.0, 1e6, 3e38):
        assert oracle.e4m3_encode(v) == 0x7E and oracle.e4m3_encode(-v) == 0xFE
    for c in list(range(0x7F)) + list(range(0x80, 0xFF)):
        assert oracle.e4m3_encode(oracle.e4m3_decode(c)) == c


def test_fp8_row_example():
    gold = _gold("fp8_row_example.txt")
    x = torch.tensor([float(v) for v in gold["x"]]).to(torch.bfloat16).view(torch.uint16).numpy()
    X8, xs = oracle.quantize_fp8_rows(x.reshape(1, -1))
    assert xs[0] == np.float32(gold["scale"][0])
    assert X8[0].tolist() == [int(c, 16) for c in gold["codes"]]
    deq = [oracle.e4m3_decode(c) * float(xs[0]) for c in X8[0]]
    assert deq == [float(v) for v in gold["deq"]]


def test_fp8_rows_properties():
    gen = np.random.Generator(np.random.PCG64(11))
    x = torch.from_numpy(gen.standard_normal((8, 96)).astype(np.float32) * 3).to(torch.bfloat16)
    x[3] = 0  # all-zero row: scale 1, codes 0
    x[5] = x[5] * 2.0 ** -110  # numerically-zero row: scale 1 as well
    bits = x.view(torch.uint16).numpy()
    X8, xs = oracle.quantize_fp8_rows(bits)
    xf = x.float().numpy()
    for m in range(8):
        amax = np.abs(xf[m]).max()
        if amax < 2.0 ** -100:
            assert xs[m] == 1.0 and not (X8[m] & 0x7F).any()
            continue
        assert xs[m] == np.float32(amax) / np.float32(448)
        # the row's largest element maps to +-448
        assert (X8[m][np.abs(xf[m]) == amax] & 0x7F == 0x7E).all()
        # same codes as torch's codec applied to the same fp32 product
        inv = np.float32(448) / np.float32(amax)
        want = torch.from_numpy(xf[m] * inv).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        assert np.array_equal(X8[m], want)
    # inputs already on the e4m3 grid times a power-of-two amax reconstruct exactly
    grid = np.array([oracle.e4m3_decode(c) for c in (0x7E, 0x40, 0x33, 0xB5, 0x08, 0x01)])
    xb = torch.tensor(grid * 2.0 ** -5, dtype=torch.float32).to(torch.bfloat16)
    X8, xs = oracle.quantize_fp8_rows(xb.view(torch.uint16).numpy().reshape(1, -1))
    assert X8[0].tolist() == [0x7E, 0x40, 0x33, 0xB5, 0x08, 0x01] and xs[0] == 2.0 ** -5


def test_nonfinite_rejected():
    x = torch.tensor([[1.0] * 31 + [float("inf")]]).to(torch.bfloat16).view(torch.uint16).numpy()
    with pytest.raises(oracle.OracleError):
        oracle.quantize_mxfp4_osc(x)
    with pytest.raises(oracle.OracleError):
        oracle.quantize_fp8_rows(x)
