"""Pins for the oracle's SwiGLU (the producer of the W_2 inputs, position 4 of Section 2.1) -- CPU only.
numpy float64 for the values, closed forms at the ends of the range, identities of the logistic
function."""
import numpy as np

import oracle
import workloads as wl
from workloads import from_bf16_bits, to_bf16_bits


def _steps(a_bits, b_bits):
    def key(b):
        b = b.astype(np.int32)
        return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)
    return np.abs(key(a_bits) - key(b_bits))


def _bf16(x64):
    return to_bf16_bits(np.asarray(x64, np.float64).astype(np.float32))


def test_against_numpy_float64():
    gen = wl.rng(95)
    g = (gen.standard_normal((64, 512)) * 3).astype(np.float32)
    u = gen.standard_normal((64, 512)).astype(np.float32)
    G, U = to_bf16_bits(g), to_bf16_bits(u)
    g64, u64 = from_bf16_bits(G).astype(np.float64), from_bf16_bits(U).astype(np.float64)
    silu = g64 / (1.0 + np.exp(-g64))
    # with up = 1 only the rounding of silu to bf16 is left: the single-precision silu must agree with
    # the float64 one everywhere except within 2^-20 of a rounding boundary
    ones = to_bf16_bits(np.ones_like(g))
    d1 = _steps(oracle.swiglu(G, ones), _bf16(silu))
    assert d1.max() <= 1 and (d1 == 0).mean() > 0.999
    # with a general up there are two roundings to 8 bits against none: one step at most
    d = _steps(oracle.swiglu(G, U), _bf16(silu * u64))
    assert d.max() <= 1 and (d == 0).mean() > 0.6
    assert np.abs(from_bf16_bits(oracle.swiglu(G, U)) - silu * u64).max() <= 2.0 ** -7 * np.abs(silu * u64).max()


def test_dense_sweep_of_the_gate():
    """every bf16 gate value between -100 and 100: silu within half a bf16 step (plus the single
    precision error) of the float64 value; zero at zero; the identity at large gates."""
    bits = np.arange(0x10000, dtype=np.uint32).astype(np.uint16)
    vals = from_bf16_bits(bits)
    keep = np.isfinite(vals) & (np.abs(vals) <= 100)
    G = bits[keep][None, :]
    g64 = from_bf16_bits(G).astype(np.float64)
    Y = from_bf16_bits(oracle.swiglu(G, to_bf16_bits(np.ones(G.shape, np.float32)))).astype(np.float64)
    ref = g64 / (1.0 + np.exp(-g64))
    mid = (np.abs(g64) >= 2.0 ** -100) & (np.abs(g64) <= 80)   # away from bf16 subnormals and from the clamp at 86
    assert (np.abs(Y - ref)[mid] <= np.abs(ref[mid]) * 2.0 ** -8 * 1.001).all()
    assert (np.abs(Y - ref)[~mid] <= 1e-30).all()
    assert (Y[g64 == 0] == 0).all()
    assert (Y[g64 >= 20] == g64[g64 >= 20]).all()
    assert (np.abs(Y[g64 <= -90]) < 1e-30).all()
    # the minimum of silu is -0.2785 near g = -1.2785: nothing goes below it
    assert -0.2794 <= Y.min() <= -0.2775   # -0.2785 rounded to 8 significant bits


def test_identities_and_edges():
    gen = wl.rng(96)
    G = to_bf16_bits((gen.standard_normal((4, 256)) * 4).astype(np.float32))
    ones = to_bf16_bits(np.ones((4, 256), np.float32))
    zeros = np.zeros((4, 256), np.uint16)
    assert (from_bf16_bits(oracle.swiglu(G, zeros)) == 0).all()
    # up = 2^k scales the result exactly; up = -1 flips the sign exactly
    y1 = from_bf16_bits(oracle.swiglu(G, ones))
    assert np.array_equal(from_bf16_bits(oracle.swiglu(G, to_bf16_bits(np.full((4, 256), 8.0, np.float32)))), y1 * 8)
    assert np.array_equal(from_bf16_bits(oracle.swiglu(G, to_bf16_bits(np.full((4, 256), -1.0, np.float32)))), -y1)
    # silu(g) - silu(-g) = g, up to the two roundings to bf16
    Gn = G ^ np.uint16(0x8000)
    diff = y1.astype(np.float64) - from_bf16_bits(oracle.swiglu(Gn, ones)).astype(np.float64)
    g = from_bf16_bits(G).astype(np.float64)
    assert (np.abs(diff - g) <= 2.0 ** -7 * np.maximum(np.abs(g), 0.3)).all()
    X = G.copy()
    X[0, 0] = 0x7F80
    try:
        oracle.swiglu(X, ones)
    except oracle.OracleError:
        return
    raise AssertionError("a non-finite input must be refused")


def test_recipe_against_the_plain_double_precision_form():
    """The fixed single-precision silu recipe against the oracle's textbook SwiGLU (libm exp in
    double, roundings only where a model made of bf16 modules has them); the plain form is pinned to
    numpy float64 here."""
    gen = wl.rng(195)
    G = to_bf16_bits((gen.standard_normal((128, 4096)) * 2.5).astype(np.float32))
    U = wl.activations_diffuse(196, 128, 4096, p=0.01)
    g64, u64 = from_bf16_bits(G).astype(np.float64), from_bf16_bits(U).astype(np.float64)
    plain1 = oracle.swiglu_plain(G, U)
    d = _steps(plain1, _bf16(g64 / (1.0 + np.exp(-g64)) * u64))
    assert d.max() <= 1 and (d == 0).mean() > 0.9999
    Y = oracle.swiglu(G, U)
    assert _steps(Y, plain1).max() <= 1                              # one rounding against two
    d2 = _steps(Y, oracle.swiglu_plain(G, U, mid_round=True))        # same roundings, plain arithmetic
    assert d2.max() <= 1 and (d2 == 0).mean() >= 0.999
    ones = to_bf16_bits(np.ones_like(g64, dtype=np.float32))
    d3 = _steps(oracle.swiglu(G, ones), oracle.swiglu_plain(G, ones))
    assert d3.max() <= 1 and (d3 == 0).mean() >= 0.999
