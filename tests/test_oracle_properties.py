"""Property tests of the oracle (hypothesis; CPU only).

1. Equivariance under channel permutations that preserve the groups of 32 (whole groups move, and
   channels move inside their group), applied alike to the columns of X, the columns of W and the
   table: scales move with their groups, B and W_L keep the protected values, Y does not change
   beyond double-precision rounding.  An arbitrary permutation changes group membership and is not
   covered (Section 3.1: the table is defined per group).
2. Protecting one more channel than necessary (Section 2.2: a channel that is wrongly listed is
   simply processed in higher precision): its values are carried exactly, no scale gets coarser, no
   other group changes, and the error of the layer against the exact product does not grow.
"""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
import workloads as wl
from workloads import from_bf16_bits

SET = dict(max_examples=30, deadline=None, derandomize=True)


def _layer(X, W, oidx):
    Xq, Xs, B = oracle.quantize_mxfp4_osc(X, oidx)
    Wq, Ws, _ = oracle.quantize_mxfp4_osc(W)
    WL = oracle.gather_wl(W, oidx) if len(oidx) else None
    return (Xq, Xs, B), oracle.dual_gemm(Xq, Xs, B if len(oidx) else None, Wq, Ws, WL)


@st.composite
def problems(draw):
    seed = draw(st.integers(0, 2 ** 31 - 1))
    M = draw(st.integers(1, 6))
    N = draw(st.integers(1, 6))
    Kg = draw(st.integers(1, 5))
    r = draw(st.integers(0, 3))
    return seed, M, N, Kg, r


@settings(**SET)
@given(problems())
def test_group_preserving_permutations(p):
    seed, M, N, Kg, r = p
    K = 32 * Kg
    gen = wl.rng(seed)
    X, table = wl.activations_persistent(seed, M, K, r) if r else (wl.activations_diffuse(seed, M, K), None)
    W = wl.weights(seed + 1, N, K)
    oidx = oracle.table_to_index(table) if r else np.zeros(0, np.int32)
    gperm = gen.permutation(Kg)
    perm = np.concatenate([32 * g + gen.permutation(32) for g in gperm])   # new column j holds old column perm[j]
    inv = np.argsort(perm)
    oidx2 = np.sort(inv[oidx]).astype(np.int32)
    (Xq, Xs, B), Y = _layer(X, W, oidx)
    (Xq2, Xs2, B2), Y2 = _layer(X[:, perm], W[:, perm], oidx2)
    assert np.array_equal(Xs2, Xs[:, gperm])
    if r:
        # the same protected values, listed in the new channel order
        order = np.argsort(inv[oidx])
        assert np.array_equal(B2[:, :len(oidx)], B[:, :len(oidx)][:, order])
    # codes move with their channels
    lo, hi = Xq & 0xF, Xq >> 4
    codes = np.stack([lo, hi], axis=2).reshape(M, K)
    lo2, hi2 = Xq2 & 0xF, Xq2 >> 4
    assert np.array_equal(np.stack([lo2, hi2], axis=2).reshape(M, K), codes[:, perm])
    assert np.allclose(Y2, Y, rtol=1e-12, atol=1e-13 * max(1.0, np.abs(Y).max()))


@settings(**SET)
@given(st.integers(0, 2 ** 31 - 1), st.integers(1, 4), st.integers(0, 2))
def test_one_more_protected_channel_never_hurts(seed, Kg, r):
    K, M, N = 32 * Kg, 64, 64
    gen = wl.rng(seed)
    X, table = wl.activations_persistent(seed, M, K, r) if r else (wl.activations_diffuse(seed, M, K), None)
    W = wl.weights(seed + 1, N, K)
    oidx = oracle.table_to_index(table) if r else np.zeros(0, np.int32)
    free = np.setdiff1d(np.arange(K), oidx)
    c = int(free[gen.integers(0, len(free))])          # an ordinary channel, listed by mistake
    oidx2 = np.sort(np.append(oidx, c)).astype(np.int32)
    (Xq, Xs, B), Y = _layer(X, W, oidx)
    (Xq2, Xs2, B2), Y2 = _layer(X, W, oidx2)
    assert np.array_equal(B2[:, int(np.searchsorted(oidx2, c))], X[:, c])          # carried exactly
    assert (Xs2 <= Xs).all()                                                       # no scale gets coarser
    g = c // 32
    other = np.ones(Kg, bool)
    other[g] = False
    assert np.array_equal(Xs2[:, other], Xs[:, other])
    keep = np.ones(K // 2, bool)
    keep[16 * g:16 * g + 16] = False
    assert np.array_equal(Xq2[:, keep], Xq[:, keep])                               # other groups untouched
    exact = from_bf16_bits(X).astype(np.float64) @ from_bf16_bits(W).astype(np.float64).T
    e_old, e_new = ((Y - exact) ** 2).sum(), ((Y2 - exact) ** 2).sum()
    assert e_new <= e_old * 1.005
