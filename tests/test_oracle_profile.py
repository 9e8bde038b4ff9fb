"""Pins for the oracle's offline profiling (Section 2.1 Eq. 1, Section 2.2 Eq. 2-4, Alg. 1) -- CPU only.

Expectations come from a hand-worked example (golden file), from numpy's own argmax / max /
bincount / argsort on the same data, from planted data whose table is known by construction, and
from invariants (additivity over token batches, token order, power-of-two scaling, limits of T).
"""
import os

import numpy as np

import oracle
import workloads as wl
from workloads import from_bf16_bits, to_bf16_bits

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _golden():
    d = {"x": [], "hist": []}
    for line in open(os.path.join(GOLD, "profile_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        v = [float(t) for t in v]
        if k in ("x", "hist"):
            d[k].append(v)
        else:
            d[k] = v
    return d


def test_hand_worked_example():
    g = _golden()
    X = to_bf16_bits(np.array(g["x"], np.float32))
    assert np.array_equal(from_bf16_bits(X), np.array(g["x"], np.float32))
    G = int(g["G"][0])
    T = oracle.profile_threshold(X, alpha=g["alpha"][0])
    assert T == g["T"][0]
    hist = oracle.profile_hist(X, T, G)
    assert np.array_equal(hist, np.array(g["hist"], np.uint32))
    table, n_total, n_hit, density, cbar = oracle.profile_table(hist, 1)
    assert list(n_total) == g["n_total"] and list(n_hit) == g["n_hit"]
    assert list(density) == g["density"] and cbar == g["cbar"][0]
    assert list(table[:, 0]) == g["table1"]
    table2 = oracle.profile_table(hist, 2)[0]
    assert list(table2.reshape(-1)) == g["table2"]


def _numpy_hist(X, T, G):
    a = np.abs(from_bf16_bits(X).astype(np.float64)).reshape(X.shape[0], -1, G)
    jstar = a.argmax(axis=2)                      # numpy: first of equal maxima
    hit = a.max(axis=2) > T
    Kg = a.shape[1]
    flat = (np.arange(Kg)[None, :] * G + jstar)[hit]
    return np.bincount(flat, minlength=Kg * G).reshape(Kg, G).astype(np.uint32)


def test_hist_against_numpy_routines():
    for G in (16, 32, 64):
        for seed, X in ((1, wl.activations_persistent(41, 96, 512, 1, jitter=0.3)[0]),
                        (2, wl.activations_diffuse(42, 96, 512, p=0.02))):
            T = float(np.float32(oracle.profile_threshold(X, 5.0)))
            h = oracle.profile_hist(X, T, G)
            assert np.array_equal(h, _numpy_hist(X, T, G)), (G, seed)
            assert h.sum() > 0


def test_threshold_against_numpy_mean_and_closed_form():
    X = wl.activations_diffuse(43, 64, 256)
    x = from_bf16_bits(X).astype(np.float64)
    assert np.isclose(oracle.profile_threshold(X, 5.0), 5.0 * np.abs(x).mean(), rtol=1e-13)
    assert np.isclose(oracle.profile_threshold(X, 1.5), 1.5 * np.abs(x).mean(), rtol=1e-13)
    c = to_bf16_bits(np.full((7, 32), -3.5, np.float32))
    assert oracle.profile_threshold(c, 5.0) == 17.5
    c[3, 4] = 0x7FC0
    try:
        oracle.profile_threshold(c, 5.0)
    except oracle.OracleError:
        return
    raise AssertionError("a non-finite input must be refused")


def test_planted_table_is_recovered_and_density_separates():
    """Token-persistent outlier channels give back the planted table with density near 1;
    independent outliers spread over the group and stay far below the 35 % line of Section 2.3."""
    Xp, planted = wl.activations_persistent(44, 512, 1024, 1)
    T = oracle.profile_threshold(Xp, 5.0)
    table, n_total, n_hit, density, cbar = oracle.profile_table(oracle.profile_hist(Xp, T), 1)
    assert np.array_equal(table, planted)
    assert (n_total > 0).all() and cbar > 0.95
    # two persistent channels per group: the two most frequent indices are the planted pair
    X2, planted2 = wl.activations_persistent(48, 512, 512, 2)
    t2 = oracle.profile_table(oracle.profile_hist(X2, oracle.profile_threshold(X2, 5.0)), 2)[0]
    assert np.array_equal(np.sort(t2, axis=1), np.sort(planted2, axis=1))
    Xd = wl.activations_diffuse(45, 4096, 256, p=0.005)
    T = oracle.profile_threshold(Xd, 5.0)
    _, n_total, _, _, cbar = oracle.profile_table(oracle.profile_hist(Xd, T), 1)
    assert n_total.min() > 300 and cbar < 0.10


def test_table_against_numpy_sort():
    gen = wl.rng(46)
    hist = gen.integers(0, 6, (40, 32)).astype(np.uint32)
    hist[3] = 0                      # an empty candidate set
    hist[4] = 0
    hist[4, 17] = 9                  # a single candidate
    hist[5, :] = 2                   # all counts equal: lowest indices first
    for R in (1, 2, 4, 32):
        table, n_total, n_hit, density, cbar = oracle.profile_table(hist, R)
        order = np.argsort(-hist.astype(np.int64), axis=1, kind="stable")[:, :R]
        cnt = np.take_along_axis(hist, order, axis=1)
        assert np.array_equal(table, np.where(cnt > 0, order, -1).astype(np.int16)), R
        assert np.array_equal(n_total, hist.sum(axis=1)) and np.array_equal(n_hit, hist.max(axis=1))
        ne = n_total > 0
        assert np.allclose(density[ne], n_hit[ne] / n_total[ne], rtol=1e-15) and (density[~ne] == 0).all()
        assert np.isclose(cbar, (n_hit[ne] / n_total[ne]).mean(), rtol=1e-14)
    assert (oracle.profile_table(hist, 1)[0][3] == -1).all()
    assert list(oracle.profile_table(hist, 3)[0][4]) == [17, -1, -1]
    assert list(oracle.profile_table(hist, 3)[0][5]) == [0, 1, 2]
    t0 = oracle.profile_table(np.zeros((4, 32), np.uint32), 1)
    assert (t0[0] == -1).all() and t0[4] == 0.0


def test_invariants():
    X, _ = wl.activations_persistent(47, 200, 256, 2, jitter=0.5)
    T = float(np.float32(oracle.profile_threshold(X, 5.0)))
    h = oracle.profile_hist(X, T)
    # additivity over token batches and independence of the token order
    acc = oracle.profile_hist(X[:77], T)
    acc = oracle.profile_hist(X[77:], T, hist=acc)
    assert np.array_equal(acc, h)
    assert np.array_equal(oracle.profile_hist(X[wl.rng(1).permutation(200)], T), h)
    # a power-of-two change of units moves the threshold with the data and nothing else
    X8 = to_bf16_bits(from_bf16_bits(X) * np.float32(2.0 ** -6))
    assert oracle.profile_threshold(X8, 5.0) == oracle.profile_threshold(X, 5.0) * 2.0 ** -6
    assert np.array_equal(oracle.profile_hist(X8, T * 2.0 ** -6), h)
    # limits of the threshold: below everything each token counts once per group, above nothing does
    assert (oracle.profile_hist(X, -1.0).sum(axis=1) == 200).all()
    assert oracle.profile_hist(X, 3e38).sum() == 0
    # the comparison is strict: a group maximum equal to T is not an outlier
    one = to_bf16_bits(np.array([[0.5] * 31 + [4.0]], np.float32))
    assert oracle.profile_hist(one, 4.0).sum() == 0 and oracle.profile_hist(one, 3.99)[0, 31] == 1
    # equal magnitudes inside a group: the lowest index wins, whatever the signs
    tie = to_bf16_bits(np.array([[0.0] * 5 + [-3.0, 1.0, 3.0] + [0.0] * 24], np.float32))
    assert oracle.profile_hist(tie, 1.0)[0, 5] == 1
