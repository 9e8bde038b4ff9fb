"""The seeded input generators: reproducible to the byte (stored CRCs), and with the structure
their recipes state (planted token-persistent channels, independent outliers, weight scale,
top-k routing).  They hold none of the method's arithmetic; bf16 rounding is checked against torch."""
import os
import sys
import zlib

import numpy as np
import torch

import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")
sys.path.insert(0, GOLD)


def test_generators_reproduce_stored_crcs():
    import make_workload_crcs as mk
    stored = dict(line.rsplit(" ", 1) for line in open(os.path.join(GOLD, "workloads_crc.txt")) if not line.startswith("#"))
    seen = 0
    for name, a in mk.cases():
        assert int(stored[name]) == zlib.crc32(np.ascontiguousarray(a).tobytes()), name
        seen += 1
    assert seen == len(stored) == 9


def test_bf16_rounding_matches_torch():
    gen = wl.rng(1)
    x = (gen.standard_normal(20000) * np.exp(gen.uniform(-30, 30, 20000))).astype(np.float32)
    x[:4] = [0.0, -0.0, 1.00390625, 1.01171875]  # the last two: exact ties, to even
    ours = wl.to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)
    assert np.array_equal(wl.from_bf16_bits(ours), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_recipes():
    X, table = wl.activations_persistent(7, 512, 1024, 2)
    assert table.shape == (32, 2) and (table >= 0).all() and (table < 32).all() and (table[:, 0] != table[:, 1]).all()
    x = wl.from_bf16_bits(X)
    ch = wl.table_channels(table)
    assert len(ch) == 64 and (np.diff(ch) > 0).all()
    rest = np.setdiff1d(np.arange(1024), ch)
    # planted channels carry a fixed factor between 20 and 100 on every token; the rest is N(0, 1)
    ratio = x[:, ch].std(axis=0) / x[:, rest].std()
    assert ratio.min() > 15 and ratio.max() < 120
    assert abs(x[:, rest].std() - 1.0) < 0.02 and abs(x[:, rest].mean()) < 0.01
    Xd = wl.from_bf16_bits(wl.activations_diffuse(8, 1024, 1024, p=0.005, factor=50.0))
    assert abs((np.abs(Xd) > 8).mean() - 0.005 * 0.87) < 0.001   # P(|50 z| > 8) = 0.873
    W = wl.from_bf16_bits(wl.weights(9, 256, 1024))
    assert abs(W.std() - 0.02) < 0.0005
    off, rm = wl.moe_routing(10, 512, 16, 4)
    assert off[0] == 0 and off[-1] == 512 * 4 and (np.diff(off) >= 0).all() and len(rm) == 512 * 4
    counts = np.bincount(rm, minlength=512)
    assert (counts == 4).all()   # every token routed to exactly top_k experts
