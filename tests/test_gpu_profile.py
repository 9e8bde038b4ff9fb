"""GPU parity of the offline profiling entry points (Section 2.1 Eq. 1, Section 2.2 Eq. 2-4, Alg. 1)
against the CPU oracle: counts, table entries, N_total and N_hit bit for bit; the threshold and the
densities (floating point) to 1e-6 relative."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from workloads import from_bf16_bits, to_bf16_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def osc():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2604_12782_amd as m
    m.lib()
    return m


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def bf(bits):
    return dev(bits.view(np.int16)).view(torch.bfloat16)


def gpu_hist(osc, X, T, G=32, hist=None):
    Td = torch.tensor([T], dtype=torch.float32, device="cuda")
    h = osc.osc_profile_hist(bf(X) if isinstance(X, np.ndarray) else X, Td, G, hist)
    return h


def as_u32(t):
    return t.cpu().numpy().view(np.uint32)


SHAPES = [(1, 64), (5, 192), (77, 1088), (333, 4096), (1030, 2112)]


@pytest.mark.parametrize("S,H", SHAPES)
def test_threshold(osc, S, H):
    X = wl.activations_diffuse(100 + S, S, H, p=0.01)
    ref = oracle.profile_threshold(X, 5.0)
    acc = osc.osc_profile_abs_sum(bf(X))
    T = osc.osc_profile_threshold(acc, S * H, 5.0)
    x = from_bf16_bits(X).astype(np.float64)
    assert abs(acc.item() - np.abs(x).sum()) <= 1e-6 * np.abs(x).sum()
    assert abs(T.item() - ref) <= 1e-6 * ref
    # in pieces: the same accumulator over two token batches
    if S > 1:
        acc2 = osc.osc_profile_abs_sum(bf(X[:S // 3]))
        acc2 = osc.osc_profile_abs_sum(bf(X[S // 3:]), acc2)
        assert abs(acc2.item() - acc.item()) <= 1e-9 * acc.item()


@pytest.mark.parametrize("G", [16, 32, 64])
@pytest.mark.parametrize("S,H", SHAPES)
def test_hist_bit_exact(osc, S, H, G):
    for kind in ("persistent", "diffuse"):
        X = (wl.activations_persistent(200 + S, S, H, 1, jitter=0.4)[0] if kind == "persistent"
             else wl.activations_diffuse(300 + S, S, H, p=0.02))
        T = float(np.float32(oracle.profile_threshold(X, 5.0)))
        ref = oracle.profile_hist(X, T, G)
        got = as_u32(gpu_hist(osc, X, T, G))
        assert np.array_equal(got, ref), (kind, S, H, G)
        assert ref.sum() > 0 or S < 8


def test_hist_threshold_limits_and_accumulation(osc):
    X = wl.activations_diffuse(401, 150, 1504 // 32 * 32, p=0.02)
    S, H = X.shape
    for T in (-1.0, 0.0, 1.0, 3e38, float("inf"), float("nan")):
        ref = oracle.profile_hist(X, T) if T == T else np.zeros((H // 32, 32), np.uint32)
        assert np.array_equal(as_u32(gpu_hist(osc, X, T)), ref), T
    assert (as_u32(gpu_hist(osc, X, -1.0)).sum(axis=1) == S).all()
    T = 2.0
    h = gpu_hist(osc, X[:60], T)
    h = gpu_hist(osc, X[60:], T, hist=h)
    assert np.array_equal(as_u32(h), oracle.profile_hist(X, T))
    # rows taken out of a wider buffer (ldx > H)
    wide = torch.zeros((S, H + 64), dtype=torch.bfloat16, device="cuda")
    wide[:, :H] = bf(X)
    assert np.array_equal(as_u32(gpu_hist(osc, wide[:, :H], T)), oracle.profile_hist(X, T))
    assert abs(osc.osc_profile_abs_sum(wide[:, :H]).item() - osc.osc_profile_abs_sum(bf(X)).item()) < 1e-6


def test_hist_edge_values(osc):
    """Zeros of both signs, subnormals, equal magnitudes of opposite sign, the largest finite value,
    a group maximum exactly at the threshold."""
    x = np.zeros((6, 128), np.float32)
    x[0, 5], x[0, 7] = -3.0, 3.0              # tie: index 5
    x[1, 32 + 31], x[1, 32 + 30] = 4.0, -4.0  # tie at the end of a group: index 30
    x[2, 64] = 4.0                            # exactly T: not counted when T = 4
    x[3, 96 + 9] = 3.3e38
    x[4, :] = 1e-39                           # bf16 subnormals everywhere: index 0 of each group
    bits = to_bf16_bits(x)
    bits[5, :] = 0x8000                       # all -0
    for G in (16, 32, 64):
        for T in (4.0, 3.99, 1.0, 0.0, -1.0, 1e-40):
            ref = oracle.profile_hist(bits, T, G)
            assert np.array_equal(as_u32(gpu_hist(osc, bits, T, G)), ref), (G, T)
    assert oracle.profile_hist(bits, 1.0)[0, 5] == 1 and oracle.profile_hist(bits, 1.0)[1, 30] == 1


@pytest.mark.parametrize("G", [16, 32, 64])
def test_table_and_density(osc, G):
    gen = wl.rng(500 + G)
    hist = gen.integers(0, 5, (300, G)).astype(np.uint32)
    hist[3] = 0
    hist[4] = 0
    hist[4, G - 1] = 9
    hist[5, :] = 2
    hist[6] = gen.integers(0, 2 ** 31, G)
    for R in (1, 2, 4, G):
        rt, rn, rh, rd, rc = oracle.profile_table(hist, R)
        table, n_total, n_hit, density, cbar = osc.osc_profile_table(dev(hist.view(np.int32)), R)
        assert np.array_equal(table.cpu().numpy(), rt), R
        assert np.array_equal(as_u32(n_total), rn) and np.array_equal(as_u32(n_hit), rh)
        assert np.allclose(density.cpu().numpy(), rd, rtol=1e-6, atol=0)
        assert abs(cbar.item() - rc) <= 1e-6 * rc
    empty = osc.osc_profile_table(torch.zeros((7, G), dtype=torch.int32, device="cuda"), 1)
    assert (empty[0].cpu().numpy() == -1).all() and empty[4].item() == 0.0


def test_planted_table_end_to_end(osc):
    """Calibrate on the device, turn the table into the channel list, quantise with it: the
    same bytes as the oracle's pipeline, and the planted channels are found."""
    X, planted = wl.activations_persistent(601, 1536, 2048, 1)
    Xd = bf(X)
    acc = osc.osc_profile_abs_sum(Xd)
    T = osc.osc_profile_threshold(acc, X.size, 5.0)
    hist = osc.osc_profile_hist(Xd, T)
    table, n_total, n_hit, density, cbar = osc.osc_profile_table(hist, 1)
    assert np.array_equal(table.cpu().numpy(), planted)
    assert cbar.item() > 0.95
    # the oracle fed with the device's threshold (a float) must give the same counts
    assert np.array_equal(as_u32(hist), oracle.profile_hist(X, T.item()))
    oidx = osc.osc_table_to_index(table.cpu().numpy())
    assert np.array_equal(oidx, oracle.table_to_index(planted))
    Xq, Xs, B = osc.osc_quantize_act(Xd, dev(oidx), osc.OSC_FMT_MXFP4_OSC)
    rq, rs, rb = oracle.quantize_mxfp4_osc(X, oidx, ldb=B.shape[1])
    assert np.array_equal(Xq.cpu().numpy(), rq) and np.array_equal(B.cpu().numpy().view(np.uint16), rb)


@pytest.mark.parametrize("S,H,G,R", [(1536, 4096, 32, 2), (300, 1088, 16, 1), (77, 2112, 64, 3), (5, 64, 32, 1)])
def test_calibrate_in_one_call(osc, S, H, G, R):
    """Alg. 1 through the single entry point (threshold, counts, table, densities with the
    intermediate results in a caller's workspace) against the oracle's three steps."""
    X, _ = wl.activations_persistent(9300 + S, S, H, 2, jitter=0.3) if G == 32 else (wl.activations_diffuse(9300 + S, S, H, p=0.02), None)
    ref_T = oracle.profile_threshold(X, 5.0)
    ws = torch.full((osc.osc_profile_workspace_bytes(H) + 512,), 0xA5, dtype=torch.uint8, device="cuda")
    ws = ws[:osc.osc_profile_workspace_bytes(H)]  # stale contents: the call clears what it needs
    table, n_total, n_hit, density, cbar, T = osc.osc_profile_calibrate(bf(X), G, 5.0, R, workspace=ws)
    assert abs(T.item() - ref_T) <= 1e-6 * ref_T
    rt, rn, rh, rd, rc = oracle.profile_table(oracle.profile_hist(X, T.item(), G), R)
    assert np.array_equal(table.cpu().numpy(), rt)
    assert np.array_equal(as_u32(n_total), rn.astype(np.uint32)) and np.array_equal(as_u32(n_hit), rh.astype(np.uint32))
    assert np.allclose(density.cpu().numpy(), rd, rtol=1e-6, atol=0) and abs(cbar.item() - rc) <= 1e-6
    # and equal to the four separate calls
    acc = osc.osc_profile_abs_sum(bf(X))
    T4 = osc.osc_profile_threshold(acc, S * H, 5.0)
    t4 = osc.osc_profile_table(osc.osc_profile_hist(bf(X), T4, G), R)
    assert torch.equal(t4[0], table) and torch.equal(t4[1], n_total) and torch.equal(t4[2], n_hit)
