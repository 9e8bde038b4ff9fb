"""GPU parity of the fused RMSNorm + OSC quantiser: the normalised row, the codes, the scales and
the gathered sub-tensor bit for bit against the oracle's RMSNorm followed by the oracle's quantiser."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from workloads import to_bf16_bits

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


def check(osc, X, gamma, eps, oidx, ldb=None):
    M, K = X.shape
    K_o = len(oidx)
    if ldb is None:
        ldb = (K_o + 63) // 64 * 64
    Xq, Xs, B, Xn = osc.osc_rmsnorm_quantize_act(dev(X), dev(gamma), eps, dev(oidx.astype(np.int32)) if K_o else None,
                                                 ldb=ldb, want_norm=True)
    y = oracle.rmsnorm(X, gamma, eps)
    rq, rs, rb = oracle.quantize_mxfp4_osc(y, oidx, ldb=ldb)
    assert np.array_equal(Xn.cpu().numpy(), y), "normalised rows differ"
    assert np.array_equal(osc.osc_unpack_act_scales(Xs, M, K).cpu().numpy(), rs), "scales differ"
    assert np.array_equal(Xq.cpu().numpy(), rq), "codes differ"
    if ldb:
        assert np.array_equal(B.cpu().numpy(), rb), "gathered sub-tensor differs"
    # and the fused call equals the unfused GPU path on the normalised rows
    Uq, Us, Ub = osc.osc_quantize_act(Xn, dev(oidx.astype(np.int32)) if K_o else None, ldb=ldb)
    assert torch.equal(Uq, Xq) and (not ldb or torch.equal(Ub, B))
    assert torch.equal(osc.osc_unpack_act_scales(Us, M, K), osc.osc_unpack_act_scales(Xs, M, K))


@pytest.mark.parametrize("M,K,r", [(1, 32, 1), (5, 96, 0), (33, 1056, 2), (70, 4096, 2), (300, 2048, 1),
                                   (9, 8192, 1), (6, 12288, 2)])
def test_fused_matches_oracle(osc, M, K, r):
    gen = wl.rng(1100 + M)
    X, table = wl.activations_persistent(1100 + M, M, K, r, jitter=0.3)
    gamma = to_bf16_bits((1.0 + 0.3 * gen.standard_normal(K)).astype(np.float32))
    check(osc, X, gamma, 1e-6, oracle.table_to_index(table) if r else np.zeros(0, np.int32))


def test_fused_scales_and_edges(osc):
    gen = wl.rng(1201)
    K = 256
    gamma = to_bf16_bits((0.5 + gen.random(K)).astype(np.float32))
    oidx = np.array([3, 40, 41, 100, 255], np.int32)
    # rows of very different magnitude, a zero row, a row with one non-zero, wide range inside a row
    x = gen.standard_normal((8, K)).astype(np.float32)
    x[0] *= 1e-20
    x[1] *= 1e20
    x[2] = 0.0
    x[3] = 0.0
    x[3, 40] = -7.0
    x[4, 0], x[4, 1] = 2.0 ** 90, 2.0 ** -90
    x[5] = 3.0
    X = to_bf16_bits(x)
    X[6, ::3] = 0x8000
    for eps in (1e-6, 1e-12, 1.0):
        check(osc, X, gamma, eps, oidx)
        check(osc, X, gamma, eps, oidx, ldb=8)
    # eps = 0 on rows without an all-zero row
    check(osc, X[[0, 1, 3, 4, 5, 7]], gamma, 0.0, oidx)


# ---- SwiGLU + MXFP8 quantiser ---------------------------------------------------------------
def check_swiglu(osc, G, U, strided=False):
    M, K = G.shape
    if strided:  # the two halves of one fused gate||up buffer
        both = torch.from_numpy(np.concatenate([G, U], axis=1)).cuda()
        dG, dU = both[:, :K], both[:, K:]
    else:
        dG, dU = dev(G), dev(U)
    Xq, Xs, Yn = osc.osc_swiglu_quantize_act(dG, dU, want_y=True)
    y = oracle.swiglu(G, U)
    rq, rs = oracle.quantize_mxfp8(y)
    assert np.array_equal(Yn.cpu().numpy(), y), "activation values differ"
    assert np.array_equal(osc.osc_unpack_act_scales(Xs, M, K).cpu().numpy(), rs), "scales differ"
    assert np.array_equal(Xq.cpu().numpy(), rq), "codes differ"
    # and equal to the unfused GPU quantiser on the same values
    Uq, Us = osc.osc_quantize_act(Yn, None, osc.OSC_FMT_MXFP8)
    assert torch.equal(Uq, Xq)
    assert torch.equal(osc.osc_unpack_act_scales(Us, M, K), osc.osc_unpack_act_scales(Xs, M, K))


# OSC_TUNE_SWIGLU_TABLE: "0" = silu evaluated per element, "1" = looked up in the 128 KB table in LDS (the
# launcher's own choice depends on the size); both must give the oracle's bits
@pytest.mark.parametrize("table", ["0", "1"])
@pytest.mark.parametrize("M,K", [(1, 32), (7, 96), (40, 1056), (130, 4096), (9, 12288)])
def test_swiglu_fused_matches_oracle(osc, tuning, table, M, K):
    tuning.swiglu_table(table)
    gen = wl.rng(1300 + M)
    G = to_bf16_bits((gen.standard_normal((M, K)) * 3).astype(np.float32))
    U = wl.activations_diffuse(1400 + M, M, K, p=0.01)
    check_swiglu(osc, G, U)
    check_swiglu(osc, G, U, strided=True)


@pytest.mark.parametrize("table", ["0", "1"])
def test_swiglu_every_gate_value(osc, tuning, table):
    """every bf16 bit pattern below 2^100 in magnitude as a gate (58 000 of them; above that the
    product with up leaves the bf16 range), against the oracle, bit for bit"""
    tuning.swiglu_table(table)
    bits = np.arange(0x10000, dtype=np.uint32).astype(np.uint16)
    bits = bits[((bits >> 7) & 0xFF) < 227]
    K = 2048
    pad = (-len(bits)) % K
    G = np.concatenate([bits, np.zeros(pad, np.uint16)]).reshape(-1, K)
    gen = wl.rng(1501)
    U = to_bf16_bits((0.5 + gen.random(G.shape)).astype(np.float32))
    check_swiglu(osc, G, U)


# ---- SwiGLU + per-token FP8 quantiser -------------------------------------------------------
def check_swiglu_fp8(osc, G, U, strided=False):
    M, K = G.shape
    if strided:
        both = torch.from_numpy(np.concatenate([G, U], axis=1)).cuda()
        dG, dU = both[:, :K], both[:, K:]
    else:
        dG, dU = dev(G), dev(U)
    X8, xs, Yn = osc.osc_swiglu_quantize_act_fp8(dG, dU, want_y=True)
    y = oracle.swiglu(G, U)
    r8, rsc = oracle.quantize_fp8_rows(y)
    assert np.array_equal(Yn.cpu().numpy(), y), "activation values differ"
    assert np.array_equal(xs.cpu().numpy().view(np.uint32), rsc.view(np.uint32)), "scales differ"
    assert np.array_equal(X8.cpu().numpy(), r8), "codes differ"
    U8, us = osc.osc_quantize_act(Yn, None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    assert torch.equal(U8, X8) and torch.equal(us, xs)
    X8b, xsb, none = osc.osc_swiglu_quantize_act_fp8(dG, dU)
    assert none is None and torch.equal(X8b, X8) and torch.equal(xsb, xs)


@pytest.mark.parametrize("table", ["0", "1"])
@pytest.mark.parametrize("M,K", [(1, 8), (7, 96), (40, 1056), (130, 4096), (9, 12288), (3, 16384), (5, 2056)])
def test_swiglu_fp8_fused_matches_oracle(osc, tuning, table, M, K):
    tuning.swiglu_table(table)
    gen = wl.rng(1600 + M)
    G = to_bf16_bits((gen.standard_normal((M, K)) * 3).astype(np.float32))
    U = wl.activations_diffuse(1700 + M, M, K, p=0.01)
    if M > 4:
        G[2] = 0  # an all-zero row: scale 1, codes 0
        U[3] = to_bf16_bits(np.full(K, 1e-36, np.float32))  # a row below 2^-100: scale 1
    check_swiglu_fp8(osc, G, U)
    check_swiglu_fp8(osc, G, U, strided=True)


@pytest.mark.parametrize("table", ["0", "1"])
def test_swiglu_fp8_every_gate_value(osc, tuning, table):
    tuning.swiglu_table(table)
    bits = np.arange(0x10000, dtype=np.uint32).astype(np.uint16)
    bits = bits[((bits >> 7) & 0xFF) < 227]
    K = 2048
    pad = (-len(bits)) % K
    G = np.concatenate([bits, np.zeros(pad, np.uint16)]).reshape(-1, K)
    U = to_bf16_bits((0.5 + wl.rng(1801).random(G.shape)).astype(np.float32))
    check_swiglu_fp8(osc, G, U)
