"""Pins for the oracle's 4-bit formats with scale groups of 16 channels (E8M0 per 16; NVFP4) -- CPU only.

Hand-worked blocks (golden file), a brute-force nearest-value quantiser written here in numpy with
none of the oracle's code, the relation to the 32-channel MXFP4 quantiser, torch's E4M3 codec for
the NVFP4 scale bytes, numpy matmuls on independently decoded operands, and the invariants of the
dual path."""
import os

import numpy as np
import torch

import oracle
import workloads as wl
from workloads import from_bf16_bits, to_bf16_bits

GOLD = os.path.join(os.path.dirname(__file__), "golden", "fp4_g16_group_examples.txt")
E2M1 = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])
FMT = {"e8m0": oracle.FMT16_E8M0, "nvfp4": oracle.FMT16_NVFP4}


def codes_of(Xq):
    return np.stack([Xq & 0xF, Xq >> 4], axis=-1).reshape(Xq.shape[0], -1)


def e4m3_values():
    return torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy().astype(np.float64)


def test_hand_worked_blocks():
    n = 0
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        fmt, name, ts, sbyte, prot = f[0], f[1], float(f[2]), int(f[3], 16), int(f[4])
        vals = np.array([float(v) for v in f[5::2]], np.float32)
        want = np.array([int(c, 16) for c in f[6::2]])
        assert len(vals) == 16 and len(want) == 16, name
        X = to_bf16_bits(vals)[None, :]
        assert np.array_equal(from_bf16_bits(X)[0], vals), f"{name}: a value is not a bf16 number"
        oidx = np.array([prot], np.int32) if prot >= 0 else None
        Xq, Xs, B = oracle.quantize_fp4_g16(X, oidx, fmt=FMT[fmt], tensor_scale=ts)
        assert Xs[0, 0] == sbyte, (name, hex(Xs[0, 0]))
        assert np.array_equal(codes_of(Xq)[0], want), (name, codes_of(Xq)[0])
        if prot >= 0:
            assert B[0, 0] == X[0, prot]
        n += 1
    assert n == 5


def brute_e2m1(v, neg):
    """nearest E2M1 code of |v| (float64 array), ties to the even mantissa bit, saturating; sign from `neg`"""
    a = np.abs(v)[..., None]
    d = np.abs(a - E2M1)
    best = np.zeros(v.shape, np.int64)
    bd = d[..., 0].copy()
    for c in range(1, 8):
        take = (d[..., c] < bd) | ((d[..., c] == bd) & (c % 2 == 0))
        best = np.where(take, c, best)
        bd = np.where(take, d[..., c], bd)
    best = np.where(np.abs(v) > 6.0, 7, best)
    return best | (neg.astype(np.int64) << 3)


def brute_quantize(X, oidx, fmt, ts):
    """the two formats straight from their definitions, in numpy, no oracle code"""
    x = from_bf16_bits(X).astype(np.float32).copy()
    bits = X.copy()
    if oidx is not None and len(oidx):
        x[:, oidx] = 0.0
        bits[:, oidx] = 0
    neg = (bits >> 15).astype(bool)
    M, K = x.shape
    xb = x.reshape(M, K // 16, 16)
    amax = np.abs(xb).max(axis=2)
    if fmt == oracle.FMT16_E8M0:
        with np.errstate(divide="ignore"):
            e = np.where(amax > 0, np.floor(np.log2(amax.astype(np.float64))) - 2, -127).astype(np.int64)
        e = np.clip(e, -127, 127)
        v = xb.astype(np.float64) / np.exp2(e.astype(np.float64))[..., None]
        return brute_e2m1(v, neg.reshape(M, K // 16, 16)).reshape(M, K), (e + 127).astype(np.uint8)
    ts = np.float32(ts)
    d = np.float32(6.0) * ts
    q = (amax / d).astype(np.float32)
    sc = torch.from_numpy(np.minimum(q, np.float32(448.0))).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    s = e4m3_values()[sc].astype(np.float32)
    with np.errstate(divide="ignore", invalid="ignore", over="ignore"):
        inv = (np.float32(1.0) / (ts * s).astype(np.float32)).astype(np.float32)
        w = (xb * inv[..., None]).astype(np.float32)
    codes = brute_e2m1(np.where(np.isfinite(w), w, 7.0).astype(np.float64), neg.reshape(M, K // 16, 16))
    codes = np.where((s == 0)[..., None], neg.reshape(M, K // 16, 16).astype(np.int64) << 3, codes)
    return codes.reshape(M, K), sc


def test_bruteforce_both_formats():
    for seed, M, K, r in ((11, 9, 256, 2), (12, 4, 1024, 1), (13, 33, 64, 0)):
        X, table = wl.activations_persistent(seed, M, K, r) if r else (wl.activations_diffuse(seed, M, K, p=0.05), None)
        oidx = oracle.table_to_index(table) if r else None
        # rough values too: tiny blocks, zero blocks, bf16 subnormals
        X[0, :16] = 0
        X[0, 16:32] = to_bf16_bits(np.full(16, 2.0 ** -20, np.float32))
        X[M - 1, 32:48] = np.arange(1, 17, dtype=np.uint16)  # subnormals
        for fmt, ts in ((oracle.FMT16_E8M0, 1.0), (oracle.FMT16_NVFP4, 1 / 64), (oracle.FMT16_NVFP4, 0.0123)):
            Xq, Xs, _ = oracle.quantize_fp4_g16(X, oidx, fmt=fmt, tensor_scale=ts)
            bc, bs = brute_quantize(X, oidx, fmt, ts)
            assert np.array_equal(Xs, bs), (seed, fmt, ts)
            assert np.array_equal(codes_of(Xq), bc), (seed, fmt, ts)


def test_relation_to_blocks_of_32():
    """E8M0 per 16: the code of a 32-channel MXFP4 block is the larger of its two 16-channel codes, and
    where the two agree the element codes are those of the MXFP4 quantiser."""
    X, table = wl.activations_persistent(21, 16, 512, 2)
    oidx = oracle.table_to_index(table)
    q16, s16, b16 = oracle.quantize_fp4_g16(X, oidx, fmt=oracle.FMT16_E8M0)
    q32, s32, b32 = oracle.quantize_mxfp4_osc(X, oidx)
    assert np.array_equal(b16, b32)
    pair = s16.reshape(16, -1, 2)
    assert np.array_equal(pair.max(axis=2), s32)
    same = np.repeat(pair[..., 0] == pair[..., 1], 32, axis=1)
    assert same.any() and (~same).any()
    assert np.array_equal(codes_of(q16)[same], codes_of(q32)[same])
    assert (s16 <= np.repeat(s32, 2, axis=1)).all()


def decode(codes_q, scales, fmt, ts):
    c = codes_of(codes_q)
    v = E2M1[c & 7] * np.where(c & 8, -1.0, 1.0)
    s = np.exp2(scales.astype(np.float64) - 127) if fmt == oracle.FMT16_E8M0 else e4m3_values()[scales]
    return v * np.repeat(s, 16, axis=1) * (1.0 if fmt == oracle.FMT16_E8M0 else float(np.float32(ts)))


def test_gemm_against_numpy_on_decoded_operands_and_invariants():
    M, N, K, r = 12, 20, 256, 2
    X, table = wl.activations_persistent(31, M, K, r)
    W = wl.weights(32, N, K)
    oidx = oracle.table_to_index(table)
    for fmt, xts, wts in ((oracle.FMT16_E8M0, 1.0, 1.0), (oracle.FMT16_NVFP4, 0.02, 0.0005)):
        Xq, Xs, B = oracle.quantize_fp4_g16(X, oidx, fmt=fmt, tensor_scale=xts)
        Wq, Ws, _ = oracle.quantize_fp4_g16(W, None, fmt=fmt, tensor_scale=wts)
        WL = oracle.gather_wl(W, oidx)
        Y = oracle.dual_gemm_g16(Xq, Xs, B, Wq, Ws, WL, fmt, xts, wts)
        ref = decode(Xq, Xs, fmt, xts) @ decode(Wq, Ws, fmt, wts).T + \
            from_bf16_bits(B).astype(np.float64) @ from_bf16_bits(WL).astype(np.float64)
        assert np.allclose(Y, ref, rtol=1e-12, atol=1e-12 * np.abs(ref).max())
        # the layer is close to the exact product (the format works), and OSC beats the same format without protection
        exact = from_bf16_bits(X).astype(np.float64) @ from_bf16_bits(W).astype(np.float64).T
        Xq0, Xs0, _ = oracle.quantize_fp4_g16(X, None, fmt=fmt, tensor_scale=xts * 40)
        Y0 = oracle.dual_gemm_g16(Xq0, Xs0, None, Wq, Ws, None, fmt, xts * 40, wts)
        assert np.abs(Y - exact).mean() < 0.5 * np.abs(Y0 - exact).mean()
        # empty table = the plain format; every channel protected = the bf16 GEMM
        Ye = oracle.dual_gemm_g16(*oracle.quantize_fp4_g16(X, None, fmt=fmt, tensor_scale=xts)[:2], None, Wq, Ws, None, fmt, xts, wts)
        assert np.allclose(Ye, decode(*oracle.quantize_fp4_g16(X, None, fmt=fmt, tensor_scale=xts)[:2], fmt, xts) @ decode(Wq, Ws, fmt, wts).T,
                           rtol=1e-12, atol=1e-12)
        allc = np.arange(K, dtype=np.int32)
        Xqa, Xsa, Ba = oracle.quantize_fp4_g16(X, allc, fmt=fmt, tensor_scale=xts)
        assert (codes_of(Xqa) == 0).all() and np.array_equal(Ba, X)
        Ya = oracle.dual_gemm_g16(Xqa, Xsa, Ba, Wq, Ws, oracle.gather_wl(W, allc), fmt, xts, wts)
        assert np.allclose(Ya, exact, rtol=1e-12, atol=1e-12)


def test_nvfp4_exact_on_the_grid():
    """values that are E2M1 x E4M3 x ts products with the block maximum at 6 x scale are reproduced exactly"""
    ts = np.float32(2.0 ** -7)
    gen = wl.rng(41)
    svals = e4m3_values()[[0x38, 0x45, 0x60, 0x2A]]        # four positive scales
    codes = gen.integers(0, 16, (4, 16))
    codes[:, 0] = 7                                          # the block's maximum sits at 6 x scale
    x = (E2M1[codes & 7] * np.where(codes & 8, -1.0, 1.0)) * svals[:, None] * float(ts)
    X = to_bf16_bits(x.reshape(1, 64).astype(np.float32))
    assert np.array_equal(from_bf16_bits(X).astype(np.float64), x.reshape(1, 64))
    Xq, Xs, _ = oracle.quantize_fp4_g16(X, None, fmt=oracle.FMT16_NVFP4, tensor_scale=ts)
    assert np.array_equal(decode(Xq, Xs, oracle.FMT16_NVFP4, ts), x.reshape(1, 64))
