#!/usr/bin/env python3
"""Benchmark of the OSC dual-path linear layer on one MI355X.

One step = the whole hot path of one Qwen3-8B attention block's linear layers at M tokens
(benchmark configuration 1, "configs[1]"): quantise+gather the attention input, dual-path GEMMs q (4096->4096),
k and v (4096->1024) on it, quantise+gather the o-projection input, dual-path GEMM o
(4096->4096).  Inputs are synthetic (seeded N(0,1) with two token-persistent outlier channels
per 32-group), resident in HBM before the timed region.  The same GEMM shapes are also run
through the library's own FP8 W8A8 path for the speed-up figure.

Prints one JSON line.  `value` = sum over the four GEMMs of 2*M*N*K, divided by the time of a
whole step (quantisers included).  Besides the headline, the line carries one object per widened
row of the path and, under "shapes", every GEMM shape of the five benchmark configurations, each
built from the seeded generators of `workloads`, with the FP8 W8A8 time of the same shape measured
in the same alternating loop.
"""
import argparse
import json
import os
import re
import sys
import time
import zlib

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MXFP4_TFLOPS = 10066.0  # MI355X dense MXFP4 matrix peak
PEAK_FP8_TFLOPS = 5033.0
PEAK_HBM_GBS = 8000.0
K_HID = 4096
PROJ = (("q", 4096), ("k", 1024), ("v", 1024), ("o", 4096))
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "dual_gemm_8192x4096x4096__hbm_traffic.txt")


def profile_figure(fname, key):
    """A figure from a tracked rocprofv3 summary under profiles/ (`KEY = value` on a line of its own): a
    profiler reading that this script cannot take itself.  None when the summary or the line is absent."""
    try:
        m = re.search(r"^" + key + r"\s*=\s*([0-9.eE+]+)", open(os.path.join(ROOT, "profiles", fname)).read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def dominant_traffic_bytes():
    """Bytes between L2 and the fabric per launch of the dominant kernel, from the tracked rocprofv3
    FETCH_SIZE / WRITE_SIZE summary (a profiler reading: this script cannot measure it itself).
    None when the summary is absent."""
    try:
        m = re.search(r"^TRAFFIC_BYTES_PER_LAUNCH\s*=\s*([0-9.eE+]+)", open(TRAFFIC_FILE).read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def cpu_baseline(rows=1280):
    """The oracle, as it stands, on a bounded sample of the same workload: `rows` tokens through
    the quantiser and the q projection.  Reported baseline only."""
    import oracle
    import workloads as wl
    c = wl.config2_attn(rows, 4096)
    oidx = oracle.table_to_index(c["table"])
    Wq, Ws, _ = oracle.quantize_mxfp4_osc(c["W"])
    WL = oracle.gather_wl(c["W"], oidx)
    t0 = time.perf_counter()
    Xq, Xs, B = oracle.quantize_mxfp4_osc(c["X"], oidx)
    oracle.dual_gemm(Xq, Xs, B, Wq, Ws, WL)
    dt = time.perf_counter() - t0
    flops = 2.0 * rows * 4096 * K_HID
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"extrapolated from {rows} of the 8192 tokens of configs[1]: quantise+gather, then the q "
                      f"projection (N=4096, K=4096, K_o=256) in {dt:.2f} s; as for `value`, the flops are the "
                      "GEMM's 2MNK and the time includes the quantiser"}


class Bench:
    """Timing helpers.  Every timed section starts with a few tens of milliseconds of GEMM work so that
    the clock is where sustained load puts it, and two things that are compared are timed in
    alternating blocks of the same loop."""

    def __init__(self, torch, osc, wl):
        self.torch, self.osc, self.wl = torch, osc, wl
        self.dev = torch.device("cuda:0")
        self._burn = None

    def up(self, a):
        return self.torch.from_numpy(np.ascontiguousarray(a)).to(self.dev)

    def ev(self):
        return self.torch.cuda.Event(enable_timing=True)

    def set_burn(self, fn, ms_each):
        self._burn = (fn, max(1, int(30.0 / max(ms_each, 1e-3))))

    def burn(self):
        if self._burn:
            fn, n = self._burn
            for _ in range(n):
                fn()

    def time_many(self, fns, reps=10, rounds=5):
        """median over `rounds` of the time of `reps` launches of each function, blocks alternating"""
        torch = self.torch
        for f in fns:
            f()
        self.burn()
        acc = [[] for _ in fns]
        for _ in range(rounds):
            evs = [self.ev() for _ in range(len(fns) + 1)]
            evs[0].record()
            for i, f in enumerate(fns):
                for _ in range(reps):
                    f()
                evs[i + 1].record()
            torch.cuda.synchronize()
            for i in range(len(fns)):
                acc[i].append(evs[i].elapsed_time(evs[i + 1]) / reps)
        return [float(np.median(a)) for a in acc]

    def time_one(self, fn, reps=10, rounds=5):
        return self.time_many([fn], reps, rounds)[0]

    def graph_many(self, fns, n=48, rounds=5):
        """The same for kernels of a few microseconds, which one launch from Python outlasts: every
        function is called n times (with the call number as its argument) inside one captured HIP graph
        and the replays are timed, alternating."""
        torch = self.torch
        graphs = []
        for f in fns:
            for i in range(n):
                f(i)
            torch.cuda.synchronize()
            side = torch.cuda.Stream()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                with torch.cuda.graph(g, stream=side):
                    for i in range(n):
                        f(i)
            torch.cuda.synchronize()
            g.replay()
            graphs.append(g)
        return [t / n for t in self.time_many([g.replay for g in graphs], reps=3, rounds=rounds)], graphs

    def host_us_per_call(self, fn, n=200):
        """wall-clock microseconds of one call through the Python binding (enqueue only)"""
        torch = self.torch
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        dt = time.perf_counter() - t0
        torch.cuda.synchronize()
        return dt / n * 1e6


def hbm(bytes_, ms):
    gbs = bytes_ / (ms * 1e-3) / 1e9
    return {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": round(gbs / PEAK_HBM_GBS, 4)}


def dual_weight_bytes(N, K, K_o):
    return N * (K // 2 + K // 32) + N * ((K_o + 63) // 64 * 64) * 2


def gemm_row(M, N, K, r, K_o, ms_osc, ms_f8, decode, cold):
    """One row of the shapes table: times, speed-up beside the model value, and the roofline that bounds
    the launch (matrix rate from about 400 rows on, weight bytes below: 10.07 PFLOP/s over 8 TB/s)."""
    row = {"M": M, "N": N, "K": K, "r": r, "K_o": K_o, "osc_ms": round(ms_osc, 4), "fp8_ms": round(ms_f8, 4),
           "speedup": round(ms_f8 / ms_osc, 3)}
    if decode:
        act = M * (K // 2 + K // 32 + ((K_o + 63) // 64 * 64) * 2) + M * N * 2
        by = dual_weight_bytes(N, K, K_o) + act
        row["roofline"] = hbm(by, ms_osc)
        row["roofline"]["weights"] = "rotated through copies larger than the last-level cache" if cold else "cache-warm"
        row["model_speedup"] = round((N * K + M * K) / (dual_weight_bytes(N, K, K_o) + M * (K // 2 + K // 32 + K_o * 2)), 3)
    else:
        tf = 2.0 * M * N * K / (ms_osc * 1e-3) / 1e12
        row["roofline"] = {"bound": "mfma", "achieved": round(tf, 1), "peak": PEAK_MXFP4_TFLOPS, "unit": "TFLOP/s",
                           "frac": round(tf / PEAK_MXFP4_TFLOPS, 4)}
        row["fp8_frac_of_fp8_peak"] = round(2.0 * M * N * K / (ms_f8 * 1e-3) / 1e12 / PEAK_FP8_TFLOPS, 4)
        row["model_speedup"] = round(2 / (1 + 4 * r / 32), 3)
    if row["speedup"] > row["model_speedup"] * 1.02:
        row["above_model"] = True  # more than the throughput ratio allows: the FP8 side is further from its roofline
    return row


def shapes_table(b, quick=False, only=None):
    """Every GEMM shape of benchmark configurations 1-4 ("configs[1..4]" of the task), inputs from the seeded
    generators, dual path against the library's FP8 W8A8 GEMM on the same X and W, bf16 output."""
    torch, osc, wl = b.torch, b.osc, b.wl
    ydt = osc.OSC_DT_BF16
    rows = {}

    cache = {}

    def packs_for(key, dW, oidx, K_o, N, K, decode, cold):
        """packed weights of one (weight, table) pair, kept while consecutive rows use the same pair"""
        if cache.get("key") != (key, decode):
            cache.clear()
            cache["key"] = (key, decode)
            if decode:
                # weights larger than the 256 MB last-level cache in total, taken in turn, so that every
                # launch streams its weights from HBM as a decode step of a whole model would
                n4 = max(2, -(-(320 << 20) // osc.osc_packed_weight_bytes(N, K, K_o))) if cold else 1
                n8 = max(2, -(-(320 << 20) // osc.osc_packed_weight_fp8_bytes(N, K))) if cold else 1
                cache["p4"] = [osc.osc_pack_weight(dW, oidx) for _ in range(n4)]
                cache["p8"] = [osc.osc_pack_weight_fp8(dW) for _ in range(n8)]
            else:
                cache["p4"], cache["p8"] = [osc.osc_pack_weight(dW, oidx)], [osc.osc_pack_weight_fp8(dW)]
        return cache["p4"], cache["p8"]

    def one(tag, X, table, W, r, wkey, cold_decode=True):
        M, K = X.shape
        N = W.shape[0]
        dX = b.up(X)
        oidx = b.up(osc.osc_table_to_index(table)) if r else None
        K_o = 0 if oidx is None else int(oidx.numel())
        q = osc.osc_quantize_act(dX, oidx)
        q8 = osc.osc_quantize_act(dX, None, osc.OSC_FMT_FP8_E4M3_TOKEN)
        Y = torch.empty((M, N), dtype=torch.bfloat16, device=b.dev)
        decode = M <= 128
        if cache.get("key") != ((wkey, r), decode):
            cache.clear()
        Wp, W8 = packs_for((wkey, r), None if cache.get("key") == ((wkey, r), decode) else b.up(W), oidx, K_o, N, K,
                           decode, cold_decode)
        if decode:
            n4, n8 = len(Wp), len(W8)
            (ms, ms8), graphs = b.graph_many(
                [lambda i: osc.osc_dual_gemm(*q, Wp[i % n4], N, K, K_o, ydt, out=Y),
                 lambda i: osc.osc_fp8_gemm(*q8, W8[i % n8], N, K, y_dtype=ydt, out=Y)])
            row = gemm_row(M, N, K, r, K_o, ms, ms8, True, cold_decode)
            row["host_us_per_call"] = round(b.host_us_per_call(lambda: osc.osc_dual_gemm(*q, Wp[0], N, K, K_o, ydt, out=Y)), 1)
            row["timing"] = "48 launches in one HIP graph"
            del graphs
        else:
            reps = 4 if M * N >= (1 << 27) else 10
            ms, ms8 = b.time_many([lambda: osc.osc_dual_gemm(*q, Wp[0], N, K, K_o, ydt, out=Y),
                                   lambda: osc.osc_fp8_gemm(*q8, W8[0], N, K, y_dtype=ydt, out=Y)], reps=reps)
            row = gemm_row(M, N, K, r, K_o, ms, ms8, False, False)
        rows[tag] = row

    if only == "cfg3":
        X, table = wl.activations_persistent(3001, 8192, K_HID, 2)
        one("cfg3 W1|W3 M=8192 N=24576", X, table, wl.weights(3002, 24576, K_HID), 2, "cfg3")
        return rows
    # configs[1]: attention projections
    Wn = {4096: wl.weights(2100, 4096, K_HID), 1024: wl.weights(2101, 1024, K_HID)}
    for N in (4096, 1024):
        for M in (1, 16, 128, 2048, 8192):
            X, table = wl.activations_persistent(2001, M, K_HID, 2)
            one(f"cfg2 M={M} N={N}", X, table, Wn[N], 2, f"cfg2-{N}")
    # fused q|k|v (one packed weight of 6144 rows, one launch) at the step's token count
    X, table = wl.activations_persistent(2001, 8192, K_HID, 2)
    Wqkv = np.concatenate([wl.weights(2100 + i, N, K_HID) for i, N in enumerate((4096, 1024, 1024))])
    one("cfg2 M=8192 N=6144 (q|k|v fused)", X, table, Wqkv, 2, "cfg2-qkv")
    del Wqkv
    # configs[2]: fused W1|W3
    if not quick:
        X, table = wl.activations_persistent(3001, 8192, K_HID, 2)
        one("cfg3 W1|W3 M=8192 N=24576", X, table, wl.weights(3002, 24576, K_HID), 2, "cfg3")
    # configs[4]: density / decode sweep
    W5 = wl.weights(5101, 12288, K_HID)
    for r in (0, 1, 2, 4):
        for M in (1, 8, 32, 64, 512, 4096):
            if quick and M not in (64, 4096):
                continue
            X, table = wl.activations_persistent(5001 + r, M, K_HID, r, factor=64.0)
            one(f"cfg5 r={r} M={M}", X, table, W5, r, "cfg5")
    del W5
    cache.clear()
    return rows


def moe_rows(b):
    """configs[3]: Qwen3-30B-A3B expert layer, 4096 tokens routed top-8 over 128 experts."""
    torch, osc, wl = b.torch, b.osc, b.wl
    ydt = osc.OSC_DT_BF16
    tokens, K, E, topk, N = 4096, 2048, 128, 8, 1536
    X, table = wl.activations_persistent(4001, tokens, K, 2)
    oidx = b.up(osc.osc_table_to_index(table))
    K_o = int(oidx.numel())
    q = osc.osc_quantize_act(b.up(X), oidx)
    off, row_map = wl.moe_routing(4002, tokens, E, topk)
    T = int(off[-1])
    d_off, d_map = b.up(off), b.up(row_map)
    stride, stride8 = osc.osc_packed_weight_bytes(N, K, K_o), osc.osc_packed_weight_fp8_bytes(N, K)
    Wp = torch.empty(E * stride, dtype=torch.uint8, device=b.dev)
    Wp8 = torch.empty(E * stride8, dtype=torch.uint8, device=b.dev)
    for e in range(E):
        W = b.up(wl.weights(4100 + e, N, K))
        osc.osc_pack_weight(W, oidx, out=Wp[e * stride:(e + 1) * stride])
        osc.osc_pack_weight_fp8(W, out=Wp8[e * stride8:(e + 1) * stride8])
    # the W8A8 form of the same layer: gathered rows quantised per token
    Xg = b.up(X[row_map])
    q8 = osc.osc_quantize_act(Xg, None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    Y = torch.empty((T, N), dtype=torch.bfloat16, device=b.dev)
    ms, ms8 = b.time_many([lambda: osc.osc_grouped_dual_gemm(*q, d_map, d_off, T, Wp, N, K, K_o, ydt, out=Y),
                           lambda: osc.osc_fp8_gemm(*q8, Wp8, N, K, expert_offsets=d_off, y_dtype=ydt, out=Y)], reps=6)
    by = E * stride + tokens * (K // 2 + K // 32 + 2 * K_o) + T * N * 2
    tf = 2.0 * T * N * K / (ms * 1e-3) / 1e12
    out = {"W1|W3 grouped dual": {
        "T": T, "E": E, "N": N, "K": K, "K_o": K_o, "osc_ms": round(ms, 4), "fp8_ms": round(ms8, 4),
        "speedup": round(ms8 / ms, 3), "model_speedup": 1.6,
        "roofline_mfma": {"bound": "mfma", "achieved": round(tf, 1), "peak": PEAK_MXFP4_TFLOPS, "unit": "TFLOP/s",
                          "frac": round(tf / PEAK_MXFP4_TFLOPS, 4)},
        "roofline_hbm": hbm(by, ms), "bytes": by}}
    del Wp, Wp8, Xg, q8, Y
    K2, N2 = 768, 2048
    X2 = b.up(wl.activations_diffuse(4003, T, K2))
    f8 = osc.osc_quantize_act(X2, None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    m8 = osc.osc_quantize_act(X2, None, osc.OSC_FMT_MXFP8)
    s8, sm = osc.osc_packed_weight_fp8_bytes(N2, K2), osc.osc_packed_weight_mxfp8_bytes(N2, K2)
    W8 = torch.empty(E * s8, dtype=torch.uint8, device=b.dev)
    Wm = torch.empty(E * sm, dtype=torch.uint8, device=b.dev)
    for e in range(E):
        W = b.up(wl.weights(4300 + e, N2, K2))
        osc.osc_pack_weight_fp8(W, out=W8[e * s8:(e + 1) * s8])
        osc.osc_pack_weight_mxfp8(W, out=Wm[e * sm:(e + 1) * sm])
    Y2 = torch.empty((T, N2), dtype=torch.bfloat16, device=b.dev)
    t8, tm = b.time_many([lambda: osc.osc_fp8_gemm(*f8, W8, N2, K2, expert_offsets=d_off, y_dtype=ydt, out=Y2),
                          lambda: osc.osc_mxfp8_gemm(*m8, Wm, N2, K2, expert_offsets=d_off, y_dtype=ydt, out=Y2)], reps=6)
    by2 = E * N2 * K2 + T * K2 + T * N2 * 2
    for name, t in (("W2 grouped fp8", t8), ("W2 grouped mxfp8", tm)):
        tf2 = 2.0 * T * N2 * K2 / (t * 1e-3) / 1e12
        out[name] = {"T": T, "E": E, "N": N2, "K": K2, "ms": round(t, 4),
                     "roofline_mfma": {"bound": "mfma", "achieved": round(tf2, 1), "peak": PEAK_FP8_TFLOPS,
                                       "unit": "TFLOP/s", "frac": round(tf2 / PEAK_FP8_TFLOPS, 4)},
                     "roofline_hbm": hbm(by2, t), "bytes": by2}
    return out


def streaming_rows(b, M=8192):
    """The HBM-side kernels once more on their bench shapes, for profiler runs: every quantiser, the producer
    fusions and the offline profiling kernels, each a few launches over a ring of inputs (event times in ms)."""
    torch, osc, wl = b.torch, b.osc, b.wl
    K, K_FF = K_HID, 12288
    X, table = wl.activations_persistent(2001, M, K, 2)
    oidx = b.up(osc.osc_table_to_index(table))
    ring = [b.up(X) for _ in range(5)]
    gam = b.up(wl.to_bf16_bits((1.0 + 0.1 * wl.rng(2200).standard_normal(K)).astype(np.float32)))
    q = osc.osc_quantize_act(ring[0], oidx)
    q64 = osc.osc_quantize_act(ring[0], oidx, osc.OSC_FMT_MXFP4_OSC_G64)
    f8 = osc.osc_quantize_act(ring[0], None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    dq = osc.osc_quantize_act_dynamic(ring[0], want_idx=True)
    g16 = [osc.osc_quantize_act_g16(ring[0], oidx, f, 1.0 / 64 if f == osc.OSC_FMT16_NVFP4 else 1.0)
           for f in (osc.OSC_FMT16_E8M0, osc.OSC_FMT16_NVFP4)]
    acc = torch.zeros(1, dtype=torch.float64, device=b.dev)
    T = osc.osc_profile_threshold(osc.osc_profile_abs_sum(ring[0]), M * K, 5.0)
    hist = torch.zeros((K // 32, 32), dtype=torch.int32, device=b.dev)
    turn = [0]

    def nxt():
        turn[0] = (turn[0] + 1) % len(ring)
        return ring[turn[0]]

    res = {}
    names = ["quant_mxfp4_osc", "quant_mxfp4_osc_g64", "quant_fp8_token", "quant_mxfp4_dynamic", "rmsnorm_quant_mxfp4",
             "quant_fp4_g16_e8m0", "quant_fp4_g16_nvfp4", "profile_abs_sum", "profile_hist"]
    fns = [lambda: osc.osc_quantize_act(nxt(), oidx, out=q),
           lambda: osc.osc_quantize_act(nxt(), oidx, osc.OSC_FMT_MXFP4_OSC_G64, out=q64),
           lambda: osc.osc_quantize_act(nxt(), None, osc.OSC_FMT_FP8_E4M3_TOKEN, out=f8),
           lambda: osc.osc_quantize_act_dynamic(nxt(), out=dq),
           lambda: osc.osc_rmsnorm_quantize_act(nxt(), gam, 1e-6, oidx, out=(q[0], q[1], q[2], None)),
           lambda: osc.osc_quantize_act_g16(nxt(), oidx, osc.OSC_FMT16_E8M0, 1.0, out=g16[0]),
           lambda: osc.osc_quantize_act_g16(nxt(), oidx, osc.OSC_FMT16_NVFP4, 1.0 / 64, out=g16[1]),
           lambda: osc.osc_profile_abs_sum(nxt(), acc),
           lambda: osc.osc_profile_hist(nxt(), T, 32, hist)]
    for n, t in zip(names, b.time_many(fns, reps=2 * len(ring))):
        res[n + f" {M}x{K}"] = round(t, 4)
    del ring, q, q64, f8, dq, g16
    Xf = b.up(wl.activations_diffuse(3003, M, K_FF))
    m8 = osc.osc_quantize_act(Xf, None, osc.OSC_FMT_MXFP8)
    t8 = osc.osc_quantize_act(Xf, None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    gen = torch.Generator(device=b.dev)
    gen.manual_seed(3005)
    gu = (torch.randn((M, 2 * K_FF), generator=gen, device=b.dev) * 2).to(torch.bfloat16).view(torch.uint16)
    names = ["quant_mxfp8", "quant_fp8_token", "swiglu_quant_mxfp8", "swiglu_quant_fp8"]
    fns = [lambda: osc.osc_quantize_act(Xf, None, osc.OSC_FMT_MXFP8, out=m8),
           lambda: osc.osc_quantize_act(Xf, None, osc.OSC_FMT_FP8_E4M3_TOKEN, out=t8),
           lambda: osc.osc_swiglu_quantize_act(gu[:, :K_FF], gu[:, K_FF:], out=(m8[0], m8[1], None)),
           lambda: osc.osc_swiglu_quantize_act_fp8(gu[:, :K_FF], gu[:, K_FF:], out=(t8[0], t8[1], None))]
    for n, t in zip(names, b.time_many(fns, reps=5)):
        res[n + f" {M}x{K_FF}"] = round(t, 4)
    return res


def vendor_library_yardstick(b, M, N, K):
    """What the GEMM library that ships with the framework reaches on the dominant shape (plain MXFP4 with
    unit scales, FP8 with one scale per tensor; random codes).  Context beside the peaks, not part of the
    path and not a target; null where this build of the framework has no such kernel."""
    torch = b.torch
    res = {}

    def t(fn):
        try:
            fn()
            return round(b.time_one(fn, reps=5), 4)
        except Exception:  # noqa: BLE001  (any refusal of the library means "not available")
            return None
    try:
        a4 = torch.randint(0, 256, (M, K // 2), device=b.dev, dtype=torch.uint8).view(torch.float4_e2m1fn_x2)
        b4 = torch.randint(0, 256, (N, K // 2), device=b.dev, dtype=torch.uint8).view(torch.float4_e2m1fn_x2)
        sa = torch.full((M, K // 32), 127, device=b.dev, dtype=torch.uint8).view(torch.float8_e8m0fnu)
        sb = torch.full((N, K // 32), 127, device=b.dev, dtype=torch.uint8).view(torch.float8_e8m0fnu)
        res["mxfp4_ms"] = t(lambda: torch._scaled_mm(a4, b4.t(), scale_a=sa, scale_b=sb, out_dtype=torch.bfloat16))
    except Exception:  # noqa: BLE001
        res["mxfp4_ms"] = None
    try:
        a8 = torch.randn((M, K), device=b.dev).to(torch.float8_e4m3fn)
        b8 = torch.randn((N, K), device=b.dev).to(torch.float8_e4m3fn)
        one = torch.ones((), device=b.dev)
        res["fp8_per_tensor_ms"] = t(lambda: torch._scaled_mm(a8, b8.t(), scale_a=one, scale_b=one, out_dtype=torch.bfloat16))
    except Exception:  # noqa: BLE001
        res["fp8_per_tensor_ms"] = None
    for k in list(res):
        if res[k]:
            res[k.replace("_ms", "_tflops")] = round(2.0 * M * N * K / (res[k] * 1e-3) / 1e12, 1)
    res["note"] = f"torch._scaled_mm at {M}x{N}x{K}, bf16 out: the framework's bundled GEMM library, timed like the kernels above"
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--tokens", type=int, default=8192)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--quick", action="store_true", help="skip most rows of the shapes table (profiler runs)")
    ap.add_argument("--only-step", action="store_true", help="the headline step only (profiler runs)")
    ap.add_argument("--section", choices=["cfg3", "moe", "streaming"], default=None,
                    help="profiler runs: only the launches of configs[2] (W1|W3 dual GEMM, W_2 FP8 and MXFP8 GEMMs), "
                         "of configs[3] (grouped GEMMs), or of the streaming kernels (quantisers, producer fusions, "
                         "offline profiling) at their bench shapes, a few times each")
    ap.add_argument("--detail", action="store_true", help="per-kernel times on stderr")
    ap.add_argument("--copy-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (a counter yardstick for profiler runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")

    import torch
    import paper_2604_12782_amd as osc
    from paper_2604_12782_amd import probe as osc_probe
    import workloads as wl
    osc.lib()
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    M = args.tokens
    b = Bench(torch, osc, wl)
    dev, up, ev = b.dev, b.up, b.ev
    if args.copy_mib:
        src = torch.zeros(args.copy_mib << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.section == "moe":
        print(json.dumps({"shapes_moe": moe_rows(b)}))
        return
    if args.section == "streaming":
        print(json.dumps({"streaming": streaming_rows(b)}))
        return
    if args.section == "cfg3":
        res = {"shapes": shapes_table(b, only="cfg3")}
        Xf = up(wl.activations_diffuse(3003, 8192, 12288))
        Wf = up(wl.weights(3004, 4096, 12288))
        wm8, wf8 = osc.osc_pack_weight_mxfp8(Wf), osc.osc_pack_weight_fp8(Wf)
        m8 = osc.osc_quantize_act(Xf, None, osc.OSC_FMT_MXFP8)
        t8 = osc.osc_quantize_act(Xf, None, osc.OSC_FMT_FP8_E4M3_TOKEN)
        Yf = torch.empty((8192, 4096), dtype=torch.bfloat16, device=dev)
        a8, a4 = b.time_many([lambda: osc.osc_mxfp8_gemm(*m8, wm8, 4096, 12288, y_dtype=osc.OSC_DT_BF16, out=Yf),
                              lambda: osc.osc_fp8_gemm(*t8, wf8, 4096, 12288, y_dtype=osc.OSC_DT_BF16, out=Yf)], reps=5)
        res["w2"] = {"mxfp8_gemm_ms": round(a8, 4), "fp8_gemm_ms": round(a4, 4)}
        print(json.dumps(res))
        return

    # ---- inputs (seeded, built on the CPU, uploaded once) -----------------------------------
    X1, table1 = wl.activations_persistent(2001, M, K_HID, 2)
    X2, table2 = wl.activations_persistent(2002, M, K_HID, 2)
    crcs = {"X1": zlib.crc32(X1.tobytes()), "X2": zlib.crc32(X2.tobytes()),
            "table1": zlib.crc32(np.ascontiguousarray(table1).tobytes())}
    oidx1 = up(osc.osc_table_to_index(table1))
    oidx2 = up(osc.osc_table_to_index(table2))
    K_o = int(oidx1.numel())
    dX1, dX2 = up(X1), up(X2)
    packs, packs8 = {}, {}
    for name, N in PROJ:
        Wh = wl.weights(2100 + len(packs), N, K_HID)
        crcs["W_" + name] = zlib.crc32(Wh.tobytes())
        W = up(Wh)
        packs[name] = osc.osc_pack_weight(W, oidx2 if name == "o" else oidx1)
        packs8[name] = osc.osc_pack_weight_fp8(W)
        del W
    ydt = osc.OSC_DT_BF16
    q1 = osc.osc_quantize_act(dX1, oidx1)
    q2 = osc.osc_quantize_act(dX2, oidx2)
    f1 = osc.osc_quantize_act(dX1, None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    f2 = osc.osc_quantize_act(dX2, None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    Y = {n: torch.empty((M, N), dtype=torch.bfloat16, device=dev) for n, N in PROJ}
    def step(events=None):
        osc.osc_quantize_act(dX1, oidx1, out=q1)
        for n, N in PROJ[:3]:
            if events is not None and n == "q":
                e0, e1 = ev(), ev()
                e0.record()
            osc.osc_dual_gemm(*q1, packs[n], N, K_HID, K_o, ydt, out=Y[n])
            if events is not None and n == "q":
                e1.record()
                events.append((e0, e1))
        osc.osc_quantize_act(dX2, oidx2, out=q2)
        osc.osc_dual_gemm(*q2, packs["o"], 4096, K_HID, K_o, ydt, out=Y["o"])

    def step_fp8():
        osc.osc_quantize_act(dX1, None, osc.OSC_FMT_FP8_E4M3_TOKEN, out=f1)
        for n, N in PROJ[:3]:
            osc.osc_fp8_gemm(*f1, packs8[n], N, K_HID, y_dtype=ydt, out=Y[n])
        osc.osc_quantize_act(dX2, None, osc.OSC_FMT_FP8_E4M3_TOKEN, out=f2)
        osc.osc_fp8_gemm(*f2, packs8["o"], 4096, K_HID, y_dtype=ydt, out=Y["o"])

    def timed_loop(fn, steps, warmup):
        # the clock needs tens of milliseconds of load to settle where sustained work puts it: a fixed
        # 40 ms of the same step first, then the W warm-up steps, then exactly K timed steps
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < 0.040:
            for _ in range(8):
                fn()
            torch.cuda.synchronize()
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    ms_step = timed_loop(step, args.steps, args.warmup)
    # The dominant kernel (the q projection): HIP events on the launch stream around batches of K launches
    # with the step's own operands.  An event pair around a single launch inside the step would put two
    # event markers next to the kernel; each costs about 6 us of dispatch gap (the kernel trace under
    # profiles/ shows them), which would slow the timed steps by 4 % and add 12 us to an 88 us kernel.
    # That reading is still taken, over a few extra untimed steps, and reported beside the batch figure.
    def q_launch():
        osc.osc_dual_gemm(*q1, packs["q"], 4096, K_HID, K_o, ydt, out=Y["q"])

    dom_ms = b.time_one(q_launch, reps=max(args.steps, 1), rounds=3)
    dom_ev = []
    for _ in range(min(args.steps, 20)):
        step(dom_ev)
    torch.cuda.synchronize()
    dom_ms_in_step = float(np.mean([a.elapsed_time(c) for a, c in dom_ev]))
    flops = sum(2.0 * M * N * K_HID for _, N in PROJ)
    value = flops / (ms_step * 1e-3) / 1e12
    dom_tflops = 2.0 * M * 4096 * K_HID / (dom_ms * 1e-3) / 1e12
    out = {
        "metric": "OSC linear TFLOP/s & % MXFP4 MFMA peak vs FP8 W8A8, Qwen3-8B shapes",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "mxfp4 x mxfp4 + bf16 x bf16, f32 accumulate, bf16 out",
        "data": "synthetic",
        "config": {"workload": f"configs[1] Qwen3-8B attention projections, M={M}: quant+gather, "
                               "q/o 4096->4096, k/v 4096->1024, 2 outliers per 32-group (K_o=256), Y bf16",
                   "tokens": M, "K": K_HID, "K_o": K_o, "input_crc32": crcs},
        "roofline": {"bound": "mfma", "achieved": round(dom_tflops, 1), "peak": PEAK_MXFP4_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(dom_tflops / PEAK_MXFP4_TFLOPS, 4),
                     "traffic": dominant_traffic_bytes() if M == 8192 else None,
                     "kernel": f"dual-path GEMM M={M} N=4096 K=4096 K_o={K_o}", "avg_ms": round(dom_ms, 4),
                     "avg_ms_single_launch_events_in_step": round(dom_ms_in_step, 4)},
        "frac_mxfp4_peak_whole_step": round(value / PEAK_MXFP4_TFLOPS, 4),
    }
    if args.only_step:
        print(json.dumps(out))
        return
    b.set_burn(lambda q=q1, p=packs["q"], y=Y["q"]: osc.osc_dual_gemm(*q, p, 4096, K_HID, K_o, ydt, out=y), dom_ms)
    ms_fp8 = timed_loop(step_fp8, max(args.steps // 2, 1), 3)
    # one more pass over both steps, alternating, for the speed-up (same clock state for both)
    ms_pair = b.time_many([step, step_fp8], reps=5, rounds=5)
    out["fp8_w8a8"] = {"ms_per_step": round(ms_fp8, 4), "tflops": round(flops / (ms_fp8 * 1e-3) / 1e12, 2),
                       "speedup_osc_over_fp8": round(ms_pair[1] / ms_pair[0], 3),
                       "alternating_ms": {"osc": round(ms_pair[0], 4), "fp8": round(ms_pair[1], 4)},
                       "model_speedup_compute_bound": round(2 / (1 + 4 * 2 / 32), 3)}

    # every kernel of the step and its FP8 counterpart, alternating blocks of one loop
    per = {}
    for n, N in PROJ:
        qq, ff = (q2, f2) if n == "o" else (q1, f1)
        per[n] = b.time_many([lambda: osc.osc_dual_gemm(*qq, packs[n], N, K_HID, K_o, ydt, out=Y[n]),
                              lambda: osc.osc_fp8_gemm(*ff, packs8[n], N, K_HID, y_dtype=ydt, out=Y[n])])

    # The quantisers are HBM-bound: time them over a ring of inputs and outputs larger than the
    # 256 MB last-level cache, so no call finds its operands left behind by the previous one.
    nring = max(2, -(-(640 << 20) // (M * K_HID * 2)))
    ringX = [dX1.clone() for _ in range(nring)]
    ringQ = [tuple(torch.empty_like(t) for t in q1) for _ in range(nring)]
    ringF = [tuple(torch.empty_like(t) for t in f1) for _ in range(nring)]
    turn = [0]

    def quant_ring(fmt, oidx, outs):
        i = turn[0] = (turn[0] + 1) % nring
        osc.osc_quantize_act(ringX[i], oidx, fmt, out=outs[i])

    ms_quant, ms_quant8 = b.time_many([lambda: quant_ring(osc.OSC_FMT_MXFP4_OSC, oidx1, ringQ),
                                       lambda: quant_ring(osc.OSC_FMT_FP8_E4M3_TOKEN, None, ringF)], reps=2 * nring)
    quant_bytes = M * (K_HID * 2 + K_HID // 2 + K_HID // 32 + 2 * K_o)
    out["kernels_ms"] = {"quant_mxfp4_gather": round(ms_quant, 4), "quant_fp8": round(ms_quant8, 4),
                         **{f"dual_gemm_{n}": round(v[0], 4) for n, v in per.items()},
                         **{f"fp8_gemm_{n}": round(v[1], 4) for n, v in per.items()}}
    out["quant_roofline"] = hbm(quant_bytes, ms_quant)
    out["speedup_with_quant"] = {
        "q_projection": round((ms_quant8 + per["q"][1]) / (ms_quant + per["q"][0]), 3),
        "note": "t(FP8 quantiser + FP8 GEMM) / t(OSC quantiser+gather + dual GEMM), M=%d, 4096x4096, K_o=%d" % (M, K_o)}

    # the quantiser at four times the tokens (a 268 MB input: nothing is cache-warm by construction)
    if M == 8192:
        Xl = torch.cat([dX1, dX2, dX1, dX2])
        ql = osc.osc_quantize_act(Xl, oidx1)
        ms_ql = b.time_one(lambda: osc.osc_quantize_act(Xl, oidx1, out=ql), reps=6)
        out["quant_roofline_M32768"] = {**hbm(4 * quant_bytes, ms_ql), "ms": round(ms_ql, 4)}
        del Xl, ql

    # offline profiling kernels (Section 2, Alg. 1) over the same ring: read-only streams of X
    p_acc = torch.zeros(1, dtype=torch.float64, device=dev)
    p_T = osc.osc_profile_threshold(osc.osc_profile_abs_sum(dX1), M * K_HID, 5.0)
    p_hist = torch.zeros((K_HID // 32, 32), dtype=torch.int32, device=dev)

    def prof_ring(which):
        i = turn[0] = (turn[0] + 1) % nring
        if which == 0:
            osc.osc_profile_abs_sum(ringX[i], p_acc)
        else:
            osc.osc_profile_hist(ringX[i], p_T, 32, p_hist)

    ms_psum, ms_phist = b.time_many([lambda: prof_ring(0), lambda: prof_ring(1)], reps=2 * nring)
    xbytes = M * K_HID * 2
    out["profiling"] = {"shape": f"S={M} H={K_HID} G=32", "abs_sum_ms": round(ms_psum, 4), "hist_ms": round(ms_phist, 4),
                        "abs_sum_roofline": hbm(xbytes, ms_psum), "hist_roofline": hbm(xbytes, ms_phist)}

    # what this machine attains next to the published peaks: a plain device copy, the FP4 MFMA alone
    # on random operands, the vendor library on the dominant shape, and the shader clock read while
    # the dominant kernel loops
    cp_src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    cp_dst = torch.empty_like(cp_src)
    ms_copy = b.time_one(lambda: cp_dst.copy_(cp_src), reps=3)
    # a bare streaming loop (16-byte non-temporal accesses, eight loads in flight per lane): read only, and four
    # bytes read per byte written (the mix of the fused SwiGLU quantisers)
    ms_rd = b.time_one(lambda: osc_probe.osc_probe_stream(cp_src, cp_dst, 0), reps=3)
    ms_rw = b.time_one(lambda: osc_probe.osc_probe_stream(cp_src, cp_dst, 4), reps=3)
    del cp_src, cp_dst
    probe_out = torch.zeros(1, dtype=torch.float32, device=dev)
    probe_flops = osc_probe.osc_probe_mfma_fp4(2048, 256, probe_out)
    ms_probe = b.time_one(lambda: osc_probe.osc_probe_mfma_fp4(2048, 256, probe_out), reps=3)

    def read_sclk():
        # current shader clock from the driver's sysfs table (the line marked with '*'); no child process
        import glob
        best = None
        for path in glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"):
            try:
                for line in open(path):
                    if "*" in line:
                        mhz = int(line.split(":")[1].strip().lower().split("mhz")[0])
                        best = mhz if best is None else max(best, mhz)
            except (OSError, ValueError, IndexError):
                pass
        return best

    for _ in range(6000):  # ~0.6 s of queued GEMMs; the clock is read while they run
        osc.osc_dual_gemm(*q1, packs["q"], 4096, K_HID, K_o, ydt, out=Y["q"])
    sclk_load = read_sclk()
    torch.cuda.synchronize()
    out["achievable"] = {
        "copy_gbs": round(2 * (1 << 30) / (ms_copy * 1e-3) / 1e9, 1),
        "stream_read_only_gbs": round((1 << 30) / (ms_rd * 1e-3) / 1e9, 1),
        "stream_read4_write1_gbs": round(1.25 * (1 << 30) / (ms_rw * 1e-3) / 1e9, 1),
        "mfma_fp4_only_tflops_random_operands": round(probe_flops / (ms_probe * 1e-3) / 1e12, 1),
        "sclk_mhz_while_dominant_kernel_loops": sclk_load, "sclk_mhz_nominal": 2400,
        "dominant_vs_mfma_only": round(dom_tflops / (probe_flops / (ms_probe * 1e-3) / 1e12), 4),
        "vendor_library": vendor_library_yardstick(b, M, 4096, K_HID),
    }

    # producer fusion: RMSNorm + OSC quantiser in one pass (same ring)
    gam = up(wl.to_bf16_bits((1.0 + 0.1 * wl.rng(2200).standard_normal(K_HID)).astype(np.float32)))

    def fused_ring():
        i = turn[0] = (turn[0] + 1) % nring
        osc.osc_rmsnorm_quantize_act(ringX[i], gam, 1e-6, oidx1, out=(ringQ[i][0], ringQ[i][1], ringQ[i][2], None))

    ms_fused = b.time_one(fused_ring, reps=2 * nring)
    out["fused_rmsnorm_quant"] = {"shape": f"M={M} K={K_HID} K_o={K_o}", "ms": round(ms_fused, 4),
                                  "roofline": hbm(quant_bytes, ms_fused), "unfused_quant_ms": round(ms_quant, 4)}
    # this kernel is limited by vector instruction issue rather than by memory: its instruction count (a
    # counter reading kept under profiles/) against the chip's issue rate, 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz
    insts = profile_figure("streaming_kernels__traffic_and_valu.txt", "RMSNORM_QUANT_VALU_WAVE_INSTS_PER_LAUNCH")
    if insts and M == 8192:
        peak = 256 * 4 * 16 * 2.4e9 / 1e12
        ach = insts * 64 / (ms_fused * 1e-3) / 1e12
        out["fused_rmsnorm_quant"]["alu_roofline"] = {"bound": "alu", "achieved": round(ach, 2), "peak": round(peak, 2),
                                                      "unit": "T lane-instructions/s", "frac": round(ach / peak, 4)}

    # Table 2 of the paper on this machine: one protected channel per group of G = 16, 32, 64
    # (K_o = K/G), a compute-bound GEMM (M tokens, 4096 x 4096) and a decode-sized one (64 tokens,
    # 4096 -> 12288), each against the FP8 W8A8 GEMM of the same shape in the same alternating loop.
    t2 = {}
    N_UP = 12288
    Wt = up(wl.weights(2100, 4096, K_HID))
    Wu = up(wl.weights(2101, N_UP, K_HID))
    wu8 = osc.osc_pack_weight_fp8(Wu)
    X64 = dX1[:64].contiguous()
    f64 = osc.osc_quantize_act(X64, None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    Y64 = torch.empty((64, N_UP), dtype=torch.bfloat16, device=dev)
    for G in (16, 32, 64):
        # G = 32 and 64: protection group = scale group (64: one shared exponent per 64 channels, held
        # in both of its hardware blocks of 32).  G = 16: the matrix core has no 16-element scale block,
        # so only the protection group is 16 wide; the scale block stays 32.
        sg = 64 if G == 64 else 32
        tab = wl.rng(7000 + G).integers(0, G, (K_HID // G, 1)).astype(np.int16)
        oi = up(osc.osc_table_to_index_g(tab, G))
        ko = int(oi.numel())
        fmt = osc.OSC_FMT_MXFP4_OSC_G64 if sg == 64 else osc.OSC_FMT_MXFP4_OSC
        pk, pu = osc.osc_pack_weight_g(Wt, oi, sg), osc.osc_pack_weight_g(Wu, oi, sg)
        qb, qs = osc.osc_quantize_act(dX1, oi, fmt), osc.osc_quantize_act(X64, oi, fmt)
        tb, tb8 = b.time_many([lambda: osc.osc_dual_gemm(*qb, pk, 4096, K_HID, ko, ydt, out=Y["q"]),
                               lambda: osc.osc_fp8_gemm(*f1, packs8["q"], 4096, K_HID, y_dtype=ydt, out=Y["q"])])
        (ts, ts8), _g = b.graph_many([lambda i: osc.osc_dual_gemm(*qs, pu, N_UP, K_HID, ko, ydt, out=Y64),
                                      lambda i: osc.osc_fp8_gemm(*f64, wu8, N_UP, K_HID, y_dtype=ydt, out=Y64)])
        model = round(2 / (1 + 4 / G), 3)
        t2[f"G={G}"] = {"K_o": ko, "scale_group": sg,
                        f"M={M} N=4096": {"osc_ms": round(tb, 4), "fp8_ms": round(tb8, 4), "speedup": round(tb8 / tb, 3),
                                          **({"above_model": True} if tb8 / tb > model * 1.02 else {})},
                        f"M=64 N={N_UP}": {"osc_ms": round(ts, 4), "fp8_ms": round(ts8, 4), "speedup": round(ts8 / ts, 3),
                                           "weights": "cache-warm"},
                        "model": model}
        del pk, pu, qb, qs, _g
    # Table 2's G = 16 row with 16 channels as the SCALE group as well (one E8M0 scale per 16), and NVFP4:
    # formats the matrix core cannot multiply as 4-bit operands, served by the weight-streaming kernel
    # that expands the codes in registers (decode regime), and, for the record, the same kernel at M tokens
    tab16 = wl.rng(7016).integers(0, 16, (K_HID // 16, 1)).astype(np.int16)
    oi16 = up(osc.osc_table_to_index_g(tab16, 16))
    ko16 = int(oi16.numel())
    for name, fmt, xts, wts in (("G=16 scale group 16 (E8M0)", osc.OSC_FMT16_E8M0, 1.0, 1.0),
                                ("NVFP4", osc.OSC_FMT16_NVFP4, 1.0 / 64, 1.0 / 4096)):
        pu = osc.osc_pack_weight_g16(Wu, oi16, fmt, wts)
        qs = osc.osc_quantize_act_g16(X64, oi16, fmt, xts)
        (ts, ts8), _g = b.graph_many([lambda i: osc.osc_dual_gemm_g16(*qs, pu, N_UP, K_HID, ko16, fmt, xts, wts, ydt, out=Y64),
                                      lambda i: osc.osc_fp8_gemm(*f64, wu8, N_UP, K_HID, y_dtype=ydt, out=Y64)])
        wbytes = N_UP * (K_HID // 2 + K_HID // 16 + ko16 * 2)
        pk = osc.osc_pack_weight_g16(Wt, oi16, fmt, wts)
        qb = osc.osc_quantize_act_g16(dX1, oi16, fmt, xts)
        tq = b.time_one(lambda: osc.osc_quantize_act_g16(dX1, oi16, fmt, xts, out=qb), reps=5)
        tb = b.time_one(lambda: osc.osc_dual_gemm_g16(*qb, pk, 4096, K_HID, ko16, fmt, xts, wts, ydt, out=Y["q"]), reps=2, rounds=3)
        t2[name] = {"K_o": ko16, "scale_group": 16,
                    f"M=64 N={N_UP}": {"osc_ms": round(ts, 4), "fp8_ms": round(ts8, 4), "speedup": round(ts8 / ts, 3),
                                       "weights": "cache-warm", "weight_bytes": wbytes,
                                       "model_memory_bound": round(N_UP * K_HID / wbytes, 3)},
                    f"M={M} N=4096": {"osc_ms": round(tb, 4), "quant_ms": round(tq, 4),
                                      "note": "codes expanded to bf16 in registers: bf16 matrix rate; the matrix core has no "
                                              "4-bit mode with a scale per 16 channels or with E4M3 scales"},
                    "model": 1.6}
        # 16 tokens with the weights streamed from HBM (copies larger than the last-level cache, in turn):
        # the regime where bytes per weight decide
        X16 = dX1[:16].contiguous()
        q16 = osc.osc_quantize_act_g16(X16, oi16, fmt, xts)
        f16 = osc.osc_quantize_act(X16, None, osc.OSC_FMT_FP8_E4M3_TOKEN)
        Y16 = torch.empty((16, N_UP), dtype=torch.bfloat16, device=dev)
        n4 = max(2, -(-(320 << 20) // osc.osc_packed_weight_g16_bytes(N_UP, K_HID, ko16)))
        n8 = max(2, -(-(320 << 20) // osc.osc_packed_weight_fp8_bytes(N_UP, K_HID)))
        p4 = [pu] + [osc.osc_pack_weight_g16(Wu, oi16, fmt, wts) for _ in range(n4 - 1)]
        p8 = [wu8] + [osc.osc_pack_weight_fp8(Wu) for _ in range(n8 - 1)]
        (tc, tc8), _g2 = b.graph_many(
            [lambda i: osc.osc_dual_gemm_g16(*q16, p4[i % n4], N_UP, K_HID, ko16, fmt, xts, wts, ydt, out=Y16),
             lambda i: osc.osc_fp8_gemm(*f16, p8[i % n8], N_UP, K_HID, y_dtype=ydt, out=Y16)])
        t2[name][f"M=16 N={N_UP}"] = {"osc_ms": round(tc, 4), "fp8_ms": round(tc8, 4), "speedup": round(tc8 / tc, 3),
                                      "weights": "rotated through copies larger than the last-level cache",
                                      "roofline": hbm(wbytes + 16 * N_UP * 2, tc), "model_memory_bound": round(N_UP * K_HID / wbytes, 3)}
        del pu, qs, _g, pk, qb, p4, p8, _g2
    del Wt, Wu, wu8
    out["table2_sweep"] = t2

    # "Dynamic" protection control (Section 4.2): run-time argmax quantiser, and the q projection
    # with the bf16 branch over all K channels (what the scheme costs without per-token gathers)
    dq = osc.osc_quantize_act_dynamic(dX1, want_idx=True)
    ringD = [tuple(torch.empty_like(t) for t in dq) for _ in range(min(nring, 4))]

    def dyn_ring():
        i = turn[0] = (turn[0] + 1) % nring
        osc.osc_quantize_act_dynamic(ringX[i], out=ringD[i % len(ringD)])

    ms_dynq = b.time_one(dyn_ring, reps=2 * nring)
    del ringD
    all_ch = torch.arange(K_HID, dtype=torch.int32, device=dev)
    pack_dyn = osc.osc_pack_weight(up(wl.weights(2100, 4096, K_HID)), all_ch)
    ms_dyng = b.time_one(lambda: osc.osc_dual_gemm(dq[0], dq[1], dq[2], pack_dyn, 4096, K_HID, K_HID, ydt, out=Y["q"]), reps=5)
    del pack_dyn, dq
    del ringX, ringQ, ringF
    out["dynamic_control"] = {
        "shape": f"M={M} K={K_HID} N=4096, one run-time protected element per group, Y bf16",
        "quant_ms": round(ms_dynq, 4),
        "quant_gbs": round(M * K_HID * (2 + 0.5 + 1 / 32 + 2 + 1 / 32) / (ms_dynq * 1e-3) / 1e9, 1),
        "gemm_ms": round(ms_dyng, 4),
        "osc_static_ms": {"quant": round(ms_quant, 4), "gemm_q": round(per["q"][0], 4)},
        "slowdown_vs_osc": round((ms_dynq + ms_dyng) / (ms_quant + per["q"][0]), 2)}

    # the W_2 fallback at the down-projection shape of configs[2] (K = 12288 -> N = 4096) on the seeded
    # diffuse-outlier input: MXFP8 (Section 4.1) next to the per-token FP8 form
    K_FF = 12288
    dXf = up(wl.activations_diffuse(3003, M, K_FF))
    Wf = up(wl.weights(3004, 4096, K_FF))
    wm8, wf8 = osc.osc_pack_weight_mxfp8(Wf), osc.osc_pack_weight_fp8(Wf)
    del Wf
    m8 = osc.osc_quantize_act(dXf, None, osc.OSC_FMT_MXFP8)
    t8 = osc.osc_quantize_act(dXf, None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    ms_m8q, ms_t8q = b.time_many([lambda: osc.osc_quantize_act(dXf, None, osc.OSC_FMT_MXFP8, out=m8),
                                  lambda: osc.osc_quantize_act(dXf, None, osc.OSC_FMT_FP8_E4M3_TOKEN, out=t8)], reps=5)
    ms_m8g, ms_t8g = b.time_many([lambda: osc.osc_mxfp8_gemm(*m8, wm8, 4096, K_FF, y_dtype=ydt, out=Y["o"]),
                                  lambda: osc.osc_fp8_gemm(*t8, wf8, 4096, K_FF, y_dtype=ydt, out=Y["o"])], reps=5)
    # the same position with its producer fused: SwiGLU on the two halves of a gate||up buffer
    gseed = torch.Generator(device=dev)
    gseed.manual_seed(3005)
    gu = (torch.randn((M, 2 * K_FF), generator=gseed, device=dev) * 2).to(torch.bfloat16).view(torch.uint16)
    ms_swq, ms_swq8 = b.time_many(
        [lambda: osc.osc_swiglu_quantize_act(gu[:, :K_FF], gu[:, K_FF:], out=(m8[0], m8[1], None)),
         lambda: osc.osc_swiglu_quantize_act_fp8(gu[:, :K_FF], gu[:, K_FF:], out=(t8[0], t8[1], None))], reps=5)
    del gu, dXf, wm8, wf8, m8, t8
    ff_flops = 2.0 * M * 4096 * K_FF

    def f8row(q_ms, g_ms, qbytes):
        tf = ff_flops / (g_ms * 1e-3) / 1e12
        return {"quant_ms": round(q_ms, 4), "gemm_ms": round(g_ms, 4), "quant_roofline": hbm(qbytes, q_ms),
                "gemm_tflops": round(tf, 1), "gemm_frac_fp8_peak": round(tf / PEAK_FP8_TFLOPS, 4)}
    out["w2_fallback"] = {"shape": f"configs[2] W_2: M={M} K={K_FF} N=4096, diffuse outliers, Y bf16",
                          "mxfp8": f8row(ms_m8q, ms_m8g, M * K_FF * (3 + 1 / 32)),
                          "fp8_per_token": f8row(ms_t8q, ms_t8g, M * K_FF * 3 + 4 * M)}
    out["fused_swiglu_quant_mxfp8"] = {"shape": f"M={M} K={K_FF}", "ms": round(ms_swq, 4),
                                       "roofline": hbm(M * K_FF * (4 + 1 + 1 / 32), ms_swq),
                                       "unfused_quant_only_ms": round(ms_m8q, 4)}
    out["fused_swiglu_quant_fp8"] = {"shape": f"M={M} K={K_FF}", "ms": round(ms_swq8, 4),
                                     "roofline": hbm(M * K_FF * 5 + 4 * M, ms_swq8),
                                     "unfused_quant_only_ms": round(ms_t8q, 4)}
    # the step with q, k and v as one launch (one packed weight of 6144 rows, Y[M, 6144] = q|k|v): the
    # same outputs with two launches fewer; a choice every caller has, reported beside the headline
    pack_qkv = osc.osc_pack_weight(up(np.concatenate([wl.weights(2100 + i, N, K_HID) for i, (_, N) in enumerate(PROJ[:3])])), oidx1)
    Yqkv = torch.empty((M, 6144), dtype=torch.bfloat16, device=dev)

    def step_fused():
        osc.osc_quantize_act(dX1, oidx1, out=q1)
        osc.osc_dual_gemm(*q1, pack_qkv, 6144, K_HID, K_o, ydt, out=Yqkv)
        osc.osc_quantize_act(dX2, oidx2, out=q2)
        osc.osc_dual_gemm(*q2, packs["o"], 4096, K_HID, K_o, ydt, out=Y["o"])

    ms_sf, ms_s3 = b.time_many([step_fused, step], reps=5, rounds=5)
    out["fused_qkv_step"] = {"ms_per_step": round(ms_sf, 4), "tflops": round(flops / (ms_sf * 1e-3) / 1e12, 2),
                             "separate_launches_ms": round(ms_s3, 4), "gain": round(ms_s3 / ms_sf, 3)}
    del Y, q1, q2, f1, f2, packs8, pack_qkv, Yqkv
    out["shapes"] = shapes_table(b, quick=args.quick)
    if not args.quick:
        out["shapes_moe"] = moe_rows(b)
    if args.detail:
        for k, v in out["kernels_ms"].items():
            print(f"  {k:24s} {v:9.4f} ms", file=sys.stderr)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
