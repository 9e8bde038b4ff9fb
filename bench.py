#!/usr/bin/env python3
"""Benchmark of the OSC dual-path linear layer on one MI355X.

One step = the whole hot path of one Qwen3-8B attention block's linear layers at M tokens
(benchmark configuration 1, "configs[1]"): quantise+gather the attention input, dual-path GEMMs q (4096->4096),
k and v (4096->1024) on it, quantise+gather the o-projection input, dual-path GEMM o
(4096->4096).  Inputs are synthetic (seeded N(0,1) with two token-persistent outlier channels
per 32-group), resident in HBM before the timed region.  The same GEMM shapes are also run
through the library's own FP8 W8A8 path for the speed-up figure.

Prints one JSON line.  `value` = sum over the four GEMMs of 2*M*N*K, divided by the time of a
whole step (quantisers included).
"""
import argparse
import zlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MXFP4_TFLOPS = 10066.0  # MI355X dense MXFP4 matrix peak
PEAK_FP8_TFLOPS = 5033.0
PEAK_HBM_GBS = 8000.0
K_HID = 4096
# Bytes between L2 and the fabric per launch of the dominant kernel (dual-path GEMM 8192x4096x4096,
# K_o=256, bf16 out), from rocprofv3 FETCH_SIZE/WRITE_SIZE runs of this script scaled by a 1 GiB
# plain copy (summary: profiles/configs1_M8192_step__hbm_traffic.txt).  A profiler reading, not
# something this script can measure itself.
DOMINANT_TRAFFIC_BYTES = {8192: 218.3e6}
PROJ = (("q", 4096), ("k", 1024), ("v", 1024), ("o", 4096))


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
    Y = oracle.dual_gemm(Xq, Xs, B, Wq, Ws, WL)
    dt = time.perf_counter() - t0
    flops = 2.0 * rows * 4096 * K_HID
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{rows} tokens of configs[1]: quantise+gather, then the q projection "
                      f"(N=4096, K=4096, K_o=256) in {dt:.2f} s"}, float(np.abs(Y).max())


def sweep(osc, wl, torch):
    """GEMM times for the other shapes of the configs (dual path against FP8 W8A8), HIP events around
    20 launches back to back, bf16 output, random N(0,1) activations.  Decode-sized shapes are bound by
    the launch from Python here; section 'table2_sweep' of the benchmark line times them inside a graph."""
    def timeit(fn, reps=20):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    gen = torch.Generator(device="cuda")
    gen.manual_seed(9001)

    def dual(tag, M, N, K, r):
        X = torch.randn((M, K), generator=gen, device="cuda").to(torch.bfloat16)
        W = (torch.randn((N, K), generator=gen, device="cuda") * 0.02).to(torch.bfloat16)
        oidx = torch.from_numpy(osc.osc_table_to_index(wl.planted_table(wl.rng(3), K, r))).cuda() if r else None
        K_o = 0 if oidx is None else int(oidx.numel())
        q, Wp = osc.osc_quantize_act(X, oidx), osc.osc_pack_weight(W, oidx)
        Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        ms = timeit(lambda: osc.osc_dual_gemm(*q, Wp, N, K, K_o, osc.OSC_DT_BF16, out=Y))
        q8 = osc.osc_quantize_act(X, None, osc.OSC_FMT_FP8_E4M3_TOKEN)
        W8 = osc.osc_pack_weight_fp8(W)
        ms8 = timeit(lambda: osc.osc_fp8_gemm(*q8, W8, N, K, y_dtype=osc.OSC_DT_BF16, out=Y))
        tf = 2.0 * M * N * K / ms / 1e9
        print(f"{tag:6s} M={M:5d} N={N:5d} K={K:5d} r={r}: dual {ms * 1e3:7.1f} us {tf:6.0f} TFLOP/s "
              f"({100 * tf / PEAK_MXFP4_TFLOPS:4.1f} % of MXFP4 peak) | fp8 {ms8 * 1e3:7.1f} us | speed-up {ms8 / ms:.2f}", flush=True)

    for M in (128, 2048, 8192):
        for N in (4096, 1024):
            dual("cfg2", M, N, 4096, 2)
    dual("cfg3", 8192, 24576, 4096, 2)
    for r in (0, 1, 2, 4):
        for M in (64, 512, 4096):
            dual("cfg5", M, 12288, 4096, r)
    # cfg4: MoE, 128 experts, top-8 routing of 4096 tokens
    tokens, K, E, topk, N = 4096, 2048, 128, 8, 1536
    X = torch.randn((tokens, K), generator=gen, device="cuda").to(torch.bfloat16)
    oidx = torch.from_numpy(osc.osc_table_to_index(wl.planted_table(wl.rng(3), K, 2))).cuda()
    K_o = int(oidx.numel())
    q = osc.osc_quantize_act(X, oidx)
    off, row_map = wl.moe_routing(4002, tokens, E, topk)
    T = int(off[-1])
    stride = osc.osc_packed_weight_bytes(N, K, K_o)
    Wp = torch.empty(E * stride, dtype=torch.uint8, device="cuda")
    for e in range(E):
        W = (torch.randn((N, K), generator=gen, device="cuda") * 0.02).to(torch.bfloat16)
        osc.osc_pack_weight(W, oidx, out=Wp[e * stride:(e + 1) * stride])
    d_off, d_map = torch.from_numpy(off).cuda(), torch.from_numpy(row_map).cuda()
    Y = torch.empty((T, N), dtype=torch.bfloat16, device="cuda")
    ms = timeit(lambda: osc.osc_grouped_dual_gemm(*q, d_map, d_off, T, Wp, N, K, K_o, osc.OSC_DT_BF16, out=Y))
    print(f"cfg4   grouped dual T={T} N={N} K={K} E={E}: {ms * 1e3:.1f} us, "
          f"{2.0 * T * N * K / ms / 1e9:.0f} TFLOP/s, weights {E * stride / 1e6:.0f} MB", flush=True)
    K2, N2 = 768, 2048
    X2 = torch.randn((T, K2), generator=gen, device="cuda").to(torch.bfloat16)
    q8 = osc.osc_quantize_act(X2, None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    s8 = osc.osc_packed_weight_fp8_bytes(N2, K2)
    Wp8 = torch.empty(E * s8, dtype=torch.uint8, device="cuda")
    for e in range(E):
        W = (torch.randn((N2, K2), generator=gen, device="cuda") * 0.02).to(torch.bfloat16)
        osc.osc_pack_weight_fp8(W, out=Wp8[e * s8:(e + 1) * s8])
    Y2 = torch.empty((T, N2), dtype=torch.bfloat16, device="cuda")
    ms = timeit(lambda: osc.osc_fp8_gemm(*q8, Wp8, N2, K2, expert_offsets=d_off, y_dtype=osc.OSC_DT_BF16, out=Y2))
    print(f"cfg4   grouped fp8  T={T} N={N2} K={K2} E={E}: {ms * 1e3:.1f} us, "
          f"{2.0 * T * N2 * K2 / ms / 1e9:.0f} TFLOP/s", flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--tokens", type=int, default=8192)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--detail", action="store_true", help="per-kernel times on stderr")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark line: time the shapes of the other benchmark configurations (table on stdout)")
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
    if args.sweep:
        return sweep(osc, wl, torch)
    M = args.tokens
    dev = torch.device("cuda:0")
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)

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

    ev = lambda: torch.cuda.Event(enable_timing=True)
    dom = []  # event pairs around the dominant kernel (q projection), on the launch stream

    def step(timed=False):
        osc.osc_quantize_act(dX1, oidx1, out=q1)
        for n, N in PROJ[:3]:
            if timed and n == "q":
                e0, e1 = ev(), ev()
                e0.record()
            osc.osc_dual_gemm(*q1, packs[n], N, K_HID, K_o, ydt, out=Y[n])
            if timed and n == "q":
                e1.record()
                dom.append((e0, e1))
        osc.osc_quantize_act(dX2, oidx2, out=q2)
        osc.osc_dual_gemm(*q2, packs["o"], 4096, K_HID, K_o, ydt, out=Y["o"])

    def step_fp8():
        osc.osc_quantize_act(dX1, None, osc.OSC_FMT_FP8_E4M3_TOKEN, out=f1)
        for n, N in PROJ[:3]:
            osc.osc_fp8_gemm(*f1, packs8[n], N, K_HID, y_dtype=ydt, out=Y[n])
        osc.osc_quantize_act(dX2, None, osc.OSC_FMT_FP8_E4M3_TOKEN, out=f2)
        osc.osc_fp8_gemm(*f2, packs8["o"], 4096, K_HID, y_dtype=ydt, out=Y["o"])

    def timed_loop(fn, steps, warmup, **kw):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn(**kw)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    if args.copy_mib:
        src = torch.zeros(args.copy_mib << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    ms_step = timed_loop(step, args.steps, args.warmup, timed=True)
    dom_ms = float(np.mean([a.elapsed_time(b) for a, b in dom]))
    ms_fp8 = timed_loop(step_fp8, max(args.steps // 2, 1), 3)

    def time_one(fn, reps=20):
        # the clock needs a few milliseconds of work to come back up after an idle stretch
        for _ in range(max(2, reps)):
            fn()
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

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

    ms_quant = time_one(lambda: quant_ring(osc.OSC_FMT_MXFP4_OSC, oidx1, ringQ), reps=4 * nring)
    ms_quant8 = time_one(lambda: quant_ring(osc.OSC_FMT_FP8_E4M3_TOKEN, None, ringF), reps=4 * nring)
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

    ms_psum = time_one(lambda: prof_ring(0), reps=4 * nring)
    ms_phist = time_one(lambda: prof_ring(1), reps=4 * nring)
    # what this machine attains next to the published peaks: a plain device copy, the FP4 MFMA alone
    # on random operands, and the shader clock read while the dominant kernel loops
    cp_src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    cp_dst = torch.empty_like(cp_src)
    ms_copy = time_one(lambda: cp_dst.copy_(cp_src), reps=5)
    del cp_src, cp_dst
    probe_out = torch.zeros(1, dtype=torch.float32, device=dev)
    probe_flops = osc_probe.osc_probe_mfma_fp4(2048, 256, probe_out)
    ms_probe = time_one(lambda: osc_probe.osc_probe_mfma_fp4(2048, 256, probe_out), reps=5)

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

    # producer fusion: RMSNorm + OSC quantiser in one pass (same ring)
    gam = up(wl.to_bf16_bits((1.0 + 0.1 * wl.rng(2200).standard_normal(K_HID)).astype(np.float32)))

    def fused_ring():
        i = turn[0] = (turn[0] + 1) % nring
        osc.osc_rmsnorm_quantize_act(ringX[i], gam, 1e-6, oidx1, out=(ringQ[i][0], ringQ[i][1], ringQ[i][2], None))

    ms_fused = time_one(fused_ring, reps=4 * nring)

    # Table 2 of the paper on this machine: one protected channel per group of G = 16, 32, 64
    # (K_o = K/G), a compute-bound GEMM (M tokens, 4096 x 4096) and a decode-sized one (64 tokens,
    # 4096 -> 12288), each against the FP8 W8A8 GEMM of the same shape.  The decode-sized kernels
    # run a few microseconds, less than one launch from Python costs, so 50 launches are captured
    # in a HIP graph and the replay is timed.
    def graph_time(fn, n=50, reps=5):
        fn()
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                for _ in range(n):
                    fn()
        torch.cuda.synchronize()
        g.replay()
        return time_one(g.replay, reps=reps) / n

    t2 = {}
    N_UP = 12288
    Wt = up(wl.weights(2100, 4096, K_HID))
    Wu = up(wl.weights(2101, N_UP, K_HID))
    wu8 = osc.osc_pack_weight_fp8(Wu)
    X64 = dX1[:64].contiguous()
    f64 = osc.osc_quantize_act(X64, None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    Y64 = torch.empty((64, N_UP), dtype=torch.bfloat16, device=dev)
    ms_f8_big = time_one(lambda: osc.osc_fp8_gemm(*f1, packs8["q"], 4096, K_HID, y_dtype=ydt, out=Y["q"]))
    ms_f8_64 = graph_time(lambda: osc.osc_fp8_gemm(*f64, wu8, N_UP, K_HID, y_dtype=ydt, out=Y64))
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
        tb = time_one(lambda: osc.osc_dual_gemm(*qb, pk, 4096, K_HID, ko, ydt, out=Y["q"]))
        ts = graph_time(lambda: osc.osc_dual_gemm(*qs, pu, N_UP, K_HID, ko, ydt, out=Y64))
        t2[f"G={G}"] = {"K_o": ko, "scale_group": sg,
                        f"M={M} N=4096": {"osc_ms": round(tb, 4), "fp8_ms": round(ms_f8_big, 4),
                                          "speedup": round(ms_f8_big / tb, 3)},
                        f"M=64 N={N_UP}": {"osc_ms": round(ts, 4), "fp8_ms": round(ms_f8_64, 4),
                                           "speedup": round(ms_f8_64 / ts, 3)},
                        "model": round(2 / (1 + 4 / G), 3)}
        del pk, pu, qb, qs
    del Wt, Wu, wu8

    # "Dynamic" protection control (Section 4.2): run-time argmax quantiser, and the q projection
    # with the bf16 branch over all K channels (what the scheme costs without per-token gathers)
    dq = osc.osc_quantize_act_dynamic(dX1, want_idx=True)
    ringD = [tuple(torch.empty_like(t) for t in dq) for _ in range(min(nring, 4))]

    def dyn_ring():
        i = turn[0] = (turn[0] + 1) % nring
        osc.osc_quantize_act_dynamic(ringX[i], out=ringD[i % len(ringD)])

    ms_dynq = time_one(dyn_ring, reps=4 * nring)
    del ringD
    all_ch = torch.arange(K_HID, dtype=torch.int32, device=dev)
    Wd = up(wl.weights(2100, 4096, K_HID))
    pack_dyn = osc.osc_pack_weight(Wd, all_ch)
    del Wd
    ms_dyng = time_one(lambda: osc.osc_dual_gemm(dq[0], dq[1], dq[2], pack_dyn, 4096, K_HID, K_HID, ydt,
                                                 out=Y["q"]), reps=10)
    del pack_dyn, dq
    del ringX, ringQ, ringF

    # the W_2 fallback at the down-projection shape of configs[2] (K = 12288 -> N = 4096), MXFP8
    # (Section 4.1) next to the per-token FP8 form
    K_FF = 12288
    dXf = torch.from_numpy(wl.activations_diffuse(3003, 64, K_FF)).to(dev).repeat(-(-M // 64), 1)[:M].contiguous()
    Wf = up(wl.weights(3004, 4096, K_FF))
    wm8, wf8 = osc.osc_pack_weight_mxfp8(Wf), osc.osc_pack_weight_fp8(Wf)
    del Wf
    m8 = osc.osc_quantize_act(dXf, None, osc.OSC_FMT_MXFP8)
    t8 = osc.osc_quantize_act(dXf, None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    ms_m8q = time_one(lambda: osc.osc_quantize_act(dXf, None, osc.OSC_FMT_MXFP8, out=m8), reps=10)
    ms_m8g = time_one(lambda: osc.osc_mxfp8_gemm(*m8, wm8, 4096, K_FF, y_dtype=ydt, out=Y["o"]), reps=10)
    ms_t8q = time_one(lambda: osc.osc_quantize_act(dXf, None, osc.OSC_FMT_FP8_E4M3_TOKEN, out=t8), reps=10)
    ms_t8g = time_one(lambda: osc.osc_fp8_gemm(*t8, wf8, 4096, K_FF, y_dtype=ydt, out=Y["o"]), reps=10)
    # the same position with its producer fused: SwiGLU on the two halves of a gate||up buffer, then MXFP8
    gseed = torch.Generator(device=dev)
    gseed.manual_seed(3005)
    gu = (torch.randn((M, 2 * K_FF), generator=gseed, device=dev) * 2).to(torch.bfloat16).view(torch.uint16)
    ms_swq = time_one(lambda: osc.osc_swiglu_quantize_act(gu[:, :K_FF], gu[:, K_FF:], out=(m8[0], m8[1], None)), reps=10)
    ms_swq8 = time_one(lambda: osc.osc_swiglu_quantize_act_fp8(gu[:, :K_FF], gu[:, K_FF:], out=(t8[0], t8[1], None)), reps=10)
    del gu
    del dXf, wm8, wf8, m8, t8
    per = {}
    for n, N in PROJ:
        qq = q2 if n == "o" else q1
        ff = f2 if n == "o" else f1
        per[n] = (time_one(lambda: osc.osc_dual_gemm(*qq, packs[n], N, K_HID, K_o, ydt, out=Y[n])),
                  time_one(lambda: osc.osc_fp8_gemm(*ff, packs8[n], N, K_HID, y_dtype=ydt, out=Y[n])))

    flops = sum(2.0 * M * N * K_HID for _, N in PROJ)
    value = flops / (ms_step * 1e-3) / 1e12
    dom_flops = 2.0 * M * 4096 * K_HID
    dom_tflops = dom_flops / (dom_ms * 1e-3) / 1e12
    quant_bytes = M * (K_HID * 2 + K_HID // 2 + K_HID // 32 + 2 * K_o)
    out = {
        "metric": "OSC linear TFLOP/s & % MXFP4 MFMA peak vs FP8 W8A8, Qwen3-8B shapes",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "mxfp4 x mxfp4 + bf16 x bf16 -> f32",
        "data": "synthetic",
        "config": {"workload": f"configs[1] Qwen3-8B attention projections, M={M}: quant+gather, "
                               "q/o 4096->4096, k/v 4096->1024, 2 outliers per 32-group (K_o=256), Y bf16",
                   "tokens": M, "K": K_HID, "K_o": K_o},
        "roofline": {"bound": "mfma", "achieved": round(dom_tflops, 1), "peak": PEAK_MXFP4_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(dom_tflops / PEAK_MXFP4_TFLOPS, 4),
                     "traffic": DOMINANT_TRAFFIC_BYTES.get(M),
                     "kernel": f"dual-path GEMM M={M} N=4096 K=4096 K_o={K_o}", "avg_ms": round(dom_ms, 4)},
        "frac_mxfp4_peak_whole_step": round(value / PEAK_MXFP4_TFLOPS, 4),
        "fp8_w8a8": {"ms_per_step": round(ms_fp8, 4), "tflops": round(flops / (ms_fp8 * 1e-3) / 1e12, 2),
                     "speedup_osc_over_fp8": round(ms_fp8 / ms_step, 3),
                     "model_speedup_compute_bound": round(2 / (1 + 4 * 2 / 32), 3)},
        "kernels_ms": {"quant_mxfp4_gather": round(ms_quant, 4), "quant_fp8": round(ms_quant8, 4),
                       **{f"dual_gemm_{n}": round(v[0], 4) for n, v in per.items()},
                       **{f"fp8_gemm_{n}": round(v[1], 4) for n, v in per.items()}},
        "quant_roofline": {"bound": "hbm", "achieved": round(quant_bytes / (ms_quant * 1e-3) / 1e9, 1),
                           "peak": PEAK_HBM_GBS, "unit": "GB/s",
                           "frac": round(quant_bytes / (ms_quant * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)},
    }
    ff_flops = 2.0 * M * 4096 * K_FF
    xbytes = M * K_HID * 2
    out["w2_fallback"] = {
        "shape": f"M={M} K={K_FF} N=4096, Y bf16",
        "mxfp8": {"quant_ms": round(ms_m8q, 4), "gemm_ms": round(ms_m8g, 4),
                  "quant_gbs": round(M * K_FF * (3 + 1 / 32) / (ms_m8q * 1e-3) / 1e9, 1),
                  "gemm_tflops": round(ff_flops / (ms_m8g * 1e-3) / 1e12, 1),
                  "gemm_frac_fp8_peak": round(ff_flops / (ms_m8g * 1e-3) / 1e12 / PEAK_FP8_TFLOPS, 4)},
        "fp8_per_token": {"quant_ms": round(ms_t8q, 4), "gemm_ms": round(ms_t8g, 4),
                          "gemm_tflops": round(ff_flops / (ms_t8g * 1e-3) / 1e12, 1),
                          "gemm_frac_fp8_peak": round(ff_flops / (ms_t8g * 1e-3) / 1e12 / PEAK_FP8_TFLOPS, 4)},
    }
    out["profiling"] = {
        "shape": f"S={M} H={K_HID} G=32",
        "abs_sum_ms": round(ms_psum, 4), "hist_ms": round(ms_phist, 4),
        "abs_sum_roofline": {"bound": "hbm", "achieved": round(xbytes / (ms_psum * 1e-3) / 1e9, 1),
                             "peak": PEAK_HBM_GBS, "unit": "GB/s",
                             "frac": round(xbytes / (ms_psum * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)},
        "hist_roofline": {"bound": "hbm", "achieved": round(xbytes / (ms_phist * 1e-3) / 1e9, 1),
                          "peak": PEAK_HBM_GBS, "unit": "GB/s",
                          "frac": round(xbytes / (ms_phist * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)},
    }
    out["config"]["input_crc32"] = crcs
    out["achievable"] = {
        "copy_gbs": round(2 * (1 << 30) / (ms_copy * 1e-3) / 1e9, 1),
        "mfma_fp4_only_tflops_random_operands": round(probe_flops / (ms_probe * 1e-3) / 1e12, 1),
        "sclk_mhz_while_dominant_kernel_loops": sclk_load, "sclk_mhz_nominal": 2400,
        "dominant_vs_mfma_only": round(dom_tflops / (probe_flops / (ms_probe * 1e-3) / 1e12), 4),
    }
    out["speedup_with_quant"] = {
        "q_projection": round((ms_quant8 + per["q"][1]) / (ms_quant + per["q"][0]), 3),
        "note": "t(FP8 quantiser + FP8 GEMM) / t(OSC quantiser+gather + dual GEMM), M=%d, 4096x4096, K_o=%d" % (M, K_o),
    }
    out["fused_rmsnorm_quant"] = {
        "shape": f"M={M} K={K_HID} K_o={K_o}", "ms": round(ms_fused, 4),
        "roofline": {"bound": "hbm", "achieved": round(quant_bytes / (ms_fused * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": round(quant_bytes / (ms_fused * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)},
        "unfused_quant_ms": round(ms_quant, 4),
    }
    sw_bytes = M * K_FF * (4 + 1 + 1 / 32)
    out["fused_swiglu_quant_mxfp8"] = {
        "shape": f"M={M} K={K_FF}", "ms": round(ms_swq, 4),
        "roofline": {"bound": "hbm", "achieved": round(sw_bytes / (ms_swq * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": round(sw_bytes / (ms_swq * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)},
        "unfused_quant_only_ms": round(ms_m8q, 4),
    }
    sw8_bytes = M * K_FF * (4 + 1) + 4 * M
    out["fused_swiglu_quant_fp8"] = {
        "shape": f"M={M} K={K_FF}", "ms": round(ms_swq8, 4),
        "roofline": {"bound": "hbm", "achieved": round(sw8_bytes / (ms_swq8 * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": round(sw8_bytes / (ms_swq8 * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)},
        "unfused_quant_only_ms": round(ms_t8q, 4),
    }
    out["table2_sweep"] = t2
    out["dynamic_control"] = {
        "shape": f"M={M} K={K_HID} N=4096, one run-time protected element per group, Y bf16",
        "quant_ms": round(ms_dynq, 4),
        "quant_gbs": round(M * K_HID * (2 + 0.5 + 1 / 32 + 2 + 1 / 32) / (ms_dynq * 1e-3) / 1e9, 1),
        "gemm_ms": round(ms_dyng, 4),
        "osc_static_ms": {"quant": round(ms_quant, 4), "gemm_q": round(per["q"][0], 4)},
        "slowdown_vs_osc": round((ms_dynq + ms_dyng) / (ms_quant + per["q"][0]), 2),
    }
    if args.detail:
        for k, v in out["kernels_ms"].items():
            print(f"  {k:24s} {v:9.4f} ms", file=sys.stderr)
    if not args.no_cpu_baseline:
        out["cpu_baseline"], _ = cpu_baseline()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
