"""The hot path under HIP graph capture: no entry point allocates, synchronises or enqueues a
memset, so a step (quantise+gather, dual GEMM, FP8 quantise, FP8 GEMM) can be captured once and
replayed.  Every replay is compared with the eager result, with eager work and synchronisations of
the same entry points between the replays."""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def osc():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2604_12782_amd as m
    m.lib()
    return m


@pytest.mark.parametrize("M", [48, 1000])
def test_step_replays_equal_eager(osc, M):
    K, N = 1024, 768
    dev = torch.device("cuda:0")
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    Xa, table = wl.activations_persistent(4001, M, K, 2)
    Xb = wl.activations_diffuse(4002, M, K)
    oidx = up(osc.osc_table_to_index(table))
    K_o = int(oidx.numel())
    W = up(wl.weights(4003, N, K))
    Wp, W8 = osc.osc_pack_weight(W, oidx), osc.osc_pack_weight_fp8(W)
    X = up(Xa)
    q = osc.osc_quantize_act(X, oidx)
    f = osc.osc_quantize_act(X, None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    Y1 = torch.empty((M, N), dtype=torch.float32, device=dev)
    Y2 = torch.empty((M, N), dtype=torch.bfloat16, device=dev)

    def step():
        osc.osc_quantize_act(X, oidx, out=q)
        osc.osc_dual_gemm(*q, Wp, N, K, K_o, osc.OSC_DT_F32, out=Y1)
        osc.osc_quantize_act(X, None, osc.OSC_FMT_FP8_E4M3_TOKEN, out=f)
        osc.osc_fp8_gemm(*f, W8, N, K, y_dtype=osc.OSC_DT_BF16, out=Y2)

    def eager(bits):
        X.copy_(up(bits))
        step()
        torch.cuda.synchronize()
        return Y1.clone(), Y2.clone(), q[0].clone()

    ref_a, ref_b = eager(Xa), eager(Xb)
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            step()
    torch.cuda.synchronize()
    for i, (bits, ref) in enumerate([(Xa, ref_a), (Xb, ref_b), (Xa, ref_a), (Xb, ref_b)]):
        X.copy_(up(bits))
        Y1.zero_(); Y2.zero_(); q[0].zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y1, ref[0]) and torch.equal(Y2, ref[1]) and torch.equal(q[0], ref[2]), f"replay {i}"
        # eager work of the same entry points between replays
        osc.osc_dual_gemm(*q, Wp, N, K, K_o, osc.OSC_DT_F32, out=torch.empty_like(Y1))
        torch.cuda.synchronize()


def test_swiglu_fusions_with_table_replay_equal_eager(osc, tuning):
    """The SwiGLU fusions on their table path (two kernels per call: the silu table, then the
    quantiser that copies it into LDS) under capture; replays on changing inputs equal eager runs."""
    tuning.swiglu_table("1")
    M, K = 300, 1536
    dev = torch.device("cuda:0")
    gen = wl.rng(4100)
    bits = [wl.to_bf16_bits((gen.standard_normal((M, 2 * K)) * s).astype(np.float32)) for s in (1.0, 4.0)]
    GU = torch.empty((M, 2 * K), dtype=torch.uint16, device=dev)
    m8 = osc.osc_swiglu_quantize_act(GU[:, :K], GU[:, K:])
    f8 = osc.osc_swiglu_quantize_act_fp8(GU[:, :K], GU[:, K:])

    def step():
        osc.osc_swiglu_quantize_act(GU[:, :K], GU[:, K:], out=(m8[0], m8[1], None))
        osc.osc_swiglu_quantize_act_fp8(GU[:, :K], GU[:, K:], out=(f8[0], f8[1], None))

    def eager(b):
        GU.copy_(torch.from_numpy(b).to(dev))
        step()
        torch.cuda.synchronize()
        return m8[0].clone(), m8[1].clone(), f8[0].clone(), f8[1].clone()

    refs = [eager(b) for b in bits]
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            step()
    torch.cuda.synchronize()
    for i in range(4):
        GU.copy_(torch.from_numpy(bits[i & 1]).to(dev))
        for t in (m8[0], f8[0], f8[1]):
            t.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        r = refs[i & 1]
        assert torch.equal(m8[0], r[0]) and torch.equal(m8[1], r[1]) and torch.equal(f8[0], r[2]) and torch.equal(f8[1], r[3]), f"replay {i}"
        tuning.swiglu_table("0")  # eager work on the other path in between
        osc.osc_swiglu_quantize_act(GU[:, :K], GU[:, K:])
        tuning.swiglu_table("1")
        torch.cuda.synchronize()


def test_persistent_kernels_replay_equal_eager(osc, tuning):
    """The persistent pipelined kernel in its three modes (dual path, per-token FP8, MXFP8; forced, with a
    ragged row tail that adds a second launch each) captured in one graph; replays on changing inputs
    equal the eager runs."""
    tuning.gemm("4,2")
    M, K, N = 552, 768, 512
    dev = torch.device("cuda:0")
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    Xa, table = wl.activations_persistent(4201, M, K, 2)
    Xb = wl.activations_diffuse(4202, M, K)
    oidx = up(osc.osc_table_to_index(table))
    K_o = int(oidx.numel())
    W = up(wl.weights(4203, N, K))
    Wp, W8, Wm = osc.osc_pack_weight(W, oidx), osc.osc_pack_weight_fp8(W), osc.osc_pack_weight_mxfp8(W)
    X = up(Xa)
    q = osc.osc_quantize_act(X, oidx)
    f = osc.osc_quantize_act(X, None, osc.OSC_FMT_FP8_E4M3_TOKEN)
    m = osc.osc_quantize_act(X, None, osc.OSC_FMT_MXFP8)
    Y = [torch.empty((M, N), dtype=torch.bfloat16, device=dev) for _ in range(3)]

    def step():
        osc.osc_quantize_act(X, oidx, out=q)
        osc.osc_dual_gemm(*q, Wp, N, K, K_o, osc.OSC_DT_BF16, out=Y[0])
        osc.osc_quantize_act(X, None, osc.OSC_FMT_FP8_E4M3_TOKEN, out=f)
        osc.osc_fp8_gemm(*f, W8, N, K, y_dtype=osc.OSC_DT_BF16, out=Y[1])
        osc.osc_quantize_act(X, None, osc.OSC_FMT_MXFP8, out=m)
        osc.osc_mxfp8_gemm(*m, Wm, N, K, y_dtype=osc.OSC_DT_BF16, out=Y[2])

    def eager(bits):
        X.copy_(up(bits))
        step()
        torch.cuda.synchronize()
        return [y.clone() for y in Y]

    refs = [eager(Xa), eager(Xb)]
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            step()
    torch.cuda.synchronize()
    for i in range(4):
        X.copy_(up(Xa if i % 2 == 0 else Xb))
        for y in Y:
            y.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for y, r in zip(Y, refs[i % 2]):
            assert torch.equal(y, r), f"replay {i}"
        osc.osc_fp8_gemm(*f, W8, N, K, y_dtype=osc.OSC_DT_BF16)  # eager work of the same kernels in between
        torch.cuda.synchronize()
