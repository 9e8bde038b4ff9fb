"""The allocation-free form of the one-call profiler (osc_profile_calibrate_static: intermediate
results in a fixed device array inside the library) against osc_profile_calibrate with a caller's
workspace, through the C ABI: two calls in a row, the second on a smaller input, so stale contents of
the shared array would show.  All outputs are preallocated; the calls themselves allocate nothing."""
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


def bf(bits):
    return torch.from_numpy(np.ascontiguousarray(bits.view(np.int16))).cuda().view(torch.bfloat16)


def outputs(H, G, R):
    Kg = H // G
    d = "cuda"
    return (torch.full((Kg, R), -7, dtype=torch.int16, device=d), torch.full((Kg,), -7, dtype=torch.int32, device=d),
            torch.full((Kg,), -7, dtype=torch.int32, device=d), torch.full((Kg,), -7.0, dtype=torch.float32, device=d),
            torch.full((1,), -7.0, dtype=torch.float32, device=d), torch.full((1,), -7.0, dtype=torch.float32, device=d))


def test_static_scratch_equals_workspace_form_twice(osc):
    cases = [(2048, 12288, 32, 2, 9501), (300, 1088, 16, 1, 9502)]   # the second is smaller in every extent
    for S, H, G, R, seed in cases:
        X = bf(wl.activations_persistent(seed, S, H, 2, jitter=0.3)[0])
        ws = torch.empty(osc.osc_profile_workspace_bytes(H), dtype=torch.uint8, device="cuda")
        ref = osc.osc_profile_calibrate(X, G, 5.0, R, workspace=ws, out=outputs(H, G, R))
        got = outputs(H, G, R)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        osc.osc_profile_calibrate_static(X, G, 5.0, R, out=got)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        names = ("table", "n_total", "n_hit", "density", "cbar", "T")
        for n, a, b in zip(names, got, ref):
            if n == "T":  # the sum behind it is added with floating-point atomics: last bits may differ
                assert abs(a.item() - b.item()) <= 1e-6 * abs(b.item()), n
            else:
                assert torch.equal(a, b), f"{n} differs at S={S} H={H}"
        assert int(got[1].sum()) > 0  # the candidate sets are not empty: the comparison is not vacuous


def test_static_form_rejects_what_its_array_cannot_hold(osc):
    H = 16384 + 64
    X = torch.zeros((4, H), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(osc.OscError) as e:
        osc.osc_profile_calibrate_static(X, 32, 5.0, 1)
    assert e.value.code == -4 and "16384" in str(e.value)
