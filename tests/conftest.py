import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


class _Tuning:
    """Kernel-choice overrides of include/osc_tuning.h for one test; everything is back to
    automatic when the test ends."""

    def __init__(self):
        import paper_2604_12782_amd as osc
        self.osc = osc

    def gemm(self, cfg):
        """cfg = "<tile rows / 64>,<kernel id>" (0 staged, 1 DMA, 2 persistent, 3 skinny) or None."""
        tile, kern = (-1, -1) if cfg is None else map(int, cfg.split(","))
        self.osc.osc_tuning_set(self.osc.OSC_TUNE_GEMM_TILE, tile)
        self.osc.osc_tuning_set(self.osc.OSC_TUNE_GEMM_KERNEL, kern)

    def gemm_ksplit(self, on):
        self.osc.osc_tuning_set(self.osc.OSC_TUNE_GEMM_KSPLIT, -1 if on is None else int(on))

    def swiglu_table(self, on):
        self.osc.osc_tuning_set(self.osc.OSC_TUNE_SWIGLU_TABLE, -1 if on is None else int(on))

    def grouped_one_tile(self, on):
        self.osc.osc_tuning_set(self.osc.OSC_TUNE_GROUPED_ONE_TILE, -1 if on is None else int(on))

    def reset(self):
        for k in range(5):
            self.osc.osc_tuning_set(k, -1)


import pytest  # noqa: E402


@pytest.fixture
def tuning():
    t = _Tuning()
    yield t
    t.reset()
