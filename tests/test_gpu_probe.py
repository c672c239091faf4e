"""The benchmark's machine probes run and report plausible rates (needs an MI355X)."""
import ctypes
import os

import pytest
import torch

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_probe_runs_and_reports_a_plausible_rate():
    torch.cuda.init()
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2506_05632_amd", "libllc_probe.so"))
    lib.llc_probe_run.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lib.llc_probe_run.restype = ctypes.c_int
    # (probe, lower and upper bound of a sane result: operations, words or bytes per second)
    sane = {0: (5e12, 6e13), 1: (2e12, 3e13), 2: (5e12, 6e13), 3: (5e11, 8e12), 4: (1e12, 9e12), 5: (1e12, 9e12), 6: (1e12, 9e12)}
    for which, (lo, hi) in sane.items():
        res, clk = ctypes.c_double(), ctypes.c_double()
        assert lib.llc_probe_run(which, 3, ctypes.byref(res), ctypes.byref(clk)) == 0
        assert lo < res.value < hi, (which, res.value)
        if which not in (4, 5):
            assert 0.5 < clk.value < 3.5, (which, clk.value)
    res = ctypes.c_double()
    assert lib.llc_probe_run(99, 3, ctypes.byref(res), None) == -1
    assert lib.llc_probe_run(0, 0, ctypes.byref(res), None) == -1
