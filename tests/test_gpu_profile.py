"""The measurement entry points of the C ABI: per-launch timing (xl_profile) and the measured peaks
(xl_measure_peaks).  Timing values are only checked for sanity; what they must not do is change results."""
import numpy as np
import pytest

import xl_workloads as W
from oracle import xlo
from paper_2007_06000_amd import binding as B
from test_gpu_parity import check

pytestmark = pytest.mark.gpu


def test_per_launch_timing_covers_every_launch_and_leaves_the_result_intact():
    import torch
    from paper_2007_06000_amd.session import Session
    wl = W.config(5, n=2, hw=63, classes=40)
    x, params = W.make_tensors(wl)
    s = Session(wl, x, params)
    for fused in (True, False):
        us = s.plan.profile(s.tensor_ptrs, s.workspace.data_ptr(), s.stream, fused, reps=3)
        assert len(us) == s.plan.num_launches(fused)
        assert all(0.5 < t < 1e5 for t in us), us
        torch.cuda.synchronize()
        check(s.y.cpu().numpy(), xlo.forward(wl, x, params), f"after profiling fused={fused}")
    # too small an output array is refused before anything runs
    import ctypes
    arr = (ctypes.c_void_p * s.plan.ntensors)()
    for t, p in s.tensor_ptrs.items():
        arr[t] = p
    out = (ctypes.c_float * 2)()
    st = B.lib().xl_profile(s.plan.handle, arr, s.plan.ntensors, ctypes.c_void_p(s.workspace.data_ptr()),
                            ctypes.c_void_p(s.stream), 1, 3, out, 2)
    assert st == B.XL_E_GRAPH


def test_measured_peaks_are_plausible_for_an_mi355x():
    import torch
    n = 256 << 20
    a = torch.ones(n // 4, dtype=torch.float32, device="cuda")
    b = torch.zeros_like(a)
    m = B.xl_measure_peaks(b.data_ptr(), a.data_ptr(), n, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert 1000 < m["copy_gbs"] < 8000 * 1.05                  # read + written bytes per second against 8 TB/s
    assert 60 < m["mfma_f32_tflops"] < 157.3 * 1.05
    assert 600 < m["mfma_bf16_tflops"] < 2500 * 1.05
    assert 30 < m["valu_f32_tflops"] < 157.3 * 1.05
    assert float(b[(2 << 20) // 4:].min()) == 1.0 and float(b[-1]) == 1.0     # the copy really copied (past the sink area)
    with pytest.raises(B.XlError):
        B.xl_measure_peaks(b.data_ptr(), a.data_ptr(), 1024)
