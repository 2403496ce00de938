"""xl_run_static: the entry point that allocates nothing (its workspace is a static device array inside the
library) must produce what xl_prepare + xl_run produce with a caller workspace.  Two calls in a row share
the array, the second with a smaller input; a third call returns to the first plan without passing weights
again only after the array was handed back to it."""
import numpy as np
import pytest

import xl_workloads as W
from oracle import xlo
from paper_2007_06000_amd import binding as B

pytestmark = pytest.mark.gpu


def outputs(s, torch, static, fused, relayout=True, weights=True):
    s.y.fill_(float("nan"))
    if static:
        s.plan.run_static(s.weight_ptrs if weights else None, s.tensor_ptrs, s.stream, fused, relayout)
    else:
        s.run(fused)
    torch.cuda.synchronize()
    return s.y.cpu().numpy()


def test_static_scratch_run_matches_the_workspace_run():
    import torch
    from paper_2007_06000_amd.session import Session
    from test_gpu_parity import check
    big = W.config(4, n=4, hw=28)           # residual block: unfused intermediates live in the scratch array
    small = W.config(3, n=1, hw=13)         # a smaller input right after it, another plan
    sessions = []
    for wl in (big, small):
        x, params = W.make_tensors(wl)
        sessions.append((wl, Session(wl, x, params), xlo.forward(wl, x, params)))
    for wl, s, ref in sessions:             # two calls in a row on the shared array, the second one smaller
        assert s.plan.workspace_bytes() <= B.XL_STATIC_SCRATCH_BYTES
        for fused in (True, False):
            print(f"[case] static run {wl.name} fused={fused}", flush=True)
            want = outputs(s, torch, False, fused)
            got = outputs(s, torch, True, fused)
            assert np.array_equal(got, want), f"{wl.name} fused={fused}: static-scratch run differs from the workspace run"
            check(got, ref, f"{wl.name} static fused={fused}")
    # the array now holds the small plan's filters: the big plan must re-lay its own before it runs
    wl, s, ref = sessions[0]
    with pytest.raises(B.XlError) as e:
        outputs(s, torch, True, True, relayout=False, weights=False)
    assert e.value.status == B.XL_E_STATE
    got = outputs(s, torch, True, True, relayout=False)                     # weights given: re-laid out on demand
    check(got, ref, "big plan after the small one")
    got = outputs(s, torch, True, False, relayout=False, weights=False)     # array still this plan's: nothing to pass
    check(got, ref, "big plan again, filters kept")


def test_plans_beyond_the_static_scratch_are_rejected():
    import torch
    from paper_2007_06000_amd.session import Session
    wl = W.config(4, n=48)                  # unfused intermediates: 2 x 38.5 MB
    x, params = W.make_tensors(wl)
    s = Session(wl, x, params)
    assert s.plan.workspace_bytes() > B.XL_STATIC_SCRATCH_BYTES
    with pytest.raises(B.XlError) as e:
        s.plan.run_static(s.weight_ptrs, s.tensor_ptrs, s.stream, True, True)
    assert e.value.status == B.XL_E_SCRATCH
    torch.cuda.synchronize()
