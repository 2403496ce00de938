"""xl_run only enqueues kernels on the caller's stream (no allocation, no synchronisation, no memset), so a
caller can capture it into a HIP graph.  The graph is replayed several times with eager work and
synchronisations in between and new input values each time; every replay is checked against the eager
result and the oracle."""
import numpy as np
import pytest

import xl_workloads as W
from oracle import xlo
from test_gpu_parity import check

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("wl,precision", [(W.config(3, n=2, hw=19), 0), (W.config(5, n=2, hw=63, classes=40), 0),
                                          (W.config(4, n=2, hw=17, c=32), 1)], ids=lambda v: getattr(v, "name", str(v)))
def test_fused_run_replayed_from_a_graph(wl, precision):
    import torch
    from paper_2007_06000_amd.session import Session
    x, params = W.make_tensors(wl)
    s = Session(wl, x, params, precision=precision)
    s.run(True)                                 # warm-up outside the capture (module load, first launch)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        s.run(True)                             # current stream = the capture stream
    rng = np.random.default_rng(3)
    for replay in range(3):
        xi = (x * (0.5 + replay) + rng.standard_normal(x.shape).astype(np.float32) * 0.1).astype(np.float32)
        s.x.copy_(torch.from_numpy(xi))         # eager work between the replays
        s.y.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = s.y.cpu().numpy()
        eager = s.output(True)
        assert np.array_equal(got, eager), f"replay {replay} differs from the eager run"
        check(got, xlo.forward(wl, xi, params), f"{wl.name} graph replay {replay}")
