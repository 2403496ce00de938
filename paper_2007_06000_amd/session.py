"""PyTorch plumbing around a Plan: device buffers, the current stream, timing.

Nothing here computes layer outputs; it moves host arrays to the device,
hands raw pointers to libxl and reads results back.
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

from .binding import Plan


class Session:
    def __init__(self, workload, x: np.ndarray, params: Dict[int, dict], device: int = 0, tune: bool = False,
                 **options):
        if not torch.cuda.is_available():
            raise RuntimeError("xl needs a GPU: libxl has no CPU path")
        self.dev = torch.device("cuda", device)
        self.workload = workload
        self.plan = Plan(workload, device=device, **options)
        self.x = torch.from_numpy(np.ascontiguousarray(x)).to(self.dev)
        self.y = torch.empty(workload.shapes[workload.output_id], dtype=torch.float32, device=self.dev)
        self._weights = []
        ptrs = self.weight_ptrs = [None] * self.plan.nweights
        for li, p in params.items():
            for j, key in enumerate(("w", "scale", "shift")):
                if p.get(key) is not None:
                    t = torch.from_numpy(np.ascontiguousarray(p[key])).to(self.dev)
                    self._weights.append(t)
                    ptrs[3 * li + j] = t.data_ptr()
        nbytes = self.plan.workspace_bytes()
        self.workspace = torch.empty((nbytes + 3) // 4, dtype=torch.float32, device=self.dev)
        assert self.workspace.data_ptr() % 256 == 0
        self.plan.prepare(ptrs, self.workspace.data_ptr(), self.stream)
        self.workspaces = [self.workspace]
        self.tensor_ptrs = {workload.input_id: self.x.data_ptr(), workload.output_id: self.y.data_ptr()}
        if tune:
            self.plan.tune(self.tensor_ptrs, self.workspace.data_ptr(), self.stream)
            torch.cuda.synchronize(self.dev)

    @property
    def stream(self) -> int:
        return torch.cuda.current_stream(self.dev).cuda_stream

    def add_workspace(self) -> int:
        """One more prepared workspace (for callers that rotate over several, e.g. cache-cold timing); returns its index."""
        ws = torch.empty_like(self.workspace)
        self.plan.prepare(self.weight_ptrs, ws.data_ptr(), self.stream)
        self.workspaces.append(ws)
        return len(self.workspaces) - 1

    def run(self, fused: bool = True, x: Optional[torch.Tensor] = None, y: Optional[torch.Tensor] = None, ws: int = 0):
        ptrs = dict(self.tensor_ptrs)
        if x is not None:
            ptrs[self.workload.input_id] = x.data_ptr()
        if y is not None:
            ptrs[self.workload.output_id] = y.data_ptr()
        self.plan.run(ptrs, self.workspaces[ws].data_ptr(), self.stream, fused)
        return self.y if y is None else y

    def output(self, fused: bool = True) -> np.ndarray:
        self.y.fill_(float("nan"))
        self.run(fused)
        torch.cuda.synchronize(self.dev)
        return self.y.cpu().numpy()
