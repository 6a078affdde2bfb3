"""Device-memory plumbing around a Plan: torch allocates buffers and provides the stream.

Nothing here computes anything: host arrays are copied to device tensors, raw pointers go
to fs_plan_run, results are copied back.  f32 tensors are float32 arrays, bf16 tensors are
uint16 arrays of raw bits, u8 tensors are uint8 arrays.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np
import torch

from .binding import Plan

_NP_DT = {"f32": np.float32, "bf16": np.uint16, "u8": np.uint8}
_TORCH_DT = {"f32": torch.float32, "bf16": torch.int16, "u8": torch.uint8}


def to_device(arr: np.ndarray, dtype: str, device) -> torch.Tensor:
    a = np.ascontiguousarray(arr, dtype=_NP_DT[dtype])
    if dtype == "bf16":
        a = a.view(np.int16)
    return torch.from_numpy(a).to(device)


def to_host(t: torch.Tensor, dtype: str) -> np.ndarray:
    a = t.cpu().numpy()
    return a.view(np.uint16) if dtype == "bf16" else a


class DeviceRun:
    """Buffers of one plan on one device; `launch()` enqueues fs_plan_run on the current stream."""

    def __init__(self, plan: Plan, device: str = "cuda:0"):
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the stitched kernels only run on a MI355X")
        self.plan = plan
        self.device = torch.device(device)
        g = plan.graph
        self.in_nodes = [g.nodes[i] for i in g.input_ids()]
        self.out_nodes = [g.nodes[o] for o in g.outputs]
        self.inputs: List[torch.Tensor] = []
        self.outputs = [torch.empty((n.rows, n.cols), dtype=_TORCH_DT[n.dtype], device=self.device) for n in self.out_nodes]
        self.ws_bytes = plan.workspace_bytes()
        self.workspace = torch.empty(max(self.ws_bytes, 256), dtype=torch.uint8, device=self.device)
        assert self.workspace.data_ptr() % 256 == 0
        plan.workspace_init(self.workspace.data_ptr(), self.ws_bytes, torch.cuda.current_stream(self.device).cuda_stream)

    def set_inputs(self, host_inputs: Sequence[np.ndarray]) -> None:
        assert len(host_inputs) == len(self.in_nodes)
        self.inputs = [to_device(a, n.dtype, self.device) for a, n in zip(host_inputs, self.in_nodes)]

    def set_device_inputs(self, tensors: Sequence[torch.Tensor]) -> None:
        self.inputs = list(tensors)

    def launch(self) -> None:
        stream = torch.cuda.current_stream(self.device).cuda_stream
        self.plan.run([t.data_ptr() for t in self.inputs], [t.data_ptr() for t in self.outputs],
                      self.workspace.data_ptr() if self.ws_bytes else 0, self.ws_bytes, stream)

    def tune(self, reps: int = 0) -> dict:
        """fs_plan_tune on this run's buffers: fills the performance library for the plan's groups."""
        stream = torch.cuda.current_stream(self.device).cuda_stream
        return self.plan.tune([t.data_ptr() for t in self.inputs], [t.data_ptr() for t in self.outputs],
                              self.workspace.data_ptr() if self.ws_bytes else 0, self.ws_bytes, stream, reps)

    def prepare(self):
        """Freeze the pointer tables and the stream; returns a zero-argument launcher for timing loops."""
        ins, outs = self.plan.pointer_tables([t.data_ptr() for t in self.inputs], [t.data_ptr() for t in self.outputs])
        ws = self.workspace.data_ptr() if self.ws_bytes else 0
        stream = torch.cuda.current_stream(self.device).cuda_stream
        run, nbytes = self.plan.run_tables, self.ws_bytes
        self._frozen = (ins, outs)  # keep the tables alive
        return lambda: run(ins, outs, ws, nbytes, stream)

    def results(self) -> List[np.ndarray]:
        torch.cuda.synchronize(self.device)
        return [to_host(t, n.dtype) for t, n in zip(self.outputs, self.out_nodes)]


def run_graph(graph, host_inputs: Sequence[np.ndarray], device: str = "cuda:0", **plan_kwargs) -> List[np.ndarray]:
    """Create a plan for `graph`, run it once on `device`, return the outputs as host arrays."""
    plan = Plan(graph, **plan_kwargs)
    try:
        r = DeviceRun(plan, device)
        r.set_inputs(host_inputs)
        r.launch()
        return r.results()
    finally:
        plan.destroy()
