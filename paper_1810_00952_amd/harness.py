"""Device-memory plumbing around the C ABI: uploads numpy arrays into torch
tensors, prepacks params, owns workspace and outputs, and hands raw pointers
and the current stream to the library.  No arithmetic happens here."""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

from .binding import Context, Plan, graph_from_spec

_TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16}


def to_device(a: np.ndarray, dtype: str, device="cuda:0") -> torch.Tensor:
    """float32 array, or uint16 bf16 bit patterns, to a device tensor (bit-exact)."""
    if dtype == "bf16":
        t = torch.from_numpy(np.asarray(a, dtype=np.uint16, order="C").view(np.int16)).to(device)
        return t.view(torch.bfloat16)
    return torch.from_numpy(np.asarray(a, dtype=np.float32, order="C")).to(device)


def to_host(t: torch.Tensor) -> np.ndarray:
    """Device tensor back to float32 array / uint16 bf16 bits."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def stream_handle() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


class Session:
    """One plan with its device buffers."""

    def __init__(self, spec, ctx: Optional[Context] = None, device="cuda:0", auto_groups: bool = False, opts: Optional[Dict[str, int]] = None):
        self.spec = spec
        self.device = device
        self.ctx = ctx or Context()
        self.graph = graph_from_spec(self.ctx, spec, auto_groups=auto_groups)
        self.plan = Plan(self.graph, opts)
        self.tensors: Dict[int, torch.Tensor] = {}    # value id -> tensor whose pointer is bound
        self.raw: Dict[int, torch.Tensor] = {}
        self.workspace = None
        self.by_name = {v.name: i for i, v in enumerate(spec.values)}

    def set_value(self, vid: int, t: torch.Tensor) -> None:
        """Bind an input or param held in boundary layout; params the plan wants
        re-laid-out are prepacked into a buffer of their own."""
        v = self.spec.values[vid]
        assert t.is_contiguous() and tuple(t.shape) == tuple(v.type.shape) and t.dtype == _TORCH_DT[v.type.dtype], v.name
        self.raw[vid] = t
        if v.role == "param":
            nb = self.plan.packed_bytes(vid)
            if nb:
                packed = torch.empty(nb, dtype=torch.uint8, device=self.device)
                self.plan.prepack(vid, t.data_ptr(), packed.data_ptr(), stream_handle())
                self.tensors[vid] = packed
                return
        self.tensors[vid] = t

    def load(self, data: Dict[str, np.ndarray]) -> None:
        for name, arr in data.items():
            if name in self.by_name:
                vid = self.by_name[name]
                self.set_value(vid, to_device(arr, self.spec.values[vid].type.dtype, self.device))

    def alloc(self) -> None:
        for vid in self.spec.outputs:
            v = self.spec.values[vid]
            if vid not in self.tensors:
                self.tensors[vid] = torch.empty(v.type.shape, dtype=_TORCH_DT[v.type.dtype], device=self.device)
        nb = self.plan.workspace_bytes()
        if self.workspace is None or self.workspace.numel() < nb:
            self.workspace = torch.empty(max(nb, 256), dtype=torch.uint8, device=self.device)

    def run(self) -> None:
        if self.workspace is None:
            self.alloc()
        self.plan.run({vid: t.data_ptr() for vid, t in self.tensors.items()}, self.workspace.data_ptr(),
                      self.workspace.numel(), stream_handle())

    def capture(self) -> "torch.cuda.CUDAGraph":
        """Record one run of the plan into a HIP graph (rl_plan_run only launches kernels: no allocation, no
        synchronisation, no memset), for callers that replay a fixed plan many times."""
        if self.workspace is None:
            self.alloc()
        self.run()                                   # first run outside the capture: lazy module loads happen here
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            self.run()
        return g

    def output(self, i: int = 0) -> torch.Tensor:
        return self.tensors[self.spec.outputs[i]]
