"""Device-memory plumbing around the C ABI: torch allocates weights, inputs, outputs and the
arena and hands raw pointers to sod2_run.  No arithmetic of the method happens here."""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from . import (sod2_graph_build, sod2_rdp_infer, sod2_plan, sod2_bind, sod2_run, sod2_binding_arena_bytes,
               sod2_binding_dump, sod2_run_decisions, sod2_run_arena_bytes, Sod2Error)

_NP = {"f32": np.float32, "i64": np.int64, "i32": np.int32}
_TORCH = {"f32": torch.float32, "bf16": torch.bfloat16, "i64": torch.int64, "i32": torch.int32}


def _bf16_bits(x: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)


def to_device(x: np.ndarray, dtype: str, device) -> torch.Tensor:
    """Host float64/int array -> device tensor in the storage type (bf16 by round-to-nearest-even)."""
    if dtype == "bf16":
        bits = _bf16_bits(np.asarray(x))
        return torch.from_numpy(bits.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x, dtype=_NP[dtype])).to(device)


def to_host(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return t.cpu().numpy().astype(np.float64 if t.dtype.is_floating_point else np.int64)


class Session:
    """One graph on one GPU: graph -> RDP -> plan once; bind + run per call."""

    def __init__(self, graph_desc, device="cuda:0", **plan_opts):
        if not torch.cuda.is_available():
            raise RuntimeError("Session needs a GPU: the HIP path has no CPU fallback")
        self.desc = graph_desc
        self.device = torch.device(device)
        self.graph = sod2_graph_build(graph_desc)
        self.rdp = sod2_rdp_infer(self.graph)
        self.plan = sod2_plan(self.graph, self.rdp, **plan_opts)
        self.weights: List[torch.Tensor] = []
        self.arena: Optional[torch.Tensor] = None
        self.stream = torch.cuda.current_stream(self.device)

    def upload_weights(self, weights: Dict[int, np.ndarray]):
        self.weights = [to_device(weights[t], self.desc.tensors[t].dtype, self.device) for t in self.desc.weights()]

    def ensure_arena(self, nbytes: int):
        if self.arena is None or self.arena.numel() < nbytes:
            self.arena = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.device)
        return self.arena

    def upload_inputs(self, inputs: Dict[int, np.ndarray]) -> List[torch.Tensor]:
        return [to_device(inputs[t], self.desc.tensors[t].dtype, self.device) for t in self.desc.inputs()]

    def alloc_outputs(self, out_shapes: Sequence[Sequence[int]]) -> List[torch.Tensor]:
        return [torch.empty(tuple(s), dtype=_TORCH[self.desc.tensors[t].dtype], device=self.device)
                for t, s in zip(self.desc.outputs(), out_shapes)]

    def bind(self, sym):
        return sod2_bind(self.plan, sym)

    def run(self, binding, inputs: List[torch.Tensor], outputs: List[torch.Tensor]):
        nbytes, _ = sod2_binding_arena_bytes(binding)
        for attempt in range(4):
            arena = self.ensure_arena(nbytes)
            try:
                sod2_run(binding, arena.data_ptr(), arena.numel(), [w.data_ptr() for w in self.weights],
                         [t.data_ptr() for t in inputs], [t.data_ptr() for t in outputs], self.stream.cuda_stream)
                return
            except Sod2Error as e:
                # with Switches the path taken can need more than the bind-time plan: grow and repeat
                if e.code != -5 or attempt == 3:
                    raise
                self.stream.synchronize()
                nbytes = max(sod2_run_arena_bytes(binding)[0], arena.numel() + 1)
                self.arena = None

    def output_shapes(self, binding) -> List[List[int]]:
        """Concrete shapes of the graph outputs, read from the binding's text dump."""
        dims = {}
        for line in sod2_binding_dump(binding).splitlines():
            if line.startswith("t") and " dims=[" in line:
                tid = int(line[1:line.index(" ")])
                dims[tid] = [int(v) for v in line[line.index("[") + 1:line.index("]")].split()]
        return [dims[t] for t in self.desc.outputs()]
