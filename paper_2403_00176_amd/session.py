"""Device-memory plumbing around the C ABI: torch allocates weights, inputs, outputs and the
arena and hands raw pointers to sod2_run.  No arithmetic of the method happens here."""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from . import (pointer_array, sod2_graph_build, sod2_rdp_infer, sod2_plan, sod2_bind, sod2_run, sod2_binding_arena_bytes,
               sod2_binding_query_tensor, sod2_run_decisions, sod2_run_arena_bytes, sod2_binding_workspace_bytes,
               sod2_replay_create, sod2_replay_launch, sod2_plan_constants_bytes, sod2_plan_prepare_constants,
               sod2_binding_set_constants, Sod2Error)

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
        with np.errstate(invalid="ignore"):            # (rows beyond an execution-determined count hold whatever was there)
            return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return t.cpu().numpy().astype(np.float64 if t.dtype.is_floating_point else np.int64)


class Session:
    """One graph on one GPU: graph -> RDP -> plan once; bind + run per call."""

    def __init__(self, graph_desc, device="cuda:0", derive_constants=True, **plan_opts):
        """``derive_constants``: hand every binding the constants derived from the weights, so that normalisations
        folded into contractions run without a kernel of their own (sod2_plan_prepare_constants)."""
        if not torch.cuda.is_available():
            raise RuntimeError("Session needs a GPU: the HIP path has no CPU fallback")
        self.desc = graph_desc
        self.device = torch.device(device)
        self.graph = sod2_graph_build(graph_desc)
        self.rdp = sod2_rdp_infer(self.graph)
        self.plan = sod2_plan(self.graph, self.rdp, **plan_opts)
        self.weights: List[torch.Tensor] = []
        self._wptrs = self._wptrs_of = None              # the weights' addresses as a C array, made once
        self.arena: Optional[torch.Tensor] = None
        self.workspace_bytes = 0
        self.stream = torch.cuda.current_stream(self.device)
        self.derive_constants = bool(derive_constants)
        self.constants: Optional[torch.Tensor] = None

    def upload_weights(self, weights: Dict[int, np.ndarray]):
        self.weights = [to_device(weights[t], self.desc.tensors[t].dtype, self.device) for t in self.desc.weights()]
        self.prepare_constants()

    def prepare_constants(self):
        """(Re)computes the derived constants from the device weights; to be called when the weights change."""
        n = sod2_plan_constants_bytes(self.plan) if self.derive_constants else 0
        if n == 0:
            self.constants = None
            return
        if self.constants is None or self.constants.numel() < n:
            with torch.cuda.stream(self.stream):
                self.constants = torch.empty(n, dtype=torch.uint8, device=self.device)
        sod2_plan_prepare_constants(self.plan, [w.data_ptr() for w in self.weights], self.constants.data_ptr(), n,
                                    self.stream.cuda_stream)

    def ensure_arena(self, nbytes: int):
        """The planned arena plus the optional workspace behind it (enables split-K)."""
        nbytes = (max(nbytes, 256) + 255) // 256 * 256 + self.workspace_bytes
        if self.arena is None or self.arena.numel() < nbytes:
            self.arena = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        return self.arena

    def upload_inputs(self, inputs: Dict[int, np.ndarray]) -> List[torch.Tensor]:
        return [to_device(inputs[t], self.desc.tensors[t].dtype, self.device) for t in self.desc.inputs()]

    def alloc_outputs(self, out_shapes: Sequence[Sequence[int]]) -> List[torch.Tensor]:
        return [torch.empty(tuple(s), dtype=_TORCH[self.desc.tensors[t].dtype], device=self.device)
                for t, s in zip(self.desc.outputs(), out_shapes)]

    def bind(self, sym):
        b = sod2_bind(self.plan, sym)
        if not self.workspace_bytes:
            self.workspace_bytes = sod2_binding_workspace_bytes(b)
        if self.constants is not None:
            sod2_binding_set_constants(b, self.constants.data_ptr(), self.constants.numel())
        return b

    def run(self, binding, inputs: List[torch.Tensor], outputs: List[torch.Tensor]):
        nbytes, _ = sod2_binding_arena_bytes(binding)
        for attempt in range(4):
            arena = self.ensure_arena(nbytes)
            try:
                if self._wptrs is None or self._wptrs_of is not self.weights:
                    self._wptrs, self._wptrs_of = pointer_array([w.data_ptr() for w in self.weights]), self.weights
                sod2_run(binding, arena.data_ptr(), arena.numel(), self._wptrs,
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
        """Concrete shapes of the graph outputs under this binding."""
        return [sod2_binding_query_tensor(binding, t)["dims"] for t in self.desc.outputs()]


class DecoderSession:
    """A prefill graph and a decode graph that declare the same weights and the same session tensors
    (the KV cache): one set of device weights, one arena whose bottom region holds the cache."""

    def __init__(self, prefill_desc, decode_desc, t_max: int, device="cuda:0", **plan_opts):
        self.pre = Session(prefill_desc, device, **plan_opts)
        self.dec = Session(decode_desc, device, **plan_opts)
        self.t_max = int(t_max)
        self.device = self.pre.device
        # a stream of its own (default priority): the decode steps can be captured in a HIP graph, which the
        # null stream does not allow.  Callers do their own torch work inside `with torch.cuda.stream(ses.stream)`.
        self.stream = torch.cuda.Stream(self.device)
        self.pre.stream = self.dec.stream = self.stream
        self.replay = None
        self.arena: Optional[torch.Tensor] = None
        self.logits_dtype = _TORCH[prefill_desc.tensors[prefill_desc.tensor_id("logits")].dtype]

    def upload_weights(self, by_name: Dict[str, np.ndarray]):
        d = self.pre.desc
        self.pre.weights = [to_device(by_name[d.tensors[t].name], d.tensors[t].dtype, self.device) for t in d.weights()]
        names = [self.dec.desc.tensors[t].name for t in self.dec.desc.weights()]
        assert names == [d.tensors[t].name for t in d.weights()], "the two graphs must declare the same weights"
        self.dec.weights = self.pre.weights
        self.pre.prepare_constants()
        self.dec.prepare_constants()

    def start(self, P: int, vocab: int):
        """Buffers of one sequence: the arena (sized for the prompt pass and the last decode step), the
        token ids and positions, one row of logits per produced token."""
        self.P = int(P)
        self.replay = None
        self.b_pre = self.pre.bind({"P": P})
        need = sod2_binding_arena_bytes(self.b_pre)[0]
        need = max(need, sod2_binding_arena_bytes(self.dec.bind({"P": P, "t": self.t_max - 1}))[0])
        need = (need + 255) // 256 * 256 + sod2_binding_workspace_bytes(self.b_pre)
        with torch.cuda.stream(self.stream):
            if self.arena is None or self.arena.numel() < need:
                self.arena = torch.empty(need, dtype=torch.uint8, device=self.device)
            self.tokens = torch.zeros(P + self.t_max + 1, dtype=torch.int64, device=self.device)
            self.positions = torch.arange(P + self.t_max + 1, dtype=torch.int64, device=self.device)
            self.logits = torch.zeros(self.t_max + 1, vocab, dtype=self.logits_dtype, device=self.device)
            self.step_counter = torch.zeros(1, dtype=torch.int32, device=self.device)

    def _run(self, ses, binding, ids_ptr, pos_ptr, logits_ptr, next_ptr):
        d = ses.desc
        ins = {d.tensor_id("ids"): ids_ptr, d.tensor_id("pos"): pos_ptr}
        outs = {d.tensor_id("logits"): logits_ptr, d.tensor_id("next"): next_ptr}
        sod2_run(binding, self.arena.data_ptr(), self.arena.numel(), [w.data_ptr() for w in ses.weights],
                 [ins[t] for t in d.inputs()], [outs[t] for t in d.outputs()], self.stream.cuda_stream)

    def prefill(self, prompt: torch.Tensor):
        """Runs the prompt pass; logits row 0 and token P (the first generated one) are written."""
        P = self.P
        with torch.cuda.stream(self.stream):
            self.tokens[:P] = prompt
        self._run(self.pre, self.b_pre, self.tokens.data_ptr(), self.positions.data_ptr(), self.logits.data_ptr(),
                  self.tokens.data_ptr() + 8 * P)

    def decode(self, t: int, binding=None):
        """Step t consumes token P+t (written by the previous step or by the caller) and writes
        logits row t+1 and token P+t+1.  Nothing is synchronised."""
        P = self.P
        b = binding if binding is not None else self.dec.bind({"P": P, "t": t})
        self._run(self.dec, b, self.tokens.data_ptr() + 8 * (P + t), self.positions.data_ptr() + 8 * (P + t),
                  self.logits.data_ptr() + (t + 1) * self.logits.stride(0) * self.logits.element_size(),
                  self.tokens.data_ptr() + 8 * (P + t + 1))
        return b

    def decode_replay(self, first_step: int, n_steps: int):
        """Steps first_step .. first_step + n_steps - 1 as replays of one captured HIP graph: the kernels
        read the step from a counter on the device, the host plans nothing per step."""
        P, d = self.P, self.dec.desc
        if self.replay is None:
            row = self.logits.stride(0) * self.logits.element_size()
            ins = {d.tensor_id("ids"): (self.tokens.data_ptr() + 8 * P, 8), d.tensor_id("pos"): (self.positions.data_ptr() + 8 * P, 8)}
            outs = {d.tensor_id("logits"): (self.logits.data_ptr() + row, row), d.tensor_id("next"): (self.tokens.data_ptr() + 8 * (P + 1), 8)}
            self.replay = sod2_replay_create(
                self.dec.plan, {"P": P, "t": 0}, "t", self.t_max, self.arena.data_ptr(), self.arena.numel(),
                [w.data_ptr() for w in self.dec.weights], [ins[t][0] for t in d.inputs()], [ins[t][1] for t in d.inputs()],
                [outs[t][0] for t in d.outputs()], [outs[t][1] for t in d.outputs()], self.step_counter.data_ptr(),
                self.stream.cuda_stream)
        sod2_replay_launch(self.replay, first_step, n_steps, self.stream.cuda_stream)
