"""Neutral description of an extended computational graph (Section 4.1, item G).

A graph is three flat lists: symbols (named dims with a declared range),
tensors and operators.  Operators follow ONNX naming (Table 2) plus the
<Switch, Combine> control-flow pair.  Nothing here computes a shape: tensors
produced by operators carry ``dims=None`` and consumers run their own analysis.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple, Union

import numpy as np

Dim = Union[int, str]

# tensor roles
INTER, INPUT, WEIGHT, HOSTCONST = "inter", "input", "weight", "hostconst"

DTYPES = ("f32", "bf16", "i64", "i32")
DTYPE_BYTES = {"f32": 4, "bf16": 2, "i64": 8, "i32": 4}

# operator kinds and their integer attributes, in the order they are marshalled
OP_ATTRS: Dict[str, Tuple[str, ...]] = {
    "Shape": (),
    "Gather": ("axis",),
    "Concat": ("axis",),
    "Reshape": (),
    "Slice": (),
    "Transpose": ("perm",),
    "MatMul": ("transB",),
    "Conv": ("stride", "pad"),
    "Add": (),
    "Mul": (),
    "Relu": (),
    "Gelu": (),
    "Sigmoid": (),
    "Cast": (),
    "Softmax": ("causal",),
    "LayerNorm": (),          # float attr eps
    "ReduceMean": ("axes", "keepdims"),
    "MaxPool": ("kernel", "stride", "pad"),
    "AveragePool": ("kernel", "stride", "pad"),   # channels last; positions in the padding do not count
    "Round": (),              # to the nearest integer, halves to the even one
    "ArgMax": (),
    "CacheAppend": (),
    "NonZero": (),
    "NMS": ("max_out",),      # inputs scores [N], boxes [N, 4] (x1, y1, x2, y2), both f32; float attr iou; result: kept box indices, i64
    "Switch": (),             # float attr threshold
    "Combine": (),
    "Range": (),              # inputs start, limit, delta (one-element int tensors)
    "Expand": (),             # input 1 = the shape to broadcast to
    "Upsample": (),           # nearest neighbour by whole factors: input 1 = host constant of one factor per dim
    "ConstantOfShape": (),    # float attr value; input 0 = the shape
    "EyeLike": ("k",),        # ones on diagonal k of a matrix shaped like input 0
    "OneHot": (),             # inputs indices, depth (one-element int tensor), values = host constant [off, on]; last axis
    "TopK": (),               # inputs x, k (one-element int tensor); results values, indices (last axis, largest first)
    "Resize": (),             # nearest neighbour, target shape = the values of input 1 ("sizes")
    "GroupNorm": ("groups",), # GroupNormalization, channels last: inputs x [N, ..., C], scale [C], bias [C]; float attr eps
    "MaxUnpool": (),          # channels last: inputs x [N, h, w, C], indices (same shape, flat positions in the result), output_shape (its values)
    "ScatterRows": (),        # ScatterND with row indices: copy of input 0 whose rows input 1 are replaced by input 2
}
OP_KINDS = tuple(OP_ATTRS)


@dataclass
class TensorDesc:
    name: str
    dtype: str
    role: str = INTER
    dims: Optional[List[Dim]] = None      # None: undeclared (to be inferred)
    data: Optional[np.ndarray] = None     # HOSTCONST only: small host array
    is_output: bool = False
    session: bool = False                 # persists across calls (KV cache): stored in the arena's session region
    capacity: Optional[List[Dim]] = None  # session inputs only: dims the storage is sized for


@dataclass
class OpDesc:
    kind: str
    inputs: List[int]
    outputs: List[int]
    attrs: Dict[str, object] = field(default_factory=dict)


@dataclass
class GraphDesc:
    symbols: List[Tuple[str, int, int]]
    tensors: List[TensorDesc]
    ops: List[OpDesc]

    def inputs(self) -> List[int]:
        """Inputs the caller passes by pointer (session inputs live in the arena instead)."""
        return [i for i, t in enumerate(self.tensors) if t.role == INPUT and not t.session]

    def session_inputs(self) -> List[int]:
        return [i for i, t in enumerate(self.tensors) if t.role == INPUT and t.session]

    def weights(self) -> List[int]:
        return [i for i, t in enumerate(self.tensors) if t.role == WEIGHT]

    def outputs(self) -> List[int]:
        return [i for i, t in enumerate(self.tensors) if t.is_output]

    def tensor_id(self, name: str) -> int:
        for i, t in enumerate(self.tensors):
            if t.name == name:
                return i
        raise KeyError(name)


class GraphBuilder:
    """Convenience front end that appends tensors and operators."""

    def __init__(self, symbols: Sequence[Tuple[str, int, int]]):
        self.g = GraphDesc(list(symbols), [], [])
        self._n = 0

    # -- tensors ---------------------------------------------------------
    def _add(self, t: TensorDesc) -> int:
        self.g.tensors.append(t)
        return len(self.g.tensors) - 1

    def input(self, name, dtype, dims) -> int:
        return self._add(TensorDesc(name, dtype, INPUT, None if dims is None else list(dims)))

    def session_input(self, name, dtype, dims, capacity) -> int:
        """A tensor that persists across calls (and across graphs that declare it alike): its storage is
        a fixed region at the bottom of the arena sized for ``capacity``; ``dims`` is what it holds now."""
        return self._add(TensorDesc(name, dtype, INPUT, list(dims), session=True, capacity=list(capacity)))

    def weight(self, name, dtype, dims) -> int:
        return self._add(TensorDesc(name, dtype, WEIGHT, list(dims)))

    def const(self, name, values, dtype="i64") -> int:
        np_dt = {"i64": np.int64, "i32": np.int32, "f32": np.float32}[dtype]
        arr = np.asarray(values, dtype=np_dt)
        return self._add(TensorDesc(name, dtype, HOSTCONST, list(arr.shape), arr))

    def _tmp(self, dtype, hint) -> int:
        self._n += 1
        return self._add(TensorDesc(f"{hint}_{self._n}", dtype))

    def mark_output(self, tid: int, name: Optional[str] = None) -> int:
        # Switch and Combine forward storage and write none: as a graph output their result gets a Cast to its own
        # type behind it, which makes the copy into the caller's buffer (the planners refuse the bare form)
        for op in self.g.ops:
            if op.kind in ("Switch", "Combine") and tid in op.outputs:
                tid = self.op("Cast", [tid], dtype=self.g.tensors[tid].dtype, hint="out")
                break
        self.g.tensors[tid].is_output = True
        if name:
            self.g.tensors[tid].name = name
        return tid

    # -- operators -------------------------------------------------------
    def op(self, kind, inputs, dtype=None, n_out=1, hint=None, **attrs):
        assert kind in OP_ATTRS, kind
        if dtype is None:
            dtype = self.g.tensors[inputs[0]].dtype
        outs = [self._tmp(dtype, hint or kind.lower()) for _ in range(n_out)]
        if kind == "CacheAppend":                       # the result lives on in the session storage of input 0
            self.g.tensors[outs[0]].session = True
        self.g.ops.append(OpDesc(kind, list(inputs), outs, dict(attrs)))
        return outs[0] if n_out == 1 else outs

    def build(self) -> GraphDesc:
        return self.g
