"""Unfused execution of the graph at concrete shapes: the value oracle.

Operators run one by one in the node order, each into a buffer of its own (no
arena, no fusion, no kernel versions).  Control flow uses dead tokens: Switch
leaves the branch it does not take dead, an operator with a dead input is not
run, Combine forwards its live input (Section 3, Fig. 1(d)).
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np

from . import ops as O

DEAD = "dead"


class Result:
    def __init__(self):
        self.values: Dict[int, object] = {}
        self.decisions: List[bool] = []       # one per executed Switch, True = skip branch taken
        self.logits: List[float] = []         # predicate value seen by each executed Switch
        self.state: Dict[str, np.ndarray] = {}   # session tensors after the run, by the session input's name
        self.exec_values: List[int] = []      # number of non-zeros found by each executed NonZero, in order


def run(graph, order: Sequence[int], weights: Dict[int, np.ndarray], inputs: Dict[int, np.ndarray],
        forced: Optional[Sequence[bool]] = None, round_weights=True,
        state: Optional[Dict[str, np.ndarray]] = None, exact: bool = False) -> Result:
    """``state``: contents of the session tensors (a KV cache) when the call starts, by name; a session
    input that is missing starts with zero rows.  ``Result.state`` is what the next call starts from.
    ``exact``: operator results (and the session state) stay in float64 instead of being rounded to the
    storage type of their tensor; weights and inputs are still what the storage holds.  This is the
    graph's plain definition; the default (every operator result rounded, as an unfused execution
    materialises it) differs from it by the rounding noise of the storage type."""
    g = graph
    res = Result()
    val = res.values
    root = {}                                 # session tensor id -> name of the session input it continues
    res.state = dict(state or {})
    for i, t in enumerate(g.tensors):
        if t.role == "input" and t.session:
            root[i] = t.name
            if t.name not in res.state:
                res.state[t.name] = np.zeros([0] + [int(d) for d in t.dims[1:]])
            st = np.asarray(res.state[t.name], np.float64)
            val[i] = st if exact else O.round_to(st, t.dtype)
        elif t.data is not None:
            val[i] = np.asarray(t.data, dtype=np.int64 if t.dtype in ("i64", "i32") else np.float64)
        elif i in weights:
            val[i] = O.round_to(np.asarray(weights[i], np.float64), t.dtype) if round_weights else weights[i]
        elif i in inputs:
            val[i] = O.round_to(np.asarray(inputs[i], np.float64), t.dtype)
    forced = list(forced) if forced is not None else None
    for n in order:
        op = g.ops[n]
        a = op.attrs
        xs = [val[t] for t in op.inputs]
        if op.kind == "Combine":
            live = [x for x in xs if x is not DEAD]
            val[op.outputs[0]] = live[0] if live else DEAD
            continue
        if any(x is DEAD for x in xs):
            for o in op.outputs:
                val[o] = DEAD
            continue
        if op.kind == "Switch":
            p = float(np.asarray(xs[1]).reshape(-1)[0])
            skip = p > a["threshold"]
            if forced is not None:
                skip = bool(forced.pop(0))
            res.decisions.append(bool(skip))
            res.logits.append(p)
            val[op.outputs[0]] = DEAD if skip else xs[0]
            val[op.outputs[1]] = xs[0] if skip else DEAD
            continue
        k = op.kind
        if k == "Shape":
            y = np.asarray(xs[0].shape, dtype=np.int64)
        elif k == "Gather":
            y = np.take(xs[0], np.asarray(xs[1], dtype=np.int64), axis=a["axis"])
        elif k == "Concat":
            y = np.concatenate(xs, axis=a["axis"])
        elif k == "Reshape":
            tgt = [xs[0].shape[i] if d == 0 else int(d) for i, d in enumerate(xs[1])]
            y = xs[0].reshape(tgt)
        elif k == "Slice":
            y = O.slice_(xs[0], xs[1], xs[2], [int(v) % xs[0].ndim for v in xs[3]])
        elif k == "Transpose":
            y = np.transpose(xs[0], a["perm"])
        elif k == "MatMul":
            y = O.matmul(xs[0], xs[1], a.get("transB", 0))
        elif k == "Conv":
            y = O.conv2d_nhwc(xs[0], xs[1], a["stride"], a["pad"])
        elif k == "Add":
            y = xs[0] + xs[1]
        elif k == "Mul":
            y = xs[0] * xs[1]
        elif k == "Relu":
            y = np.maximum(xs[0], 0.0)
        elif k == "Gelu":
            y = O.gelu(xs[0])
        elif k == "Sigmoid":
            y = O.sigmoid(xs[0])
        elif k == "Cast":
            y = xs[0]
        elif k == "Softmax":
            y = O.softmax(xs[0], a.get("causal", 0))
        elif k == "LayerNorm":
            y = O.layernorm(xs[0], xs[1], xs[2], a["eps"])
        elif k == "MaxUnpool":
            y = O.maxunpool(xs[0], xs[1], xs[2])
        elif k == "GroupNorm":
            y = O.groupnorm(xs[0], xs[1], xs[2], int(a["groups"]), a["eps"])
        elif k == "ReduceMean":
            y = xs[0].mean(axis=tuple(a["axes"]), keepdims=bool(a.get("keepdims", 1)))
        elif k == "MaxPool":
            y = O.maxpool_nhwc(xs[0], a["kernel"], a["stride"], a["pad"])
        elif k == "AveragePool":
            y = O.avgpool_nhwc(xs[0], a["kernel"], a["stride"], a["pad"])
        elif k == "Round":
            y = np.rint(xs[0])
        elif k == "ArgMax":
            y = np.argmax(xs[0], axis=-1)
        elif k == "CacheAppend":
            y = np.concatenate([xs[0], xs[1]], axis=0)
        elif k == "NonZero":
            y = O.nonzero(xs[0])
            res.exec_values.append(int(y.shape[1]))
        elif k == "NMS":
            y = O.nms(xs[0], xs[1], int(a.get("max_out", 0)), a["iou"])
            res.exec_values.append(int(y.shape[0]))
        elif k == "Range":
            y = np.arange(int(np.asarray(xs[0]).reshape(-1)[0]), int(np.asarray(xs[1]).reshape(-1)[0]),
                          int(np.asarray(xs[2]).reshape(-1)[0]), dtype=np.int64)
        elif k == "Expand":
            tgt = np.broadcast_shapes(xs[0].shape, tuple(int(v) for v in xs[1]))
            y = np.broadcast_to(xs[0], tgt)
        elif k == "Resize":
            y = O.resize_nearest(xs[0], xs[1])
        elif k == "TopK":
            vals, idx = O.topk(xs[0], int(np.asarray(xs[1]).reshape(-1)[0]))
            val[op.outputs[1]] = idx
            y = vals
        elif k == "Upsample":
            y = O.resize_nearest(xs[0], [int(d) * int(f) for d, f in zip(xs[0].shape, np.asarray(xs[1]).reshape(-1))])
        elif k == "ConstantOfShape":
            y = np.full(tuple(int(v) for v in np.asarray(xs[0]).reshape(-1)), float(a.get("value", 0.0)))
        elif k == "EyeLike":
            y = np.eye(xs[0].shape[0], xs[0].shape[1], k=int(a.get("k", 0)))
        elif k == "OneHot":
            depth = int(np.asarray(xs[1]).reshape(-1)[0])
            off, on = (float(v) for v in np.asarray(xs[2]).reshape(-1))
            idx = np.asarray(xs[0], dtype=np.int64)
            idx = np.where(idx < 0, idx + depth, idx)
            y = np.where(idx[..., None] == np.arange(depth), on, off)
        elif k == "ScatterRows":
            y = np.array(xs[0], copy=True)
            for j, r in enumerate(np.asarray(xs[1], dtype=np.int64).reshape(-1)):
                y[int(r)] = xs[2][j]
        else:
            raise ValueError(k)
        od = g.tensors[op.outputs[0]].dtype
        val[op.outputs[0]] = np.asarray(y, np.float64) if (exact and od in ("f32", "bf16")) else O.round_to(np.asarray(y), od)
        if k == "CacheAppend":
            root[op.outputs[0]] = root[op.inputs[0]]
            res.state[root[op.outputs[0]]] = val[op.outputs[0]]
    return res
