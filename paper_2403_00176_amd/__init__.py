"""Python binding of libsod2 (argument marshalling only; every step runs in the library).

The functions carry the names of the C entry points (see include/sod2.h):
sod2_graph_build, sod2_rdp_infer, sod2_plan, sod2_bind, sod2_run and the queries.
The library must have been built (``python -m paper_2403_00176_amd.build`` or
``__graft_entry__.build()``); importing fails loudly otherwise.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch  # noqa: F401  -- first, so that libsod2 binds to the HIP runtime torch has already loaded

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsod2.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2403_00176_amd.build`")
_lib = C.CDLL(LIB_PATH)

DTYPES = {"f32": 0, "bf16": 1, "i64": 2, "i32": 3}
ROLES = {"inter": 0, "input": 1, "weight": 2, "hostconst": 3}
OP_KINDS = ["Shape", "Gather", "Concat", "Reshape", "Slice", "Transpose", "MatMul", "Conv", "Add", "Mul",
            "Relu", "Gelu", "Sigmoid", "Cast", "Softmax", "LayerNorm", "ReduceMean", "MaxPool", "ArgMax",
            "CacheAppend", "NonZero", "Switch", "Combine", "ScatterRows", "Resize", "Range", "Expand",
            "Upsample", "ConstantOfShape", "EyeLike", "OneHot", "TopK", "GroupNorm", "MaxUnpool", "AveragePool", "Round", "NMS"]
OP_CLASS_NAMES = ["ISDO", "ISDOS", "ISVDOS", "EDO"]

EXPORTS = [
    "sod2_graph_build", "sod2_graph_destroy", "sod2_graph_op_class", "sod2_op_kind_class", "sod2_rdp_infer", "sod2_rdp_infer_ordered",
    "sod2_rdp_destroy", "sod2_rdp_query", "sod2_rdp_sweeps", "sod2_rdp_dump", "sod2_plan", "sod2_plan_destroy",
    "sod2_plan_counts", "sod2_plan_dump", "sod2_plan_query_group", "sod2_bind", "sod2_bind_decided", "sod2_bind_executed",
    "sod2_binding_destroy",
    "sod2_binding_arena_bytes", "sod2_binding_dump", "sod2_binding_query_tensor", "sod2_run_query_tensor", "sod2_run_trace", "sod2_binding_force_decisions", "sod2_binding_force_variant",
    "sod2_binding_force_splits", "sod2_binding_workspace_bytes",
    "sod2_plan_constants_bytes", "sod2_plan_prepare_constants", "sod2_binding_set_constants",
    "sod2_run", "sod2_run_static", "sod2_run_decisions", "sod2_run_exec_values", "sod2_run_plan_dump", "sod2_run_arena_bytes", "sod2_binding_set_profiling",
    "sod2_binding_launch_records", "sod2_replay_create", "sod2_replay_launch", "sod2_replay_destroy",
    "sod2_last_error", "sod2_version",
]


class Sod2Error(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"sod2 error {code}: {msg}")
        self.code = code


class _TensorDesc(C.Structure):
    _fields_ = [("name", C.c_char_p), ("dtype", C.c_int32), ("role", C.c_int32), ("rank", C.c_int32),
                ("dims", C.POINTER(C.c_char_p)), ("host_data", C.c_void_p), ("host_count", C.c_int64),
                ("is_output", C.c_int32), ("session", C.c_int32), ("capacity_dims", C.POINTER(C.c_char_p))]


class _OpDesc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("n_inputs", C.c_int32), ("inputs", C.POINTER(C.c_int32)),
                ("n_outputs", C.c_int32), ("outputs", C.POINTER(C.c_int32)), ("n_iattr", C.c_int32),
                ("iattr", C.POINTER(C.c_int64)), ("fattr", C.c_double)]


class _GraphDesc(C.Structure):
    _fields_ = [("n_symbols", C.c_int32), ("symbol_names", C.POINTER(C.c_char_p)),
                ("symbol_lo", C.POINTER(C.c_int64)), ("symbol_hi", C.POINTER(C.c_int64)),
                ("n_tensors", C.c_int32), ("tensors", C.POINTER(_TensorDesc)),
                ("n_ops", C.c_int32), ("ops", C.POINTER(_OpDesc))]


class PlanOpts(C.Structure):
    _fields_ = [("fusion", C.c_int32), ("sep", C.c_int32), ("dmp", C.c_int32), ("mvc", C.c_int32),
                ("inplace", C.c_int32), ("max_versions", C.c_int32), ("attn_head_dim", C.c_int32),
                ("append_max_rows", C.c_int32), ("prologue_max_rows", C.c_int32), ("prologue_max_k", C.c_int32),
                ("prologue_k_multiple", C.c_int32), ("fold_ln", C.c_int32), ("fold_k_multiple", C.c_int32)]


class DimInfo(C.Structure):
    _fields_ = [("cls", C.c_int32), ("value", C.c_int64), ("expr", C.c_char * 120)]


class LaunchRecord(C.Structure):
    _fields_ = [("group", C.c_int32), ("kernel", C.c_int32), ("variant", C.c_int32), ("reserved", C.c_int32),
                ("ms", C.c_float), ("flops", C.c_double), ("bytes", C.c_double)]


KERNEL_NAMES = ["gemm", "conv", "layernorm", "softmax", "eltwise", "pool", "reduce", "other", "gather", "append", "argmax", "attention",
                "nonzero", "scatter", "resize", "concat", "range", "fill", "onehot", "topk", "groupnorm", "maxunpool", "nms"]

_lib.sod2_last_error.restype = C.c_char_p
_lib.sod2_version.restype = C.c_char_p
for _n in EXPORTS:
    if _n not in ("sod2_last_error", "sod2_version") and not _n.endswith("_destroy"):
        getattr(_lib, _n).restype = C.c_int32
for _n in ("sod2_graph_destroy", "sod2_rdp_destroy", "sod2_plan_destroy", "sod2_binding_destroy", "sod2_replay_destroy"):
    getattr(_lib, _n).restype = None
    getattr(_lib, _n).argtypes = [C.c_void_p]


def _check(rc):
    if rc != 0:
        raise Sod2Error(rc, _lib.sod2_last_error().decode())


def _attrs(kind: str, attrs: dict):
    ia: List[int] = []
    fa = 0.0
    if kind in ("Gather", "Concat"):
        ia = [int(attrs["axis"])]
    elif kind == "Transpose":
        ia = [int(v) for v in attrs["perm"]]
    elif kind == "MatMul":
        ia = [int(attrs.get("transB", 0))]
    elif kind == "Conv":
        ia = [int(attrs["stride"]), int(attrs["pad"])]
    elif kind == "Softmax":
        ia = [int(attrs.get("causal", 0))]
    elif kind == "ReduceMean":
        ia = [int(attrs.get("keepdims", 1))] + [int(a) for a in attrs["axes"]]
    elif kind in ("MaxPool", "AveragePool"):
        ia = [int(attrs["kernel"]), int(attrs["stride"]), int(attrs["pad"])]
    elif kind == "LayerNorm":
        fa = float(attrs["eps"])
    elif kind == "Switch":
        fa = float(attrs["threshold"])
    elif kind == "ConstantOfShape":
        fa = float(attrs.get("value", 0.0))
    elif kind == "EyeLike":
        ia = [int(attrs.get("k", 0))]
    elif kind == "NMS":
        ia = [int(attrs.get("max_out", 0))]
        fa = float(attrs["iou"])
    elif kind == "GroupNorm":
        ia = [int(attrs["groups"])]
        fa = float(attrs["eps"])
    return ia, fa


class _Handle:
    _destroy = None

    def __init__(self, ptr, keep=()):
        self.ptr = ptr
        self._keep = keep

    def __del__(self):
        if getattr(self, "ptr", None) and _lib is not None:      # _lib is gone at interpreter exit
            getattr(_lib, self._destroy)(self.ptr)
            self.ptr = None


class Graph(_Handle):
    _destroy = "sod2_graph_destroy"


class Rdp(_Handle):
    _destroy = "sod2_rdp_destroy"


class Plan(_Handle):
    _destroy = "sod2_plan_destroy"


class Binding(_Handle):
    _destroy = "sod2_binding_destroy"


def sod2_graph_build(desc) -> Graph:
    """desc: a workloads.GraphDesc-like object (symbols, tensors, ops)."""
    keep = []

    def cstr(s):
        b = C.c_char_p(str(s).encode())
        keep.append(b)
        return b

    ns = len(desc.symbols)
    names = (C.c_char_p * max(ns, 1))(*[str(s[0]).encode() for s in desc.symbols])
    lo = (C.c_int64 * max(ns, 1))(*[int(s[1]) for s in desc.symbols])
    hi = (C.c_int64 * max(ns, 1))(*[int(s[2]) for s in desc.symbols])
    tds = (_TensorDesc * max(len(desc.tensors), 1))()
    for i, t in enumerate(desc.tensors):
        td = tds[i]
        td.name = str(t.name).encode()
        td.dtype = DTYPES[t.dtype]
        td.role = ROLES[t.role]
        td.is_output = int(t.is_output)
        td.session = int(getattr(t, "session", False))
        if t.dims is None:
            td.rank = -1
        else:
            td.rank = len(t.dims)
            arr = (C.c_char_p * max(len(t.dims), 1))(*[str(d).encode() for d in t.dims])
            keep.append(arr)
            td.dims = arr
            cap = getattr(t, "capacity", None)
            if cap is not None:
                carr = (C.c_char_p * max(len(cap), 1))(*[str(d).encode() for d in cap])
                keep.append(carr)
                td.capacity_dims = carr
        if t.data is not None:
            np_dt = {"i64": np.int64, "i32": np.int32, "f32": np.float32}[t.dtype]
            a = np.ascontiguousarray(t.data, dtype=np_dt)
            keep.append(a)
            td.host_data = a.ctypes.data
            td.host_count = a.size
    ods = (_OpDesc * max(len(desc.ops), 1))()
    for i, op in enumerate(desc.ops):
        od = ods[i]
        od.kind = OP_KINDS.index(op.kind)
        ins = (C.c_int32 * max(len(op.inputs), 1))(*op.inputs)
        outs = (C.c_int32 * max(len(op.outputs), 1))(*op.outputs)
        ia, fa = _attrs(op.kind, op.attrs)
        iarr = (C.c_int64 * max(len(ia), 1))(*ia)
        keep += [ins, outs, iarr]
        od.n_inputs, od.inputs = len(op.inputs), ins
        od.n_outputs, od.outputs = len(op.outputs), outs
        od.n_iattr, od.iattr, od.fattr = len(ia), iarr, fa
    gd = _GraphDesc(ns, names, lo, hi, len(desc.tensors), tds, len(desc.ops), ods)
    out = C.c_void_p()
    _check(_lib.sod2_graph_build(C.byref(gd), C.byref(out)))
    g = Graph(out)
    g.desc = desc
    return g


def sod2_graph_op_class(g: Graph, op: int) -> str:
    c = C.c_int32()
    _check(_lib.sod2_graph_op_class(g.ptr, op, C.byref(c)))
    return OP_CLASS_NAMES[c.value]


def sod2_op_kind_class(kind: str) -> str:
    c = C.c_int32()
    _check(_lib.sod2_op_kind_class(OP_KINDS.index(kind), C.byref(c)))
    return OP_CLASS_NAMES[c.value]


def sod2_rdp_infer(g: Graph, order: Optional[Sequence[int]] = None) -> Rdp:
    out = C.c_void_p()
    if order is None:
        _check(_lib.sod2_rdp_infer(g.ptr, C.byref(out)))
    else:
        arr = (C.c_int32 * len(order))(*order)
        _check(_lib.sod2_rdp_infer_ordered(g.ptr, arr, len(order), C.byref(out)))
    return Rdp(out, keep=(g,))


def sod2_rdp_query(r: Rdp, tensor: int):
    rank = C.c_int32()
    dims = (DimInfo * 8)()
    _check(_lib.sod2_rdp_query(r.ptr, tensor, C.byref(rank), dims))
    return rank.value, [(d.cls, d.value, d.expr.decode()) for d in dims[:max(rank.value, 0)]]


def sod2_rdp_sweeps(r: Rdp) -> int:
    n = C.c_int32()
    _check(_lib.sod2_rdp_sweeps(r.ptr, C.byref(n)))
    return n.value


def _text(fn, ptr) -> str:
    need = C.c_size_t()
    fn(ptr, None, 0, C.byref(need))
    buf = C.create_string_buffer(need.value)
    _check(fn(ptr, buf, need.value, C.byref(need)))
    return buf.value.decode()


def sod2_rdp_dump(r: Rdp) -> str:
    return _text(_lib.sod2_rdp_dump, r.ptr)


def sod2_plan(g: Graph, r: Rdp, fusion=1, sep=1, dmp=1, mvc=1, inplace=1, max_versions=0, attn_head_dim=0,
              append_max_rows=0, prologue_max_rows=0, prologue_max_k=0, prologue_k_multiple=0, fold_ln=1,
              fold_k_multiple=0) -> Plan:
    """The last six options are limits of the fusion rules; 0 = the library's default (see sod2_plan_opts)."""
    out = C.c_void_p()
    opts = PlanOpts(int(fusion), int(sep), int(dmp), int(mvc), int(inplace), int(max_versions), int(attn_head_dim),
                    int(append_max_rows), int(prologue_max_rows), int(prologue_max_k), int(prologue_k_multiple),
                    int(fold_ln), int(fold_k_multiple))
    _check(_lib.sod2_plan(g.ptr, r.ptr, C.byref(opts), C.byref(out)))
    p = Plan(out, keep=(g, r))
    p.graph = g
    return p


def sod2_plan_counts(p: Plan):
    a, b, c = C.c_int32(), C.c_int32(), C.c_int32()
    _check(_lib.sod2_plan_counts(p.ptr, C.byref(a), C.byref(b), C.byref(c)))
    return a.value, b.value, c.value


def sod2_plan_dump(p: Plan) -> str:
    return _text(_lib.sod2_plan_dump, p.ptr)


def _symbols(p: Plan, sym) -> "C.Array":
    if isinstance(sym, dict):
        sym = [sym[s[0]] for s in p.graph.desc.symbols]
    return (C.c_int64 * max(len(sym), 1))(*[int(v) for v in sym]), len(sym)


def sod2_bind(p: Plan, sym, decisions: Optional[Sequence[int]] = None,
              exec_values: Optional[Sequence[int]] = None) -> Binding:
    """decisions / exec_values: plan for given Switch decisions / NonZero counts (no run needed)."""
    arr, n = _symbols(p, sym)
    out = C.c_void_p()
    if decisions is None and exec_values is None:
        _check(_lib.sod2_bind(p.ptr, arr, n, C.byref(out)))
    elif exec_values is not None:
        decisions = decisions or []
        d = (C.c_int32 * max(len(decisions), 1))(*[int(bool(v)) for v in decisions])
        e = (C.c_int64 * max(len(exec_values), 1))(*[int(v) for v in exec_values])
        _check(_lib.sod2_bind_executed(p.ptr, arr, n, d, len(decisions), e, len(exec_values), C.byref(out)))
    else:
        d = (C.c_int32 * max(len(decisions), 1))(*[int(bool(v)) for v in decisions])
        _check(_lib.sod2_bind_decided(p.ptr, arr, n, d, len(decisions), C.byref(out)))
    b = Binding(out, keep=(p,))
    b.plan = p
    return b


def sod2_binding_arena_bytes(b: Binding):
    a, pk = C.c_size_t(), C.c_size_t()
    _check(_lib.sod2_binding_arena_bytes(b.ptr, C.byref(a), C.byref(pk)))
    return a.value, pk.value


def sod2_run_arena_bytes(b: Binding):
    a, pk = C.c_size_t(), C.c_size_t()
    _check(_lib.sod2_run_arena_bytes(b.ptr, C.byref(a), C.byref(pk)))
    return a.value, pk.value


def sod2_binding_dump(b: Binding) -> str:
    return _text(_lib.sod2_binding_dump, b.ptr)


def sod2_run_plan_dump(b: Binding) -> str:
    return _text(_lib.sod2_run_plan_dump, b.ptr)


def sod2_binding_force_decisions(b: Binding, decisions: Sequence[int]):
    d = (C.c_int32 * max(len(decisions), 1))(*[int(bool(v)) for v in decisions])
    _check(_lib.sod2_binding_force_decisions(b.ptr, d, len(decisions)))


def sod2_binding_force_variant(b: Binding, variant: int):
    _check(_lib.sod2_binding_force_variant(b.ptr, int(variant)))


def sod2_binding_force_splits(b: Binding, n: int):
    _check(_lib.sod2_binding_force_splits(b.ptr, int(n)))


def sod2_binding_workspace_bytes(b: Binding) -> int:
    n = C.c_size_t()
    _check(_lib.sod2_binding_workspace_bytes(b.ptr, C.byref(n)))
    return n.value


def sod2_plan_constants_bytes(p) -> int:
    n = C.c_size_t()
    _check(_lib.sod2_plan_constants_bytes(p.ptr, C.byref(n)))
    return n.value


def sod2_plan_prepare_constants(p, weight_ptrs: Sequence[int], constants_ptr: int, nbytes: int, stream: int = 0):
    """Computes the plan's derived constants (device memory of the caller) from the weights, on ``stream``."""
    w = weight_ptrs if isinstance(weight_ptrs, C.Array) else pointer_array(weight_ptrs)
    _check(_lib.sod2_plan_prepare_constants(p.ptr, w, len(weight_ptrs), C.c_void_p(constants_ptr), C.c_size_t(nbytes),
                                            C.c_void_p(stream)))


def sod2_binding_set_constants(b: Binding, constants_ptr: int, nbytes: int):
    _check(_lib.sod2_binding_set_constants(b.ptr, C.c_void_p(constants_ptr or None), C.c_size_t(nbytes)))


def sod2_binding_set_profiling(b: Binding, on: bool):
    _check(_lib.sod2_binding_set_profiling(b.ptr, int(on)))


def sod2_binding_launch_records(b: Binding):
    n = C.c_int32()
    _check(_lib.sod2_binding_launch_records(b.ptr, None, 0, C.byref(n)))
    recs = (LaunchRecord * max(n.value, 1))()
    _check(_lib.sod2_binding_launch_records(b.ptr, recs, n.value, C.byref(n)))
    return [dict(group=r.group, kernel=KERNEL_NAMES[r.kernel], variant=r.variant, ms=r.ms, flops=r.flops,
                 bytes=r.bytes) for r in recs[:n.value]]


def sod2_run_decisions(b: Binding) -> List[int]:
    n = C.c_int32()
    _check(_lib.sod2_run_decisions(b.ptr, None, 0, C.byref(n)))
    arr = (C.c_int32 * max(n.value, 1))()
    _check(_lib.sod2_run_decisions(b.ptr, arr, n.value, C.byref(n)))
    return list(arr[:n.value])


def pointer_array(ptrs: Sequence[int]):
    """Device addresses as the `const void* const*` argument of sod2_run (reusable across calls)."""
    return (C.c_void_p * len(ptrs))(*ptrs)


def sod2_run_exec_values(b: Binding) -> List[int]:
    n = C.c_int32()
    _check(_lib.sod2_run_exec_values(b.ptr, None, 0, C.byref(n)))
    arr = (C.c_int64 * max(n.value, 1))()
    _check(_lib.sod2_run_exec_values(b.ptr, arr, n.value, C.byref(n)))
    return list(arr[:n.value])


def sod2_run(b: Binding, arena_ptr: int, arena_bytes: int, weight_ptrs: Sequence[int], input_ptrs: Sequence[int],
             output_ptrs: Sequence[int], stream: int = 0):
    """All pointers are raw device addresses (e.g. torch.Tensor.data_ptr()); stream is a hipStream_t value.
    weight_ptrs may be an array made once by pointer_array()."""
    w = weight_ptrs if isinstance(weight_ptrs, C.Array) else pointer_array(weight_ptrs)
    i = (C.c_void_p * max(len(input_ptrs), 1))(*input_ptrs)
    o = (C.c_void_p * max(len(output_ptrs), 1))(*output_ptrs)
    _check(_lib.sod2_run(b.ptr, C.c_void_p(arena_ptr), C.c_size_t(arena_bytes), w, len(weight_ptrs), i,
                         len(input_ptrs), o, len(output_ptrs), C.c_void_p(stream)))


STATIC_SCRATCH_BYTES = 8 << 20

GROUP_KINDS = ["GEMM", "CONV", "LAYERNORM", "SOFTMAX", "MAXPOOL", "REDUCEMEAN", "ARGMAX", "CACHEAPPEND", "NONZERO", "GATHER",
               "ELTWISE", "ATTENTION", "SCATTER", "RESIZE", "CONCAT", "RANGE", "FILL", "ONEHOT", "TOPK", "GROUPNORM", "MAXUNPOOL", "AVGPOOL", "NMS", "COPY"]
SG_CLASSES = ["known", "mixed", "nac"]


class GroupInfo(C.Structure):
    _fields_ = [("gid", C.c_int32), ("kind", C.c_int32), ("out", C.c_int32), ("out2", C.c_int32), ("n_ops", C.c_int32),
                ("n_ins", C.c_int32), ("subgraph", C.c_int32), ("sg_class", C.c_int32), ("inplace_of", C.c_int32),
                ("versions", C.c_int32)]


class TensorInfo(C.Structure):
    _fields_ = [("executed", C.c_int32), ("where", C.c_int32), ("base", C.c_int32), ("rank", C.c_int32),
                ("dims", C.c_int64 * 8), ("offset", C.c_int64), ("bytes", C.c_int64), ("life_start", C.c_int32),
                ("life_end", C.c_int32)]


class TraceEntry(C.Structure):
    _fields_ = [("is_group", C.c_int32), ("ref", C.c_int32), ("kernel", C.c_int32), ("variant", C.c_int32),
                ("splits", C.c_int32), ("decision", C.c_int32), ("fold", C.c_int32)]


def sod2_plan_query_group(p: "Plan", index: int) -> dict:
    """Group `index` (planned execution order) as a dict: gid, kind, out, out2, ops, ins, subgraph, sg_class, ..."""
    info = GroupInfo()
    _check(_lib.sod2_plan_query_group(p.ptr, index, C.byref(info), None, 0, None, 0))
    ops = (C.c_int32 * max(info.n_ops, 1))()
    ins = (C.c_int32 * max(info.n_ins, 1))()
    _check(_lib.sod2_plan_query_group(p.ptr, index, C.byref(info), ops, info.n_ops, ins, info.n_ins))
    return dict(gid=info.gid, kind=GROUP_KINDS[info.kind], out=info.out, out2=info.out2, ops=list(ops[:info.n_ops]),
                ins=list(ins[:info.n_ins]), subgraph=info.subgraph, sg_class=SG_CLASSES[info.sg_class],
                inplace_of=info.inplace_of, versions=info.versions)


def _tensor_info(fn, b: "Binding", tensor: int) -> dict:
    info = TensorInfo()
    _check(fn(b.ptr, int(tensor), C.byref(info)))
    return dict(executed=bool(info.executed), where=["arena", "session", "inplace", "external"][info.where], base=info.base,
                dims=list(info.dims[:info.rank]), offset=info.offset, bytes=info.bytes, life=(info.life_start, info.life_end))


def sod2_binding_query_tensor(b: "Binding", tensor: int) -> dict:
    return _tensor_info(_lib.sod2_binding_query_tensor, b, tensor)


def sod2_run_query_tensor(b: "Binding", tensor: int) -> dict:
    return _tensor_info(_lib.sod2_run_query_tensor, b, tensor)


def sod2_run_trace(b: "Binding") -> list:
    """Executed steps of the last run: dicts with is_group, ref, kernel, variant, splits, decision, fold."""
    n = C.c_int32()
    _check(_lib.sod2_run_trace(b.ptr, None, 0, C.byref(n)))
    arr = (TraceEntry * max(n.value, 1))()
    _check(_lib.sod2_run_trace(b.ptr, arr, n.value, C.byref(n)))
    return [dict(is_group=bool(e.is_group), ref=e.ref, kernel=e.kernel, variant=e.variant, splits=e.splits, decision=e.decision,
                 fold=e.fold)
            for e in arr[:n.value]]


def sod2_run_static(b: Binding, arena_ptr: int, arena_bytes: int, weight_ptrs: Sequence[int], input_ptrs: Sequence[int],
                    output_ptrs: Sequence[int], stream: int = 0):
    """sod2_run for callers that cannot allocate: split-K partials go to the library's static device buffer."""
    w = weight_ptrs if isinstance(weight_ptrs, C.Array) else pointer_array(weight_ptrs)
    i = (C.c_void_p * max(len(input_ptrs), 1))(*input_ptrs)
    o = (C.c_void_p * max(len(output_ptrs), 1))(*output_ptrs)
    _check(_lib.sod2_run_static(b.ptr, C.c_void_p(arena_ptr), C.c_size_t(arena_bytes), w, len(weight_ptrs), i,
                                len(input_ptrs), o, len(output_ptrs), C.c_void_p(stream)))


class Replay(_Handle):
    _destroy = "sod2_replay_destroy"


def sod2_replay_create(p: Plan, sym, step_symbol: str, max_steps: int, arena_ptr: int, arena_bytes: int,
                       weight_ptrs: Sequence[int], input_ptrs: Sequence[int], input_step_bytes: Sequence[int],
                       output_ptrs: Sequence[int], output_step_bytes: Sequence[int], step_counter_ptr: int,
                       stream: int) -> Replay:
    arr, n = _symbols(p, sym)
    names = [s[0] for s in p.graph.desc.symbols]
    w = (C.c_void_p * max(len(weight_ptrs), 1))(*weight_ptrs)
    i = (C.c_void_p * max(len(input_ptrs), 1))(*input_ptrs)
    o = (C.c_void_p * max(len(output_ptrs), 1))(*output_ptrs)
    isb = (C.c_int64 * max(len(input_ptrs), 1))(*[int(v) for v in input_step_bytes])
    osb = (C.c_int64 * max(len(output_ptrs), 1))(*[int(v) for v in output_step_bytes])
    out = C.c_void_p()
    _check(_lib.sod2_replay_create(p.ptr, arr, n, names.index(step_symbol), int(max_steps), C.c_void_p(arena_ptr),
                                   C.c_size_t(arena_bytes), w, len(weight_ptrs), i, isb, len(input_ptrs), o, osb,
                                   len(output_ptrs), C.c_void_p(step_counter_ptr), C.c_void_p(stream), C.byref(out)))
    return Replay(out, keep=(p,))


def sod2_replay_launch(r: Replay, first_step: int, n_steps: int, stream: int):
    _check(_lib.sod2_replay_launch(r.ptr, int(first_step), int(n_steps), C.c_void_p(stream)))


def sod2_version() -> str:
    return _lib.sod2_version().decode()
