"""Static planning on top of RDP: fusion groups (Section 4.2), sub-graph
partition and execution order (Section 4.3).

The paper delegates the fusion rules to an earlier system and gives the
partition and the search only in outline, so the concrete rules below are this
build's reading; the library follows the same written rules independently.

R0  An operator whose outputs are all integer tensors with a fully resolved
    value map is *folded*: its result is known from RDP (Fig. 1(a)), nothing runs.
R1  Reshape, Slice, Transpose, Expand and Gather-with-a-scalar-host-index are *views*:
    their output aliases the input's storage; no kernel, no arena tensor.  One
    whose result is a graph output is a group of its own (COPY): the view is
    written out densely into the caller's buffer.  Likewise an operator with a
    known value map is not folded when its result is a graph output.  A view that
    a kernel could not walk is a COPY group too (its result an arena tensor): a
    strided view (a permutation, a slice or index of a dim other than the first,
    an Expand, or a view of such a view) read by an operator whose kernel wants
    dense operands (Concat, ReduceMean, pools, GroupNorm, Conv, the table of a
    Gather by an index tensor, ...), and a permuted view read by LayerNorm,
    Softmax or Reshape (regrouping the dims of a permutation needs its elements
    in the new order).  "Read by" looks through Switch and Combine, which hand
    the storage on under another name.
R2  MatMul / Conv seeds a group and absorbs the chain of its sole consumers, in
    this order and each at most once: Mul by a host scalar; Add of a rank-1
    weight equal to the last dim (bias); activation; Add of a non-constant
    tensor whose shape RDP proves equal to the output's (residual);
    activation; Transpose (stored permuted).  The chain stops at the first
    operator that does not fit.  With fusion switched off only a directly
    following Transpose is still taken: the permuted store is a layout choice
    of the contraction, and without it the Reshape behind it would need a copy.
R3  LayerNorm, GroupNorm, MaxUnpool, Softmax, MaxPool, AveragePool, ReduceMean, ArgMax, CacheAppend, NonZero, NMS,
    ScatterRows, Resize, Upsample, OneHot, TopK (one group, two results), and a Concat, Range, ConstantOfShape or EyeLike that is not folded are groups of their own; a non-view Gather absorbs one following Add whose
    other operand has a proven-equal shape.
R4  Remaining elementwise operators chain, up to 8 ops (a Round joins a chain
    only behind an fp32 value, otherwise it starts one: it has to round what
    would have been stored).  An aligned dim pair of
    the two operands of a binary member is *proven* when RDP shows the two
    extents equal or one of them 1 (the condition of Fig. 4): the fused loop nest
    then has one form.  A pair of two resolved but unrelated extents is
    *unproven*: each such pair doubles the number of code versions of the fused
    nest (Fig. 4: 8 versions for three unproven pairs), of which one is selected
    when the symbols are bound (Section 4.2).  The chain stops before the member
    that would take the group beyond ``Opts.max_versions`` versions (8, the
    largest bucket of Fig. 8; 1 = fuse proven chains only), and at any pair with
    an unresolved extent.  A group of a single operator has one version (the
    plain operator with run-time broadcast strides).
R5  Group id = smallest operator id in it; groups are ordered by the position
    of their last member in the node order (a topological order of groups).
R6  Attention: a GEMM group that is only MatMul [+ Mul by a host scalar], whose
    result is read by one Softmax alone, whose result in turn is the first
    operand of one MatMul alone that leads a GEMM group of MatMul [+ Transpose]:
    the three groups become one ATTENTION group (scores and probabilities are
    never materialised: Section 4.2, fusion reduces the materialisation of
    intermediate results).  Only for bf16 tensors with a known head size among
    ``Opts.attn_head_dims`` (what the executing backend declares it can fuse).
R8  Cache append inside attention: when the key operand and the value operand
    of an ATTENTION group are, through views only and with no other reader, the
    results of two CacheAppend operators that each append a known number of at
    most ``Opts.append_max_rows`` bf16 rows (the decode step), the two CACHEAPPEND groups join the
    ATTENTION group: its kernel writes the new rows into the session slots and
    reads them from where they were produced.
R7  LayerNorm as a prologue: a LAYERNORM group whose result is read by one
    MatMul alone, as its first operand, joins that MatMul's GEMM group when the
    row count is a known constant of at most ``Opts.prologue_max_rows`` (the
    decode step), the normalised dim (= the contraction dim) is a known constant
    of at most ``Opts.prologue_max_k`` and a multiple of
    ``Opts.prologue_k_multiple``, and everything is bf16.  The LayerNorm result
    is never materialised.
R9  LayerNorm behind a contraction: a LAYERNORM group whose input is the result
    of a GEMM group (MatMul with any epilogue but a permuted store; no LayerNorm
    prologue, no second result yet) and whose result is read by one MatMul alone
    -- as its first operand, against a rank-2 weight [n, k] stored k-contiguous,
    leading its GEMM group -- joins the *producing* group: that group gets a
    second result, the LayerNorm's tensor, and the consuming group is marked
    (``lnfold``).  Everything bf16; the normalised extent a known constant that
    is a multiple of ``Opts.fold_k_multiple``.  What the producing kernel writes
    into the second result is its business (the normalised rows, or the rows
    scaled by gamma together with per-row partial sums from which the consumer
    finishes the normalisation in its epilogue): the tensor is sized for the
    latter, 2.25 bytes per element instead of 2 (per row and 32 columns an
    8-byte pair of partial sums).  The group keeps its place in the order.
The limits of R6-R9 are capabilities of whatever executes the plan, handed in
with the options (the same numbers go to the library's planner); they shape
the groups, never a value.

Execution-determined extents (Section 4.3: what follows an EDO can only be
planned once it has executed).  When the graph holds a NonZero or an NMS the plan uses
the analysis with *named* EDO extents (``RDP(named_edo=True)``): sizes after
such an operator are expressions in its execution symbol, evaluated at run time as
soon as the count is known.  A tensor that is nac or mentions an execution
symbol counts as nac for the partition: a cut follows every item that writes
one, and such sub-graphs keep the node order (no search).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

from .expr import Expr
from . import rdp as R

ALIGN = 256
MAX_SG = 14
DT_BYTES = {"f32": 4, "bf16": 2, "i64": 8, "i32": 4}
VIEW_KINDS = ("Reshape", "Slice", "Transpose", "Expand")
ACTS = ("Relu", "Gelu", "Sigmoid")
DENSE_ONLY = ("Concat", "ReduceMean", "MaxPool", "AveragePool", "GroupNorm", "Conv", "MaxUnpool", "Resize", "Upsample",
              "ScatterRows", "TopK", "ArgMax", "NonZero", "NMS")        # operators whose kernels want dense operands
ROW_OPS = ("LayerNorm", "Softmax")                 # a dense last dim and evenly spaced rows suffice: a permutation breaks that
COUNTING = ("NonZero", "NMS")                  # execution-determined operators whose result has a length found by running
COUNTING_GROUPS = ("NONZERO", "NMS")
ELTWISE = ("Add", "Mul", "Relu", "Gelu", "Sigmoid", "Cast", "Round")
SOLO = {"LayerNorm": "LAYERNORM", "Softmax": "SOFTMAX", "MaxPool": "MAXPOOL",
        "ReduceMean": "REDUCEMEAN", "ArgMax": "ARGMAX", "CacheAppend": "CACHEAPPEND",
        "NonZero": "NONZERO", "NMS": "NMS", "ScatterRows": "SCATTER", "Resize": "RESIZE", "Concat": "CONCAT", "Range": "RANGE",
        "Upsample": "RESIZE", "ConstantOfShape": "FILL", "EyeLike": "FILL", "OneHot": "ONEHOT", "TopK": "TOPK", "GroupNorm": "GROUPNORM", "MaxUnpool": "MAXUNPOOL",
        "AveragePool": "AVGPOOL"}


@dataclass
class Opts:
    fusion: bool = True      # RDP-enabled fusion (R2-R4); off: every operator is its own group
    sep: bool = True         # static execution planning; off: node order
    dmp: bool = True         # peak-first arena plan; off: best-fit greedy in execution order
    mvc: bool = True         # multi-version kernels (library only; no effect on structure)
    inplace: bool = True     # a group's result may take over the storage of an operand that dies there
    max_versions: int = 8    # R4: most code versions a fused elementwise group may need (1: proven chains only)
    # what the executing backend can fuse (R6-R8); structure only
    attn_head_dims: tuple = (64,)
    append_max_rows: int = 4
    prologue_max_rows: int = 8
    prologue_max_k: int = 1024
    prologue_k_multiple: int = 64
    fold_ln: bool = True     # R9: a LayerNorm behind a contraction becomes that contraction's second result
    fold_k_multiple: int = 64


@dataclass
class Group:
    gid: int
    kind: str
    ops: List[int]
    out: int                              # tensor id written by the group
    ins: List[int] = field(default_factory=list)   # base tensors read from outside the group
    also: List[int] = field(default_factory=list)  # further results of the same operator (TopK: the indices)
    versions: int = 1                              # code versions of the fused loop nest (Fig. 4)
    unproven: List[tuple] = field(default_factory=list)   # (operand a, operand b, aligned dim) pairs behind them
    lnfold: int = -1                               # R9: the LayerNorm operator whose result this contraction reads
    key: int = -1                                  # position in the node order that places the group among the items


@dataclass
class Item:                               # a step candidate: a group or a control operator
    is_group: bool
    ref: int                              # group id or operator id
    reads: List[int] = field(default_factory=list)     # static bases read
    writes: List[int] = field(default_factory=list)    # static bases produced


@dataclass
class Plan:
    graph: object
    rdp: R.RDP
    opts: Opts
    order: List[int]
    folded: List[bool]
    view: List[bool]
    groups: Dict[int, Group]
    group_of_op: Dict[int, int]
    items: List[Item]
    subgraphs: List[List[int]]            # item indices, in planned execution order
    sg_class: List[str]
    sbase: List[int]                      # static base of every tensor
    versions_unfused: int = 0             # broadcast versions a shape-blind fuser would need
    paper_rdp: R.RDP = None               # Alg. 1 as printed (EDO outputs nac); == rdp without a NonZero
    exec_ops: List[int] = field(default_factory=list)    # NonZero operators, in the node order
    inplace: Dict[int, int] = field(default_factory=dict)   # group result -> the operand whose storage it takes over
    fold_y: Dict[int, int] = field(default_factory=dict)    # R9: LayerNorm result produced by a contraction -> the LayerNorm


def _shape_equal(a, b) -> bool:
    return isinstance(a, list) and isinstance(b, list) and len(a) == len(b) and \
        all(R.is_expr(x) and R.is_expr(y) and x == y for x, y in zip(a, b))


def _unproven_pairs(rdp, op):
    """Aligned dim pairs of the two operands of a binary elementwise operator that RDP cannot prove equal or 1, as
    (operand a, operand b, dim counted from the last); [] for a unary operator; None when an extent is unresolved."""
    if len(op.inputs) != 2:
        return []
    a, b = op.inputs
    sa, sb = rdp.S[a], rdp.S[b]
    if not isinstance(sa, list) or not isinstance(sb, list):
        return None
    out = []
    for k in range(1, max(len(sa), len(sb)) + 1):
        x = sa[-k] if k <= len(sa) else R.C(1)
        y = sb[-k] if k <= len(sb) else R.C(1)
        if R.pair_proven(x, y):
            continue
        if not (R.is_expr(x) and R.is_expr(y)):
            return None
        out.append((a, b, k))
    return out


def tensor_bytes_expr(plan_or_rdp, graph, tid) -> Optional[Expr]:
    s = plan_or_rdp.S[tid]
    if not isinstance(s, list) or any(not R.is_expr(d) for d in s):
        return None
    e = R.C(DT_BYTES[graph.tensors[tid].dtype])
    for d in s:
        e = e * d
    return e


def align_up(n: int) -> int:
    return (n + ALIGN - 1) // ALIGN * ALIGN


def build_plan(graph, rdp: R.RDP, opts: Opts = None) -> Plan:
    opts = opts or Opts()
    g = graph
    paper_rdp = rdp
    if any(op.kind in COUNTING for op in g.ops):
        rdp = R.RDP(g, named_edo=True).analyse()
    order = rdp.sorted_nodes()
    pos = {n: i for i, n in enumerate(order)}
    nops = len(g.ops)

    for t, d in enumerate(g.tensors):
        if d.is_output and rdp.producer[t] < 0:
            raise ValueError(f"graph output {d.name} is produced by no operator")
    # R0 / R1 ---------------------------------------------------------------
    folded, view = [False] * nops, [False] * nops
    for i, op in enumerate(g.ops):
        if op.kind in ("Switch", "Combine"):
            if any(g.tensors[o].is_output for o in op.outputs):
                # control operators forward storage, they write none: nothing would reach the caller's buffer
                raise ValueError("a graph output must not be the direct result of a Switch or Combine "
                                 "(put an operator behind it: a Cast to its own type copies it)")
            continue
        outs_int = all(g.tensors[o].dtype in ("i64", "i32") for o in op.outputs)
        to_caller = any(g.tensors[o].is_output for o in op.outputs)      # its result must reach the caller's buffer
        if outs_int and not to_caller and all(isinstance(rdp.V[o], list) and all(R.is_expr(e) for e in rdp.V[o])
                                              for o in op.outputs):
            folded[i] = True
        elif op.kind in VIEW_KINDS:
            view[i] = not to_caller
        elif op.kind == "Gather":
            idx = g.tensors[op.inputs[1]]
            view[i] = idx.data is not None and idx.data.ndim == 0 and not to_caller

    # R1, second half: a view that a kernel could not walk is written out.  Decided from the graph alone, in the node
    # order so that a view of a view inherits: a view is *strided* when it permutes dims, slices or indexes a dim other
    # than the first, or repeats elements (Expand); *permuted* when a Transpose is involved.
    nt = len(g.tensors)
    strided, permuted = [False] * nt, [False] * nt     # per tensor: it is such a view (control operators pass it on)

    def readers(t):
        """The operators that get to read tensor t, with the tensor they read it as: its consumers, looking through
        Switch and Combine (which hand the storage on under another name)."""
        out, stack, seen = [], [t], set()
        while stack:
            u = stack.pop()
            for c in rdp.consumers[u]:
                if (c, u) in seen or folded[c]:
                    continue
                seen.add((c, u))
                if g.ops[c].kind in ("Switch", "Combine"):
                    stack.extend(g.ops[c].outputs)
                else:
                    out.append((c, u))
        return sorted(out)

    for n in order:
        op = g.ops[n]
        if op.kind == "Switch":
            for o in op.outputs:
                strided[o], permuted[o] = strided[op.inputs[0]], permuted[op.inputs[0]]
            continue
        if op.kind == "Combine":
            strided[op.outputs[0]] = any(strided[t] for t in op.inputs)
            permuted[op.outputs[0]] = any(permuted[t] for t in op.inputs)
            continue
        if not view[n]:
            continue
        src, res = op.inputs[0], op.outputs[0]
        rank = len(rdp.S[src]) if isinstance(rdp.S[src], list) else None
        s = p = False
        if op.kind == "Transpose":
            s = p = list(op.attrs["perm"]) != list(range(len(op.attrs["perm"])))
        elif op.kind == "Slice":
            ax = rdp.V[op.inputs[3]]
            known = rank is not None and isinstance(ax, list) and all(R.is_expr(e) and e.is_const() for e in ax)
            s = not known or any(e.const_value() % rank != 0 for e in ax)
        elif op.kind == "Expand":
            s = True
        elif op.kind == "Gather":
            s = rank is None or op.attrs["axis"] % rank != 0
        strided[res], permuted[res] = s or strided[src], p or permuted[src]
        for c, u in readers(res):
            k = g.ops[c].kind
            table = k == "Gather" and not view[c] and g.ops[c].inputs[0] == u      # rows picked by an index tensor
            if ((k in DENSE_ONLY or table) and strided[res]) or (k in ROW_OPS + ("Reshape",) and permuted[res]):
                view[n] = False                    # a COPY group: its result is dense
                strided[res] = permuted[res] = False
                break

    def sole_consumer(t) -> Optional[int]:
        if g.tensors[t].is_output or len(rdp.consumers[t]) != 1:
            return None
        return rdp.consumers[t][0]

    def other(op, cur):
        return op.inputs[1] if op.inputs[0] == cur else op.inputs[0]

    def is_host_scalar(t) -> bool:
        d = g.tensors[t]
        return d.data is not None and d.data.size == 1

    # R2-R4: fusion -----------------------------------------------------------
    assigned: Dict[int, int] = {}
    groups: Dict[int, Group] = {}
    absorbed_transpose = set()

    def new_group(kind, members):
        gid = min(members)
        last = max(members, key=lambda n: pos[n])
        groups[gid] = Group(gid, kind, sorted(members), g.ops[last].outputs[0], also=list(g.ops[last].outputs[1:]))
        for n in members:
            assigned[n] = gid

    for n in order:
        op = g.ops[n]
        if folded[n] or n in assigned or op.kind in ("Switch", "Combine"):
            continue
        if view[n] and n not in absorbed_transpose:
            continue
        if op.kind in ("MatMul", "Conv"):
            members, cur, state = [n], op.outputs[0], 0
            while True:
                c = sole_consumer(cur)
                if c is None or folded[c] or c in assigned:
                    break
                cop = g.ops[c]
                if not opts.fusion and cop.kind != "Transpose":
                    break           # fusion off: only the permuted store (a layout choice, no arithmetic merged) remains
                nxt = None
                if cop.kind == "Mul" and state < 1 and is_host_scalar(other(cop, cur)):
                    nxt = 1
                elif cop.kind == "Add":
                    o = other(cop, cur)
                    so, sc = rdp.S[o], rdp.S[cur]
                    if state < 2 and g.tensors[o].role == "weight" and isinstance(so, list) and \
                            len(so) == 1 and isinstance(sc, list) and R.is_expr(sc[-1]) and so[0] == sc[-1]:
                        nxt = 2
                    elif state < 4 and g.tensors[o].role not in ("weight", "hostconst") and \
                            _shape_equal(so, sc):
                        nxt = 4
                elif cop.kind in ACTS:
                    nxt = 3 if state < 3 else (5 if state == 4 else None)
                elif cop.kind == "Transpose" and state < 6:
                    nxt = 6
                    absorbed_transpose.add(c)
                if nxt is None:
                    break
                members.append(c)
                cur, state = cop.outputs[0], nxt
                if state == 6:
                    break
            new_group("GEMM" if op.kind == "MatMul" else "CONV", members)
        elif op.kind in SOLO:
            new_group(SOLO[op.kind], [n])
        elif op.kind in VIEW_KINDS or (op.kind == "Gather" and g.tensors[op.inputs[1]].data is not None
                                       and g.tensors[op.inputs[1]].data.ndim == 0):
            new_group("COPY", [n])           # a view whose result is a graph output: materialised in the caller's buffer
        elif op.kind == "Gather":
            members = [n]
            c = sole_consumer(op.outputs[0])
            if opts.fusion and c is not None and g.ops[c].kind == "Add" and c not in assigned and \
                    _shape_equal(rdp.S[other(g.ops[c], op.outputs[0])], rdp.S[op.outputs[0]]):
                members.append(c)
            new_group("GATHER", members)
        elif op.kind in ELTWISE:
            members, cur = [n], op.outputs[0]
            pairs = _unproven_pairs(rdp, op) or []           # of the seed itself; they count once it has company
            while opts.fusion and len(members) < 8:
                c = sole_consumer(cur)
                if c is None or c in assigned or g.ops[c].kind not in ELTWISE:
                    break
                cop = g.ops[c]
                if cop.kind == "Round" and g.tensors[cur].dtype != "f32":
                    break                # Round decides an integer: it must see the value as stored, not the chain's fp32
                more = _unproven_pairs(rdp, cop)
                if more is None or 2 ** (len(pairs) + len(more)) > max(opts.max_versions, 1):
                    break
                pairs = pairs + more
                members.append(c)
                cur = cop.outputs[0]
            new_group("ELTWISE", members)
            if len(members) > 1 and pairs:
                groups[min(members)].versions = 2 ** len(pairs)
                groups[min(members)].unproven = pairs
        else:
            raise ValueError(f"no grouping rule for {op.kind}")
    for c in absorbed_transpose:
        view[c] = False

    def _append_behind(t) -> Optional[int]:
        """The CacheAppend whose result reaches tensor t through views only, each link read by nobody
        else, when it appends a known number of at most 4 bf16 rows (R8); else None."""
        while True:
            p = rdp.producer[t]
            if p < 0 or g.tensors[t].is_output or len(rdp.consumers[t]) != 1:
                return None
            if view[p]:
                t = g.ops[p].inputs[0]
                continue
            op = g.ops[p]
            if op.kind != "CacheAppend" or p not in assigned or groups[assigned[p]].kind != "CACHEAPPEND":
                return None
            rows = rdp.S[op.inputs[1]]
            if g.tensors[t].dtype != "bf16" or not isinstance(rows, list) or not rows or not R.is_expr(rows[0]) \
                    or not rows[0].is_const() or rows[0].const_value() > opts.append_max_rows:
                return None
            return p

    # R6: attention --------------------------------------------------------------
    if opts.fusion:
        for n in order:
            op = g.ops[n]
            if op.kind != "Softmax" or n not in assigned or groups[assigned[n]].kind != "SOFTMAX":
                continue
            x, y = op.inputs[0], op.outputs[0]
            p1 = rdp.producer[x]
            if p1 < 0 or p1 not in assigned or sole_consumer(x) != n:
                continue
            g1 = groups[assigned[p1]]
            kinds1 = [g.ops[m].kind for m in g1.ops]
            if g1.kind != "GEMM" or g1.out != x or kinds1 not in (["MatMul"], ["MatMul", "Mul"]):
                continue
            c2 = sole_consumer(y)
            if c2 is None or g.ops[c2].kind != "MatMul" or g.ops[c2].inputs[0] != y or g.ops[c2].inputs[1] == y:
                continue
            g2 = groups[assigned[c2]]
            kinds2 = [g.ops[m].kind for m in g2.ops]
            if g2.kind != "GEMM" or min(g2.ops) != c2 or kinds2 not in (["MatMul"], ["MatMul", "Transpose"]):
                continue
            mm1 = g.ops[g1.ops[0]]
            tensors = [mm1.inputs[0], mm1.inputs[1], g.ops[c2].inputs[1], x, y, g2.out]
            if any(g.tensors[t].dtype != "bf16" for t in tensors):
                continue
            sq, sv = rdp.S[mm1.inputs[0]], rdp.S[g.ops[c2].inputs[1]]
            if not (isinstance(sq, list) and isinstance(sv, list) and sq and sv and R.is_expr(sq[-1]) and
                    R.is_expr(sv[-1]) and sq[-1] == sv[-1] and sq[-1].is_const() and
                    sq[-1].const_value() in opts.attn_head_dims):
                continue
            members = g1.ops + [n] + g2.ops
            for gid in (g1.gid, assigned[n], g2.gid):
                del groups[gid]
            # R8: the decode step's attention appends the new key / value rows itself
            appends = []
            for t in (mm1.inputs[1], g.ops[c2].inputs[1]):
                ca = _append_behind(t)
                if ca is not None:
                    appends.append(ca)
            if len(appends) == 2 and appends[0] != appends[1]:
                for ca in appends:
                    del groups[assigned[ca]]
                members = appends + members
            gid = min(members)
            groups[gid] = Group(gid, "ATTENTION", sorted(members), g2.out)
            for m in members:
                assigned[m] = gid

    # R7: LayerNorm as the prologue of a contraction ------------------------------
    if opts.fusion:
        for n in order:
            op = g.ops[n]
            if op.kind != "LayerNorm" or n not in assigned or groups[assigned[n]].kind != "LAYERNORM":
                continue
            y = op.outputs[0]
            c = sole_consumer(y)
            if c is None or g.ops[c].kind != "MatMul" or g.ops[c].inputs[0] != y or g.ops[c].inputs[1] == y:
                continue
            gm = groups[assigned[c]]
            if gm.kind != "GEMM" or min(gm.ops) != c:
                continue
            sx = rdp.S[op.inputs[0]]
            tensors = list(op.inputs) + [y, g.ops[c].inputs[1], gm.out]
            if any(g.tensors[t].dtype != "bf16" for t in tensors):
                continue
            if not (isinstance(sx, list) and sx and all(R.is_expr(d) and d.is_const() for d in sx)):
                continue
            kdim, rows = sx[-1].const_value(), 1
            for d in sx[:-1]:
                rows *= d.const_value()
            if kdim > opts.prologue_max_k or kdim % opts.prologue_k_multiple != 0 or rows > opts.prologue_max_rows:
                continue
            members = [n] + gm.ops
            del groups[assigned[n]]
            del groups[gm.gid]
            gid = min(members)
            groups[gid] = Group(gid, "GEMM", sorted(members), gm.out)
            for m in members:
                assigned[m] = gid

    # R9: LayerNorm as the second result of the contraction that produces its input ----------
    fold_y: Dict[int, int] = {}
    for gr in groups.values():
        gr.key = max(pos[m] for m in gr.ops)
    if opts.fusion and opts.fold_ln:
        for n in order:
            op = g.ops[n]
            if op.kind != "LayerNorm" or n not in assigned or groups[assigned[n]].kind != "LAYERNORM":
                continue
            x, y = op.inputs[0], op.outputs[0]
            px = rdp.producer[x]
            if px < 0 or px not in assigned:
                continue
            gp = groups[assigned[px]]
            kinds = [g.ops[m].kind for m in gp.ops]
            if gp.kind != "GEMM" or gp.out != x or gp.also or kinds[0] != "MatMul" or \
                    any(k in ("Transpose", "LayerNorm", "CacheAppend") for k in kinds):
                continue
            c = sole_consumer(y)
            if c is None or g.ops[c].kind != "MatMul" or g.ops[c].inputs[0] != y or g.ops[c].inputs[1] == y:
                continue
            gm = groups[assigned[c]]
            wt = g.ops[c].inputs[1]
            sw, sx = rdp.S[wt], rdp.S[x]
            if gm.kind != "GEMM" or min(gm.ops) != c or gm.lnfold >= 0 or not g.ops[c].attrs.get("transB", 0) or \
                    g.tensors[wt].role != "weight" or not isinstance(sw, list) or len(sw) != 2:
                continue
            if any(g.tensors[t].dtype != "bf16" for t in list(op.inputs) + [y, wt, gm.out]):
                continue
            if not (isinstance(sx, list) and sx and all(R.is_expr(d) for d in sx) and sx[-1].is_const()
                    and sx[-1].const_value() % opts.fold_k_multiple == 0 and sx[-1].const_value() > 0):
                continue
            del groups[assigned[n]]
            gp.ops = sorted(gp.ops + [n])
            gp.also = [y]
            assigned[n] = gp.gid
            gm.lnfold = n
            fold_y[y] = n

    # statistic: loop-nest versions a fuser without RDP results would emit (Fig. 4)
    versions = 0
    for i, op in enumerate(g.ops):
        if op.kind in ("Add", "Mul") and not folded[i]:
            versions += 2 ** max(len(rdp.S[t]) if isinstance(rdp.S[t], list) else 0 for t in op.inputs)

    # static alias bases --------------------------------------------------------
    sbase = list(range(len(g.tensors)))
    for n in order:
        op = g.ops[n]
        if view[n] or op.kind == "Switch":
            for o in op.outputs:
                sbase[o] = sbase[op.inputs[0]]

    def reads_of(members) -> List[int]:
        inside = {o for n in members for o in g.ops[n].outputs}
        seen, out = set(), []
        for n in members:
            for t in g.ops[n].inputs:
                b = sbase[t]
                if t in inside or b in inside or b in seen:
                    continue
                seen.add(b)
                out.append(b)
        return out

    for gr in groups.values():
        gr.ins = reads_of(gr.ops)

    # items in topological order (R5) --------------------------------------------
    entries = [(gr.key if gr.key >= 0 else max(pos[n] for n in gr.ops), True, gid) for gid, gr in groups.items()]
    entries += [(pos[n], False, n) for n, op in enumerate(g.ops) if op.kind in ("Switch", "Combine")]
    items: List[Item] = []
    for _, is_group, ref in sorted(entries):
        if is_group:
            items.append(Item(True, ref, list(groups[ref].ins), [groups[ref].out] + groups[ref].also))
        else:
            op = g.ops[ref]
            reads = []
            for t in op.inputs:
                if sbase[t] not in reads:
                    reads.append(sbase[t])
            items.append(Item(False, ref, reads, list(op.outputs) if op.kind == "Combine" else []))

    plan = Plan(g, rdp, opts, order, folded, view, groups, assigned, items, [], [], sbase, versions,
                paper_rdp, [n for n in order if g.ops[n].kind in COUNTING])
    plan.fold_y = fold_y
    _partition(plan)
    if opts.inplace:
        _mark_inplace(plan)
    return plan


def _mark_inplace(plan: Plan):
    """In-place reuse (a refinement of the lifetime rule of Section 4.4.1; the paper does not spell it
    out).  The result of a contraction group with a residual operand, or of an elementwise group,
    takes over the storage of one operand r when, whatever path is executed,
      * r is the result of a group, lives in the arena, and has the type and (provably) the shape of
        the result, which lives in the arena too;
      * the group reads the storage of r through that operand only (each kernel thread reads the
        elements of r it is about to write, nothing else of r), and stores without a permutation;
      * the group is the last item, in the planned execution order, that reads the storage of r, and
        no Combine forwards r (its output would keep the storage alive on some paths)."""
    g, rdp = plan.graph, plan.rdp
    position = {}
    for sg in plan.subgraphs:
        for i in sg:
            position[i] = len(position)
    combined = {t for it in plan.items if not it.is_group and g.ops[it.ref].kind == "Combine" for t in it.reads}
    readers: Dict[int, List[int]] = {}
    for i, it in enumerate(plan.items):
        for t in it.reads:
            readers.setdefault(t, []).append(i)
    prod = rdp.producer
    for i, it in enumerate(plan.items):
        if not it.is_group:
            continue
        gr = plan.groups[it.ref]
        if gr.kind not in ("GEMM", "CONV", "ELTWISE") or not arena_candidate(plan, gr.out):
            continue
        if any(g.ops[n].kind in ("Transpose", "CacheAppend") or
               (g.ops[n].kind == "LayerNorm" and n not in plan.fold_y.values()) for n in gr.ops):
            continue                     # (a LayerNorm that is the group's second result, R9, reads the finished rows)
        inside = {o for n in gr.ops for o in g.ops[n].outputs}
        outer = [t for n in gr.ops for t in g.ops[n].inputs if t not in inside and plan.sbase[t] not in inside]
        if gr.kind == "ELTWISE":
            cands = [t for t in outer]
        else:                            # the operand added in the epilogue: an Add member's outside operand
            cands = [t for n in gr.ops if g.ops[n].kind == "Add" for t in g.ops[n].inputs if t in outer]
        for r in cands:
            d = g.tensors[r]
            if d.role != "inter" or not arena_candidate(plan, r) or r in combined or r in plan.inplace.values():
                continue
            pr = prod[r]
            if pr < 0 or plan.folded[pr] or plan.view[pr] or g.ops[pr].kind in ("Switch", "Combine") + COUNTING:
                continue
            if plan.groups[plan.group_of_op[pr]].out != r:
                continue
            if d.dtype != g.tensors[gr.out].dtype or not _shape_equal(rdp.S[r], rdp.S[gr.out]):
                continue
            if [t for t in outer if plan.sbase[t] == r] != [r]:
                continue
            if any(position[j] > position[i] for j in readers.get(r, []) if j != i):
                continue
            plan.inplace[gr.out] = r
            break


def arena_candidate(plan: Plan, t: int) -> bool:
    """Static test: tensor t is produced by an item and is not written to a caller buffer."""
    d = plan.graph.tensors[t]
    return d.role == "inter" and not d.is_output and not d.session


def execution_determined(plan: Plan, t: int) -> bool:
    """nac in the paper's lattice: unresolved, or an expression in an execution symbol."""
    s = plan.rdp.S[t]
    return not isinstance(s, list) or any(not R.is_expr(d) or R.mentions_exec(d) for d in s)


def _item_has_nac(plan: Plan, it: Item) -> bool:
    return any(execution_determined(plan, t) for t in it.writes)


def _partition(plan: Plan):
    items = plan.items
    n = len(items)
    last_read = {}
    for i, it in enumerate(items):
        for t in it.reads:
            last_read[t] = i
    cut_after = [False] * n
    live = set()
    for i, it in enumerate(items):
        for t in it.writes:
            if arena_candidate(plan, t) and last_read.get(t, -1) > i:
                live.add(t)
        live = {t for t in live if last_read[t] > i}
        is_edo = (not it.is_group) or plan.groups[it.ref].kind in COUNTING_GROUPS
        if is_edo:
            cut_after[i] = True
            if i > 0:
                cut_after[i - 1] = True
        elif _item_has_nac(plan, it) or len(live) <= 1:
            cut_after[i] = True
    pieces, cur = [], []
    for i in range(n):
        cur.append(i)
        if cut_after[i] or len(cur) == MAX_SG:
            pieces.append(cur)
            cur = []
    if cur:
        pieces.append(cur)
    plan.subgraphs = [_order_subgraph(plan, p, last_read) for p in pieces]
    plan.sg_class = [_classify(plan, p) for p in pieces]


def _classify(plan: Plan, piece) -> str:
    cls = "known"
    for i in piece:
        for t in plan.items[i].writes:
            if execution_determined(plan, t):
                return "nac"
            if any(not d.is_const() for d in plan.rdp.S[t]):
                cls = "mixed"
    return cls


def _bytes_at(plan: Plan, t: int, env) -> int:
    """Size used by the order search; an execution-determined tensor counts as 0 (unknown)."""
    e = tensor_bytes_expr(plan.rdp, plan.graph, t)
    if e is None or execution_determined(plan, t):
        return 0
    n = e.eval(env)
    return align_up(n * 9 // 8 if t in plan.fold_y else n)      # R9: the partial sums behind the rows


def subgraph_peak(plan: Plan, seq, last_read, env) -> int:
    """Peak of the summed bytes of live tensors when the items run in the order ``seq``."""
    first, end = min(seq), max(seq)
    inside = set(seq)
    produced_in = {t: i for i in seq for t in plan.items[i].writes if arena_candidate(plan, t)}
    incoming = []
    for i in seq:
        for t in plan.items[i].reads:
            if t not in produced_in and t not in incoming and _incoming_arena(plan, t, first):
                incoming.append(t)
    done, peak = set(), 0
    for cur in seq:
        mem = 0
        for t in incoming + list(produced_in):
            if t in produced_in and produced_in[t] not in done and produced_in[t] != cur:
                continue
            readers = [i for i in inside if t in plan.items[i].reads]
            alive = last_read.get(t, -1) > end or any(i not in done for i in readers) or produced_in.get(t) == cur
            if alive:
                mem += _bytes_at(plan, t, env)
        peak = max(peak, mem)
        done.add(cur)
    return peak


def _incoming_arena(plan: Plan, t: int, first_item: int) -> bool:
    if not arena_candidate(plan, t):
        return False
    return any(t in it.writes for it in plan.items[:first_item])


def _order_subgraph(plan: Plan, piece, last_read) -> List[int]:
    """Section 4.3: exhaustive search (dynamic programme over executed subsets) for the order with
    the smallest peak, sizes taken at the symbols' upper bounds; ties -> smallest group ids first."""
    if not plan.opts.sep or len(piece) <= 2 or _classify(plan, piece) == "nac":
        return list(piece)
    items = plan.items
    env = {name: hi for name, lo, hi in plan.graph.symbols}
    k = len(piece)
    idx = {it: j for j, it in enumerate(piece)}
    first, end = piece[0], piece[-1]
    produced_in = {}
    for i in piece:
        for t in items[i].writes:
            if arena_candidate(plan, t):
                produced_in[t] = idx[i]
    tensors = list(produced_in)
    for i in piece:
        for t in items[i].reads:
            if t not in produced_in and t not in tensors and _incoming_arena(plan, t, first):
                tensors.append(t)
    size = {t: _bytes_at(plan, t, env) for t in tensors}
    readers = {t: [idx[i] for i in piece if t in items[i].reads] for t in tensors}
    live_out = {t: last_read.get(t, -1) > end for t in tensors}
    writer = {t: idx[i] for i in piece for t in items[i].writes}    # includes graph outputs
    deps = [0] * k
    for i in piece:
        for t in items[i].reads:
            if t in writer:
                deps[idx[i]] |= 1 << writer[t]

    def step_mem(S: int, j: int) -> int:
        mem = 0
        for t in tensors:
            p = produced_in.get(t, -1)
            if p >= 0 and p != j and not (S >> p) & 1:
                continue
            if p == j or live_out[t] or any(not (S >> r) & 1 for r in readers[t]):
                mem += size[t]
        return mem

    full = (1 << k) - 1
    INF = float("inf")
    best = [INF] * (full + 1)
    best[full] = 0
    for S in range(full - 1, -1, -1):
        b = INF
        for j in range(k):
            if (S >> j) & 1 or (deps[j] & ~S):
                continue
            b = min(b, max(step_mem(S, j), best[S | (1 << j)]))
        best[S] = b
    target, S, seq = best[0], 0, []
    by_id = sorted(range(k), key=lambda j: (items[piece[j]].ref, j))
    while S != full:
        for j in by_id:
            if (S >> j) & 1 or (deps[j] & ~S):
                continue
            if max(step_mem(S, j), best[S | (1 << j)]) <= target:
                seq.append(piece[j])
                S |= 1 << j
                break
    return seq


# ---------------------------------------------------------------------------
# canonical text dump
# ---------------------------------------------------------------------------

def dump(plan: Plan) -> str:
    g = plan.graph
    lines = ["order" + "".join(f" {n}" for n in plan.order)]
    lines.append("folded" + "".join(f" {i}" for i, f in enumerate(plan.folded) if f))
    lines.append("views" + "".join(f" {i}" for i, f in enumerate(plan.view) if f))
    for t in range(len(g.tensors)):                      # shapes that wait for an EDO to execute
        s = plan.rdp.S[t]
        if isinstance(s, list) and any(R.mentions_exec(d) for d in s):
            lines.append(f"named t{t} S={R.fmt_list(s)}")
    for it in plan.items:
        if it.is_group:
            gr = plan.groups[it.ref]
            also = "".join(f" also=t{t}" for t in gr.also)
            ver = ""
            if gr.versions > 1:
                ver = f" versions={gr.versions} unproven=[" + " ".join(f"t{a}~t{b}@{k}" for a, b, k in gr.unproven) + "]"
            if gr.lnfold >= 0:
                ver += f" lnfold={gr.lnfold}"
            lines.append(f"g{gr.gid} {gr.kind} ops=[{' '.join(map(str, gr.ops))}] out=t{gr.out}{also} "
                         f"ins=[{' '.join('t%d' % t for t in gr.ins)}]{ver}")
        else:
            lines.append(f"c{it.ref} {g.ops[it.ref].kind}")
    for t in sorted(plan.inplace):
        lines.append(f"inplace t{t}=t{plan.inplace[t]}")
    for s, (sg, cls) in enumerate(zip(plan.subgraphs, plan.sg_class)):
        names = [("g%d" % plan.items[i].ref) if plan.items[i].is_group else ("c%d" % plan.items[i].ref)
                 for i in sg]
        lines.append(f"sg{s} {cls} " + " ".join(names))
    return "\n".join(lines) + "\n"
