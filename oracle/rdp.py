"""Rank and Dimension Propagation (Section 4.1; Alg. 1; Tables 3 and 4).

Per tensor the analysis keeps a shape S and, for small integer tensors, a
value V.  Both live in the lattice of Fig. 2: undef (top) > {known constant,
symbolic constant, operation-inferred constant} > nac (bottom), taken per
component (rank, each dim, each element) as a product lattice.

Readings where the paper is silent (all listed in the design notes):
  * every visit re-applies the transfer function and *meets* the result into
    the stored state, so the fixed point does not depend on the visiting order;
    the early return of Alg. 1 is the shortcut that holds for the sorted order;
  * Switch forwards the shape and value of its data input to every output;
  * Combine takes the meet over its inputs that are not undef;
  * a backward transfer assigns only what is unique (Section 3: for Add each
    input dim may be 1 or the output dim, so nothing is assigned);
  * whatever is still undef at the fixed point becomes nac.
"""
from __future__ import annotations

from typing import List, Optional

from .expr import Expr

UNDEF = None
NAC = "nac"
MAX_V = 16            # value maps are kept for int tensors up to this many elements
INT_MAX = 2 ** 31 - 1

ISDO, ISDOS, ISVDOS, EDO = "ISDO", "ISDOS", "ISVDOS", "EDO"
OP_CLASS = {
    "Shape": ISDO, "ConstantOfShape": ISDO, "EyeLike": ISDO,
    "Gather": ISDOS, "Concat": ISDOS, "Transpose": ISDOS, "MatMul": ISDOS, "Conv": ISDOS,
    "Add": ISDOS, "Mul": ISDOS, "Relu": ISDOS, "Gelu": ISDOS, "Sigmoid": ISDOS, "Cast": ISDOS,
    "Softmax": ISDOS, "LayerNorm": ISDOS, "ReduceMean": ISDOS, "MaxPool": ISDOS, "AveragePool": ISDOS, "Round": ISDOS,
    "ArgMax": ISDOS, "CacheAppend": ISDOS, "ScatterRows": ISDOS,
    "Reshape": ISVDOS, "Slice": ISVDOS, "Resize": ISVDOS, "Range": ISVDOS, "Expand": ISVDOS,
    "OneHot": ISVDOS, "Upsample": ISVDOS, "TopK": ISVDOS, "GroupNorm": ISVDOS, "MaxUnpool": ISVDOS,
    "NonZero": EDO, "NMS": EDO, "Switch": EDO, "Combine": EDO,
}
UNARY = ("Relu", "Gelu", "Sigmoid", "Round", "Cast", "Softmax", "LayerNorm", "GroupNorm")   # result shaped like input 0
EXEC_PREFIX = "@nz"   # name of an execution symbol: EXEC_PREFIX + operator id


def exec_symbol(op_id: int) -> str:
    return f"{EXEC_PREFIX}{op_id}"


def mentions_exec(e) -> bool:
    """Does a lattice value depend on an execution symbol (nested floordiv / mod atoms included)?"""
    return is_expr(e) and EXEC_PREFIX in str(e)


class ShapeMismatch(Exception):
    pass


# ---------------------------------------------------------------------------
# lattice
# ---------------------------------------------------------------------------

def is_expr(x) -> bool:
    return isinstance(x, Expr)


def meet(a, b):
    """Meet of two scalar lattice values (a dim, a rank or an element)."""
    if a is UNDEF:
        return b
    if b is UNDEF:
        return a
    if a == NAC or b == NAC:
        return NAC
    if a == b:
        return a
    if a.is_const() and b.is_const():
        raise ShapeMismatch(f"{a} vs {b}")
    return NAC


def meet_list(a, b):
    """Meet of two shapes (or value vectors): undef | nac | list of scalar lattice values."""
    if a is UNDEF:
        return b
    if b is UNDEF:
        return a
    if a == NAC or b == NAC:
        return NAC
    if len(a) != len(b):
        raise ShapeMismatch(f"rank {len(a)} vs {len(b)}")
    return [meet(x, y) for x, y in zip(a, b)]


def same(a, b) -> bool:
    if a is UNDEF or b is UNDEF or a == NAC or b == NAC:
        return a is b or a == b
    if isinstance(a, list) != isinstance(b, list):
        return False
    if isinstance(a, list):
        return len(a) == len(b) and all(same(x, y) for x, y in zip(a, b))
    return a == b


def g_is_int(g, t) -> bool:
    return g.tensors[t].dtype in ("i64", "i32")


def has_undef(x) -> bool:
    if x is UNDEF:
        return True
    if isinstance(x, list):
        return any(e is UNDEF for e in x)
    return False


def arith(op, a, b):
    """Arithmetic on scalar lattice values: nac absorbs, then undef, else the expression."""
    if a == NAC or b == NAC:
        return NAC
    if a is UNDEF or b is UNDEF:
        return UNDEF
    return op(a, b)


def d_add(a, b): return arith(lambda x, y: x + y, a, b)
def d_sub(a, b): return arith(lambda x, y: x - y, a, b)
def d_mul(a, b): return arith(lambda x, y: x * y, a, b)


def d_floordiv(a, b):
    def f(x, y):
        return x.floordiv(y.const_value()) if (y.is_const() and y.const_value() > 0) else NAC
    return arith(f, a, b)


def C(v: int) -> Expr:
    return Expr.const(v)


def broadcast_dim(a, b):
    """Output dim of an elementwise op with broadcasting for one aligned pair of input dims."""
    if is_expr(a) and is_expr(b):
        if a == b:
            return a
        if a.is_const() and a.const_value() == 1:
            return b
        if b.is_const() and b.const_value() == 1:
            return a
        if a.is_const() and b.is_const():
            raise ShapeMismatch(f"broadcast {a} vs {b}")
        # unproven: could be equal, one of them could be 1 (Fig. 4).  The extent is still a function of the
        # symbols -- an operation-inferred constant, evaluated (and checked) when they are bound
        return a.bcast(b)
    for x, y in ((a, b), (b, a)):
        if is_expr(x) and x.is_const() and x.const_value() != 1 and (y is UNDEF or y == NAC):
            return x                     # the other side is 1 or x: the output is x either way
    if a is UNDEF or b is UNDEF:
        return UNDEF
    return NAC


def broadcast_shapes(a: list, b: list) -> list:
    r = max(len(a), len(b))
    a = [C(1)] * (r - len(a)) + a
    b = [C(1)] * (r - len(b)) + b
    return [broadcast_dim(x, y) for x, y in zip(a, b)]


def pair_proven(a, b) -> bool:
    """Fig. 4 condition for one aligned dim pair: equal, or one side is the constant 1."""
    if not (is_expr(a) and is_expr(b)):
        return False
    return a == b or (a.is_const() and a.const_value() == 1) or (b.is_const() and b.const_value() == 1)


def fused_versions(a, b) -> int:
    """Number of fused loop nests needed for an elementwise pair (Fig. 4): 2 per unproven dim pair."""
    if not isinstance(a, list) or not isinstance(b, list):
        return -1                        # rank unknown: unbounded
    r = max(len(a), len(b))
    a = [C(1)] * (r - len(a)) + a
    b = [C(1)] * (r - len(b)) + b
    n = 1
    for x, y in zip(a, b):
        if not pair_proven(x, y):
            n *= 2
    return n


# ---------------------------------------------------------------------------
# the analysis
# ---------------------------------------------------------------------------

class RDP:
    """``named_edo=False`` is Alg. 1 as printed: every output of an execution-determined operator is
    nac.  ``named_edo=True`` runs the same transfer functions with one change: the extent NonZero
    produces (unknown until it has executed, then a constant for the rest of the call) is given a
    name, the execution symbol ``@nz<operator id>``, so that everything downstream is an expression
    in it and can be evaluated, not re-inferred, once the operator has run.  The second analysis
    refines the first: where the first has a value the second has the same one, and whatever is nac
    or mentions an execution symbol in the second is nac in the first."""

    def __init__(self, graph, named_edo: bool = False):
        self.g = graph
        self.named_edo = named_edo
        nt = len(graph.tensors)
        self.S: List = [UNDEF] * nt
        self.V: List = [UNDEF] * nt
        self.sweeps = 0
        self.producer = [-1] * nt
        self.consumers = [[] for _ in range(nt)]
        for i, op in enumerate(graph.ops):
            for t in op.outputs:
                self.producer[t] = i
            for t in op.inputs:
                self.consumers[t].append(i)

    # -- node order: reverse post-order of a depth-first walk ---------------
    def sorted_nodes(self) -> List[int]:
        g = self.g
        succ = []
        for i, op in enumerate(g.ops):
            s = sorted({c for t in op.outputs for c in self.consumers[t]})
            succ.append(s)
        roots = [i for i, op in enumerate(g.ops) if all(self.producer[t] < 0 for t in op.inputs)]
        seen, post = set(), []
        for r in roots:
            if r in seen:
                continue
            seen.add(r)
            stack = [(r, 0)]
            while stack:
                u, k = stack.pop()
                if k < len(succ[u]):
                    stack.append((u, k + 1))
                    v = succ[u][k]
                    if v not in seen:
                        seen.add(v)
                        stack.append((v, 0))
                else:
                    post.append(u)
        return post[::-1]

    # -- initial state ---------------------------------------------------------
    def set_model_input_shape(self):
        for i, t in enumerate(self.g.tensors):
            if t.dims is not None:
                self.S[i] = [Expr.parse(d) for d in t.dims]
            if t.data is not None and t.dtype in ("i64", "i32") and t.data.size <= MAX_V and t.data.ndim <= 1:
                self.V[i] = [C(int(v)) for v in t.data.reshape(-1)]

    # -- state update: meet the new information into the stored one ------------
    def _refine(self, store: list, tid: int, new) -> bool:
        if new is UNDEF:
            return False
        old = store[tid]
        upd = meet_list(old, new)
        if same(old, upd):
            return False
        store[tid] = upd
        return True

    def analyse(self, order: Optional[List[int]] = None):
        g = self.g
        order = self.sorted_nodes() if order is None else order
        self.set_model_input_shape()
        changed = True
        while changed:
            changed = False
            self.sweeps += 1
            for n in order:
                op = g.ops[n]
                if op.kind == "Combine":
                    changed |= self._merge(op)
                    continue
                if op.kind == "Switch":
                    for o in op.outputs:                       # transit to all successors
                        changed |= self._refine(self.S, o, self.S[op.inputs[0]])
                        changed |= self._refine(self.V, o, self.V[op.inputs[0]])
                    for o in op.outputs:                       # and back (input = output)
                        changed |= self._refine(self.S, op.inputs[0], self.S[o])
                    continue
                changed |= self._forward(op, n)
                for k, t in enumerate(op.inputs):
                    if has_undef(self.S[t]) or (g.tensors[t].dtype in ("i64", "i32") and has_undef(self.V[t])):
                        changed |= self._backward(op, k)
        # an undef left at the fixed point cannot be planned: lower it to nac
        for store in (self.S, self.V):
            for i, x in enumerate(store):
                if x is UNDEF:
                    store[i] = NAC
                elif isinstance(x, list):
                    store[i] = [NAC if e is UNDEF else e for e in x]
        return self

    def _merge(self, op) -> bool:
        ch = False
        s = v = UNDEF
        for t in op.inputs:
            s = meet_list(s, self.S[t])
            v = meet_list(v, self.V[t]) if self.V[t] is not UNDEF else v
        for o in op.outputs:
            ch |= self._refine(self.S, o, s)
            ch |= self._refine(self.V, o, v)
        return ch

    # -- forward transfer ----------------------------------------------------
    def _forward(self, op, n: int) -> bool:
        cls = OP_CLASS[op.kind]
        if cls == EDO and self.named_edo and op.kind == "NonZero":
            s = self.S[op.inputs[0]]                    # result [rank of the input, number of non-zeros]
            if s is UNDEF:
                return False
            res = [(NAC if s == NAC else [C(len(s)), Expr.sym(exec_symbol(n))], NAC)]
        elif cls == EDO and self.named_edo and op.kind == "NMS":
            if self.S[op.inputs[0]] is UNDEF:
                return False
            res = [([Expr.sym(exec_symbol(n))], NAC)]   # the kept boxes' indices: a vector whose length is found by running
        elif cls == EDO:
            res = [(NAC, NAC) for _ in op.outputs]
        else:
            r = getattr(self, "_f_" + op.kind if op.kind not in UNARY else "_f_unary")(op)
            if r is None:
                return False
            res = [r] * len(op.outputs)                 # (TopK: values and indices have one shape)
        ch = False
        for o, (s, v) in zip(op.outputs, res):
            ch |= self._refine(self.S, o, s)
            if self.g.tensors[o].dtype in ("i64", "i32"):
                ch |= self._refine(self.V, o, v)
        return ch

    def _shape(self, t):
        return self.S[t]

    def _f_Shape(self, op):
        s = self.S[op.inputs[0]]
        if s is UNDEF:
            return None
        if s == NAC:
            return NAC, NAC
        return [C(len(s))], list(s)          # ISDO: the value is the symbolic shape of the input

    def _f_unary(self, op):
        s = self.S[op.inputs[0]]
        return None if s is UNDEF else ((NAC if s == NAC else list(s)), UNDEF)

    def _f_Transpose(self, op):
        s = self.S[op.inputs[0]]
        if s is UNDEF:
            return None
        if s == NAC:
            return NAC, UNDEF
        perm = op.attrs["perm"]
        if len(perm) != len(s):
            raise ShapeMismatch("Transpose rank")
        return [s[p] for p in perm], UNDEF

    def _f_Gather(self, op):
        d, i = self.S[op.inputs[0]], self.S[op.inputs[1]]
        if d is UNDEF or i is UNDEF:
            return None
        if d == NAC or i == NAC:
            return NAC, NAC
        ax = op.attrs["axis"] % len(d)
        s = d[:ax] + list(i) + d[ax + 1:]
        dv, iv = self.V[op.inputs[0]], self.V[op.inputs[1]]
        v = UNDEF
        if isinstance(dv, list) and isinstance(iv, list) and len(d) == 1:
            if all(is_expr(e) and e.is_const() for e in iv):
                v = [dv[e.const_value() % len(dv)] for e in iv]
            else:
                v = NAC
        elif dv == NAC or iv == NAC:
            v = NAC
        return s, v

    def _f_Concat(self, op):
        shapes = [self.S[t] for t in op.inputs]
        if any(s is UNDEF for s in shapes):
            return None
        if any(s == NAC for s in shapes):
            return NAC, NAC
        r = len(shapes[0])
        if any(len(s) != r for s in shapes):
            raise ShapeMismatch("Concat rank")
        ax = op.attrs["axis"] % r
        out = []
        for k in range(r):
            if k == ax:
                tot = C(0)
                for s in shapes:
                    tot = d_add(tot, s[k])
                out.append(tot)
            else:
                m = UNDEF
                for s in shapes:
                    m = meet(m, s[k])
                out.append(m)
        vals = [self.V[t] for t in op.inputs]
        v = UNDEF
        if r == 1 and all(isinstance(x, list) for x in vals):
            v = [e for x in vals for e in x]
        elif any(x == NAC for x in vals):
            v = NAC
        return out, v

    def _f_Reshape(self, op):
        x, tv = self.S[op.inputs[0]], self.V[op.inputs[1]]
        ts = self.S[op.inputs[1]]
        if x is UNDEF or ts is UNDEF or tv is UNDEF:
            return None
        if tv == NAC:                                   # only the rank may be known
            if ts != NAC and is_expr(ts[0]) and ts[0].is_const():
                return [NAC] * ts[0].const_value(), UNDEF
            return NAC, UNDEF
        out, infer = [], -1
        for k, e in enumerate(tv):
            if is_expr(e) and e.is_const() and e.const_value() == 0:
                out.append(x[k] if isinstance(x, list) and k < len(x) else NAC)
            elif is_expr(e) and e.is_const() and e.const_value() == -1:
                infer = k
                out.append(UNDEF)
            else:
                out.append(e)
        if infer >= 0:
            if x == NAC:
                out[infer] = NAC
            else:
                total, known = C(1), C(1)
                for d in x:
                    total = d_mul(total, d)
                for k, d in enumerate(out):
                    if k != infer:
                        known = d_mul(known, d)
                if total is UNDEF or known is UNDEF:
                    return None
                if total == NAC or known == NAC:
                    out[infer] = NAC
                else:
                    q = total.exact_div(known)
                    out[infer] = q if q is not None else NAC
        return out, UNDEF

    def _f_Slice(self, op):
        x = self.S[op.inputs[0]]
        st, en, ax = (self.V[t] for t in op.inputs[1:4])
        if x is UNDEF or st is UNDEF or en is UNDEF or ax is UNDEF:
            return None
        if x == NAC or ax == NAC:
            return NAC, NAC
        out = list(x)
        bounds = []
        for s, e, a in zip(st, en, ax):
            a = a.const_value() % len(x)
            D = x[a]
            if not (is_expr(s) and is_expr(e)):
                out[a] = NAC
                bounds.append(None)
                continue
            # a constant bound follows the usual conventions (negative: counted from the end; INT_MAX: the end);
            # a computed one -- an expression carried by the value map (Section 3: input shape and value determined
            # output shape) -- is a position as it stands: 0 <= start <= end <= extent is checked when it is bound
            lo = (d_add(D, s) if s.const_value() < 0 else s) if s.is_const() else s
            if e.is_const():
                hi = D if e.const_value() >= INT_MAX else (d_add(D, e) if e.const_value() < 0 else e)
            else:
                hi = e
            out[a] = d_sub(hi, lo)
            bounds.append((lo, hi))
        v = UNDEF
        xv = self.V[op.inputs[0]]
        if isinstance(xv, list) and len(x) == 1 and bounds and bounds[0] is not None:
            lo, hi = bounds[0]
            if is_expr(lo) and is_expr(hi) and lo.is_const() and hi.is_const():
                v = xv[lo.const_value():hi.const_value()]
            else:
                v = NAC
        return out, v

    def _f_MatMul(self, op):
        a, b = self.S[op.inputs[0]], self.S[op.inputs[1]]
        if a is UNDEF or b is UNDEF:
            return None
        if a == NAC or b == NAC:
            return NAC, UNDEF
        if len(a) < 2 or len(b) < 2:
            raise ShapeMismatch("MatMul rank")
        if op.attrs.get("transB", 0):
            n, kb = b[-2], b[-1]
        else:
            kb, n = b[-2], b[-1]
        meet(a[-1], kb)                                 # raises when both are known and differ
        return broadcast_shapes(a[:-2], b[:-2]) + [a[-2], n], UNDEF

    def _window(self, d, k, stride, pad):
        """floor((d + 2*pad - k) / stride) + 1."""
        return d_add(d_floordiv(d_add(d, C(2 * pad - k)), C(stride)), C(1))

    def _f_Conv(self, op):
        x, w = self.S[op.inputs[0]], self.S[op.inputs[1]]
        if x is UNDEF or w is UNDEF:
            return None
        if x == NAC or w == NAC:
            return NAC, UNDEF
        if len(x) != 4 or len(w) != 4:
            raise ShapeMismatch("Conv rank")
        meet(x[3], w[3])
        s, p = op.attrs["stride"], op.attrs["pad"]
        kh, kw = w[1].const_value(), w[2].const_value()
        return [x[0], self._window(x[1], kh, s, p), self._window(x[2], kw, s, p), w[0]], UNDEF

    def _f_MaxPool(self, op):
        x = self.S[op.inputs[0]]
        if x is UNDEF:
            return None
        if x == NAC:
            return NAC, UNDEF
        k, s, p = op.attrs["kernel"], op.attrs["stride"], op.attrs["pad"]
        return [x[0], self._window(x[1], k, s, p), self._window(x[2], k, s, p), x[3]], UNDEF

    _f_AveragePool = _f_MaxPool

    def _binary(self, op, vfun):
        a, b = self.S[op.inputs[0]], self.S[op.inputs[1]]
        if a == NAC or b == NAC:
            return NAC, NAC
        if a is UNDEF or b is UNDEF:
            return None
        s = broadcast_shapes(list(a), list(b))
        av, bv = self.V[op.inputs[0]], self.V[op.inputs[1]]
        v = UNDEF
        if isinstance(av, list) and isinstance(bv, list) and len(a) <= 1 and len(b) <= 1:
            n = max(len(av), len(bv))
            if len(av) in (1, n) and len(bv) in (1, n):
                v = [vfun(av[i % len(av)], bv[i % len(bv)]) for i in range(n)]
        return s, v

    def _f_Add(self, op):
        return self._binary(op, d_add)

    def _f_Mul(self, op):
        return self._binary(op, d_mul)

    def _f_ReduceMean(self, op):
        x = self.S[op.inputs[0]]
        if x is UNDEF:
            return None
        if x == NAC:
            return NAC, UNDEF
        axes = {a % len(x) for a in op.attrs["axes"]}
        if op.attrs.get("keepdims", 1):
            return [C(1) if k in axes else d for k, d in enumerate(x)], UNDEF
        return [d for k, d in enumerate(x) if k not in axes], UNDEF

    def _f_ArgMax(self, op):
        x = self.S[op.inputs[0]]
        if x is UNDEF:
            return None
        return (NAC if x == NAC else list(x[:-1])), UNDEF

    def _f_Range(self, op):
        """[start, start + delta, ...) below limit: the length is ceil((limit - start) / delta) for a known
        positive delta (the expression assumes limit >= start); the values are kept while they are few."""
        vs = [self.V[t] for t in op.inputs]
        if any(v is UNDEF for v in vs):
            return None
        if any(not isinstance(v, list) or len(v) != 1 or not is_expr(v[0]) for v in vs):
            return [NAC], NAC
        start, limit, delta = (v[0] for v in vs)
        if not delta.is_const() or delta.const_value() <= 0:
            return [NAC], NAC
        d = delta.const_value()
        n = (limit - start + C(d - 1)).floordiv(d)
        if n.is_const() and n.const_value() < 0:
            n = C(0)
        vals = NAC
        if n.is_const() and n.const_value() <= MAX_V:
            vals = [start + C(i * d) for i in range(n.const_value())]
        return [n], vals

    def _f_Expand(self, op):
        """Broadcast of input 0 against the shape held by the values of input 1."""
        x, tv = self.S[op.inputs[0]], self.V[op.inputs[1]]
        if x is UNDEF or tv is UNDEF:
            return None
        if not isinstance(x, list) or not isinstance(tv, list):
            return NAC, UNDEF
        return broadcast_shapes(list(x), list(tv)), UNDEF

    def _f_ConstantOfShape(self, op):
        """A tensor of the shape held by the *values* of the input, every element the attribute value
        (Table 2 lists it with Shape: the result is known from the input alone, nothing is computed)."""
        ts, tv = self.S[op.inputs[0]], self.V[op.inputs[0]]
        if ts is UNDEF or tv is UNDEF:
            return None
        if isinstance(tv, list):
            v = UNDEF
            if len(tv) <= 1 and all(is_expr(d) and d.is_const() for d in tv):
                n = tv[0].const_value() if tv else 1
                if n <= MAX_V:
                    v = [C(int(op.attrs.get("value", 0)))] * n
            return list(tv), v
        if isinstance(ts, list) and len(ts) == 1 and is_expr(ts[0]) and ts[0].is_const():
            return [NAC] * ts[0].const_value(), UNDEF    # the rank is the length of the shape tensor
        return NAC, UNDEF

    def _f_EyeLike(self, op):
        """The shape of the input, ones on one diagonal (Table 2 lists it with Shape: nothing of the
        input's values is read)."""
        s = self.S[op.inputs[0]]
        if s is UNDEF:
            return None
        if isinstance(s, list) and len(s) != 2:
            raise ShapeMismatch("EyeLike needs a matrix")
        return (NAC if s == NAC else list(s)), UNDEF

    def _f_OneHot(self, op):
        """indices.shape + [depth], the depth read from the value of input 1 (last axis): an input shape
        and value determined output shape (Table 2)."""
        s, dv = self.S[op.inputs[0]], self.V[op.inputs[1]]
        if s is UNDEF or dv is UNDEF:
            return None
        if s == NAC:
            return NAC, UNDEF
        depth = dv[0] if isinstance(dv, list) and len(dv) == 1 and is_expr(dv[0]) else NAC
        return list(s) + [depth], UNDEF

    def _f_TopK(self, op):
        """The k largest entries along the last axis, and their positions: the input's shape with the
        last extent replaced by the value of input 1 (Fig. 3(c): the shape waits for that value)."""
        x, kv = self.S[op.inputs[0]], self.V[op.inputs[1]]
        if x is UNDEF or kv is UNDEF:
            return None
        if x == NAC:
            return NAC, UNDEF
        k = kv[0] if isinstance(kv, list) and len(kv) == 1 and is_expr(kv[0]) else NAC
        return list(x[:-1]) + [k], UNDEF

    def _f_Upsample(self, op):
        """Nearest-neighbour enlargement by whole-number factors held in a host constant: every extent is
        the input's times its factor (with constant factors the operator is as tractable as an ISDOS one,
        the case Section 3 mentions for Upsample)."""
        x = self.S[op.inputs[0]]
        sc = self.g.tensors[op.inputs[1]].data
        if sc is None or any(float(v) != int(v) or int(v) < 1 for v in sc.reshape(-1)):
            raise ShapeMismatch("Upsample factors must be whole host constants >= 1")
        if x is UNDEF:
            return None
        if x == NAC:
            return NAC, UNDEF
        f = [int(v) for v in sc.reshape(-1)]
        if len(f) != len(x):
            raise ShapeMismatch("Upsample rank")
        return [d_mul(d, C(k)) for d, k in zip(x, f)], UNDEF

    def _f_Resize(self, op):
        """Output shape = the values of the sizes input (ISVDOS; lowered when they are resolved)."""
        x, ts, tv = self.S[op.inputs[0]], self.S[op.inputs[1]], self.V[op.inputs[1]]
        if x is UNDEF or ts is UNDEF or tv is UNDEF:
            return None
        if isinstance(tv, list):
            if isinstance(x, list) and len(x) != len(tv):
                raise ShapeMismatch("Resize rank")
            return list(tv), UNDEF
        if isinstance(x, list):
            return [NAC] * len(x), UNDEF               # the rank survives, the extents do not
        return NAC, UNDEF

    def _f_MaxUnpool(self, op):
        """Output shape = the values of the output_shape input (Table 2 lists MaxUnpool under ISVDOS)."""
        x, ts, tv = self.S[op.inputs[0]], self.S[op.inputs[2]], self.V[op.inputs[2]]
        if x is UNDEF or ts is UNDEF or tv is UNDEF:
            return None
        if isinstance(tv, list):
            if isinstance(x, list) and len(x) != len(tv):
                raise ShapeMismatch("MaxUnpool rank")
            return list(tv), UNDEF
        if isinstance(x, list):
            return [NAC] * len(x), UNDEF
        return NAC, UNDEF

    def _f_ScatterRows(self, op):
        s = self.S[op.inputs[0]]                        # a copy of input 0 with some rows replaced
        return None if s is UNDEF else ((NAC if s == NAC else list(s)), UNDEF)

    def _f_CacheAppend(self, op):
        p, n = self.S[op.inputs[0]], self.S[op.inputs[1]]
        if p is UNDEF or n is UNDEF:
            return None
        if p == NAC or n == NAC:
            return NAC, UNDEF
        return [d_add(p[0], n[0])] + [meet(x, y) for x, y in zip(p[1:], n[1:])], UNDEF

    # -- backward transfer: IS <- F^bs(OS), IV <- F^bv(OS, OV), only where the answer is unique ----
    def _backward(self, op, k) -> bool:
        out = self.S[op.outputs[0]]
        t = op.inputs[k]
        new = UNDEF
        ch0 = False
        if op.kind == "Shape" and k == 0:
            v = self.V[op.outputs[0]]                    # the value of the result *is* the input's shape
            if isinstance(v, list):
                new = list(v)
        elif op.kind == "ConstantOfShape" and k == 0:
            if not isinstance(out, list):                # the result's shape is the value of the input
                return False
            ch = self._refine(self.V, t, [UNDEF if d == NAC else d for d in out])
            return self._refine(self.S, t, [C(len(out))]) or ch
        elif op.kind in UNARY and k == 0:
            new = out if out != NAC else UNDEF
            if op.kind == "Cast" and g_is_int(self.g, t) and g_is_int(self.g, op.outputs[0]):
                ch0 = self._backward_values(op, t, self.V[op.outputs[0]])     # F^bv: an integer Cast changes no value
        elif op.kind == "Add" and g_is_int(self.g, t):
            # F^bv: with the other operand's values known, in = out - other (unique when this operand has as
            # many elements as the result: a broadcast one could not be told from its repeats)
            ov, other = self.V[op.outputs[0]], self.V[op.inputs[1 - k]]
            if isinstance(ov, list) and isinstance(other, list) and len(other) in (1, len(ov)) and \
                    not any(e is UNDEF or e == NAC for e in other):
                return self._backward_values(op, t, [d_sub(ov[i], other[i % len(other)]) for i in range(len(ov))])
            return False
        elif op.kind == "Concat" and g_is_int(self.g, t):
            # F^bv: input k of a Concat of vectors holds the elements behind those of the inputs before it
            ov = self.V[op.outputs[0]]
            lens = [self.S[i] for i in op.inputs]
            if isinstance(ov, list) and all(isinstance(x, list) and len(x) == 1 and is_expr(x[0]) and x[0].is_const() for x in lens):
                n = [x[0].const_value() for x in lens]
                if sum(n) == len(ov):
                    return self._backward_values(op, t, ov[sum(n[:k]):sum(n[:k + 1])])
            return False
        elif op.kind == "Transpose" and isinstance(out, list):
            perm = op.attrs["perm"]
            new = [UNDEF] * len(perm)
            for i, p in enumerate(perm):
                new[p] = out[i]
        elif op.kind == "MatMul" and k == 0:
            b = self.S[op.inputs[1]]
            if isinstance(b, list) and len(b) == 2:
                kdim = b[1] if op.attrs.get("transB", 0) else b[0]
                if isinstance(out, list):
                    new = out[:-1] + [kdim]
                elif isinstance(self.S[t], list):
                    new = [UNDEF] * (len(self.S[t]) - 1) + [kdim]
        elif op.kind == "Conv" and k == 0:
            w = self.S[op.inputs[1]]
            if isinstance(w, list):
                n = out[0] if isinstance(out, list) else UNDEF
                new = [n, UNDEF, UNDEF, w[3]]
        if new is UNDEF:
            return ch0
        new = [UNDEF if d == NAC else d for d in new]    # a nac carries no backward information
        return self._refine(self.S, t, new) or ch0

    def _backward_values(self, op, t, vals) -> bool:
        """IV <- F^bv(OV): the values of input t, as many as it has elements (a vector or a scalar, known to RDP)."""
        s = self.S[t]
        if not isinstance(vals, list) or not isinstance(s, list) or len(s) > 1:
            return False
        if len(s) == 1 and not (is_expr(s[0]) and s[0].is_const() and s[0].const_value() == len(vals)):
            return False
        if len(s) == 0 and len(vals) != 1:
            return False
        return self._refine(self.V, t, [UNDEF if d == NAC else d for d in vals])


# ---------------------------------------------------------------------------
# canonical text dump (compared byte for byte with the library's)
# ---------------------------------------------------------------------------

def fmt_scalar(d) -> str:
    if d is UNDEF:
        return "undef"
    if d == NAC:
        return "nac"
    return {"known": "k", "symbolic": "s", "opinf": "e"}[d.kind()] + ":" + str(d)


def fmt_list(x) -> str:
    if x is UNDEF:
        return "undef"
    if x == NAC:
        return "nac"
    return "[" + ", ".join(fmt_scalar(d) for d in x) + "]"


def dump(r: RDP) -> str:
    lines = []
    for i, t in enumerate(r.g.tensors):
        v = fmt_list(r.V[i]) if t.dtype in ("i64", "i32") else "-"
        lines.append(f"t{i} {t.name} S={fmt_list(r.S[i])} V={v}")
    return "\n".join(lines) + "\n"
