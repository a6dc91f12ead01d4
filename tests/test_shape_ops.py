"""Pins for the input-shape-and-value determined operators added for the detection-style neck
(Table 2, ISVDOS): Resize whose target shape is computed from Shape of another tensor, arithmetic on
value maps, and Concat of activations.  CPU only."""
import numpy as np
import pytest

import paper_2403_00176_amd as S
from oracle import ops as O
from oracle import execute, rdp as R, plan as P, arena as A
from workloads import configs, GraphBuilder


def test_resize_nearest_brute_force_and_repeat():
    rs = np.random.RandomState(9)
    x = rs.randn(2, 3, 5, 4)
    for sizes in ((2, 6, 10, 4), (2, 7, 3, 4), (2, 3, 5, 4), (4, 1, 11, 4)):
        got = O.resize_nearest(x, sizes)
        ref = np.zeros(sizes)
        for i0 in range(sizes[0]):
            for i1 in range(sizes[1]):
                for i2 in range(sizes[2]):
                    ref[i0, i1, i2] = x[i0 * 2 // sizes[0], i1 * 3 // sizes[1], i2 * 5 // sizes[2]]
        assert np.array_equal(got, ref)
    # an exact doubling repeats every pixel (what the neck does on images in multiples of 32)
    assert np.array_equal(O.resize_nearest(x, (2, 6, 10, 4)), np.repeat(np.repeat(x, 2, axis=1), 2, axis=2))


def test_resize_is_lowered_when_its_sizes_are_known_symbolically():
    # sizes = [Shape(x)[0], 2 * Shape(x)[1:3], Shape(x)[3]]: arithmetic on a value map, then Resize
    b = GraphBuilder([("H", 2, 64), ("W", 2, 64)])
    x = b.input("x", "f32", [1, "H", "W", 8])
    shp = b.op("Shape", [x], dtype="i64")
    ax0 = b.const("ax0", [0])
    n = b.op("Slice", [shp, b.const("c0", [0]), b.const("c1", [1]), ax0], dtype="i64")
    hw = b.op("Slice", [shp, b.const("d1", [1]), b.const("d3", [3]), ax0], dtype="i64")
    hw2 = b.op("Mul", [hw, b.const("two", [2, 2])], dtype="i64")
    c = b.op("Slice", [shp, b.const("e3", [3]), b.const("e4", [4]), ax0], dtype="i64")
    sizes = b.op("Concat", [n, hw2, c], axis=0, dtype="i64")
    y = b.op("Resize", [x, sizes])
    b.mark_output(y, "y")
    g = b.build()
    r = R.RDP(g).analyse()
    assert R.fmt_list(r.V[sizes]) == "[k:1, e:2*H, e:2*W, k:8]"
    assert R.fmt_list(r.S[y]) == "[k:1, e:2*H, e:2*W, k:8]"
    assert R.OP_CLASS["Resize"] == R.ISVDOS
    plan = P.build_plan(g, r)
    assert all(plan.folded[n_] for n_, op in enumerate(g.ops) if op.kind != "Resize")     # only the Resize runs
    # brute force over a box of symbol values: the expression equals the shape the operator really produces
    for H in (2, 3, 7):
        for W in (2, 5):
            res = execute.run(g, plan.order, {}, {0: np.zeros((1, H, W, 8))})
            assert list(res.values[y].shape) == [d.eval({"H": H, "W": W}) for d in r.S[y]]
    # the library agrees byte for byte
    gl = S.sod2_graph_build(g)
    rl = S.sod2_rdp_infer(gl)
    assert S.sod2_rdp_dump(rl) == R.dump(r)
    assert S.sod2_plan_dump(S.sod2_plan(gl, rl)) == P.dump(plan)
    assert S.sod2_graph_op_class(gl, len(g.ops) - 1) == "ISVDOS"


def test_resize_with_unknown_sizes_is_nac():
    b = GraphBuilder([("H", 2, 64)])
    x = b.input("x", "f32", [1, "H", 4, 8])
    sizes = b.input("sizes", "i64", [4])                  # values arrive at run time: nothing to propagate
    y = b.op("Resize", [x, sizes])
    b.mark_output(y)
    g = b.build()
    r = R.RDP(g).analyse()
    assert r.S[y] == R.NAC                                 # an ISVDOS operator that cannot be lowered
    gl = S.sod2_graph_build(g)
    assert S.sod2_rdp_dump(S.sod2_rdp_infer(gl)) == R.dump(r)
    mismatch = GraphBuilder([])
    x2 = mismatch.input("x", "f32", [1, 4, 4, 8])
    mismatch.mark_output(mismatch.op("Resize", [x2, mismatch.const("s", [8, 8, 8])]))
    with pytest.raises(R.ShapeMismatch):
        R.RDP(mismatch.build()).analyse()
    with pytest.raises(S.Sod2Error) as e:
        S.sod2_rdp_infer(S.sod2_graph_build(mismatch.build()))
    assert e.value.code == -3


def small_fpn():
    return configs.fpn(7, 4, sizes=(64, 96, 128), stages=(1, 1, 1, 1))


def test_neck_shapes_groups_and_arena():
    w = small_fpn()
    g = w.graph
    r = R.RDP(g).analyse()
    plan = P.build_plan(g, r)
    # the enlarged map has, symbolically, the shape of the map it is concatenated with: no nac anywhere
    assert all(isinstance(s, list) and all(R.is_expr(d) for d in s) for s in r.S)
    for op in g.ops:
        if op.kind == "Resize":
            like = [o for o in g.ops if o.kind == "Concat" and op.outputs[0] in o.inputs and g.tensors[o.outputs[0]].dtype == "bf16"][0]
            other = [t for t in like.inputs if t != op.outputs[0]][0]
            assert [str(d) for d in r.S[op.outputs[0]]] == [str(d) for d in r.S[other]]
    kinds = [plan.groups[it.ref].kind for it in plan.items if it.is_group]
    assert kinds.count("RESIZE") == 2 and kinds.count("CONCAT") == 2
    for n_, op in enumerate(g.ops):                        # every shape computation is folded
        if op.kind in ("Shape", "Slice") or (op.kind == "Concat" and g.tensors[op.outputs[0]].dtype == "i64"):
            assert plan.folded[n_]
    for call in w.calls + [{"H": 96, "W": 64}]:
        b = A.bind(plan, call)
        A.check_no_overlap(b)
        assert b.arena_bytes == b.peak_live
        res = execute.run(g, plan.order, w.make_weights(), w.make_inputs(0, call)) if call is w.calls[0] else None
        if res is not None:
            for t, dims in b.dims.items():
                assert list(res.values[t].shape) == dims
            for t in g.outputs():                          # strides 8, 16, 32
                s_ = {"out8": 8, "out16": 16, "out32": 32}[g.tensors[t].name]
                assert list(res.values[t].shape) == [1, call["H"] // s_, call["W"] // s_, 256]
    # library: same maps, plan and bindings
    gl = S.sod2_graph_build(g)
    rl = S.sod2_rdp_infer(gl)
    assert S.sod2_rdp_dump(rl) == R.dump(r)
    pl = S.sod2_plan(gl, rl)
    assert S.sod2_plan_dump(pl) == P.dump(plan)
    for call in w.calls + [{"H": 96, "W": 64}]:
        assert S.sod2_binding_dump(S.sod2_bind(pl, call)) == A.dump(A.bind(plan, call))


def _positions_graph(dtype="bf16"):
    """x[B, L, 8] + table[Range(0, L)] broadcast over the batch: position ids made in the graph (Range
    with a limit read from Shape), rows gathered by them, Expand to the shape of x."""
    b = GraphBuilder([("B", 1, 8), ("L", 1, 300)])
    x = b.input("x", dtype, ["B", "L", 8])
    table = b.weight("table", dtype, [512, 8])
    shp = b.op("Shape", [x], dtype="i64")
    L = b.op("Gather", [shp, b.const("i1", [1])], axis=0, dtype="i64")
    pos = b.op("Range", [b.const("zero", [0]), L, b.const("one", [1])], dtype="i64", hint="pos")
    rows = b.op("Gather", [table, pos], axis=0, hint="rows")                 # [L, 8]
    wide = b.op("Expand", [rows, shp], hint="wide")                         # [B, L, 8]
    b.mark_output(b.op("Add", [x, wide]), "y")
    b.mark_output(pos, "positions")
    return b.build(), pos, rows, wide


def test_range_and_expand_are_lowered():
    g, pos, rows, wide = _positions_graph()
    r = R.RDP(g).analyse()
    assert R.fmt_list(r.S[pos]) == "[s:L]" and r.V[pos] == R.NAC            # too many values to carry
    assert R.fmt_list(r.S[rows]) == "[s:L, k:8]"
    assert R.fmt_list(r.S[wide]) == "[s:B, s:L, k:8]"
    plan = P.build_plan(g, r)
    kinds = [plan.groups[it.ref].kind for it in plan.items if it.is_group]
    assert kinds == ["RANGE", "GATHER", "ELTWISE"]                           # Expand is a view, the shape ops fold
    for B, L in ((1, 1), (3, 7), (2, 40)):
        res = execute.run(g, plan.order, {1: np.arange(512 * 8).reshape(512, 8) / 64.0}, {0: np.zeros((B, L, 8))})
        assert list(res.values[pos]) == list(range(L))
        assert list(res.values[wide].shape) == [d.eval({"B": B, "L": L}) for d in r.S[wide]]
        assert np.array_equal(res.values[g.tensor_id("y")][B - 1], res.values[rows])
    # a short constant range keeps its values; a step of 3; an empty one
    for start, limit, delta, expect in ((2, 11, 3, [2, 5, 8]), (0, 4, 1, [0, 1, 2, 3]), (5, 5, 2, []), (7, 3, 1, [])):
        b = GraphBuilder([])
        t = b.op("Range", [b.const("s", [start]), b.const("l", [limit]), b.const("d", [delta])], dtype="i64")
        b.mark_output(b.op("Cast", [t], dtype="f32"))
        gd = b.build()
        rr = R.RDP(gd).analyse()
        assert [e.const_value() for e in rr.V[t]] == expect and rr.S[t][0].const_value() == len(expect)
        assert list(np.arange(start, limit, delta)) == expect
        gl = S.sod2_graph_build(gd)
        assert S.sod2_rdp_dump(S.sod2_rdp_infer(gl)) == R.dump(rr)
    gl = S.sod2_graph_build(g)
    rl = S.sod2_rdp_infer(gl)
    assert S.sod2_rdp_dump(rl) == R.dump(r)
    pl = S.sod2_plan(gl, rl)
    assert S.sod2_plan_dump(pl) == P.dump(plan)
    for sym in ({"B": 3, "L": 7}, {"B": 8, "L": 300}):
        assert S.sod2_binding_dump(S.sod2_bind(pl, sym)) == A.dump(A.bind(plan, sym))


def _generators_graph(dtype="f32"):
    """The remaining shape-driven operators of Table 2 in one graph: a constant tensor shaped like x
    (ConstantOfShape of Shape), an identity shaped like a square input (EyeLike), a one-hot code whose
    depth is a dim of another tensor (read through Shape), and an enlargement by whole factors."""
    b = GraphBuilder([("B", 1, 8), ("L", 1, 64), ("N", 1, 48), ("D", 2, 40)])
    x = b.input("x", dtype, ["B", "L", 8])
    sq = b.input("sq", dtype, ["N", "N"])
    ids = b.input("ids", "i64", ["B", "L"])
    table = b.input("table", dtype, ["D", 8])
    half = b.op("ConstantOfShape", [b.op("Shape", [x], dtype="i64")], dtype=dtype, value=0.5, hint="half")
    b.mark_output(b.op("Add", [x, half]), "shifted")
    eye = b.op("EyeLike", [sq], k=1, hint="eye")
    b.mark_output(b.op("Add", [b.op("Mul", [eye, b.const("three", 3.0, "f32")]), sq]), "diag")
    depth = b.op("Gather", [b.op("Shape", [table], dtype="i64"), b.const("i0", [0])], axis=0, dtype="i64")
    hot = b.op("OneHot", [ids, depth, b.const("offon", [0.0, 1.0], "f32")], dtype=dtype, hint="hot")
    b.mark_output(b.op("MatMul", [hot, table]), "picked")                     # [B, L, D] x [D, 8]
    img = b.op("Reshape", [x, b.const("to4", [1, 0, -1, 4])], hint="img")     # [1, L, 2 B... ] any 4-d view
    b.mark_output(b.op("Upsample", [img, b.const("f", [1.0, 2.0, 3.0, 1.0], "f32")], hint="up"), "bigger")
    return b.build(), half, eye, hot


def test_constantofshape_eyelike_onehot_upsample():
    g, half, eye, hot = _generators_graph()
    r = R.RDP(g).analyse()
    assert R.fmt_list(r.S[half]) == "[s:B, s:L, k:8]"
    assert R.fmt_list(r.S[eye]) == "[s:N, s:N]"
    assert R.fmt_list(r.S[hot]) == "[s:B, s:L, s:D]"                            # the depth is a dim of the table
    up = g.tensor_id("bigger")
    assert [str(d) for d in r.S[up]][0] == "1" and [str(d) for d in r.S[up]][3] == "4"
    plan = P.build_plan(g, r)
    kinds = sorted(plan.groups[it.ref].kind for it in plan.items if it.is_group)
    assert kinds == sorted(["FILL", "ELTWISE", "FILL", "ELTWISE", "ONEHOT", "GEMM", "RESIZE"])
    rs = np.random.RandomState(4)
    for B, L, N, D in ((1, 1, 1, 2), (3, 7, 5, 11), (8, 64, 48, 40)):
        sym = {"B": B, "L": L, "N": N, "D": D}
        ins = {g.tensor_id("x"): rs.randn(B, L, 8), g.tensor_id("sq"): rs.randn(N, N),
               g.tensor_id("ids"): rs.randint(-D, D, size=(B, L)), g.tensor_id("table"): rs.randn(D, 8)}
        res = execute.run(g, plan.order, {}, ins)
        f32 = lambda a: O.round_to(a, "f32")
        x, sq, table = (f32(ins[g.tensor_id(n)]) for n in ("x", "sq", "table"))
        ids = ins[g.tensor_id("ids")]
        # closed forms: a shift by the constant, the super-diagonal, a table lookup, pixel repetition
        assert np.array_equal(res.values[g.tensor_id("shifted")], f32(x + 0.5))
        ref = sq.copy()
        ref[np.arange(N - 1), np.arange(1, N)] += 3.0
        assert np.array_equal(res.values[g.tensor_id("diag")], f32(ref))
        assert np.allclose(res.values[g.tensor_id("picked")], table[np.where(ids < 0, ids + D, ids)], rtol=1e-6, atol=1e-6)
        img = x.reshape(1, L, -1, 4)
        assert np.array_equal(res.values[up], np.repeat(np.repeat(img, 2, axis=1), 3, axis=2))
        for t, d in ((half, [B, L, 8]), (eye, [N, N]), (hot, [B, L, D])):
            assert list(res.values[t].shape) == d == [e.eval(sym) for e in r.S[t]]
    # a short integer constant is known to the analysis and folds: nothing runs for it
    b = GraphBuilder([])
    c = b.op("ConstantOfShape", [b.const("s", [3])], dtype="i64", value=7)
    b.mark_output(b.op("Cast", [b.op("Range", [b.const("z", [0]), b.op("Gather", [c, b.const("i", [1])], axis=0, dtype="i64"),
                                              b.const("o", [2])], dtype="i64")], dtype="f32"))
    gd = b.build()
    rr = R.RDP(gd).analyse()
    assert [e.const_value() for e in rr.V[c]] == [7, 7, 7]
    assert P.build_plan(gd, rr).folded[0]
    assert S.sod2_rdp_dump(S.sod2_rdp_infer(S.sod2_graph_build(gd))) == R.dump(rr)
    # whole factors only
    b = GraphBuilder([])
    b.mark_output(b.op("Upsample", [b.input("x", "f32", [1, 4, 4, 2]), b.const("f", [1.0, 1.5, 2.0, 1.0], "f32")]))
    with pytest.raises(R.ShapeMismatch):
        R.RDP(b.build()).analyse()
    with pytest.raises(S.Sod2Error):
        S.sod2_rdp_infer(S.sod2_graph_build(b.build()))
    # the library: identical analysis, plan and bindings
    gl = S.sod2_graph_build(g)
    rl = S.sod2_rdp_infer(gl)
    assert S.sod2_rdp_dump(rl) == R.dump(r)
    pl = S.sod2_plan(gl, rl)
    assert S.sod2_plan_dump(pl) == P.dump(plan)
    for sym in ({"B": 3, "L": 7, "N": 5, "D": 11}, {"B": 8, "L": 64, "N": 48, "D": 40}):
        assert S.sod2_binding_dump(S.sod2_bind(pl, sym)) == A.dump(A.bind(plan, sym))


def _backward_value_graph():
    """Nothing is declared for the input x; the only declared shape is that of an output two operators
    behind a ConstantOfShape(Shape(x)).  The shape reaches x backwards: through the unary operator (shape),
    through ConstantOfShape (the result's shape is the *value* of its input) and through Shape (the
    result's value is the input's shape): the backward value transfer of Table 3."""
    b = GraphBuilder([("B", 1, 8), ("L", 1, 64)])
    x = b.input("x", "f32", None)
    s = b.op("Shape", [x], dtype="i64", hint="s")
    z = b.op("ConstantOfShape", [s], dtype="f32", value=1.0, hint="z")
    y = b.op("Relu", [z])
    b.g.tensors[y].dims = ["B", "L", 8]
    b.mark_output(y, "y")
    b.mark_output(b.op("Add", [x, z]), "sum")
    return b.build(), x, s, z


def test_backward_value_transfer_through_shape_and_constantofshape():
    g, x, s, z = _backward_value_graph()
    r = R.RDP(g).analyse()
    for t in (x, z, g.tensor_id("sum")):
        assert R.fmt_list(r.S[t]) == "[s:B, s:L, k:8]"
    assert R.fmt_list(r.V[s]) == "[s:B, s:L, k:8]" and R.fmt_list(r.S[s]) == "[k:3]"
    # the same fixed point whatever the visiting order
    import random
    order = list(range(len(g.ops)))
    for seed in range(6):
        random.Random(seed).shuffle(order)
        assert R.dump(R.RDP(g).analyse(list(order))) == R.dump(r)
    # without the declared output nothing is known: the transfer invents nothing
    g2, x2, s2, z2 = _backward_value_graph()
    g2.tensors[g2.tensor_id("y")].dims = None
    r2 = R.RDP(g2).analyse()
    assert r2.S[x2] == R.NAC and r2.S[z2] == R.NAC and r2.V[s2] == R.NAC
    # a declared shape that contradicts a constant the forward pass finds is an error, not a silent choice
    g3, x3, _, _ = _backward_value_graph()
    g3.tensors[x3].dims = [2, 5, 9]
    with pytest.raises(R.ShapeMismatch):
        R.RDP(g3).analyse()
    gl = S.sod2_graph_build(g)
    rl = S.sod2_rdp_infer(gl)
    assert S.sod2_rdp_dump(rl) == R.dump(r)
    assert S.sod2_rdp_dump(S.sod2_rdp_infer(S.sod2_graph_build(g2))) == R.dump(r2)
    plan = P.build_plan(g, r)
    pl = S.sod2_plan(gl, rl)
    assert S.sod2_plan_dump(pl) == P.dump(plan)
    sym = {"B": 3, "L": 7}
    assert S.sod2_binding_dump(S.sod2_bind(pl, sym)) == A.dump(A.bind(plan, sym))
    res = execute.run(g, plan.order, {}, {x: np.arange(3 * 7 * 8, dtype=np.float64).reshape(3, 7, 8)})
    assert np.array_equal(res.values[g.tensor_id("sum")], np.arange(168.0).reshape(3, 7, 8) + 1.0)


def _runtime_sizes_graph(declared=True):
    """A target size that arrives as a run-time integer input (`sz`, two values nobody knows ahead of time) and is
    used twice: a Reshape of x to it, and -- through Add, Concat and an integer Cast -- the shape of a zero tensor
    whose extents the graph declares.  That declaration is the only source of knowledge about the values of `sz`."""
    b = GraphBuilder([("B", 1, 8), ("L", 1, 64)])
    x = b.input("x", "f32", ["B", 2, "L", 2])
    sz = b.input("sz", "i64", [2])
    plus = b.op("Add", [sz, b.const("off", [0, 3])])                      # [2 B, 2 L + 3]
    cat = b.op("Concat", [b.const("lead", [2]), plus], axis=0)            # [2, 2 B, 2 L + 3]
    z = b.op("ConstantOfShape", [b.op("Cast", [cat], dtype="i32")], dtype="f32", value=0.0)
    if declared:
        b.g.tensors[z].dims = [2, "B+B", "L+L+3"]
    b.mark_output(z, "zeros")
    y = b.op("Reshape", [x, sz])
    b.mark_output(b.op("Relu", [y]), "y")
    return b.build(), sz, y


def test_backward_value_transfer_through_add_concat_and_cast():
    """Table 3's F^bv beyond Shape / ConstantOfShape: values flow backwards through an integer Cast (unchanged),
    a Concat of vectors (each input gets its own stretch) and an Add whose other operand is known (the
    difference).  The Reshape that reads the same run-time sizes then has a resolved symbolic shape instead of
    nac, so what follows it is planned ahead of time."""
    g, sz, y = _runtime_sizes_graph()
    r = R.RDP(g).analyse()
    assert R.fmt_list(r.V[sz]) == "[e:2*B, e:2*L]"
    assert R.fmt_list(r.S[y]) == "[e:2*B, e:2*L]"
    import random
    order = list(range(len(g.ops)))
    for seed in range(6):
        random.Random(seed).shuffle(order)
        assert R.dump(R.RDP(g).analyse(list(order))) == R.dump(r)
    # without the declaration the sizes stay unknown and the Reshape's result is not a constant of any kind
    g2, sz2, y2 = _runtime_sizes_graph(declared=False)
    r2 = R.RDP(g2).analyse()
    assert r2.V[sz2] == R.NAC and r2.S[y2] == R.NAC
    # an Add never hands values to an operand it may have broadcast (a scalar against a vector result)
    b = GraphBuilder([("B", 1, 8)])
    one = b.input("one", "i64", [1])
    zz = b.op("ConstantOfShape", [b.op("Add", [one, b.const("c", [1, 2])])], dtype="f32", value=0.0)
    b.g.tensors[zz].dims = ["B", "B+1"]
    b.mark_output(zz, "z")
    r3 = R.RDP(b.build()).analyse()
    assert r3.V[one] == R.NAC
    for gg, rr in ((g, r), (g2, r2), (b.build(), r3)):
        assert S.sod2_rdp_dump(S.sod2_rdp_infer(S.sod2_graph_build(gg))) == R.dump(rr)
    plan = P.build_plan(g, r)
    gl = S.sod2_graph_build(g)
    pl = S.sod2_plan(gl, S.sod2_rdp_infer(gl))
    assert S.sod2_plan_dump(pl) == P.dump(plan)
    sym = {"B": 3, "L": 5}
    assert S.sod2_binding_dump(S.sod2_bind(pl, sym)) == A.dump(A.bind(plan, sym))
    xs = np.arange(3 * 2 * 5 * 2, dtype=np.float64).reshape(3, 2, 5, 2) - 20.0
    res = execute.run(g, plan.order, {}, {g.tensor_id("x"): xs, sz: np.array([6, 10])})
    assert np.array_equal(res.values[g.tensor_id("y")], np.maximum(xs.reshape(6, 10), 0.0))
    assert res.values[g.tensor_id("zeros")].shape == (2, 6, 13)


def _router_graph(dtype="f32"):
    """A routing head: scores = x W^T, the K best of them per row (K is a dim of another input, read
    through Shape), softmax over those, and the table rows of the chosen columns picked with a one-hot
    product.  TopK is the paper's own example of an operator whose output shape waits for a value
    (Fig. 3(c)); it is also the one operator here with two results."""
    b = GraphBuilder([("B", 1, 64), ("K", 1, 16)])
    x = b.input("x", dtype, ["B", 64])
    sel = b.input("sel", dtype, ["K", 8])
    wr = b.weight("wr", dtype, [40, 64])
    table = b.weight("table", dtype, [40, 8])
    scores = b.op("MatMul", [x, wr], transB=1, hint="scores")
    kdim = b.op("Gather", [b.op("Shape", [sel], dtype="i64"), b.const("i0", [0])], axis=0, dtype="i64")
    vals, idx = b.op("TopK", [scores, kdim], n_out=2, hint="top")
    b.g.tensors[idx].dtype = "i64"
    b.mark_output(b.op("Softmax", [vals]), "gates")
    hot = b.op("OneHot", [idx, b.const("depth", [40]), b.const("offon", [0.0, 1.0], "f32")], dtype=dtype)
    b.mark_output(b.op("MatMul", [hot, table]), "rows")
    return b.build(), scores, vals, idx


def test_topk_brute_force_and_ties():
    rs = np.random.RandomState(11)
    for shape, k in (((5, 9), 3), ((2, 3, 7), 7), ((4, 6), 1), ((3, 5), 0)):
        x = rs.randint(-2, 3, size=shape).astype(np.float64)         # few distinct values: many ties
        vals, idx = O.topk(x, k)
        assert vals.shape == shape[:-1] + (k,) and idx.shape == vals.shape
        if k == 0:
            continue
        for row, v, i in zip(x.reshape(-1, shape[-1]), vals.reshape(-1, k), idx.reshape(-1, k)):
            taken = []
            for _ in range(k):                                       # pick the largest left, the first of equals
                best = max((j for j in range(len(row)) if j not in taken), key=lambda j: (row[j], -j))
                taken.append(best)
            assert list(i) == taken and list(v) == [row[j] for j in taken]


def test_topk_two_results_one_group():
    g, scores, vals, idx = _router_graph()
    r = R.RDP(g).analyse()
    assert R.fmt_list(r.S[vals]) == "[s:B, s:K]" == R.fmt_list(r.S[idx])
    assert R.OP_CLASS["TopK"] == "ISVDOS"
    plan = P.build_plan(g, r)
    top = [gr for gr in plan.groups.values() if gr.kind == "TOPK"]
    assert len(top) == 1 and top[0].out == vals and top[0].also == [idx]
    item = [it for it in plan.items if it.is_group and it.ref == top[0].gid][0]
    assert item.writes == [vals, idx]
    weights = {g.tensor_id("wr"): np.random.RandomState(1).randn(40, 64) * 0.1,
               g.tensor_id("table"): np.random.RandomState(2).randn(40, 8)}
    for B, K in ((1, 1), (5, 3), (64, 16)):
        sym = {"B": B, "K": K}
        bd = A.bind(plan, sym)
        A.check_no_overlap(bd)
        assert bd.dims[vals] == [B, K] == bd.dims[idx]
        assert bd.tensors[vals].start == bd.tensors[idx].start and bd.tensors[idx].bytes == (B * K * 8 + 255) // 256 * 256
        ins = {g.tensor_id("x"): np.random.RandomState(B).randn(B, 64), g.tensor_id("sel"): np.zeros((K, 8))}
        res = execute.run(g, plan.order, weights, ins)
        sc, iv = res.values[scores], res.values[idx]
        assert np.array_equal(np.sort(sc, axis=-1)[:, ::-1][:, :K], res.values[vals])
        assert np.allclose(res.values[g.tensor_id("gates")].sum(-1), 1.0)
        assert np.allclose(res.values[g.tensor_id("rows")], O.round_to(weights[g.tensor_id("table")], "f32")[iv], atol=1e-6)
    # a k that only a run-time value fixes: the shapes behind it wait (nac), as in Fig. 3(c)
    b = GraphBuilder([("B", 1, 8)])
    v2, i2 = b.op("TopK", [b.input("x", "f32", ["B", 32]), b.input("k", "i64", [1])], n_out=2)
    b.mark_output(v2)
    r2 = R.RDP(b.build()).analyse()
    assert R.fmt_list(r2.S[v2]) == "nac" == R.fmt_list(r2.S[i2])
    gl = S.sod2_graph_build(g)
    rl = S.sod2_rdp_infer(gl)
    assert S.sod2_rdp_dump(rl) == R.dump(r)
    assert S.sod2_rdp_dump(S.sod2_rdp_infer(S.sod2_graph_build(b.build()))) == R.dump(r2)
    pl = S.sod2_plan(gl, rl)
    assert S.sod2_plan_dump(pl) == P.dump(plan)
    for sym in ({"B": 5, "K": 3}, {"B": 64, "K": 16}):
        assert S.sod2_binding_dump(S.sod2_bind(pl, sym)) == A.dump(A.bind(plan, sym))


def _computed_slice_graph(dtype="f32"):
    """Slice whose bounds are computed from shapes (Table 2 lists Slice as input shape *and value* determined): the
    difference of neighbouring tokens x[:, 1:L] - x[:, 0:L-1] with L read through Shape (and L - 1 made by arithmetic
    on the value map), and the first M tokens x[:, :M] with M the extent of another input."""
    b = GraphBuilder([("B", 1, 8), ("L", 2, 300), ("M", 1, 300)])
    x = b.input("x", dtype, ["B", "L", 8])
    m = b.input("m", dtype, ["M", 8])
    L = b.op("Gather", [b.op("Shape", [x], dtype="i64"), b.const("i1", [1])], axis=0, dtype="i64")
    Lm1 = b.op("Add", [L, b.const("minus1", [-1])], dtype="i64")
    ax = b.const("ax1", [1])
    late = b.op("Slice", [x, b.const("one", [1]), L, ax], hint="late")           # [B, L - 1, 8]
    early = b.op("Slice", [x, b.const("zero", [0]), Lm1, ax], hint="early")      # [B, L - 1, 8]
    diff = b.op("Add", [late, b.op("Mul", [early, b.const("neg", -1.0, "f32")])], hint="diff")
    b.mark_output(diff, "diff")
    M = b.op("Gather", [b.op("Shape", [m], dtype="i64"), b.const("i0", [0])], axis=0, dtype="i64")
    head = b.op("Slice", [x, b.const("zero2", [0]), M, ax], hint="head")         # [B, M, 8]
    b.mark_output(b.op("Add", [head, m]), "shifted")
    return b.build(), late, early, head


def test_slice_with_computed_bounds_is_lowered():
    g, late, early, head = _computed_slice_graph()
    r = R.RDP(g).analyse()
    assert R.fmt_list(r.S[late]) == "[s:B, e:-1 + L, k:8]" == R.fmt_list(r.S[early])
    assert R.fmt_list(r.S[head]) == "[s:B, s:M, k:8]"
    p = P.build_plan(g, r)
    # both slices are views, the token difference is one fused group with a single code version (the two extents
    # are provably equal: L - 1 both times), and so is the shifted head (M against M)
    kinds = sorted(gr.kind for gr in p.groups.values())
    assert kinds == ["ELTWISE", "ELTWISE"] and all(gr.versions == 1 for gr in p.groups.values())
    rs = np.random.RandomState(3)
    for sym in ({"B": 2, "L": 7, "M": 4}, {"B": 1, "L": 2, "M": 2}, {"B": 3, "L": 33, "M": 1}):
        xv, mv = rs.randn(sym["B"], sym["L"], 8), rs.randn(sym["M"], 8)
        res = execute.run(g, p.order, {}, {g.tensor_id("x"): xv, g.tensor_id("m"): mv})
        x32, m32 = xv.astype(np.float32).astype(np.float64), mv.astype(np.float32).astype(np.float64)
        assert np.allclose(res.values[g.tensor_id("diff")], x32[:, 1:] - x32[:, :-1], atol=1e-6)
        assert np.allclose(res.values[g.tensor_id("shifted")], x32[:, :sym["M"]] + m32, atol=1e-6)
        bd = A.bind(p, sym)
        for t, v in res.values.items():
            if t in bd.dims:
                assert bd.dims[t] == list(np.shape(v))
    lg = S.sod2_graph_build(g)
    lr = S.sod2_rdp_infer(lg)
    assert S.sod2_rdp_dump(lr) == R.dump(r)
    lp = S.sod2_plan(lg, lr)
    assert S.sod2_plan_dump(lp) == P.dump(p)
    for sym in ({"B": 2, "L": 7, "M": 4}, {"B": 8, "L": 300, "M": 300}):
        assert S.sod2_binding_dump(S.sod2_bind(lp, sym)) == A.dump(A.bind(p, sym))


def _groupnorm_graph(dtype="f32", groups=4, channels=32):
    """conv-free block around GroupNormalization (Table 2): y = Relu(GroupNorm(x)) + x on a channels-last image."""
    b = GraphBuilder([("H", 1, 64), ("W", 1, 64)])
    x = b.input("x", dtype, [2, "H", "W", channels])
    gam = b.weight("gn.g", dtype, [channels])
    bet = b.weight("gn.b", dtype, [channels])
    y = b.op("GroupNorm", [x, gam, bet], groups=groups, eps=1e-5, hint="gn")
    b.mark_output(b.op("Add", [b.op("Relu", [y]), x]), "y")
    return b.build(), y


def test_groupnorm_closed_forms_and_structure():
    rs = np.random.RandomState(9)
    # against explicit loops over (sample, group)
    x = rs.randn(2, 5, 3, 12) * 2 + 1
    g_, b_ = rs.randn(12), rs.randn(12)
    got = O.groupnorm(x, g_, b_, 3, 1e-5)
    for n in range(2):
        for gi in range(3):
            slab = x[n, :, :, gi * 4:(gi + 1) * 4]
            ref = (slab - slab.mean()) / np.sqrt(slab.var() + 1e-5) * g_[gi * 4:(gi + 1) * 4] + b_[gi * 4:(gi + 1) * 4]
            assert np.allclose(got[n, :, :, gi * 4:(gi + 1) * 4], ref, atol=1e-12)
    # one group over one position = LayerNorm over the channels; as many groups as channels and a constant image = bias
    row = rs.randn(4, 1, 1, 16)
    assert np.allclose(O.groupnorm(row, g_[:1].repeat(16), b_[:1].repeat(16), 1, 1e-5).reshape(4, 16),
                       O.layernorm(row.reshape(4, 16), g_[:1].repeat(16), b_[:1].repeat(16), 1e-5))
    assert np.allclose(O.groupnorm(np.full((1, 3, 3, 12), 2.5), g_, b_, 12, 1e-5), np.broadcast_to(b_, (1, 3, 3, 12)))
    # eps inside the root: a slab of +-a has variance a^2; eps = 3 a^2 -> the result is +-gamma / 2 + beta
    a = 0.5
    img = np.tile(np.array([a, -a]), (1, 2, 2, 2))                 # [1, 2, 2, 4], two groups of (+a, -a)
    assert np.allclose(O.groupnorm(img, np.ones(4), np.zeros(4), 2, 3 * a * a), img / (2 * a))
    g, y = _groupnorm_graph()
    r = R.RDP(g).analyse()
    assert R.fmt_list(r.S[y]) == "[k:2, s:H, s:W, k:32]" and R.OP_CLASS["GroupNorm"] == "ISVDOS"
    p = P.build_plan(g, r)
    assert sorted(gr.kind for gr in p.groups.values()) == ["ELTWISE", "GROUPNORM"]
    lg = S.sod2_graph_build(g)
    lr = S.sod2_rdp_infer(lg)
    lp = S.sod2_plan(lg, lr)
    assert S.sod2_rdp_dump(lr) == R.dump(r) and S.sod2_plan_dump(lp) == P.dump(p)
    assert S.sod2_op_kind_class("GroupNorm") == "ISVDOS"
    for sym in ({"H": 7, "W": 9}, {"H": 64, "W": 64}):
        assert S.sod2_binding_dump(S.sod2_bind(lp, sym)) == A.dump(A.bind(p, sym))


def _unpool_graph(dtype="f32", known_sizes=True):
    """x [N, h, w, C] and the positions of its elements in a map twice as large per side, whose shape is computed
    in the graph from the shape of x (Shape, Mul by [1, 2, 2, 1]): MaxUnpool's output_shape input."""
    b = GraphBuilder([("N", 1, 4), ("H", 1, 32), ("W", 1, 32)])
    x = b.input("x", dtype, ["N", "H", "W", 8])
    idx = b.input("idx", "i64", ["N", "H", "W", 8])
    if known_sizes:
        shp = b.op("Mul", [b.op("Shape", [x], dtype="i64"), b.const("two", [1, 2, 2, 1])])
    else:
        shp = b.input("shp", "i64", [4])
    y = b.op("MaxUnpool", [x, idx, shp], dtype=dtype)
    b.mark_output(b.op("Relu", [y]), "y")
    return b.build(), y


def _pool_positions(big):
    """Non-overlapping 2 x 2 max-pool of a channels-last map: the maxima and their positions in the flattened map."""
    n, hh, ww, c = big.shape
    h, w = hh // 2, ww // 2
    win = big.reshape(n, h, 2, w, 2, c).transpose(0, 1, 3, 5, 2, 4).reshape(n, h, w, c, 4)
    arg = win.argmax(-1)
    dy, dx = arg // 2, arg % 2
    nn, yy, xx, cc = np.meshgrid(np.arange(n), np.arange(h), np.arange(w), np.arange(c), indexing="ij")
    pos = ((nn * hh + 2 * yy + dy) * ww + 2 * xx + dx) * c + cc
    return win.max(-1), pos


def test_maxunpool_against_its_definition_and_structure():
    """MaxUnpool (Table 2, ISVDOS) puts each pooled value back where the pooling found it, zeros elsewhere:
    pooling the result again returns the pooled values; the sum is preserved; out-of-range positions are dropped.
    The result's shape comes from a value map (computed from Shape here; nac when it is a run-time input)."""
    rs = np.random.RandomState(4)
    big = rs.randn(2, 6, 10, 3) + 3.0                               # positive: the zeros never win a window
    pooled, pos = _pool_positions(big)
    back = O.maxunpool(pooled, pos, [2, 6, 10, 3])
    assert back.shape == big.shape and np.count_nonzero(back) == pooled.size
    assert np.array_equal(back.reshape(-1)[pos.reshape(-1)], pooled.reshape(-1))
    assert np.array_equal(_pool_positions(back)[0], pooled) and np.isclose(back.sum(), pooled.sum())
    assert np.array_equal(back != 0, big == np.repeat(np.repeat(pooled, 2, 1), 2, 2))
    # a hand-made case, and positions outside the result are ignored
    assert np.array_equal(O.maxunpool([5.0, 7.0], [3, 0], [4]), [7.0, 0.0, 0.0, 5.0])
    assert np.array_equal(O.maxunpool([5.0, 7.0, 9.0], [3, -1, 4], [4]), [0.0, 0.0, 0.0, 5.0])
    g, y = _unpool_graph()
    r = R.RDP(g).analyse()
    assert R.fmt_list(r.S[y]) == "[s:N, e:2*H, e:2*W, k:8]" and R.OP_CLASS["MaxUnpool"] == "ISVDOS"
    g2, y2 = _unpool_graph(known_sizes=False)
    assert R.RDP(g2).analyse().S[y2] == R.NAC
    p = P.build_plan(g, r)
    assert sorted(gr.kind for gr in p.groups.values()) == ["ELTWISE", "MAXUNPOOL"]
    lg = S.sod2_graph_build(g)
    lr = S.sod2_rdp_infer(lg)
    lp = S.sod2_plan(lg, lr)
    assert S.sod2_rdp_dump(lr) == R.dump(r) and S.sod2_plan_dump(lp) == P.dump(p)
    assert S.sod2_rdp_dump(S.sod2_rdp_infer(S.sod2_graph_build(g2))) == R.dump(R.RDP(g2).analyse())
    assert S.sod2_op_kind_class("MaxUnpool") == "ISVDOS"
    for sym in ({"N": 1, "H": 3, "W": 5}, {"N": 4, "H": 32, "W": 32}):
        assert S.sod2_binding_dump(S.sod2_bind(lp, sym)) == A.dump(A.bind(p, sym))
    pooled8, pos8 = _pool_positions(rs.randn(2, 6, 10, 8) + 3.0)
    res = execute.run(g, p.order, {}, {g.tensor_id("x"): pooled8, g.tensor_id("idx"): pos8})
    assert np.array_equal(_pool_positions(res.values[g.tensor_id("y")])[0], O.round_to(pooled8, "f32"))


def _avgpool_round_graph(dtype="f32", channels=16, kernel=3, stride=2, pad=1):
    """A quantising pooling block on a channels-last image: q = Round(AveragePool(x) * 4) / 4, and Round(x).
    (Table 2 lists AveragePool and Round with the operators whose output shape follows from the input shapes.)"""
    b = GraphBuilder([("N", 1, 8), ("H", 1, 128), ("W", 1, 128)])
    x = b.input("x", dtype, ["N", "H", "W", channels])
    p = b.op("AveragePool", [x], kernel=kernel, stride=stride, pad=pad, hint="avg")
    q = b.op("Mul", [p, b.const("four", 4.0, "f32")])
    q = b.op("Round", [q])
    q = b.op("Mul", [q, b.const("quarter", 0.25, "f32")])
    b.mark_output(q, "q")
    b.mark_output(b.op("Round", [x]), "rx")
    return b.build(), p


def test_averagepool_and_round_against_their_definitions_and_structure():
    rs = np.random.RandomState(12)
    # explicit loops over every output position, padding positions not counted
    x = rs.randn(2, 7, 6, 3)
    for k, s, p in ((3, 2, 1), (2, 2, 0), (3, 1, 1), (2, 1, 1), (5, 3, 2)):
        got = O.avgpool_nhwc(x, k, s, p)
        oh, ow = (7 + 2 * p - k) // s + 1, (6 + 2 * p - k) // s + 1
        assert got.shape == (2, oh, ow, 3)
        for i in range(oh):
            for j in range(ow):
                vals = [x[:, a, b_, :] for a in range(i * s - p, i * s - p + k) for b_ in range(j * s - p, j * s - p + k)
                        if 0 <= a < 7 and 0 <= b_ < 6]
                assert np.allclose(got[:, i, j, :], np.mean(vals, axis=0), atol=1e-13)
    # a constant image stays that constant, padding or not (a divisor of k*k at the border would lower the rim);
    # the window covering the whole image is the mean over it; a 1 x 1 window is the identity
    assert np.allclose(O.avgpool_nhwc(np.full((1, 5, 5, 2), 3.25), 3, 2, 1), 3.25)
    assert np.allclose(O.avgpool_nhwc(x, 6, 1, 0)[:, 0, 0, :], x[:, :6, :6, :].mean(axis=(1, 2)))
    assert np.array_equal(O.avgpool_nhwc(x, 1, 1, 0), x)
    # a hand-made corner: 2 x 2 image [[1, 2], [3, 4]], window 3, pad 1, stride 1: every window sees all four values
    # except that nothing beyond the image counts -> all four results are 2.5
    assert np.allclose(O.avgpool_nhwc(np.array([1.0, 2, 3, 4]).reshape(1, 2, 2, 1), 3, 1, 1), 2.5)
    # the mean never exceeds the maximum over the same window
    assert (O.avgpool_nhwc(x, 3, 2, 1) <= O.maxpool_nhwc(x, 3, 2, 1) + 1e-12).all()

    g, p = _avgpool_round_graph()
    # Round: halves go to the even integer, the sign survives
    ins = {g.tensor_id("x"): np.array([0.5, 1.5, 2.5, -0.5, -1.5, 2.4999, 2.5001, -3.0] * 2, dtype=np.float64).reshape(1, 1, 1, 16)}
    r = R.RDP(g).analyse()
    po = P.build_plan(g, r)
    out = execute.run(g, po.order, {}, ins)
    assert out.values[g.tensor_id("rx")].reshape(-1)[:8].tolist() == [0.0, 2.0, 2.0, -0.0, -2.0, 2.0, 3.0, -3.0]
    assert np.signbit(out.values[g.tensor_id("rx")].reshape(-1)[3])
    assert R.fmt_list(r.S[p]) == "[s:N, e:1 + floordiv(-1 + H, 2), e:1 + floordiv(-1 + W, 2), k:16]"   # the window formula
    assert R.OP_CLASS["AveragePool"] == "ISDOS" and R.OP_CLASS["Round"] == "ISDOS"
    kinds = sorted(gr.kind for gr in po.groups.values())
    assert kinds == ["AVGPOOL", "ELTWISE", "ELTWISE"]
    chain = [gr for gr in po.groups.values() if gr.kind == "ELTWISE" and len(gr.ops) == 3]
    assert len(chain) == 1                      # Mul, Round, Mul in one loop nest (fp32: the Round sees the stored value)
    gb, _ = _avgpool_round_graph("bf16")
    pb = P.build_plan(gb, R.RDP(gb).analyse())
    assert sorted(len(gr.ops) for gr in pb.groups.values() if gr.kind == "ELTWISE") == [1, 1, 2]   # bf16: the Round starts a chain
    for gg, pp in ((g, po), (gb, pb)):
        lg = S.sod2_graph_build(gg)
        lr = S.sod2_rdp_infer(lg)
        lp = S.sod2_plan(lg, lr)
        assert S.sod2_rdp_dump(lr) == R.dump(R.RDP(gg).analyse()) and S.sod2_plan_dump(lp) == P.dump(pp)
        for sym in ({"N": 1, "H": 1, "W": 1}, {"N": 2, "H": 7, "W": 9}, {"N": 8, "H": 128, "W": 128}):
            assert S.sod2_binding_dump(S.sod2_bind(lp, sym)) == A.dump(A.bind(pp, sym))
    assert S.sod2_op_kind_class("AveragePool") == "ISDOS" and S.sod2_op_kind_class("Round") == "ISDOS"


def _nms_graph(max_out=0, iou=0.5):
    """Detection post-processing: the kept boxes and their scores, gathered by the indices NMS returns
    (Table 2 lists NMS with the execution-determined operators)."""
    b = GraphBuilder([("N", 0, 4096)])
    sc = b.input("scores", "f32", ["N"])
    bx = b.input("boxes", "f32", ["N", 4])
    sel = b.op("NMS", [sc, bx], dtype="i64", max_out=max_out, iou=iou, hint="sel")
    b.mark_output(b.op("Gather", [bx, sel], axis=0), "kept_boxes")
    b.mark_output(b.op("Gather", [sc, sel], axis=0), "kept_scores")
    return b.build(), sel


def _grid_boxes(rs, n, span=40, side=12):
    """Boxes with integer corners (areas, intersections and the products with a dyadic threshold are exact in
    every precision) clustered so that many overlap; scores with ties."""
    x1 = rs.randint(0, span, n)
    y1 = rs.randint(0, span, n)
    boxes = np.stack([x1, y1, x1 + rs.randint(1, side, n), y1 + rs.randint(1, side, n)], axis=1).astype(np.float64)
    scores = rs.randint(0, max(n // 2, 2), n) / 64.0
    return scores, boxes


def _iou64(a, b_):
    iw = max(0.0, min(a[2], b_[2]) - max(a[0], b_[0]))
    ih = max(0.0, min(a[3], b_[3]) - max(a[1], b_[1]))
    inter = iw * ih
    return inter / ((a[2] - a[0]) * (a[3] - a[1]) + (b_[2] - b_[0]) * (b_[3] - b_[1]) - inter)


def test_nms_against_its_definition_and_structure():
    # hand-made: A and B overlap by 2 / 6, C is far away
    boxes = np.array([[0, 0, 2, 2], [1, 0, 3, 2], [10, 10, 12, 12]], dtype=np.float64)
    scores = np.array([0.9, 0.8, 0.7])
    assert O.nms(scores, boxes, 0, 0.3).tolist() == [0, 2]
    assert O.nms(scores, boxes, 0, 0.4).tolist() == [0, 1, 2]
    assert O.nms(scores[::-1].copy(), boxes, 0, 0.3).tolist() == [2, 1]          # visiting order follows the scores
    assert O.nms(scores, boxes, 1, 0.4).tolist() == [0] and O.nms(scores, boxes, 2, 0.4).tolist() == [0, 1]
    # the comparison is strict: an overlap of exactly the threshold survives (1 / 2 here), one just above does not
    half = np.array([[0, 0, 2, 1], [0, 0, 1, 1]], dtype=np.float64)
    assert O.nms(np.array([1.0, 0.5]), half, 0, 0.5).tolist() == [0, 1]
    assert O.nms(np.array([1.0, 0.5]), half, 0, 0.49).tolist() == [0]
    # equal scores: the lower index first (and -0 is the same score as +0); a box never suppresses itself
    same = np.array([[0, 0, 4, 4], [0, 0, 4, 4], [0, 0, 4, 4]], dtype=np.float64)
    assert O.nms(np.array([0.5, 0.5, 0.5]), same, 0, 0.5).tolist() == [0]
    assert O.nms(np.array([0.0, -0.0, 0.0]), np.array([[0, 0, 1, 1], [5, 5, 6, 6], [9, 9, 10, 10]], dtype=np.float64), 0, 0.5).tolist() == [0, 1, 2]
    assert O.nms(np.zeros(0), np.zeros((0, 4)), 0, 0.5).tolist() == []
    # degenerate boxes (zero area) have no overlap with anything: all kept
    assert O.nms(np.array([3.0, 2.0, 1.0]), np.array([[1, 1, 1, 5], [1, 1, 1, 5], [0, 0, 9, 9]], dtype=np.float64), 0, 0.1).tolist() == [0, 1, 2]
    # what fixes the result without naming the procedure: kept boxes in visiting order, no two of them overlap by
    # more than the threshold, and every dropped box overlaps a kept one visited before it
    rs = np.random.RandomState(21)
    for n, thr in ((40, 0.5), (300, 0.25), (300, 0.5), (1000, 0.125)):
        scores, boxes = _grid_boxes(rs, n)
        kept = O.nms(scores, boxes, 0, thr).tolist()
        rank = {int(i): r for r, i in enumerate(np.argsort(-scores, kind="stable"))}
        assert [rank[i] for i in kept] == sorted(rank[i] for i in kept) and len(set(kept)) == len(kept)
        for a_ in range(len(kept)):
            for c_ in range(a_):
                assert _iou64(boxes[kept[a_]], boxes[kept[c_]]) <= thr
        ks = set(kept)
        for i in range(n):
            if i not in ks:
                assert any(rank[j] < rank[i] and _iou64(boxes[i], boxes[j]) > thr for j in kept), i
        assert 0 < len(kept) < n
        lim = O.nms(scores, boxes, 7, thr).tolist()
        assert lim == kept[:7]

    g, sel = _nms_graph()
    assert R.OP_CLASS["NMS"] == "EDO" and S.sod2_op_kind_class("NMS") == "EDO"
    r = R.RDP(g).analyse()
    assert r.S[sel] == R.NAC                               # Alg. 1 as printed: an EDO's output is nac
    po = P.build_plan(g, r)
    assert R.fmt_list(po.rdp.S[sel]) == "[s:@nz0]" and po.exec_ops == [0]   # named: a vector whose length is found by running
    assert [gr.kind for gr in po.groups.values()] == ["NMS", "GATHER", "GATHER"]
    lg = S.sod2_graph_build(g)
    lr = S.sod2_rdp_infer(lg)
    lp = S.sod2_plan(lg, lr)
    assert S.sod2_rdp_dump(lr) == R.dump(r) and S.sod2_plan_dump(lp) == P.dump(po)
    for sym, ev in (({"N": 100}, ()), ({"N": 100}, [0]), ({"N": 100}, [37]), ({"N": 100}, [100]), ({"N": 1}, [1]), ({"N": 4096}, ()), ({"N": 0}, ())):
        assert S.sod2_binding_dump(S.sod2_bind(lp, sym, exec_values=list(ev))) == A.dump(A.bind(po, sym, exec_values=list(ev))), (sym, ev)
    assert "exec @nz0=100 bound" in S.sod2_binding_dump(S.sod2_bind(lp, {"N": 100}))
    with pytest.raises(S.Sod2Error):
        S.sod2_bind(lp, {"N": 100}, exec_values=[101])
    scores, boxes = _grid_boxes(np.random.RandomState(3), 50)
    out = execute.run(g, po.order, {}, {g.tensor_id("scores"): scores, g.tensor_id("boxes"): boxes})
    kept = O.nms(scores, boxes, 0, 0.5)
    assert out.exec_values == [len(kept)] and np.array_equal(out.values[g.tensor_id("kept_boxes")], boxes[kept])
