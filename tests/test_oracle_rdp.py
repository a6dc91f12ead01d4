"""Pins for the oracle's expressions and RDP (Section 4.1): brute-force execution, the
worked examples of Sections 3 and 4.2, lattice laws and order independence."""
import itertools
import os
import random

import numpy as np
import pytest

from oracle import rdp as R
from oracle import execute, plan
from oracle.expr import Expr
from workloads import configs, GraphBuilder

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def analyse(g, order=None):
    return R.RDP(g).analyse(order)


def test_expr_matches_integer_arithmetic():
    H, W = Expr.sym("H"), Expr.sym("W")
    e = ((H + Expr.const(6) - Expr.const(7)).floordiv(2) + Expr.const(1))
    e2 = (e + Expr.const(2) - Expr.const(3)).floordiv(2) + Expr.const(1)
    prod = (e2 * W * Expr.const(3) - W).mod(5)
    for h in range(1, 70):
        a = (h + 6 - 7) // 2 + 1
        b = (a + 2 - 3) // 2 + 1
        assert e.eval({"H": h}) == a and e2.eval({"H": h}) == b
        for w in (1, 2, 7):
            assert prod.eval({"H": h, "W": w}) == (b * w * 3 - w) % 5
    assert str(e2) == "1 + floordiv(-1 + H, 4)"                 # nested floors merge
    assert (H * W + W * H - Expr.const(2) * H * W) == Expr.const(0)
    assert (H * Expr.const(4)).floordiv(2) == H * Expr.const(2)
    assert (Expr.const(-3)).floordiv(2).const_value() == -2      # floor, not truncation
    assert (H * W * Expr.const(2304)).exact_div(H * Expr.const(36)) == W * Expr.const(64)
    assert (H + W).exact_div(H) is None


def test_meet_is_a_lattice_meet():
    a, b, k = Expr.sym("a"), Expr.sym("b"), Expr.const(3)
    vals = [R.UNDEF, R.NAC, a, b, k, a + k]
    for x, y in itertools.product(vals, repeat=2):
        assert R.same(R.meet(x, y), R.meet(y, x))
        for z in vals:
            assert R.same(R.meet(R.meet(x, y), z), R.meet(x, R.meet(y, z)))
    for x in vals:
        assert R.same(R.meet(x, x), x)
        assert R.same(R.meet(R.UNDEF, x), x)
        assert R.meet(R.NAC, x) == R.NAC
    assert R.meet(a, b) == R.NAC
    with pytest.raises(R.ShapeMismatch):
        R.meet(Expr.const(3), Expr.const(4))


def _tiny_graphs():
    # (graph, dict of symbol ranges to sweep)
    b = GraphBuilder([("I", 1, 6), ("J", 1, 6)])
    x = b.input("x", "f32", ["I", "J", 8])
    w = b.weight("w", "f32", [12, 8])
    y = b.op("MatMul", [x, w], transB=1)
    shp = b.op("Shape", [y], dtype="i64")
    d0 = b.op("Gather", [shp, b.const("i0", [0])], axis=0, dtype="i64")
    d1 = b.op("Gather", [shp, b.const("i1", [1])], axis=0, dtype="i64")
    tgt = b.op("Concat", [b.op("Mul", [d0, d1], dtype="i64"), b.const("m1", [-1])], axis=0, dtype="i64")
    z = b.op("Reshape", [y, tgt])
    z = b.op("Transpose", [z], perm=(1, 0))
    z = b.op("Slice", [z, b.const("s", [2]), b.const("e", [2 ** 31 - 1]), b.const("a", [0])])
    z = b.op("ReduceMean", [z], axes=(0,), keepdims=0)
    b.mark_output(b.op("Softmax", [z], causal=0))
    g1 = b.build()

    b = GraphBuilder([("H", 5, 40), ("W", 5, 40)])
    x = b.input("x", "f32", [2, "H", "W", 3])
    w1 = b.weight("w1", "f32", [4, 3, 3, 3])
    y = b.op("Conv", [x, w1], stride=2, pad=1)
    y = b.op("MaxPool", [y], kernel=3, stride=2, pad=1)
    w2 = b.weight("w2", "f32", [4, 1, 1, 4])
    y2 = b.op("Conv", [y, w2], stride=1, pad=0)
    y = b.op("Relu", [b.op("Add", [y2, y])])
    b.mark_output(b.op("ReduceMean", [y], axes=(1, 2), keepdims=0))
    g2 = b.build()
    return [g1, g2]


@pytest.mark.parametrize("gi", [0, 1])
def test_rdp_shapes_equal_brute_force_execution(gi):
    """Every inferred dim, evaluated at the symbols, equals the shape obtained by running the op."""
    g = _tiny_graphs()[gi]
    r = analyse(g)
    rs = np.random.RandomState(0)
    ranges = [range(lo, hi + 1, 1 if gi == 0 else 3) for _, lo, hi in g.symbols]
    for vals in itertools.product(*ranges):
        env = dict(zip([s[0] for s in g.symbols], vals))
        ins = {t: rs.randn(*[env.get(d, d) for d in g.tensors[t].dims]) for t in g.inputs()}
        ws = {t: rs.randn(*g.tensors[t].dims) for t in g.weights()}
        res = execute.run(g, r.sorted_nodes(), ws, ins)
        for t, v in res.values.items():
            s = r.S[t]
            assert isinstance(s, list), g.tensors[t].name
            assert [d.eval(env) for d in s] == list(np.shape(v)), (g.tensors[t].name, env)
            if isinstance(r.V[t], list):
                assert [e.eval(env) for e in r.V[t]] == [int(q) for q in np.reshape(v, -1)]


@pytest.mark.parametrize("cfg,draws", [(1, [{"L": 16}, {"L": 37}]), (3, [{"H": 225, "W": 97}, {"H": 64, "W": 64}])])
def test_rdp_shapes_on_configs(cfg, draws):
    w = configs.config1() if cfg == 1 else configs.resnet50(3, 2, sizes=(64, 225), stages=(1, 1, 1, 1))
    g = w.graph
    g.symbols = [(n, 1, 10 ** 4) for n, _, _ in g.symbols]
    r = analyse(g)
    W = w.make_weights()
    for env in draws:
        res = execute.run(g, r.sorted_nodes(), W, w.make_inputs(0, env))
        for t, v in res.values.items():
            assert [d.eval(env) for d in r.S[t]] == list(np.shape(v))


def test_fig4_fusion_versions_match_paper():
    gold = dict(l.split() for l in open(os.path.join(GOLD, "fig4_fusion_versions.txt")) if l[0] != "#")
    I, J, K = Expr.sym("I"), Expr.sym("J"), Expr.sym("K")
    B = [I, J, K]
    assert R.fused_versions([R.NAC] * 3, B) == int(gold["unknown_A"])
    assert R.fused_versions([I, Expr.const(1), Expr.const(1)], B) == int(gold["rdp_I_1_1"])
    # and through the analysis + fusion rule.  With the RDP result (A = [I, 1, 1]) the pair fuses into one group with
    # a single code version; with nothing known about A it still fuses, as the paper's second option, with the 8
    # versions the figure counts; 2 and 4 versions in between; with multi-versioning off (max_versions = 1) or a cap
    # below the need the pair stays two groups (the paper's first option: no fusion)
    def graph(dimsA):
        b = GraphBuilder([(s, 1, 9) for s in "IJKPQR"])
        A = b.input("A", "f32", dimsA)
        Bt = b.input("B", "f32", ["I", "J", "K"])
        b.mark_output(b.op("Add", [b.op("Sigmoid", [A]), Bt]))
        return b.build()
    for dimsA, versions in ((["I", 1, 1], int(gold["rdp_I_1_1"])), (["I", "Q", 1], 2), (["P", "Q", 1], 4),
                            (["P", "Q", "R"], int(gold["unknown_A"]))):
        g = graph(dimsA)
        p = plan.build_plan(g, analyse(g))
        assert len(p.groups) == 1 and p.groups[0].versions == versions, dimsA
        assert len(p.groups[0].unproven) == {1: 0, 2: 1, 4: 2, 8: 3}[versions]
        p1 = plan.build_plan(g, analyse(g), plan.Opts(max_versions=1))
        assert len(p1.groups) == (1 if versions == 1 else 2)
        p4 = plan.build_plan(g, analyse(g), plan.Opts(max_versions=4))
        assert len(p4.groups) == (1 if versions <= 4 else 2)
    # a rank-4 pair with four unrelated extents would need 16 versions: beyond the cap, not fused
    b = GraphBuilder([(s, 1, 9) for s in "IJKLPQRS"])
    A = b.input("A", "f32", ["P", "Q", "R", "S"])
    Bt = b.input("B", "f32", ["I", "J", "K", "L"])
    b.mark_output(b.op("Add", [b.op("Sigmoid", [A]), Bt]))
    g = b.build()
    assert len(plan.build_plan(g, analyse(g)).groups) == 2


def test_unproven_broadcast_extent_is_an_operation_inferred_constant():
    """Two unrelated symbolic extents broadcast to bcast(a, b): resolved once the symbols are bound (the common value,
    or the other one when one is 1), an error when they cannot broadcast; the version selected at bind says which
    case held, and the values equal the plain operator-by-operator run whatever the version."""
    from oracle import arena
    from oracle.expr import BroadcastMismatch
    b = GraphBuilder([(s, 1, 9) for s in "IJKPQR"])
    A = b.input("A", "f32", ["P", "Q", "R"])
    Bt = b.input("B", "f32", ["I", "J", "K"])
    out = b.mark_output(b.op("Mul", [b.op("Add", [b.op("Sigmoid", [A]), Bt]), b.const("two", 2.0, "f32")]))
    g = b.build()
    r = analyse(g)
    assert R.fmt_list(r.S[out]) == "[e:bcast(I, P), e:bcast(J, Q), e:bcast(K, R)]"
    I, P = Expr.sym("I"), Expr.sym("P")
    e = I.bcast(P)
    assert e == P.bcast(I) and e.kind() == "opinf"
    assert I.bcast(I) == I and I.bcast(Expr.const(1)) == I and Expr.const(1).bcast(P) == P
    assert [e.eval({"I": i, "P": p}) for i, p in ((5, 5), (5, 1), (1, 7))] == [5, 5, 7]
    with pytest.raises(BroadcastMismatch):
        e.eval({"I": 5, "P": 3})
    with pytest.raises(BroadcastMismatch):
        Expr.const(3).bcast(Expr.const(4))
    p = plan.build_plan(g, r)
    assert len(p.groups) == 1 and p.groups[0].versions == 8 and len(p.groups[0].ops) == 3
    rs = np.random.RandomState(5)
    seen = set()
    for sym in (dict(I=3, J=4, K=5, P=3, Q=4, R=5), dict(I=3, J=4, K=5, P=1, Q=4, R=1), dict(I=1, J=4, K=5, P=6, Q=1, R=5),
                dict(I=3, J=1, K=1, P=3, Q=7, R=2)):
        bd = arena.bind(p, sym)
        seen.add(bd.versions[0])
        a = rs.randn(sym["P"], sym["Q"], sym["R"])
        bb = rs.randn(sym["I"], sym["J"], sym["K"])
        res = execute.run(g, p.order, {}, {A: a, Bt: bb})
        ref = ((1.0 / (1.0 + np.exp(-a.astype(np.float32).astype(np.float64)))).astype(np.float32).astype(np.float64)
               + bb.astype(np.float32).astype(np.float64)).astype(np.float32).astype(np.float64) * 2.0
        assert bd.dims[out] == list(ref.shape) == list(res.values[out].shape)
        assert np.allclose(res.values[out], ref, rtol=1e-6)
        # letters: per unproven pair (last dim first) e = equal, a = the Sigmoid result is broadcast, b = B is
        want = "".join("e" if x == y else ("a" if x == 1 else "b")
                       for x, y in ((sym["R"], sym["K"]), (sym["Q"], sym["J"]), (sym["P"], sym["I"])))
        assert bd.versions[0] == want
    assert len(seen) == 4
    with pytest.raises(BroadcastMismatch):
        arena.bind(p, dict(I=3, J=4, K=5, P=2, Q=4, R=5))


def test_backward_add_does_not_invent_a_dim():
    """Section 3: an input dim of Add is 1 or the output dim -- not unique, so nothing is assigned."""
    b = GraphBuilder([("I", 1, 9)])
    a = b.input("a", "f32", None)
    c = b.input("c", "f32", ["I", 4])
    b.mark_output(b.op("Add", [a, c]))
    g = b.build()
    r = analyse(g)
    assert r.S[g.tensor_id("a")] == R.NAC


def test_backward_recovers_input_of_matmul_and_unary():
    b = GraphBuilder([("I", 1, 9)])
    x = b.input("x", "f32", None)
    y = b.op("Relu", [x])
    w = b.weight("w", "f32", [768, 3072])
    z = b.op("MatMul", [y, w], transB=0)
    ref = b.input("ref", "f32", ["I", 5, 3072])
    b.mark_output(b.op("Add", [b.op("Relu", [z]), ref]))
    g = b.build()
    r = analyse(g)
    # rank and last dim come backwards from the weight; leading dims stay unknown (Add is ambiguous)
    assert R.fmt_list(r.S[g.tensor_id("x")]) in ("nac", "[nac, nac, k:768]")
    b2 = GraphBuilder([("I", 1, 9)])
    x = b2.input("x", "f32", None)
    z = b2.op("MatMul", [b2.op("Gelu", [x]), b2.weight("w", "f32", [16, 8])], transB=1)
    b2.mark_output(z)
    g2 = b2.build()
    g2.tensors[z].dims = ["I", 4, 16]        # declared output shape
    r2 = analyse(g2)
    assert R.fmt_list(r2.S[g2.tensor_id("x")]) == "[s:I, k:4, k:8]"


def test_fig1_examples():
    # (a) Shape's value reaches a Reshape through ISDOS operators
    w = configs.config1()
    r = analyse(w.graph)
    g = w.graph
    qkv5 = [i for i, t in enumerate(g.tensors) if t.name.startswith("qkv5")][0]
    assert R.fmt_list(r.S[qkv5]) == "[k:1, s:L, k:3, k:4, k:64]"
    # (b) one known input shape resolves a whole ISDOS sub-graph
    assert all(isinstance(s, list) and all(R.is_expr(d) for d in s) for s in r.S)
    # (c) an execution-determined operator leaves everything after it nac
    b = GraphBuilder([("I", 1, 9)])
    x = b.input("x", "f32", ["I", 4])
    nz = b.op("NonZero", [x], dtype="i64")
    b.mark_output(b.op("Cast", [nz], dtype="f32"))
    g = b.build()
    r = analyse(g)
    assert r.S[nz] == R.NAC and r.S[g.outputs()[0]] == R.NAC
    # (d) Switch / Combine: equal branch shapes survive the merge, a differing dim becomes nac
    for wdim, expect in ((8, "[s:I, k:8]"), (6, None)):
        b = GraphBuilder([("I", 1, 9)])
        x = b.input("x", "f32", ["I", 8])
        p = b.input("p", "f32", [1])
        run, skip = b.op("Switch", [x, p], n_out=2, threshold=0.5)
        y = b.op("MatMul", [run, b.weight("w", "f32", [wdim, 8])], transB=1)
        out = b.op("Combine", [y, skip])
        b.mark_output(out)
        g = b.build()
        if expect:
            assert R.fmt_list(analyse(g).S[out]) == expect
        else:
            with pytest.raises(R.ShapeMismatch):      # two different known constants: an error
                analyse(g)
    b = GraphBuilder([("I", 1, 9), ("J", 1, 9)])
    x = b.input("x", "f32", ["I", 8])
    z = b.input("z", "f32", ["J", 8])
    run, skip = b.op("Switch", [x, b.input("p", "f32", [1])], n_out=2, threshold=0.5)
    out = b.op("Combine", [b.op("Relu", [run]), z])
    b.mark_output(out)
    assert R.fmt_list(analyse(b.build()).S[out]) == "[nac, k:8]"


@pytest.mark.parametrize("cfg", [1, 3, 4])
def test_fixed_point_does_not_depend_on_visiting_order(cfg):
    w = {1: configs.config1, 3: lambda: configs.resnet50(3, 1, stages=(1, 1, 1, 1)),
         4: lambda: configs.config4(1, layers=2)}[cfg]()
    ref = R.dump(analyse(w.graph))
    rnd = random.Random(cfg)
    n = len(w.graph.ops)
    for trial in range(8):
        order = list(range(n))
        rnd.shuffle(order)
        assert R.dump(analyse(w.graph, order)) == ref
    # re-applying every transfer function at the fixed point changes nothing
    r = analyse(w.graph)
    before = R.dump(r)
    for n_ in r.sorted_nodes():
        op = w.graph.ops[n_]
        if op.kind not in ("Switch", "Combine"):
            assert not r._forward(op, n_)
    assert R.dump(r) == before


def test_known_constant_conflict_is_an_error():
    b = GraphBuilder([])
    x = b.input("x", "f32", [4, 8])
    b.mark_output(b.op("MatMul", [x, b.weight("w", "f32", [7, 16])], transB=0))
    with pytest.raises(R.ShapeMismatch):
        analyse(b.build())


def test_operator_classes_follow_table2():
    """The classes of Table 2 for the operators it lists (fixture: tests/golden/table2_operator_classes.txt;
    "Reduce" and "Elementwise w/ broadcast" of the table appear as ReduceMean and Mul), in the oracle and
    in the library."""
    import os
    import paper_2403_00176_amd as S
    rows = [l.split() for l in open(os.path.join(os.path.dirname(__file__), "golden", "table2_operator_classes.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) >= 19
    for name, cls in rows:
        assert R.OP_CLASS[name] == cls, name
        assert S.sod2_op_kind_class(name) == cls, name


def _printed_sweeps(g):
    """Alg. 1 taken literally: the sorted order only, a forward transfer skipped as soon as no output shape
    is undef, a backward transfer towards a predecessor skipped as soon as that predecessor's shape is not
    undef, Combine merged and then passed over, Switch passed over (its outputs take the data input's maps,
    the "transit to all successors" of the listing), until a sweep changes nothing.  Uses the oracle's
    transfer functions but none of analyse()'s control: no re-application, no meet on every visit."""
    r = R.RDP(g)
    r.set_model_input_shape()
    order = r.sorted_nodes()
    changed = True
    while changed:
        changed = False
        r.sweeps += 1
        for n in order:
            op = g.ops[n]
            if op.kind == "Combine":
                changed |= r._merge(op)
                continue
            if op.kind == "Switch":
                for o in op.outputs:
                    if R.has_undef(r.S[o]):
                        changed |= r._refine(r.S, o, r.S[op.inputs[0]])
                        changed |= r._refine(r.V, o, r.V[op.inputs[0]])
                if R.has_undef(r.S[op.inputs[0]]):
                    for o in op.outputs:
                        changed |= r._refine(r.S, op.inputs[0], r.S[o])
                continue
            if any(R.has_undef(r.S[o]) for o in op.outputs):           # forward_transfer's first test
                changed |= r._forward(op, n)
            for k, t in enumerate(op.inputs):
                if R.has_undef(r.S[t]) or (g.tensors[t].dtype in ("i64", "i32") and R.has_undef(r.V[t])):
                    changed |= r._backward(op, k)                       # backward_transfer's first test
    for store in (r.S, r.V):
        for i, x in enumerate(store):
            if x is R.UNDEF:
                store[i] = R.NAC
            elif isinstance(x, list):
                store[i] = [R.NAC if e is R.UNDEF else e for e in x]
    return r


def _alg1_graphs():
    from tests.test_shape_ops import _backward_value_graph, _positions_graph, _generators_graph, _router_graph, small_fpn
    from tests.test_compaction import small
    dec = configs.decoder(5, layers=2, hidden=128, heads=2, ffn=256, vocab=64, p_range=(4, 12), t_max=6)
    return {"config1": configs.config1().graph,
            "config2": configs.config2(1, layers=2).graph,
            "config3": configs.resnet50(3, 1, stages=(1, 1, 1, 1)).graph,
            "config4": configs.config4(1, layers=2).graph,
            "config5_prefill": dec.prefill, "config5_decode": dec.decode,
            "config6": small().graph, "config7": small_fpn().graph,
            "tiny0": _tiny_graphs()[0], "tiny1": _tiny_graphs()[1],
            "positions": _positions_graph()[0], "generators": _generators_graph()[0],
            "router": _router_graph()[0], "backward_value": _backward_value_graph()[0]}


def test_printed_algorithm_reaches_the_same_fixed_point():
    """The reading "every visit re-applies the transfer function and meets the result in" must not change
    what Alg. 1 computes: run literally (sorted order, early returns), the listing gives the same S- and
    V-maps on the configs and on every small graph of this suite, backward-only cases included."""
    for name, g in _alg1_graphs().items():
        assert R.dump(_printed_sweeps(g)) == R.dump(analyse(g)), name
    # graphs whose input shape is recoverable only backwards
    b2 = GraphBuilder([("I", 1, 9)])
    x = b2.input("x", "f32", None)
    z = b2.op("MatMul", [b2.op("Gelu", [x]), b2.weight("w", "f32", [16, 8])], transB=1)
    b2.mark_output(z)
    g2 = b2.build()
    g2.tensors[z].dims = ["I", 4, 16]
    assert R.dump(_printed_sweeps(g2)) == R.dump(analyse(g2))
    assert R.fmt_list(_printed_sweeps(g2).S[g2.tensor_id("x")]) == "[s:I, k:4, k:8]"
