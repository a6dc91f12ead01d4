"""Differential test on seeded random graphs (CPU only): the library's RDP, plan and binding against the oracle's,
byte for byte, and the oracle's inferred shapes against the shapes of an actual execution.  The graphs mix what the
configurations use one at a time: broadcasting elementwise chains, contractions and convolutions with epilogues, row
operators, pools, GroupNorm, views (Transpose, Slice, Expand, Reshape through computed shapes), Gather by an index
tensor, Concat, ReduceMean, Cast and Round, over two symbols."""
import random

import numpy as np
import pytest

import paper_2403_00176_amd as S
from oracle import rdp as R, plan as P, arena as A, execute
from workloads import GraphBuilder


def random_graph(seed, dtype="f32", wide=False, gates=False, compact=False):
    """``wide``: inner extents of 64 and more and symbols up to 70 x 130, so that contractions take the tiled
    matrix-core kernels with ragged row counts, epilogues and the LayerNorm-behind-a-contraction rule.
    ``gates``: <Switch, Combine> pairs around short branches, each decided by a one-element graph input (so that a
    test sets the decisions exactly).  ``compact``: rows picked by NonZero of a 0 / 1 graph input, a short branch on
    the picked rows only, ScatterRows back (batch compaction with an execution-determined row count)."""
    rnd = random.Random(seed)
    C0 = 64 if wide else 8                       # the inner extent of the inputs
    b = GraphBuilder([("A", 1, 70), ("B", 1, 130)] if wide else [("A", 1, 9), ("B", 1, 12)])
    pool = []                                  # (tensor id, dims as tokens: "A", "B" or an int)
    weights = {}

    def add(t, dims):
        pool.append((t, list(dims)))
        return t

    def weight(dims):
        t = b.weight(f"w{len(weights)}", dtype, dims)
        weights[t] = tuple(dims)
        return t

    add(b.input("x0", dtype, ["A", "B", C0]), ["A", "B", C0])
    add(b.input("x1", dtype, ["A", 1, C0]), ["A", 1, C0])
    add(b.input("x2", dtype, ["B", C0]), ["B", C0])
    add(b.input("img", dtype, [2, "A", "B", C0]), [2, "A", "B", C0])            # channels last
    idx = b.input("idx", "i64", ["B"])                                         # row numbers below 8
    n_const = [0]

    def const(values, dtype="i64"):
        n_const[0] += 1
        return b.const(f"c{n_const[0]}", values, dtype)

    def broadcastable(x, y):
        for p, q in zip(reversed(x), reversed(y)):
            if p != q and p != 1 and q != 1:
                return False
        return True

    def bshape(x, y):
        n = max(len(x), len(y))
        x, y = [1] * (n - len(x)) + list(x), [1] * (n - len(y)) + list(y)
        return [q if p == 1 else p for p, q in zip(x, y)]

    for _ in range(rnd.randint(6, 14)):
        t, d = rnd.choice(pool)
        kind = rnd.choice(["unary", "unary", "binary", "binary", "scalar", "matmul", "layernorm", "softmax", "transpose",
                           "reduce", "concat", "slice", "flatten", "cast", "conv", "pool", "groupnorm", "gather", "expand"] +
                          (["matmul", "matmul", "mlp", "mlp"] if wide else []) + (["gate"] * 4 if gates else []) + (["compact"] * 4 if compact else []))
        if kind == "compact" and b.g.tensors[t].dtype == dtype and len(d) >= 2 and d[0] in ("A", "B"):
            n_masks = sum(1 for op in b.g.ops if op.kind == "NonZero")
            mask = b.input(f"m{n_masks}{d[0]}", "f32", [d[0]])                     # 0 / 1 per row
            nz = b.op("NonZero", [mask], dtype="i64")                               # [1, count]
            rows = b.op("Gather", [nz, const(0)], axis=0, dtype="i64")              # [count]
            x = b.op("Gather", [t, rows], axis=0)                                   # the picked rows
            for _ in range(rnd.randint(1, 3)):
                c = rnd.choice(["unary", "scalar", "softmax", "layernorm"])
                if c == "unary":
                    x = b.op(rnd.choice(["Relu", "Gelu", "Sigmoid"]), [x])
                elif c == "scalar":
                    x = b.op(rnd.choice(["Add", "Mul"]), [x, const(rnd.choice([0.5, 2.0, -1.0]), "f32")])
                elif c == "softmax":
                    x = b.op("Softmax", [x], causal=0)
                elif isinstance(d[-1], int):
                    x = b.op("LayerNorm", [x, weight([d[-1]]), weight([d[-1]])], eps=1e-5)
            add(b.op("ScatterRows", [t, rows, x]), d)
        elif kind == "gate" and b.g.tensors[t].dtype == dtype:
            n_gates = sum(1 for op in b.g.ops if op.kind == "Switch")
            pred = b.input(f"p{n_gates}", "f32", [1])
            taken, other = b.op("Switch", [t, pred], n_out=2, threshold=0.5)

            def branch(x, n_ops):
                for _ in range(n_ops):
                    c = rnd.choice(["unary", "scalar", "softmax", "layernorm"])
                    if c == "unary":
                        x = b.op(rnd.choice(["Relu", "Gelu", "Sigmoid"]), [x])
                    elif c == "scalar":
                        x = b.op(rnd.choice(["Add", "Mul"]), [x, const(rnd.choice([0.5, 2.0, -1.0]), "f32")])
                    elif c == "softmax":
                        x = b.op("Softmax", [x], causal=0)
                    elif isinstance(d[-1], int):
                        x = b.op("LayerNorm", [x, weight([d[-1]]), weight([d[-1]])], eps=1e-5)
                return x
            merged = b.op("Combine", [branch(taken, rnd.randint(1, 3)), branch(other, rnd.randint(0, 2))])
            # (a Combine forwards storage and writes none: behind it an operator, so that the result may be an output)
            add(b.op("Cast", [merged], dtype=dtype) if rnd.random() < 0.5 else b.op("Relu", [merged]), d)
        elif kind == "unary":
            add(b.op(rnd.choice(["Relu", "Gelu", "Sigmoid", "Round"]), [t]), d)
        elif kind == "scalar":
            add(b.op(rnd.choice(["Add", "Mul"]), [t, const(rnd.choice([0.5, 2.0, -1.0]), "f32")]), d)
        elif kind == "binary":
            cands = [(u, e) for u, e in pool if u != t and broadcastable(d, e)]
            if cands:
                u, e = rnd.choice(cands)
                args = [t, u] if rnd.random() < 0.5 else [u, t]
                add(b.op(rnd.choice(["Add", "Mul"]), args), bshape(d, e))
        elif kind == "matmul" and isinstance(d[-1], int) and len(d) >= 2:
            n = rnd.choice([64, 96, 136, 256] if wide else [4, 8, 16])
            y = b.op("MatMul", [t, weight([n, d[-1]])], transB=1)
            if rnd.random() < 0.6:
                y = b.op("Add", [y, weight([n])])
            if rnd.random() < 0.4:
                y = b.op(rnd.choice(["Relu", "Gelu"]), [y])
            add(y, d[:-1] + [n])
        elif kind == "mlp" and isinstance(d[-1], int) and len(d) >= 2:
            # contraction (+ bias, residual) -> LayerNorm -> contraction (+ bias, activation): the pair rule R9 looks for
            n1, n2 = rnd.choice([64, 128, 192]), rnd.choice([64, 96, 256])
            y = b.op("Add", [b.op("MatMul", [t, weight([n1, d[-1]])], transB=1), weight([n1])])
            if n1 == d[-1] and rnd.random() < 0.5:
                y = b.op("Add", [y, t])
            y = b.op("LayerNorm", [y, weight([n1]), weight([n1])], eps=1e-5)
            y = b.op("Add", [b.op("MatMul", [y, weight([n2, n1])], transB=1), weight([n2])])
            if rnd.random() < 0.5:
                y = b.op("Gelu", [y])
            add(y, d[:-1] + [n2])
        elif kind == "layernorm" and isinstance(d[-1], int):
            add(b.op("LayerNorm", [t, weight([d[-1]]), weight([d[-1]])], eps=1e-5), d)
        elif kind == "softmax":
            add(b.op("Softmax", [t], causal=0), d)
        elif kind == "transpose" and len(d) >= 2:
            perm = list(range(len(d)))
            rnd.shuffle(perm)
            add(b.op("Transpose", [t], perm=tuple(perm)), [d[p] for p in perm])
        elif kind == "reduce" and len(d) >= 2:
            ax = rnd.randrange(len(d))
            keep = rnd.randint(0, 1)
            add(b.op("ReduceMean", [t], axes=(ax,), keepdims=keep), [1 if i == ax else e for i, e in enumerate(d)] if keep
                else [e for i, e in enumerate(d) if i != ax])
        elif kind == "concat":
            cands = [(u, e) for u, e in pool if e == d]
            u, e = rnd.choice(cands)
            ax = rnd.randrange(len(d))
            if isinstance(d[ax], int):
                add(b.op("Concat", [t, u], axis=ax), [2 * e2 if i == ax else e2 for i, e2 in enumerate(d)])
        elif kind == "slice" and isinstance(d[-1], int) and d[-1] >= 4:
            lo, hi = 1, d[-1] - 1
            add(b.op("Slice", [t, const([lo]), const([hi]), const([len(d) - 1])]), d[:-1] + [hi - lo])
        elif kind == "flatten" and len(d) >= 3:
            # [.., p, q] -> [.., p * q] through Shape, Slice of the leading dims and Concat with -1
            shp = b.op("Shape", [t], dtype="i64")
            lead = b.op("Slice", [shp, const([0]), const([len(d) - 2]), const([0])], dtype="i64")
            tgt = b.op("Concat", [lead, const([-1])], axis=0, dtype="i64")
            p, q = d[-2], d[-1]
            merged = p * q if isinstance(p, int) and isinstance(q, int) else None
            if merged is not None:
                add(b.op("Reshape", [t, tgt]), d[:-2] + [merged])
        elif kind == "conv" and len(d) == 4 and isinstance(d[3], int):
            k = rnd.choice([1, 3])                      # stride 1 and pad k // 2 keep the image dims
            o = rnd.choice([64, 128] if wide else [4, 8, 16])
            y = b.op("Conv", [t, weight([o, k, k, d[3]])], stride=1, pad=k // 2)
            if rnd.random() < 0.6:
                y = b.op("Add", [y, weight([o])])
            if rnd.random() < 0.5:
                y = b.op("Relu", [y])
            add(y, d[:3] + [o])
        elif kind == "pool" and len(d) == 4:
            add(b.op(rnd.choice(["MaxPool", "AveragePool"]), [t], kernel=3, stride=1, pad=1), d)
        elif kind == "groupnorm" and len(d) >= 2 and isinstance(d[-1], int) and d[-1] % 4 == 0:
            add(b.op("GroupNorm", [t, weight([d[-1]]), weight([d[-1]])], groups=rnd.choice([1, 2, 4]), eps=1e-5), d)
        elif kind == "gather" and len(d) >= 2 and isinstance(d[0], int) and d[0] >= 8:
            add(b.op("Gather", [t, idx], axis=0), ["B"] + d[1:])
        elif kind == "expand":
            cands = [(u, e) for u, e in pool if u != t and len(e) >= len(d) and broadcastable(d, e) and bshape(d, e) == e and e != d]
            if cands:
                u, e = rnd.choice(cands)
                add(b.op("Expand", [t, b.op("Shape", [u], dtype="i64")]), e)
        elif kind == "cast":
            other_dt = "bf16" if dtype == "f32" else "f32"
            add(b.op("Cast", [b.op("Cast", [t], dtype=other_dt)], dtype=dtype), d)
    outs = {pool[-1][0]}
    outs.add(rnd.choice(pool[3:] or pool)[0])
    for k, t in enumerate(sorted(outs)):
        if b.g.tensors[t].role == "inter":
            b.mark_output(t, f"out{k}")
    g = b.build()
    if not g.outputs():
        return None, None, None
    return g, weights, dict(pool)


def concrete(dims, sym):
    return tuple(sym[d] if isinstance(d, str) else d for d in dims)


def make_inputs(g, shapes, sym, rs):
    ins = {}
    for t in g.inputs():
        if g.tensors[t].dtype == "i64":
            ins[t] = rs.randint(0, 8, size=(sym["B"],)).astype(np.int64)
        elif g.tensors[t].name[0] == "m" and g.tensors[t].name[-1] in "AB" and g.tensors[t].name[1:-1].isdigit():
            n = sym[g.tensors[t].name[-1]]                                     # a row mask: none, all, or some rows
            how = rs.randint(0, 4)
            ins[t] = np.zeros(n) if how == 0 else (np.ones(n) if how == 1 else (rs.rand(n) < 0.5).astype(np.float64))
        elif g.tensors[t].name.startswith("p") and g.tensors[t].name[1:].isdigit():
            ins[t] = np.array([float(rs.randint(0, 2))])              # a gate's predicate: 0 or 1 against the threshold 0.5
        else:
            ins[t] = rs.randn(*concrete(shapes[t], sym))
    return ins


def _has(g, *kinds):
    return g is not None and all(any(op.kind == k for op in g.ops) for k in kinds)


def _seeds(n, kinds, **modes):
    """The seeds below n whose draw holds every operator kind named (decided when the tests are collected)."""
    return [s for s in range(n) if _has(random_graph(s, **modes)[0], *kinds)]


@pytest.mark.parametrize("seed,wide", [(s, False) for s in range(60)] + [(s, True) for s in range(25)])
def test_random_graph_library_equals_oracle(seed, wide):
    g, weights, shapes = random_graph(seed, "bf16" if wide else "f32", wide)
    if g is None:
        pytest.skip("no operator survived the draw")
    lg = S.sod2_graph_build(g)
    lr = S.sod2_rdp_infer(lg)
    ro = R.RDP(g).analyse()
    assert S.sod2_rdp_dump(lr) == R.dump(ro)
    # the generator's own bookkeeping of the shapes (plain token arithmetic) agrees with RDP
    for t, d in shapes.items():
        if g.tensors[t].role == "inter":
            got = ro.S[t]
            assert isinstance(got, list) and len(got) == len(d), (g.tensors[t].name, R.fmt_list(got), d)
    for opts in ({}, {"fusion": 0}, {"sep": 0, "inplace": 0}):
        lp = S.sod2_plan(lg, lr, **opts)
        po = P.build_plan(g, ro, P.Opts(**{k: bool(v) for k, v in opts.items()}))
        assert S.sod2_plan_dump(lp) == P.dump(po), opts
        for sym in ({"A": 1, "B": 1}, {"A": 3, "B": 7}, {"A": 70, "B": 130} if wide else {"A": 9, "B": 12}):
            bo = A.bind(po, sym)
            assert S.sod2_binding_dump(S.sod2_bind(lp, sym)) == A.dump(bo), (opts, sym)
            # the layout itself: tensors alive at the same step never share a byte, the arena is at least the peak
            ts = sorted(bo.tensors.values(), key=lambda a: a.offset)
            for i, x in enumerate(ts):
                assert x.offset >= 0 and x.offset % 256 == 0 and x.offset + x.bytes <= bo.arena_bytes
                for y in ts[i + 1:]:
                    if y.offset >= x.offset + x.bytes:
                        break
                    assert x.end < y.start or y.end < x.start, (g.tensors[x.tid].name, g.tensors[y.tid].name, sym)
            assert bo.arena_bytes >= bo.peak_live
    # executed shapes == inferred shapes, values finite
    rs = np.random.RandomState(seed)
    sym = {"A": 3, "B": 5}
    ins = make_inputs(g, shapes, sym, rs)
    W = {t: rs.randn(*d) * 0.3 for t, d in weights.items()}
    po = P.build_plan(g, ro)
    ref = execute.run(g, po.order, W, ins)
    bo = A.bind(po, sym)
    for t in g.outputs():
        assert ref.values[t].shape == concrete(shapes[t], sym) == tuple(bo.dims[t])
        assert np.isfinite(ref.values[t]).all()


@pytest.mark.parametrize("seed", range(40))
def test_random_graph_with_an_undeclared_input(seed):
    """One input loses its declared shape: what backward transfer recovers (and what it leaves nac) must be the same on
    both sides, and so must the outcome of planning and binding: equal dumps, or the same kind of refusal."""
    import copy
    g, weights, shapes = random_graph(seed)
    if g is None:
        pytest.skip("no operator survived the draw")
    g = copy.deepcopy(g)
    floats = [t for t in g.inputs() if g.tensors[t].dtype != "i64"]
    g.tensors[floats[seed % len(floats)]].dims = None
    lg = S.sod2_graph_build(g)

    def oracle():
        ro = R.RDP(g).analyse()
        po = P.build_plan(g, ro)
        return R.dump(ro), P.dump(po), A.dump(A.bind(po, {"A": 3, "B": 7}))

    def library():
        lr = S.sod2_rdp_infer(lg)
        lp = S.sod2_plan(lg, lr)
        return S.sod2_rdp_dump(lr), S.sod2_plan_dump(lp), S.sod2_binding_dump(S.sod2_bind(lp, {"A": 3, "B": 7}))

    def outcome(f):
        try:
            return ("ok",) + f()
        except S.Sod2Error as e:
            return ("refused", {-3: "mismatch", -4: "unresolved", -6: "unsupported"}.get(e.code, e.code))
        except R.ShapeMismatch:
            return ("refused", "mismatch")
        except A.UnresolvedShape:
            return ("refused", "unresolved")
        except ValueError as e:                      # the oracle's "no grouping rule for ..."
            assert "no grouping rule" in str(e)
            return ("refused", "unsupported")

    assert outcome(library) == outcome(oracle)


@pytest.mark.parametrize("seed", _seeds(30, ("Switch",), gates=True))
def test_random_graph_with_gates(seed):
    """<Switch, Combine> pairs in random places: the analysis (a Combine merges its branches), the partition around the
    control operators, and the plan for every decision vector tried -- the one a run of the oracle takes on random
    predicates, all-run, all-skip -- agree between the library and the oracle; the plan with nothing decided binds."""
    g, weights, shapes = random_graph(seed, gates=True)
    lg = S.sod2_graph_build(g)
    lr = S.sod2_rdp_infer(lg)
    ro = R.RDP(g).analyse()
    assert S.sod2_rdp_dump(lr) == R.dump(ro)
    lp = S.sod2_plan(lg, lr)
    po = P.build_plan(g, ro)
    assert S.sod2_plan_dump(lp) == P.dump(po)
    n_sw = sum(1 for op in g.ops if op.kind == "Switch")
    rs = np.random.RandomState(seed)
    sym = {"A": 3, "B": 5}
    W = {t: rs.randn(*d) * 0.3 for t, d in weights.items()}
    vectors = [[False] * n_sw, [True] * n_sw]
    for _ in range(3):
        ref = execute.run(g, po.order, W, make_inputs(g, shapes, sym, rs))
        assert len(ref.decisions) == n_sw                # gates are never nested here: every Switch executes
        vectors.append(list(ref.decisions))
        for t in g.outputs():
            assert ref.values[t].shape == concrete(shapes[t], sym)
    for dec in vectors:
        assert S.sod2_binding_dump(S.sod2_bind(lp, sym, decisions=dec)) == A.dump(A.bind(po, sym, dec)), dec
    arena, peak = S.sod2_binding_arena_bytes(S.sod2_bind(lp, sym))     # nothing decided yet: every branch is planned
    assert arena >= peak > 0


def test_control_results_cannot_be_graph_outputs():
    """A Switch or Combine forwards storage and writes none; as a graph output its result would never reach the
    caller's buffer.  Both planners refuse such a graph, and accept it with a Cast behind the Combine."""
    def graph(cast):
        b = GraphBuilder([("A", 1, 9)])
        x = b.input("x", "f32", ["A", 8])
        run, skip = b.op("Switch", [x, b.input("p", "f32", [1])], n_out=2, threshold=0.5)
        y = b.op("Combine", [b.op("Relu", [run]), skip])
        if cast:
            b.mark_output(y, "y")                     # the builder puts the Cast behind the Combine itself
            assert b.g.ops[-1].kind == "Cast"
        else:
            b.g.tensors[y].is_output = True            # the bare form, as a raw description could state it
        return b.build()
    g = graph(False)
    with pytest.raises(ValueError):
        P.build_plan(g, R.RDP(g).analyse())
    lg = S.sod2_graph_build(g)
    with pytest.raises(S.Sod2Error) as e:
        S.sod2_plan(lg, S.sod2_rdp_infer(lg))
    assert e.value.code == -6
    g = graph(True)
    lg = S.sod2_graph_build(g)
    assert S.sod2_plan_dump(S.sod2_plan(lg, S.sod2_rdp_infer(lg))) == P.dump(P.build_plan(g, R.RDP(g).analyse()))


@pytest.mark.parametrize("seed", _seeds(30, ("NonZero",), compact=True))
def test_random_graph_with_compaction(seed):
    """NonZero / Gather / ScatterRows around short branches in random places: the two analyses (Alg. 1 as printed, and
    with the row counts named), the plan, and the bindings -- at the upper bounds, and with the counts a run of the
    oracle finds, also partly known -- agree between the library and the oracle."""
    g, weights, shapes = random_graph(seed, compact=True)
    lg = S.sod2_graph_build(g)
    lr = S.sod2_rdp_infer(lg)
    ro = R.RDP(g).analyse()
    assert S.sod2_rdp_dump(lr) == R.dump(ro)
    lp = S.sod2_plan(lg, lr)
    po = P.build_plan(g, ro)
    assert S.sod2_plan_dump(lp) == P.dump(po)
    rs = np.random.RandomState(seed)
    W = {t: rs.randn(*d) * 0.3 for t, d in weights.items()}
    for sym in ({"A": 3, "B": 5}, {"A": 9, "B": 12}, {"A": 1, "B": 1}):
        assert S.sod2_binding_dump(S.sod2_bind(lp, sym)) == A.dump(A.bind(po, sym))
        for _ in range(2):
            ref = execute.run(g, po.order, W, make_inputs(g, shapes, sym, rs))
            ev = list(ref.exec_values)
            assert len(ev) == sum(1 for op in g.ops if op.kind == "NonZero")
            for known in (ev, ev[:1]):
                assert S.sod2_binding_dump(S.sod2_bind(lp, sym, exec_values=known)) == A.dump(A.bind(po, sym, exec_values=known)), (sym, known)
            for t in g.outputs():
                assert ref.values[t].shape == concrete(shapes[t], sym)


@pytest.mark.parametrize("seed", _seeds(80, ("Switch", "NonZero"), gates=True, compact=True))
def test_random_graph_with_gates_and_compaction(seed):
    """Both kinds of execution-determined operators in one graph: the plan, and the bindings for the decisions and
    counts a run of the oracle takes, agree between the library and the oracle."""
    g, weights, shapes = random_graph(seed, gates=True, compact=True)
    lg = S.sod2_graph_build(g)
    lr = S.sod2_rdp_infer(lg)
    ro = R.RDP(g).analyse()
    assert S.sod2_rdp_dump(lr) == R.dump(ro)
    lp = S.sod2_plan(lg, lr)
    po = P.build_plan(g, ro)
    assert S.sod2_plan_dump(lp) == P.dump(po)
    rs = np.random.RandomState(seed)
    W = {t: rs.randn(*d) * 0.3 for t, d in weights.items()}
    for sym in ({"A": 3, "B": 5}, {"A": 9, "B": 12}):
        for _ in range(3):
            ref = execute.run(g, po.order, W, make_inputs(g, shapes, sym, rs))
            dec, ev = list(ref.decisions), list(ref.exec_values)
            assert S.sod2_binding_dump(S.sod2_bind(lp, sym, decisions=dec, exec_values=ev)) == \
                A.dump(A.bind(po, sym, dec, ev)), (sym, dec, ev)
