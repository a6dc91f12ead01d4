"""Host half of the library against the oracle, byte for byte: RDP maps, fusion groups,
execution order, executed steps, lifetimes and arena offsets.  No GPU needed."""
import random
import re

import pytest

import paper_2403_00176_amd as S
from oracle import rdp as R, plan as P, arena as A
from workloads import configs, GraphBuilder


def small(cfg):
    return {1: configs.config1, 2: lambda: configs.config2(8, layers=3),
            3: lambda: configs.resnet50(3, 6, stages=(2, 2, 1, 1)),
            4: lambda: configs.config4(6, layers=3),
            6: lambda: configs.config6(6, layers=3)}[cfg]()


def test_library_exports_every_declared_symbol():
    header = open(S.LIB_PATH.replace("paper_2403_00176_amd/libsod2.so", "include/sod2.h")).read()
    declared = set(re.findall(r"\b(sod2_[a-z_0-9]+)\s*\(", header))
    assert declared, "no declarations found"
    for name in declared:
        assert hasattr(S._lib, name), name
    assert declared == set(S.EXPORTS)
    assert "gfx950" in S.sod2_version()


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 6])
def test_rdp_plan_bind_match_oracle(cfg):
    w = small(cfg)
    g = S.sod2_graph_build(w.graph)
    r = S.sod2_rdp_infer(g)
    ro = R.RDP(w.graph).analyse()
    assert S.sod2_rdp_dump(r) == R.dump(ro)
    assert S.sod2_rdp_sweeps(r) == ro.sweeps
    for opts in (dict(), dict(fusion=0), dict(sep=0), dict(dmp=0)):
        p = S.sod2_plan(g, r, **{k: v for k, v in opts.items()})
        po = P.build_plan(w.graph, ro, P.Opts(**{k: bool(v) for k, v in opts.items()}))
        assert S.sod2_plan_dump(p) == P.dump(po)
        n_sw = sum(1 for op in w.graph.ops if op.kind == "Switch")
        assert S.sod2_plan_counts(p) == (len(po.groups), len(po.subgraphs), n_sw)
        rnd = random.Random(cfg)
        for call in w.calls:
            dec = [rnd.random() < 0.5 for _ in range(n_sw)]
            b = S.sod2_bind(p, call, dec)
            bo = A.bind(po, call, dec)
            assert S.sod2_binding_dump(b) == A.dump(bo)
            assert S.sod2_binding_arena_bytes(b) == (bo.arena_bytes, bo.peak_live)
            # execution-determined extents: none, some and all of the NonZero counts known
            n_nz = len(po.exec_ops)
            for known in sorted({0, n_nz // 2, n_nz} - {0} if n_nz else ()):
                ev = [rnd.randint(0, call.get("B", 1)) for _ in range(known)]
                assert S.sod2_binding_dump(S.sod2_bind(p, call, exec_values=ev)) == A.dump(A.bind(po, call, exec_values=ev))


def test_full_size_configs_match_oracle():
    for cfg in (2, 3):
        w = configs.BUILDERS[cfg]()
        g = S.sod2_graph_build(w.graph)
        r = S.sod2_rdp_infer(g)
        ro = R.RDP(w.graph).analyse()
        assert S.sod2_rdp_dump(r) == R.dump(ro)
        p = S.sod2_plan(g, r)
        po = P.build_plan(w.graph, ro)
        assert S.sod2_plan_dump(p) == P.dump(po)
        for call in w.calls[:6]:
            assert S.sod2_binding_dump(S.sod2_bind(p, call)) == A.dump(A.bind(po, call))


def test_order_independence_and_classes():
    w = configs.config4(1, layers=2)
    g = S.sod2_graph_build(w.graph)
    ref = S.sod2_rdp_dump(S.sod2_rdp_infer(g))
    rnd = random.Random(3)
    for _ in range(5):
        order = list(range(len(w.graph.ops)))
        rnd.shuffle(order)
        assert S.sod2_rdp_dump(S.sod2_rdp_infer(g, order)) == ref
    for i, op in enumerate(w.graph.ops):
        assert S.sod2_graph_op_class(g, i) == R.OP_CLASS[op.kind]
    rank, dims = S.sod2_rdp_query(S.sod2_rdp_infer(g), w.graph.tensor_id("x"))
    assert rank == 3 and dims[0][:2] == (0, 4) and dims[1][0] == 1 and dims[1][2] == "L"


def test_error_paths():
    w = configs.config2(1, layers=1)
    g = S.sod2_graph_build(w.graph)
    r = S.sod2_rdp_infer(g)
    p = S.sod2_plan(g, r)
    with pytest.raises(S.Sod2Error) as e:
        S.sod2_bind(p, {"B": 9, "L": 64})
    assert e.value.code == -2
    with pytest.raises(S.Sod2Error) as e:
        S.sod2_bind(p, [1])
    assert e.value.code == -1
    b = GraphBuilder([])
    x = b.input("x", "f32", [4, 8])
    b.mark_output(b.op("MatMul", [x, b.weight("w", "f32", [7, 16])], transB=0))
    with pytest.raises(S.Sod2Error) as e:
        S.sod2_rdp_infer(S.sod2_graph_build(b.build()))
    assert e.value.code == -3
    # a nac shape reaching a kernel is refused at bind
    # (branches whose symbolic dims differ meet in a Combine: those dims are nac, Section 3 / Fig. 1(d))
    b = GraphBuilder([("I", 1, 9), ("J", 1, 9)])
    x = b.input("x", "f32", ["I", "J"])
    pr = b.input("p", "f32", [1])
    run, skip = b.op("Switch", [x, pr], n_out=2, threshold=0.5)
    y = b.op("Gelu", [b.op("Transpose", [run], perm=(1, 0))])
    b.mark_output(b.op("Relu", [b.op("Combine", [y, skip])]))
    gd = b.build()
    g2 = S.sod2_graph_build(gd)
    r2 = S.sod2_rdp_infer(g2)
    p2 = S.sod2_plan(g2, r2)
    with pytest.raises(S.Sod2Error) as e:
        S.sod2_bind(p2, {"I": 3, "J": 4})
    assert e.value.code == -4
    # an execution-determined extent is not an error: it is planned at its upper bound until known
    b = GraphBuilder([("I", 1, 9)])
    x = b.input("x", "f32", ["I", 4])
    nz = b.op("NonZero", [x], dtype="i64")
    b.mark_output(b.op("Cast", [nz], dtype="f32"))
    g3 = S.sod2_graph_build(b.build())
    p3 = S.sod2_plan(g3, S.sod2_rdp_infer(g3))
    assert "exec @nz0=12 bound" in S.sod2_binding_dump(S.sod2_bind(p3, {"I": 3}))
    assert "exec @nz0=5 known" in S.sod2_binding_dump(S.sod2_bind(p3, {"I": 3}, exec_values=[5]))
    with pytest.raises(S.Sod2Error) as e:
        S.sod2_bind(p3, {"I": 3}, exec_values=[13])
    assert e.value.code == -1
    # run without a device: bad pointers are refused before any launch
    bnd = S.sod2_bind(p, {"B": 1, "L": 32})
    with pytest.raises(S.Sod2Error) as e:
        S.sod2_run(bnd, 0, 0, [1] * len(w.graph.weights()), [1], [1])
    assert e.value.code == -5
    w4 = configs.config4(1, layers=2)
    g4 = S.sod2_graph_build(w4.graph)
    p4 = S.sod2_plan(g4, S.sod2_rdp_infer(g4))
    with pytest.raises(S.Sod2Error):
        S.sod2_bind(p4, {"L": 128}, [1])          # one decision short
    assert S.sod2_binding_arena_bytes(S.sod2_bind(p4, {"L": 128}))[0] > 0   # undecided: plans every branch


def test_tiny_fixture_graphs_match_oracle():
    from tests.test_oracle_rdp import _tiny_graphs
    for gd in _tiny_graphs():
        g = S.sod2_graph_build(gd)
        r = S.sod2_rdp_infer(g)
        ro = R.RDP(gd).analyse()
        assert S.sod2_rdp_dump(r) == R.dump(ro)
        assert S.sod2_plan_dump(S.sod2_plan(g, r)) == P.dump(P.build_plan(gd, ro))


@pytest.mark.parametrize("cfg", [2, 3, 4])
def test_structured_queries_agree_with_the_oracle(cfg):
    """sod2_plan_query_group and sod2_binding_query_tensor (records, not text) against the oracle's plan and
    binding objects: groups in planned order with members, inputs, sub-graph and class; per tensor the
    concrete dims, where it lives, offset, bytes and lifetime."""
    w = small(cfg)
    g = S.sod2_graph_build(w.graph)
    r = S.sod2_rdp_infer(g)
    p = S.sod2_plan(g, r)
    po = P.build_plan(w.graph, R.RDP(w.graph).analyse())
    n_groups = S.sod2_plan_counts(p)[0]
    expect = [(s, po.items[i].ref) for s, sg in enumerate(po.subgraphs) for i in sg if po.items[i].is_group]
    assert n_groups == len(expect)
    for k, (sg, gid) in enumerate(expect):
        q = S.sod2_plan_query_group(p, k)
        gr = po.groups[gid]
        assert (q["gid"], q["kind"], q["out"], q["ops"], q["ins"]) == (gr.gid, gr.kind, gr.out, gr.ops, gr.ins)
        assert q["out2"] == (gr.also[0] if gr.also else -1)
        assert (q["subgraph"], q["sg_class"]) == (sg, po.sg_class[sg])
        assert q["inplace_of"] == po.inplace.get(gr.out, -1)
    with pytest.raises(S.Sod2Error):
        S.sod2_plan_query_group(p, n_groups)
    call = w.calls[0]
    n_sw = sum(1 for op in w.graph.ops if op.kind == "Switch")
    dec = [k % 2 == 0 for k in range(n_sw)]
    b = S.sod2_bind(p, call, dec)
    bo = A.bind(po, call, dec)
    for t in range(len(w.graph.tensors)):
        q = S.sod2_binding_query_tensor(b, t)
        assert q["executed"] == (t in bo.dims), t
        if not q["executed"]:
            continue
        assert q["dims"] == list(bo.dims[t])
        if t in bo.tensors:
            a = bo.tensors[t]
            assert (q["where"], q["offset"], q["bytes"], q["life"]) == ("arena", a.offset, a.bytes, (a.start, a.end))
        elif w.graph.tensors[t].is_output:
            assert q["where"] == "external"
    with pytest.raises(S.Sod2Error):
        S.sod2_binding_query_tensor(b, len(w.graph.tensors))


def _multi_version_graph(dimsA=("P", "Q", "R"), dtype="f32"):
    """Sigmoid(A) + B, then * 2: the example of Fig. 4 with one more member; nothing relates A's extents to B's."""
    b = GraphBuilder([(s, 1, 600) for s in "IJKPQR"])
    A = b.input("A", dtype, list(dimsA))
    Bt = b.input("B", dtype, ["I", "J", "K"])
    y = b.op("Mul", [b.op("Add", [b.op("Sigmoid", [A]), Bt]), b.const("two", 2.0, "f32")])
    b.mark_output(y, "y")
    return b.build()


def test_multi_version_groups_match_the_oracle():
    """Section 4.2: a fused chain over extents RDP cannot relate is planned with 2 code versions per unproven dim pair
    (Fig. 4) and the version is selected at bind.  RDP maps (bcast extents), groups, version counts, the selected
    version and the refusal of symbols that do not broadcast: library == oracle."""
    for dimsA in (("I", 1, 1), ("I", "Q", 1), ("P", "Q", 1), ("P", "Q", "R")):
        gd = _multi_version_graph(dimsA)
        g = S.sod2_graph_build(gd)
        r = S.sod2_rdp_infer(g)
        ro = R.RDP(gd).analyse()
        assert S.sod2_rdp_dump(r) == R.dump(ro)
        for mv in (0, 1, 2, 4):
            p = S.sod2_plan(g, r, max_versions=mv)
            po = P.build_plan(gd, ro, P.Opts(max_versions=mv or 8))
            assert S.sod2_plan_dump(p) == P.dump(po), (dimsA, mv)
            q = S.sod2_plan_query_group(p, 0)
            assert q["versions"] == po.groups[q["gid"]].versions
            for sym in (dict(I=3, J=4, K=5, P=3, Q=4, R=5), dict(I=3, J=4, K=5, P=1, Q=1, R=1),
                        dict(I=1, J=4, K=1, P=3, Q=4, R=5), dict(I=3, J=1, K=5, P=3, Q=4, R=1)):
                assert S.sod2_binding_dump(S.sod2_bind(p, sym)) == A.dump(A.bind(po, sym))
    gd = _multi_version_graph()
    g = S.sod2_graph_build(gd)
    r = S.sod2_rdp_infer(g)
    p = S.sod2_plan(g, r)
    with pytest.raises(S.Sod2Error) as e:
        S.sod2_bind(p, dict(I=3, J=4, K=5, P=2, Q=4, R=5))
    assert e.value.code == -3                       # SOD2_ERR_SHAPE_MISMATCH


def test_backend_limits_of_the_fusion_rules_are_options():
    """R6-R8 take their limits (fused head size, rows appended inside attention, LayerNorm-prologue rows / extent)
    from the plan options on both sides: other values change the groups alike."""
    dec = configs.decoder(5, layers=2, hidden=128, heads=2, ffn=256, vocab=64, p_range=(4, 12), t_max=6)
    enc = configs.config2(1, layers=1)
    for gd in (dec.decode, dec.prefill, enc.graph):
        g = S.sod2_graph_build(gd)
        r = S.sod2_rdp_infer(g)
        ro = R.RDP(gd).analyse()
        base = S.sod2_plan_dump(S.sod2_plan(g, r))
        assert base == P.dump(P.build_plan(gd, ro))
        variants = [(dict(attn_head_dim=32), dict(attn_head_dims=(32,))),
                    (dict(append_max_rows=1, prologue_max_rows=1), dict(append_max_rows=1, prologue_max_rows=1)),
                    (dict(prologue_max_k=64), dict(prologue_max_k=64)),
                    (dict(prologue_k_multiple=256), dict(prologue_k_multiple=256))]
        changed = 0
        for lib_opts, ora_opts in variants:
            d = S.sod2_plan_dump(S.sod2_plan(g, r, **lib_opts))
            assert d == P.dump(P.build_plan(gd, ro, P.Opts(**ora_opts))), lib_opts
            changed += d != base
        assert changed >= 1


def test_derived_constants_layout_and_argument_checks():
    """The constants a plan's folded LayerNorms need (R9): two fp32 vectors over the columns of every contraction
    that reads such a LayerNorm, each block rounded up to 256 bytes; none with the rule off or when no pair exists.
    Argument errors are reported on the host (no kernel is launched for them)."""
    w = configs.config2(4, layers=2)
    g = S.sod2_graph_build(w.graph)
    r = S.sod2_rdp_infer(g)
    po = P.build_plan(w.graph, R.RDP(w.graph).analyse())
    readers = [gr for gr in po.groups.values() if gr.lnfold >= 0]
    assert len(readers) == 3
    want = 0
    for gr in readers:
        wt = w.graph.ops[gr.ops[0]].inputs[1]
        n = int(w.graph.tensors[wt].dims[0])
        want += (2 * n * 4 + 255) // 256 * 256
    p = S.sod2_plan(g, r)
    assert S.sod2_plan_constants_bytes(p) == want == 2 * (2 * 3072 * 4) + 2 * 2304 * 4   # FFN1 of both layers, QKV of the second
    assert S.sod2_plan_constants_bytes(S.sod2_plan(g, r, fold_ln=0)) == 0
    w1 = configs.config1()
    g1 = S.sod2_graph_build(w1.graph)
    assert S.sod2_plan_constants_bytes(S.sod2_plan(g1, S.sod2_rdp_infer(g1))) == 0      # fp32 graph: the rule wants bf16
    b = S.sod2_bind(p, {"B": 1, "L": 32})
    with pytest.raises(S.Sod2Error):
        S.sod2_binding_set_constants(b, 0x1008, want)                 # not 256-byte aligned
    S.sod2_binding_set_constants(b, 0, 0)                             # back to the default
    with pytest.raises(S.Sod2Error):
        S.sod2_plan_prepare_constants(p, [0x1000] * 3, 0x1000, want)  # wrong number of weight pointers
    n_w = len(w.graph.weights())
    with pytest.raises(S.Sod2Error):
        S.sod2_plan_prepare_constants(p, [0x1000] * n_w, 0x1000, want - 256)   # buffer too small
    with pytest.raises(S.Sod2Error):
        S.sod2_plan_prepare_constants(p, [0x1000] * n_w, 0x1010, want)         # buffer misaligned


def test_malformed_graphs_are_refused_not_crashed():
    """Descriptors a caller could get wrong are turned into errors at graph build: a cycle (also one through an
    operator that is only a view), a Transpose whose attribute is no permutation, pooling and convolution windows
    that later stages would divide by, an axis outside the rank.  Then a seeded batch of random corruptions of real
    graphs (attributes, ids, types, ranks, roles, dropped operators): each must end in an error or in a plan."""
    import copy
    import random
    w = small(2)

    def build(g):
        h = S.sod2_graph_build(g)
        p = S.sod2_plan(h, S.sod2_rdp_infer(h))
        return S.sod2_bind(p, {"B": 2, "L": 40})

    def mutated(f):
        g = copy.deepcopy(w.graph)
        f(g)
        return g

    def first(g, kind):
        return next(op for op in g.ops if op.kind == kind)

    def self_loop(g):
        op = first(g, "Reshape")
        op.inputs[0] = op.outputs[0]

    def two_cycle(g):
        a, b = [op for op in g.ops if op.kind == "Add"][:2]
        a.inputs[0], b.inputs[0] = b.outputs[0], a.outputs[0]

    cases = {
        "cycle": [self_loop, two_cycle],
        "permutation": [lambda g: first(g, "Transpose").attrs.update(perm=(7, -5, 9, 8, 1)),
                        lambda g: first(g, "Transpose").attrs.update(perm=(0, 0, 1, 2, 3))],
        "axis": [lambda g: first(g, "Concat").attrs.update(axis=5),
                 lambda g: first(g, "Gather").inputs.reverse()],
    }
    for what, fs in cases.items():
        for f in fs:
            with pytest.raises(S.Sod2Error) as e:
                build(mutated(f))
            assert e.value.code in (-1, -3), (what, str(e.value))
    w3 = small(3)
    for attrs in (dict(kernel=0, stride=2, pad=0), dict(kernel=3, stride=0, pad=1), dict(kernel=3, stride=2, pad=3)):
        g = copy.deepcopy(w3.graph)
        first(g, "MaxPool").attrs.update(attrs)
        with pytest.raises(S.Sod2Error):
            S.sod2_graph_build(g)
    g = copy.deepcopy(w3.graph)
    first(g, "Conv").attrs.update(stride=0)
    with pytest.raises(S.Sod2Error):
        S.sod2_graph_build(g)

    # an output that no operator produces (a graph input, a weight, a dangling tensor): nothing would write it
    for what in ("input", "weight", "dangling"):
        gb = GraphBuilder([("A", 1, 9)])
        x = gb.input("x", "f32", ["A", 8])
        wt = gb.weight("w", "f32", [8])
        gb.mark_output(gb.op("Add", [x, wt]), "y")
        gb.mark_output({"input": x, "weight": wt, "dangling": gb._tmp("f32", "lost")}[what])
        with pytest.raises(S.Sod2Error) as e:
            S.sod2_graph_build(gb.build())
        assert e.value.code == -1 and "produced by no operator" in str(e.value)
        with pytest.raises(ValueError):
            P.build_plan(gb.build(), R.RDP(gb.build()).analyse())

    # extents at the bound symbols: a window larger than its input gives an empty or a negative extent (the latter is
    # refused), a tensor beyond 2^44 bytes is refused before any byte count can overflow
    gb = GraphBuilder([("H", 1, 2 ** 40)])
    x = gb.input("x", "f32", [1, "H", "H", 8])
    gb.mark_output(gb.op("MaxPool", [x], kernel=5, stride=1, pad=0), "y")
    hg = S.sod2_graph_build(gb.build())
    hp = S.sod2_plan(hg, S.sod2_rdp_infer(hg))
    assert S.sod2_binding_arena_bytes(S.sod2_bind(hp, {"H": 4}))[0] == 0       # nothing to compute
    for H in (2, 2 ** 20, 2 ** 31, 2 ** 40):
        with pytest.raises(S.Sod2Error) as e:
            S.sod2_bind(hp, {"H": H})
        assert e.value.code == -3

    rnd = random.Random(2024)
    outcomes = {"refused": 0, "planned": 0}
    for trial in range(120):
        g = copy.deepcopy((w, w3)[trial % 2].graph)
        for _ in range(rnd.randint(1, 3)):
            op = rnd.choice(g.ops)
            m = rnd.randint(0, 7)
            if m == 0 and op.attrs:
                k = rnd.choice(sorted(op.attrs))
                v = op.attrs[k]
                op.attrs[k] = [rnd.randint(-9, 9) for _ in v] if isinstance(v, (list, tuple)) else \
                    (rnd.choice([0.0, -1.0, 1e30]) if isinstance(v, float) else rnd.choice([-3, -1, 0, 1, 7, 1000, 2 ** 31]))
            elif m == 1:
                rnd.choice(g.tensors).dtype = rnd.choice(["f32", "bf16", "i64", "i32"])
            elif m == 2:
                t = rnd.choice([t for t in g.tensors if t.dims])
                t.dims = list(t.dims) + [3] if rnd.random() < 0.5 else list(t.dims)[:-1]
            elif m == 3 and len(op.inputs) >= 2:
                op.inputs[0], op.inputs[1] = op.inputs[1], op.inputs[0]
            elif m == 4:
                op.inputs[rnd.randrange(len(op.inputs))] = rnd.randrange(len(g.tensors))
            elif m == 5:
                t = rnd.choice([t for t in g.tensors if t.dims])
                t.dims = list(t.dims)
                t.dims[rnd.randrange(len(t.dims))] = rnd.choice([0, 1, 7, "B", "L", "B+L", 2 ** 40])
            elif m == 6:
                g.ops.remove(op)
            else:
                op.outputs = list(op.outputs) + [rnd.randrange(len(g.tensors))]
        try:
            h = S.sod2_graph_build(g)
            p = S.sod2_plan(h, S.sod2_rdp_infer(h))
            b = S.sod2_bind(p, {name: min(hi, lo + 7) for name, lo, hi in g.symbols})
            S.sod2_binding_dump(b)
            outcomes["planned"] += 1
        except S.Sod2Error:
            outcomes["refused"] += 1
        except (KeyError, TypeError, ValueError, OverflowError):
            outcomes["refused"] += 1          # stopped by the binding's own marshalling
    assert outcomes["refused"] > 40 and outcomes["planned"] > 0, outcomes
