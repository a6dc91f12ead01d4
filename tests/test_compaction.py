"""Pins for the execution-determined path (Table 2's EDO class, Section 4.3): NonZero, batch
compaction with Gather, ScatterRows, the analysis with named EDO extents and the two-stage arena
plan (upper bound before the NonZero has run, exact after).  CPU only."""
import numpy as np
import pytest

from oracle import ops as O
from oracle import execute, rdp as R, plan as P, arena as A
from workloads import configs, GraphBuilder


def small(gate_bias=None, layers=2, n_calls=6, gated="sample"):
    # hidden 128 = 2 heads of 64; short sequences keep the float64 runs quick
    return configs.encoder(6, layers, 128, 2, 256, "bf16", (2, 6), (8, 24), n_calls, final_ln=True,
                           gated=gated, gate_bias=gate_bias)


def run(w, ci, weights=None, sym=None, x=None):
    sym = sym or w.calls[ci]
    order = R.RDP(w.graph).sorted_nodes()
    x = x if x is not None else w.make_inputs(ci, sym)
    return execute.run(w.graph, order, weights or w.make_weights(), x), x


def by_name(g, values):
    return {g.tensors[t].name: v for t, v in values.items()}


def test_nonzero_row_major_coordinates():
    rs = np.random.RandomState(3)
    for shape in ((7,), (3, 5), (2, 3, 4), (0,), (4, 0)):
        x = rs.randn(*shape) * (rs.rand(*shape) < 0.4)
        got = O.nonzero(x)
        ref = np.stack(np.nonzero(x)).astype(np.int64) if x.ndim else None
        assert got.shape == (x.ndim, int(np.count_nonzero(x)))
        assert np.array_equal(got, ref)
    assert O.nonzero(np.zeros(5)).shape == (1, 0)
    assert np.array_equal(O.nonzero(np.array([0.0, -2.0, 0.0, 1e-30])), [[1, 3]])


def test_scatter_rows_replaces_exactly_the_indexed_rows():
    b = GraphBuilder([("B", 1, 8)])
    x = b.input("x", "f32", ["B", 3])
    i = b.input("i", "i64", None)
    y = b.input("y", "f32", None)
    b.mark_output(b.op("ScatterRows", [x, i, y]), "out")
    g = b.build()
    xv = np.arange(15, dtype=np.float64).reshape(5, 3)
    yv = -np.ones((2, 3)) * [[1], [2]]
    res = execute.run(g, [0], {}, {0: xv, 1: np.array([3, 0]), 2: yv})
    out = res.values[g.tensor_id("out")]
    assert np.array_equal(out[[1, 2, 4]], xv[[1, 2, 4]])
    assert np.array_equal(out[3], yv[0]) and np.array_equal(out[0], yv[1])
    assert np.array_equal(xv, np.arange(15).reshape(5, 3))          # the input is not modified
    same = execute.run(g, [0], {}, {0: xv, 1: np.zeros(0, np.int64), 2: np.zeros((0, 3))})
    assert np.array_equal(same.values[g.tensor_id("out")], xv)


def test_named_analysis_agrees_with_the_printed_algorithm():
    """Alg. 1 makes every EDO output nac.  Naming the extent only refines that: wherever the printed
    analysis has a value the named one has the same value, and wherever the named one has nac or an
    execution symbol the printed one has nac."""
    w = small()
    paper = R.RDP(w.graph).analyse()
    named = R.RDP(w.graph, named_edo=True).analyse()
    n_exec = 0
    for t in range(len(w.graph.tensors)):
        for store_p, store_n in ((paper.S, named.S), (paper.V, named.V)):
            sp, sn = store_p[t], store_n[t]
            if isinstance(sp, list):
                assert isinstance(sn, list) and len(sn) == len(sp)
                for dp, dn in zip(sp, sn):
                    if dp != R.NAC:
                        assert dp == dn and not R.mentions_exec(dn)
            if sn == R.NAC:
                assert sp == R.NAC
            elif isinstance(sn, list):
                for k, dn in enumerate(sn):
                    if dn == R.NAC or R.mentions_exec(dn):
                        assert sp == R.NAC or sp[k] == R.NAC
                        n_exec += store_n is named.S
    assert n_exec > 20
    # the compacted activations are [count, L, hidden] with the count of *their own* layer's NonZero
    nz_ops = [n for n, op in enumerate(w.graph.ops) if op.kind == "NonZero"]
    assert len(nz_ops) == 2
    for n in nz_ops:
        out = w.graph.ops[n].outputs[0]
        assert [str(d) for d in named.S[out]] == ["1", R.exec_symbol(n)]
    xs0 = w.graph.tensor_id([t.name for t in w.graph.tensors if t.name.startswith("g0.xs")][0])
    assert [str(d) for d in named.S[xs0]] == [R.exec_symbol(nz_ops[0]), "L", "128"]
    # the merged stream has the full batch again
    merged = w.graph.ops[[n for n, op in enumerate(w.graph.ops) if op.kind == "ScatterRows"][0]].outputs[0]
    assert [str(d) for d in named.S[merged]] == ["B", "L", "128"]
    # a graph without an EDO: both analyses are identical
    w2 = configs.config1()
    assert R.dump(R.RDP(w2.graph).analyse()) == R.dump(R.RDP(w2.graph, named_edo=True).analyse())


def plain_twin(w_gated, layers=2):
    """The ungated encoder with the same block weights (matched by name)."""
    wp = small(layers=layers, gated=False)
    vals = by_name(w_gated.graph, w_gated.make_weights())
    return wp, {t: vals[wp.graph.tensors[t].name] for t in wp.graph.weights()}


def test_every_sequence_kept_equals_the_plain_encoder():
    w = small(gate_bias=10.0)
    wp, weights_p = plain_twin(w)
    for ci in (0, 1):
        res, x = run(w, ci)
        B = w.calls[ci]["B"]
        assert res.exec_values == [B, B]
        ref = execute.run(wp.graph, R.RDP(wp.graph).sorted_nodes(), weights_p,
                          {wp.graph.tensor_id("x"): x[w.graph.tensor_id("x")]})
        assert np.array_equal(res.values[w.graph.tensor_id("y")], ref.values[wp.graph.tensor_id("y")])


def test_no_sequence_kept_is_the_final_layernorm_of_the_input():
    w = small(gate_bias=-10.0)
    res, x = run(w, 0)
    assert res.exec_values == [0, 0]
    xv = O.round_to(x[w.graph.tensor_id("x")], "bf16")
    weights = by_name(w.graph, w.make_weights())
    gamma, beta = O.round_to(weights["lnf.g"], "bf16"), O.round_to(weights["lnf.beta"], "bf16")
    mu = xv.mean(-1, keepdims=True)
    var = ((xv - mu) ** 2).mean(-1, keepdims=True)
    ref = O.round_to((xv - mu) / np.sqrt(var + 1e-5) * gamma + beta, "bf16")
    assert np.array_equal(res.values[w.graph.tensor_id("y")], ref)


def test_a_batch_equals_its_sequences_run_one_by_one():
    """Decisions are per sequence and no operator mixes sequences: row b of a batched call equals the
    call on sequence b alone (this fails if compaction or the scatter mis-index a single row)."""
    w = small(n_calls=12)
    weights = w.make_weights()
    w1 = configs.encoder(6, 2, 128, 2, 256, "bf16", (1, 6), (8, 24), 1, final_ln=True, gated="sample")
    weights1 = {t: by_name(w.graph, weights)[w1.graph.tensors[t].name] for t in w1.graph.weights()}
    mixed = 0
    for ci in range(12):
        sym = w.calls[ci]
        res, x = run(w, ci, weights)
        xv = x[w.graph.tensor_id("x")]
        y = res.values[w.graph.tensor_id("y")]
        per_layer = np.zeros(2, dtype=int)
        for bi in range(sym["B"]):
            one = execute.run(w1.graph, R.RDP(w1.graph).sorted_nodes(), weights1,
                              {w1.graph.tensor_id("x"): xv[bi:bi + 1]})
            per_layer += np.array(one.exec_values)
            assert np.allclose(one.values[w1.graph.tensor_id("y")][0], y[bi], rtol=0, atol=2e-2 * np.abs(y).max())
        assert list(per_layer) == res.exec_values
        mixed += any(0 < c < sym["B"] for c in res.exec_values)
    assert mixed >= 3, "the calls must include partly kept batches"


def test_upper_bound_plan_then_exact_plan():
    w = small(n_calls=12)
    ro = R.RDP(w.graph).analyse()
    plan = P.build_plan(w.graph, ro)
    assert plan.paper_rdp is ro and plan.rdp is not ro and len(plan.exec_ops) == 2
    weights = w.make_weights()
    for ci in range(12):
        sym = w.calls[ci]
        res, _ = run(w, ci, weights)
        before = A.bind(plan, sym)                                   # nothing executed yet
        half = A.bind(plan, sym, exec_values=res.exec_values[:1])    # first NonZero done
        after = A.bind(plan, sym, exec_values=res.exec_values)
        for b in (before, half, after):
            A.check_no_overlap(b)
        assert [v for _, v, _ in before.exec] == [sym["B"], sym["B"]]
        assert [k for _, _, k in half.exec] == [True, False]
        # (no order between the three arena sizes is asserted: first fit is not monotone in the tensor
        #  sizes, so the exact plan may need more than the upper-bound plan; a run that meets this
        #  reports it before launching anything that follows the NonZero)
        assert after.arena_bytes >= after.peak_live and before.arena_bytes >= before.peak_live
        # causality: what was placed before a NonZero ran keeps its offset when the count arrives
        nz_steps = [k for k, i in enumerate(after.steps)
                    if plan.items[i].is_group and plan.groups[plan.items[i].ref].kind == "NONZERO"]
        for t, at in after.tensors.items():
            if at.start <= nz_steps[0]:
                assert before.tensors[t].offset == at.offset and before.tensors[t].bytes == at.bytes
            if at.start <= nz_steps[1]:
                assert half.tensors[t].offset == at.offset and half.tensors[t].bytes == at.bytes
        # the NonZero result is allocated for its upper bound plus the count slot
        for n in plan.exec_ops:
            out = w.graph.ops[n].outputs[0]
            assert after.tensors[out].bytes == (sym["B"] * 8 + 8 + 255) // 256 * 256
            assert after.dims[out] == [1, dict((o, v) for o, v, _ in after.exec)[n]]
        # executed shapes equal the shapes the value oracle produced
        for t, dims in after.dims.items():
            assert list(res.values[t].shape) == dims, w.graph.tensors[t].name
    with pytest.raises(ValueError):
        A.bind(plan, w.calls[0], exec_values=[w.calls[0]["B"] + 1])
    # a count that is known is not the same as the upper bound assumed for an unknown one, even when the
    # numbers agree: with the count known the sub-graphs behind the NonZero are planned together, so a
    # run must plan again after every NonZero (the library once skipped that when count == bound)
    sym = w.calls[0]
    assumed, known = A.bind(plan, sym), A.bind(plan, sym, exec_values=[sym["B"]])
    assert [v for _, v, _ in assumed.exec][:1] == [v for _, v, _ in known.exec][:1]
    assert len(A.planning_regions(plan, known)) < len(A.planning_regions(plan, assumed))


def test_partition_cuts_after_every_execution_determined_item():
    w = small()
    plan = P.build_plan(w.graph, R.RDP(w.graph).analyse())
    for sg, cls in zip(plan.subgraphs, plan.sg_class):
        writes = [t for i in sg for t in plan.items[i].writes]
        if any(P.execution_determined(plan, t) for t in writes):
            assert cls == "nac" and len(sg) == 1
    kinds = [plan.groups[plan.items[i].ref].kind for sg in plan.subgraphs for i in sg]
    assert kinds.count("NONZERO") == 2 and kinds.count("SCATTER") == 2 and kinds.count("ATTENTION") == 2
    # the shape arithmetic on the compacted batch is folded: Shape / Gather / Concat of dims never run
    for n, op in enumerate(w.graph.ops):
        if op.kind in ("Shape", "Concat"):
            assert plan.folded[n]
