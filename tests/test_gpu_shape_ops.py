"""Resize (nearest) and Concat kernels and the detection-style neck on the GPU against the oracle."""
import numpy as np
import pytest

from oracle import rdp as R, plan as P, arena as A, execute
from workloads import configs, GraphBuilder, rng

pytestmark = pytest.mark.gpu


def rel_err(got, ref):
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


@pytest.fixture(scope="module")
def S():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2403_00176_amd as S
    return S


@pytest.mark.parametrize("dtype,c", [("bf16", 256), ("bf16", 5), ("f32", 6), ("f32", 64)])
def test_resize_and_concat_kernels(S, dtype, c):
    """Pure copies: exact.  Channel counts with and without 16-byte rows; enlarging, shrinking, identity."""
    import torch
    from paper_2403_00176_amd.session import Session, to_host
    b = GraphBuilder([("H", 1, 64), ("W", 1, 64), ("OH", 1, 128), ("OW", 1, 128)])
    x = b.input("x", dtype, [2, "H", "W", c])
    like = b.input("like", dtype, [2, "OH", "OW", 3 * c])
    shp_x = b.op("Shape", [x], dtype="i64")
    shp_l = b.op("Shape", [like], dtype="i64")
    ax0 = b.const("ax0", [0])
    sizes = b.op("Concat", [b.op("Slice", [shp_x, b.const("a0", [0]), b.const("a1", [1]), ax0], dtype="i64"),
                            b.op("Slice", [shp_l, b.const("b1", [1]), b.const("b3", [3]), ax0], dtype="i64"),
                            b.op("Slice", [shp_x, b.const("c3", [3]), b.const("c4", [4]), ax0], dtype="i64")], axis=0, dtype="i64")
    up = b.op("Resize", [x, sizes], hint="up")
    b.mark_output(b.op("Concat", [up, like, up], axis=3, hint="cat"), "y")
    g = b.build()
    ses = Session(g)
    ses.upload_weights({})
    po = P.build_plan(g, R.RDP(g).analyse())
    rs = np.random.RandomState(c)
    for H, W, OH, OW in ((3, 5, 6, 10), (8, 8, 3, 5), (4, 4, 4, 4), (1, 1, 7, 2), (16, 12, 32, 24)):
        sym = {"H": H, "W": W, "OH": OH, "OW": OW}
        print(f"case resize/concat {dtype} c={c} {sym}", flush=True)
        ins = {0: rs.randn(2, H, W, c), 1: rs.randn(2, OH, OW, 3 * c)}
        bnd = ses.bind(sym)
        assert S.sod2_binding_dump(bnd) == A.dump(A.bind(po, sym))
        outs = ses.alloc_outputs(ses.output_shapes(bnd))
        ses.run(bnd, ses.upload_inputs(ins), outs)
        torch.cuda.synchronize()
        ref = execute.run(g, po.order, {}, ins)
        assert np.array_equal(to_host(outs[0]), ref.values[g.tensor_id("y")])


def test_detection_neck(S):
    """Reduced backbone + the full neck at three image sizes: structure byte for byte, the three output
    maps within the bf16 bar."""
    import torch
    from paper_2403_00176_amd.session import Session, to_host
    w = configs.fpn(7, 3, sizes=(64, 96, 128), stages=(1, 1, 1, 1))
    ses = Session(w.graph)
    W = w.make_weights()
    ses.upload_weights(W)
    po = P.build_plan(w.graph, R.RDP(w.graph).analyse())
    for ci, sym in [(0, {"H": 96, "W": 64}), (1, {"H": 64, "W": 64}), (2, {"H": 128, "W": 96})]:
        print(f"case neck {sym}", flush=True)
        ins = w.make_inputs(ci, sym)
        b = ses.bind(sym)
        assert S.sod2_binding_dump(b) == A.dump(A.bind(po, sym))
        outs = ses.alloc_outputs(ses.output_shapes(b))
        ses.run(b, ses.upload_inputs(ins), outs)
        torch.cuda.synchronize()
        ref = execute.run(w.graph, po.order, W, ins)
        for t, o in zip(w.graph.outputs(), outs):
            got = to_host(o)
            assert got.shape == ref.values[t].shape and np.isfinite(got).all()
            assert rel_err(got, ref.values[t]) <= 2e-2, (w.graph.tensors[t].name, sym, rel_err(got, ref.values[t]))


def test_range_gather_expand(S):
    """Position ids made in the graph (Range up to a dim read from Shape), table rows gathered by them and
    broadcast over the batch through an Expand view (stride 0) into an elementwise Add."""
    import torch
    from paper_2403_00176_amd.session import Session, to_host
    from tests.test_shape_ops import _positions_graph
    g, pos, rows, wide = _positions_graph()
    ses = Session(g)
    rs = np.random.RandomState(2)
    table = rs.randn(512, 8)
    ses.upload_weights({g.tensor_id("table"): table})
    po = P.build_plan(g, R.RDP(g).analyse())
    for B, L in ((1, 1), (3, 7), (8, 300), (2, 257)):
        sym = {"B": B, "L": L}
        print(f"case positions {sym}", flush=True)
        ins = {g.tensor_id("x"): rs.randn(B, L, 8)}
        b = ses.bind(sym)
        assert S.sod2_binding_dump(b) == A.dump(A.bind(po, sym))
        outs = ses.alloc_outputs(ses.output_shapes(b))
        ses.run(b, ses.upload_inputs(ins), outs)
        torch.cuda.synchronize()
        ref = execute.run(g, po.order, {g.tensor_id("table"): table}, ins)
        by_name = dict(zip([g.tensors[t].name for t in g.outputs()], outs))
        assert np.array_equal(to_host(by_name["positions"]), np.arange(L))
        assert rel_err(to_host(by_name["y"]), ref.values[g.tensor_id("y")]) <= 1e-2


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_constantofshape_eyelike_onehot_upsample(S, dtype):
    """The fill, identity, one-hot and whole-factor enlargement kernels against the oracle; the one-hot
    code times a table equals the table rows the indices name (negative indices count from the depth)."""
    import torch
    from paper_2403_00176_amd.session import Session, to_host
    from tests.test_shape_ops import _generators_graph
    g, half, eye, hot = _generators_graph(dtype)
    ses = Session(g)
    po = P.build_plan(g, R.RDP(g).analyse())
    rs = np.random.RandomState(7)
    tol = 1e-5 if dtype == "f32" else 1e-2
    for B, L, N, D in ((1, 1, 1, 2), (3, 7, 5, 11), (8, 64, 48, 40), (2, 33, 17, 3)):
        sym = {"B": B, "L": L, "N": N, "D": D}
        print(f"case generators {dtype} {sym}", flush=True)
        ins = {g.tensor_id("x"): rs.randn(B, L, 8), g.tensor_id("sq"): rs.randn(N, N),
               g.tensor_id("ids"): rs.randint(-D, D, size=(B, L)), g.tensor_id("table"): rs.randn(D, 8)}
        b = ses.bind(sym)
        assert S.sod2_binding_dump(b) == A.dump(A.bind(po, sym))
        outs = ses.alloc_outputs(ses.output_shapes(b))
        ses.run(b, ses.upload_inputs(ins), outs)
        torch.cuda.synchronize()
        ref = execute.run(g, po.order, {}, ins)
        for t, o in zip(g.outputs(), outs):
            got = to_host(o)
            assert got.shape == ref.values[t].shape
            assert rel_err(got, ref.values[t]) <= tol, (g.tensors[t].name, sym, rel_err(got, ref.values[t]))
        names = [g.tensors[t].name for t in g.outputs()]
        assert np.array_equal(to_host(outs[names.index("bigger")]), ref.values[g.tensor_id("bigger")])   # a copy: exact


def test_input_shape_found_by_backward_value_transfer(S):
    """The graph declares no shape for its input: RDP finds it backwards through Shape and ConstantOfShape,
    and the run uses it."""
    import torch
    from paper_2403_00176_amd.session import Session, to_host
    from tests.test_shape_ops import _backward_value_graph
    g, x, s, z = _backward_value_graph()
    ses = Session(g)
    for B, L in ((1, 1), (3, 7), (8, 64)):
        sym = {"B": B, "L": L}
        print(f"case backward value {sym}", flush=True)
        xv = np.random.RandomState(B).randn(B, L, 8)
        b = ses.bind(sym)
        outs = ses.alloc_outputs(ses.output_shapes(b))
        ses.run(b, ses.upload_inputs({x: xv}), outs)
        torch.cuda.synchronize()
        names = [g.tensors[t].name for t in g.outputs()]
        assert np.array_equal(to_host(outs[names.index("sum")]), (xv.astype(np.float32) + np.float32(1.0)).astype(np.float64))
        assert np.array_equal(to_host(outs[names.index("y")]), np.ones((B, L, 8)))


def test_runtime_sizes_found_by_backward_value_transfer(S):
    """Sizes that arrive as a run-time integer input: RDP knows their values backwards from a declared extent
    (through ConstantOfShape, an integer Cast, Concat and Add), so the Reshape that reads them is planned ahead of
    time and runs as a view."""
    import torch
    from paper_2403_00176_amd.session import Session, to_host
    from tests.test_shape_ops import _runtime_sizes_graph
    g, sz, y = _runtime_sizes_graph()
    po = P.build_plan(g, R.RDP(g).analyse())
    ses = Session(g)
    ses.upload_weights({})
    for B, L in ((1, 1), (3, 5), (8, 64)):
        sym = {"B": B, "L": L}
        print(f"case run-time sizes {sym}", flush=True)
        xv = np.random.RandomState(L).randn(B, 2, L, 2)
        ins = {g.tensor_id("x"): xv, sz: np.array([2 * B, 2 * L])}
        b = ses.bind(sym)
        assert S.sod2_binding_dump(b) == A.dump(A.bind(po, sym))
        outs = ses.alloc_outputs(ses.output_shapes(b))
        ses.run(b, ses.upload_inputs(ins), outs)
        torch.cuda.synchronize()
        ref = execute.run(g, po.order, {}, ins)
        for t, o in zip(g.outputs(), outs):
            assert np.array_equal(to_host(o), ref.values[t])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_topk_router(S, dtype):
    """TopK (values and positions from one kernel), softmax over the chosen scores and a one-hot product
    that picks the chosen table rows.  Positions are compared exactly where the oracle's chosen scores
    are distinct after rounding; where scores tie the kernel must still return valid positions."""
    import torch
    from paper_2403_00176_amd.session import Session, to_host
    from tests.test_shape_ops import _router_graph
    g, scores, vals, idx = _router_graph(dtype)
    g.tensors[idx].is_output = True                    # also hand the positions to the caller
    g.tensors[vals].is_output = True
    ses = Session(g)
    weights = {g.tensor_id("wr"): np.random.RandomState(1).randn(40, 64) * 0.1,
               g.tensor_id("table"): np.random.RandomState(2).randn(40, 8)}
    ses.upload_weights(weights)
    po = P.build_plan(g, R.RDP(g).analyse())
    tol = 1e-4 if dtype == "f32" else 2e-2
    for B, K in ((1, 1), (5, 3), (64, 16), (33, 40 if False else 16)):
        sym = {"B": B, "K": K}
        print(f"case router {dtype} {sym}", flush=True)
        ins = {g.tensor_id("x"): np.random.RandomState(B + K).randn(B, 64), g.tensor_id("sel"): np.zeros((K, 8))}
        b = ses.bind(sym)
        assert S.sod2_binding_dump(b) == A.dump(A.bind(po, sym))
        outs = ses.alloc_outputs(ses.output_shapes(b))
        ses.run(b, ses.upload_inputs(ins), outs)
        torch.cuda.synchronize()
        ref = execute.run(g, po.order, weights, ins)
        got = {g.tensors[t].name: to_host(o) for t, o in zip(g.outputs(), outs)}
        gv, gi = got[g.tensors[vals].name], got[g.tensors[idx].name].astype(np.int64)
        rv = ref.values[vals]
        assert gv.shape == (B, K) == gi.shape
        assert rel_err(gv, rv) <= tol
        assert (np.diff(gv, axis=-1) <= 0).all()                        # largest first
        assert all(len(set(row)) == K for row in gi) and gi.min() >= 0 and gi.max() < 40
        # every returned position holds the returned value in the scores the kernel saw; the scores are
        # not an output, so check against the oracle's within the storage tolerance
        assert np.abs(np.take_along_axis(ref.values[scores], gi, axis=-1) - gv).max() <= tol * np.abs(rv).max()
        gap = np.abs(np.diff(np.sort(ref.values[scores], axis=-1), axis=-1)).min(axis=-1)   # per row: closest pair
        clear = gap > 4 * tol * np.abs(rv).max()
        assert np.array_equal(gi[clear], ref.values[idx][clear])
        assert rel_err(got["gates"], ref.values[g.tensor_id("gates")]) <= tol
        if clear.all():
            assert rel_err(got["rows"], ref.values[g.tensor_id("rows")]) <= tol


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_multi_version_fused_chain(S_lib, dtype):
    """Fig. 4 on the GPU: Sigmoid(A) + B, * 2 with nothing relating A's extents to B's.  The chain runs as ONE
    kernel (8 code versions planned; the broadcast strides of the version that holds are selected at bind) and gives
    the oracle's values in every case: equal extents, A broadcast in some dims, B broadcast in others; the same graph
    planned without fusion runs three kernels and gives the same values; symbols that do not broadcast are refused."""
    import torch
    from tests.test_host_parity import _multi_version_graph
    from paper_2403_00176_amd.session import Session, to_host
    S = S_lib
    g = _multi_version_graph(dtype=dtype)
    po = P.build_plan(g, R.RDP(g).analyse())
    a_id, b_id, out = g.tensor_id("A"), g.tensor_id("B"), g.outputs()[0]
    tol = 1e-4 if dtype == "f32" else 2e-2
    runs = {}
    for fusion in (1, 0):
        ses = Session(g, fusion=fusion)
        ses.upload_weights({})
        for k, sym in enumerate((dict(I=37, J=70, K=129, P=37, Q=70, R=129), dict(I=37, J=70, K=129, P=1, Q=70, R=1),
                                 dict(I=1, J=70, K=1, P=53, Q=1, R=129), dict(I=37, J=1, K=129, P=37, Q=90, R=1),
                                 dict(I=5, J=3, K=600, P=5, Q=3, R=600))):
            ins = {a_id: rng.normal(800 + k, (sym["P"], sym["Q"], sym["R"])), b_id: rng.normal(900 + k, (sym["I"], sym["J"], sym["K"]))}
            b = ses.bind(sym)
            if fusion:
                assert S.sod2_binding_dump(b) == A.dump(A.bind(po, sym))
            outs = ses.alloc_outputs(ses.output_shapes(b))
            ses.run(b, ses.upload_inputs(ins), outs)
            torch.cuda.synchronize()
            ref = execute.run(g, po.order, {}, ins).values[out]
            got = to_host(outs[0])
            assert got.shape == ref.shape
            assert np.abs(got - ref).max() / np.abs(ref).max() <= tol, (fusion, sym)
            launches = [e for e in S.sod2_run_trace(b) if e["is_group"]]
            assert len(launches) == (1 if fusion else 3)
            runs[(fusion, k)] = got
    ses = Session(g)
    with pytest.raises(S.Sod2Error) as e:
        ses.bind(dict(I=3, J=4, K=5, P=2, Q=4, R=5))
    assert e.value.code == -3


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_slice_with_computed_bounds(S_lib, dtype):
    """Slices whose bounds are values computed from shapes run as views (offset and extent evaluated at bind) feeding
    fused elementwise kernels; a bound outside the tensor is refused when the launch is prepared."""
    import torch
    from tests.test_shape_ops import _computed_slice_graph
    from paper_2403_00176_amd.session import Session, to_host
    g = _computed_slice_graph(dtype)[0]
    po = P.build_plan(g, R.RDP(g).analyse())
    ses = Session(g)
    ses.upload_weights({})
    tol = 1e-4 if dtype == "f32" else 2e-2
    for k, sym in enumerate(({"B": 2, "L": 7, "M": 4}, {"B": 1, "L": 2, "M": 2}, {"B": 8, "L": 300, "M": 300}, {"B": 5, "L": 129, "M": 65})):
        ins = {g.tensor_id("x"): rng.normal(700 + k, (sym["B"], sym["L"], 8)), g.tensor_id("m"): rng.normal(750 + k, (sym["M"], 8))}
        b = ses.bind(sym)
        assert S_lib.sod2_binding_dump(b) == A.dump(A.bind(po, sym))
        outs = ses.alloc_outputs(ses.output_shapes(b))
        ses.run(b, ses.upload_inputs(ins), outs)
        torch.cuda.synchronize()
        ref = execute.run(g, po.order, {}, ins)
        for t, o in zip(g.outputs(), outs):
            got = to_host(o)
            assert got.shape == ref.values[t].shape
            assert rel_err(got, ref.values[t]) <= tol, (sym, g.tensors[t].name)
    # M beyond L: the head slice would end outside x
    sym = {"B": 1, "L": 4, "M": 9}
    b = ses.bind(sym)
    ins = {g.tensor_id("x"): rng.normal(1, (1, 4, 8)), g.tensor_id("m"): rng.normal(2, (9, 8))}
    outs = ses.alloc_outputs(ses.output_shapes(b))
    with pytest.raises(S_lib.Sod2Error) as e:
        ses.run(b, ses.upload_inputs(ins), outs)
    assert e.value.code == -1 and "Slice bounds" in str(e.value)
    torch.cuda.synchronize()


@pytest.mark.parametrize("dtype,groups,channels", [("f32", 4, 32), ("bf16", 32, 256), ("bf16", 1, 8), ("f32", 6, 6)])
def test_groupnorm_kernel(S_lib, dtype, groups, channels):
    import torch
    from tests.test_shape_ops import _groupnorm_graph
    from paper_2403_00176_amd.session import Session, to_host
    g = _groupnorm_graph(dtype, groups, channels)[0]
    po = P.build_plan(g, R.RDP(g).analyse())
    ses = Session(g)
    W = {g.tensor_id("gn.g"): rng.normal(31, (channels,), 1.0, 0.2), g.tensor_id("gn.b"): rng.normal(32, (channels,), 0.0, 0.2)}
    ses.upload_weights(W)
    for k, sym in enumerate(({"H": 1, "W": 1}, {"H": 7, "W": 9}, {"H": 64, "W": 64})):
        ins = {g.tensor_id("x"): rng.normal(600 + k, (2, sym["H"], sym["W"], channels), 0.5, 2.0)}
        b = ses.bind(sym)
        assert S_lib.sod2_binding_dump(b) == A.dump(A.bind(po, sym))
        outs = ses.alloc_outputs(ses.output_shapes(b))
        ses.run(b, ses.upload_inputs(ins), outs)
        torch.cuda.synchronize()
        ref = execute.run(g, po.order, W, ins).values[g.outputs()[0]]
        assert rel_err(to_host(outs[0]), ref) <= (1e-4 if dtype == "f32" else 2e-2), sym


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_maxunpool_kernel(S_lib, dtype):
    """MaxUnpool on the GPU: bit-exact (a copy of stored values to computed positions, zeros elsewhere), several
    sizes including one whose element count is no multiple of the workgroup size; positions outside the result
    are dropped."""
    import torch
    from paper_2403_00176_amd.session import Session, to_host
    from oracle import ops as O
    from tests.test_shape_ops import _unpool_graph, _pool_positions
    g, y = _unpool_graph(dtype)
    po = P.build_plan(g, R.RDP(g).analyse())
    ses = Session(g)
    ses.upload_weights({})
    rs = np.random.RandomState(2)
    for N, H, W in ((1, 1, 1), (2, 3, 5), (4, 32, 32), (3, 17, 9)):
        sym = {"N": N, "H": H, "W": W}
        print(f"case maxunpool {dtype} {sym}", flush=True)
        pooled, pos = _pool_positions(rs.randn(N, 2 * H, 2 * W, 8) + 3.0)
        if H > 1:
            pos[0, 0, 0, 0] = -5                         # outside: dropped
            pos[-1, -1, -1, -1] = N * 4 * H * W * 8      # one past the end: dropped
        ins = {g.tensor_id("x"): pooled, g.tensor_id("idx"): pos}
        b = ses.bind(sym)
        assert S_lib.sod2_binding_dump(b) == A.dump(A.bind(po, sym))
        outs = ses.alloc_outputs(ses.output_shapes(b))
        ses.run(b, ses.upload_inputs(ins), outs)
        torch.cuda.synchronize()
        ref = execute.run(g, po.order, {}, ins)
        got = to_host(outs[0])
        assert got.shape == (N, 2 * H, 2 * W, 8) and np.array_equal(got, ref.values[g.tensor_id("y")])
        assert np.count_nonzero(got) == pooled.size - (2 if H > 1 else 0)


@pytest.mark.parametrize("dtype,channels,kernel,stride,pad", [("f32", 16, 3, 2, 1), ("bf16", 16, 3, 2, 1), ("bf16", 64, 2, 2, 0),
                                                                ("bf16", 5, 3, 1, 1), ("f32", 3, 5, 3, 2)])
def test_averagepool_and_round_kernels(S_lib, dtype, channels, kernel, stride, pad):
    """AveragePool (wide bf16 kernel and the plain one) within the bar; Round is exact: in fp32 the chain
    Mul, Round, Mul is one kernel whose Round sees the same fp32 product as the definition, in bf16 the Round starts
    its own kernel on the stored value.  Inputs of Round(x) include exact halves."""
    import torch
    from tests.test_shape_ops import _avgpool_round_graph
    from paper_2403_00176_amd.session import Session, to_host
    g, _ = _avgpool_round_graph(dtype, channels, kernel, stride, pad)
    po = P.build_plan(g, R.RDP(g).analyse())
    ses = Session(g)
    ses.upload_weights({})
    for k, sym in enumerate(({"N": 1, "H": 5, "W": 5}, {"N": 2, "H": 7, "W": 9}, {"N": 3, "H": 128, "W": 96}, {"N": 8, "H": 33, "W": 1 + kernel})):
        print(f"case avgpool {dtype} c={channels} k={kernel} s={stride} p={pad} {sym}", flush=True)
        x = np.round(rng.normal(700 + k, (sym["N"], sym["H"], sym["W"], channels), 0.0, 3.0) * 8) / 8     # multiples of 1/8: halves occur
        ins = {g.tensor_id("x"): x}
        b = ses.bind(sym)
        assert S_lib.sod2_binding_dump(b) == A.dump(A.bind(po, sym))
        outs = ses.alloc_outputs(ses.output_shapes(b))
        ses.run(b, ses.upload_inputs(ins), outs)
        torch.cuda.synchronize()
        ref = execute.run(g, po.order, {}, ins)
        got = {t: to_host(o) for t, o in zip(g.outputs(), outs)}
        assert np.array_equal(got[g.tensor_id("rx")], ref.values[g.tensor_id("rx")])           # Round of stored values: exact
        q, qr = got[g.tensor_id("q")], ref.values[g.tensor_id("q")]
        assert q.shape == qr.shape
        # the pooled mean is a float result (fp32 sum / count against the exact one): a mean within rounding distance of
        # a quantisation boundary may land on the neighbouring step, nothing else may differ
        d = np.abs(q - qr)
        print("  quantised means that differ:", int((d > 1e-6).sum()), "of", d.size, "max", float(d.max()), flush=True)
        assert d.max() <= 0.25 + 1e-6 and np.mean(d > 1e-6) <= 1e-4, (sym, d.max(), np.mean(d > 1e-6))


@pytest.mark.parametrize("max_out,iou", [(0, 0.5), (0, 0.3), (10, 0.25)])
def test_nms_kernel(S_lib, max_out, iou):
    """Non-maximum suppression on the GPU: the count read back in mid-run, the kept indices (through the two
    Gathers behind them) bit-exact against the definition, whose overlap test is taken in fp32 on both sides.
    Integer-corner boxes with tied scores, and arbitrary float boxes; none, one, a few, and the largest number of
    boxes the kernel takes (several sort passes per thread, a padded sort for sizes that are no power of two)."""
    import torch
    from tests.test_shape_ops import _nms_graph, _grid_boxes
    from paper_2403_00176_amd.session import Session, to_host
    from oracle import ops as O
    g, sel = _nms_graph(max_out, iou)
    po = P.build_plan(g, R.RDP(g).analyse())
    ses = Session(g)
    ses.upload_weights({})
    rs = np.random.RandomState(17)
    for N, kind in ((0, "grid"), (1, "grid"), (5, "grid"), (100, "grid"), (1000, "float"), (1500, "grid"), (4096, "grid"), (4096, "float")):
        print(f"case nms max_out={max_out} iou={iou} N={N} {kind}", flush=True)
        if kind == "grid":
            scores, boxes = _grid_boxes(rs, N, span=30 + N // 8, side=14)
        else:
            c = rs.rand(N, 2) * (20 + N / 16.0)
            wh = rs.rand(N, 2) * 9 + 0.5
            boxes = np.concatenate([c - wh / 2, c + wh / 2], axis=1).astype(np.float32).astype(np.float64)
            scores = rs.rand(N).astype(np.float32).astype(np.float64)
        ins = {g.tensor_id("scores"): scores, g.tensor_id("boxes"): boxes.reshape(N, 4)}
        sym = {"N": N}
        bnd = ses.bind(sym)
        outs = ses.alloc_outputs(ses.output_shapes(bnd))               # sized for the upper bound
        ses.run(bnd, ses.upload_inputs(ins), outs)
        torch.cuda.synchronize()
        kept = O.nms(scores, boxes.reshape(N, 4), max_out, iou)
        assert S_lib.sod2_run_exec_values(bnd) == [len(kept)]
        assert S_lib.sod2_run_plan_dump(bnd) == A.dump(A.bind(po, sym, exec_values=[len(kept)]))
        n = len(kept)
        got_b = to_host(outs[0]).reshape(-1, 4)[:n]
        got_s = to_host(outs[1]).reshape(-1)[:n]
        assert np.array_equal(got_b, boxes.reshape(N, 4)[kept]) and np.array_equal(got_s, scores[kept])
        if N >= 100:
            assert 0 < n < N
        if N > 512:
            # with a workspace behind the arena (Session hands one over) that many boxes take the three-kernel path;
            # without one the single workgroup does all of it: the same indices
            outs2 = ses.alloc_outputs(ses.output_shapes(bnd))
            bnd2 = ses.bind(sym)
            arena = torch.empty(S_lib.sod2_binding_arena_bytes(bnd2)[0], dtype=torch.uint8, device="cuda")
            S_lib.sod2_run(bnd2, arena.data_ptr(), arena.numel(), [], [x.data_ptr() for x in ses.upload_inputs(ins)],
                           [x.data_ptr() for x in outs2], ses.stream.cuda_stream)
            torch.cuda.synchronize()
            assert S_lib.sod2_run_exec_values(bnd2) == [n]
            assert np.array_equal(to_host(outs2[0]).reshape(-1, 4)[:n], got_b) and np.array_equal(to_host(outs2[1]).reshape(-1)[:n], got_s)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_views_as_graph_outputs_are_written_out(S_lib, dtype):
    """A Transpose, Slice, Reshape, Expand or scalar-index Gather whose result is a graph output has no storage of its
    own to alias: the planner makes it a COPY group and the view is written densely into the caller's buffer (bit
    exact), also when the same view is read by another operator."""
    import torch
    from paper_2403_00176_amd.session import Session, to_host
    b = GraphBuilder([("A", 1, 40), ("B", 1, 40)])
    x = b.input("x", dtype, ["A", "B", 8])
    y = b.op("Mul", [x, b.const("two", 2.0, "f32")])                                  # a computed tensor in the arena
    t = b.mark_output(b.op("Transpose", [y], perm=(2, 0, 1)), "transposed")
    b.mark_output(b.op("Slice", [y, b.const("s", [1]), b.const("e", [7]), b.const("ax", [2])]), "sliced")
    shp = b.op("Shape", [y], dtype="i64")
    lead = b.op("Slice", [shp, b.const("l0", [0]), b.const("l1", [1]), b.const("lax", [0])], dtype="i64")
    b.mark_output(b.op("Reshape", [y, b.op("Concat", [lead, b.const("m1", [-1])], axis=0, dtype="i64")]), "flat")
    b.mark_output(b.op("Gather", [y, b.const("i3", 3)], axis=2), "column")
    b.mark_output(b.op("Expand", [b.op("ReduceMean", [y], axes=(1,), keepdims=1), shp]), "expanded")
    b.mark_output(b.op("Relu", [t]), "relu_of_view")                                  # the view is also read
    # a permutation regrouped by a Reshape: [A, B, 8] -> [B, A, 8] -> [B, A * 8] needs the elements in the new order
    yt = b.op("Transpose", [y], perm=(1, 0, 2))
    lead_t = b.op("Slice", [b.op("Shape", [yt], dtype="i64"), b.const("t0", [0]), b.const("t1", [1]), b.const("tax", [0])], dtype="i64")
    b.mark_output(b.op("Relu", [b.op("Reshape", [yt, b.op("Concat", [lead_t, b.const("tm1", [-1])], axis=0, dtype="i64")])]),
                  "regrouped")
    b.mark_output(b.op("Transpose", [x], perm=(1, 0, 2)), "input_transposed")         # a view of a graph input
    g = b.build()
    po = P.build_plan(g, R.RDP(g).analyse())
    assert sum(1 for gr in po.groups.values() if gr.kind == "COPY") == 7
    ses = Session(g)
    ses.upload_weights({})
    for k, sym in enumerate(({"A": 1, "B": 1}, {"A": 3, "B": 5}, {"A": 40, "B": 33})):
        ins = {g.tensor_id("x"): rng.normal(900 + k, (sym["A"], sym["B"], 8))}
        bnd = ses.bind(sym)
        assert S_lib.sod2_binding_dump(bnd) == A.dump(A.bind(po, sym))
        outs = ses.alloc_outputs(ses.output_shapes(bnd))
        ses.run(bnd, ses.upload_inputs(ins), outs)
        torch.cuda.synchronize()
        ref = execute.run(g, po.order, {}, ins)
        for t_, o in zip(g.outputs(), outs):
            got = to_host(o)
            assert got.shape == ref.values[t_].shape, (g.tensors[t_].name, sym)
            if g.tensors[t_].name == "expanded":            # a computed mean under the view: within the bar, and constant along B
                assert rel_err(got, ref.values[t_]) <= (1e-5 if dtype == "f32" else 2e-2)
                assert np.array_equal(got, np.broadcast_to(got[:, :1, :], got.shape))
            else:                                           # copies of exactly computed values: bit exact
                assert np.array_equal(got, ref.values[t_]), (g.tensors[t_].name, sym)


@pytest.mark.parametrize("opts", [{}, {"fusion": 0}, {"sep": 0, "inplace": 0}], ids=["default", "unfused", "node-order-no-inplace"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_random_graphs_against_the_oracle(S_lib, dtype, opts):
    """The seeded random graphs of tests/test_random_graphs.py (broadcasting chains, small contractions and
    convolutions with epilogues, row operators, pools, GroupNorm, views also as outputs, Concat, ReduceMean) through
    the C ABI in fp32 and bf16: every output within the bar of the oracle's values.  None of these graphs is refused:
    a strided view handed to an operator whose kernel wants dense operands is written out first (a COPY group)."""
    import torch
    from tests.test_random_graphs import random_graph, concrete, make_inputs
    from paper_2403_00176_amd.session import Session, to_host
    ran = refused = 0
    worst = 0.0
    for seed in range(40):
        g, weights, shapes = random_graph(seed, dtype)
        if g is None:
            continue
        po = P.build_plan(g, R.RDP(g).analyse(), P.Opts(**{k: bool(v) for k, v in opts.items()}))
        ses = Session(g, **opts)
        rs = np.random.RandomState(seed)
        W = {t: rs.randn(*d) * 0.3 for t, d in weights.items()}
        ses.upload_weights(W)
        for sym in ({"A": 3, "B": 5}, {"A": 9, "B": 12}, {"A": 1, "B": 1}):
            print(f"case random graph seed {seed} {sym} groups {[gr.kind for gr in po.groups.values()]}", flush=True)
            ins = make_inputs(g, shapes, sym, rs)
            bnd = ses.bind(sym)
            assert S_lib.sod2_binding_dump(bnd) == A.dump(A.bind(po, sym))
            outs = ses.alloc_outputs(ses.output_shapes(bnd))
            try:
                ses.run(bnd, ses.upload_inputs(ins), outs)
            except S_lib.Sod2Error as e:
                assert e.code == -6, (seed, sym, str(e))
                refused += 1
                print("  refused:", str(e)[:120], flush=True)
                continue
            torch.cuda.synchronize()
            ran += 1
            ref = execute.run(g, po.order, W, ins)
            for t, o in zip(g.outputs(), outs):
                got = to_host(o)
                assert got.shape == ref.values[t].shape and np.isfinite(got).all()
                err = rel_err(got, ref.values[t])
                worst = max(worst, err)
                assert err <= (1e-4 if dtype == "f32" else 2e-2), (seed, sym, g.tensors[t].name, err)
    print("random graphs", dtype, ": ran", ran, "refused", refused, "worst rel err", worst)
    assert ran >= 100 and refused == 0


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_wide_random_graphs_against_the_oracle(S_lib, dtype):
    """The same generator with inner extents of 64 and more and up to 6400 rows: contractions on the tiled
    matrix-core kernels with ragged row counts and every epilogue, the LayerNorm behind a contraction folded into
    its neighbours (constants derived by the session), convolutions with 64 and 128 channels."""
    import torch
    from tests.test_random_graphs import random_graph, make_inputs
    from paper_2403_00176_amd.session import Session, to_host
    ran = folds = 0
    worst = 0.0
    for seed in range(16):
        g, weights, shapes = random_graph(seed, dtype, wide=True)
        if g is None:
            continue
        po = P.build_plan(g, R.RDP(g).analyse())
        # a Cast to bf16 quantises: a value that the two sides compute a rounding error apart may fall on either side
        # of a bf16 boundary, so behind such a Cast the bf16 bar applies also in an fp32 graph
        narrowing = any(op.kind == "Cast" and g.tensors[op.outputs[0]].dtype == "bf16" for op in g.ops)
        bar = 2e-4 if dtype == "f32" and not narrowing else 2e-2
        ses = Session(g)
        rs = np.random.RandomState(seed)
        W = {t: rs.randn(*d) * (0.5 / np.sqrt(d[-1])) for t, d in weights.items()}
        ses.upload_weights(W)
        for sym in ({"A": 3, "B": 33}, {"A": 64, "B": 100}, {"A": 1, "B": 1}):
            print(f"case wide random graph {dtype} seed {seed} {sym} groups {[gr.kind for gr in po.groups.values()]}", flush=True)
            ins = make_inputs(g, shapes, sym, rs)
            bnd = ses.bind(sym)
            assert S_lib.sod2_binding_dump(bnd) == A.dump(A.bind(po, sym))
            outs = ses.alloc_outputs(ses.output_shapes(bnd))
            ses.run(bnd, ses.upload_inputs(ins), outs)
            torch.cuda.synchronize()
            ran += 1
            folds += sum(1 for e in S_lib.sod2_run_trace(bnd) if e["is_group"] and e["fold"] == 2)
            ref = execute.run(g, po.order, W, ins)
            for t, o in zip(g.outputs(), outs):
                got = to_host(o)
                assert got.shape == ref.values[t].shape and np.isfinite(got).all()
                err = rel_err(got, ref.values[t])
                worst = max(worst, err)
                assert err <= bar, (seed, sym, g.tensors[t].name, err)
    print("wide random graphs", dtype, ": ran", ran, "LayerNorms finished in a contraction's epilogue", folds, "worst rel err", worst)
    assert ran >= 40 and (dtype == "f32" or folds > 0)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_random_graphs_with_gates_against_the_oracle(S_lib, dtype):
    """Random graphs with <Switch, Combine> pairs whose predicates are graph inputs (0 or 1 against the threshold 0.5, so
    the decisions are exact): the decisions the run takes, the plan it ends with (made in mid-run as each predicate
    is read back) and every output against the oracle."""
    import torch
    from tests.test_random_graphs import random_graph, make_inputs
    from paper_2403_00176_amd.session import Session, to_host
    ran = switches = 0
    worst = 0.0
    for seed in range(30):
        g, weights, shapes = random_graph(seed, dtype, gates=True)
        if g is None or not any(op.kind == "Switch" for op in g.ops):
            continue
        po = P.build_plan(g, R.RDP(g).analyse())
        ses = Session(g)
        rs = np.random.RandomState(seed)
        W = {t: rs.randn(*d) * 0.3 for t, d in weights.items()}
        ses.upload_weights(W)
        for sym in ({"A": 3, "B": 5}, {"A": 9, "B": 12}, {"A": 1, "B": 1}, {"A": 4, "B": 7}):
            ins = make_inputs(g, shapes, sym, rs)
            ref = execute.run(g, po.order, W, ins)
            print(f"case gated random graph {dtype} seed {seed} {sym} decisions {ref.decisions}", flush=True)
            bnd = ses.bind(sym)
            outs = ses.alloc_outputs(ses.output_shapes(bnd))
            ses.run(bnd, ses.upload_inputs(ins), outs)
            torch.cuda.synchronize()
            ran += 1
            switches += len(ref.decisions)
            assert [bool(d) for d in S_lib.sod2_run_decisions(bnd)] == ref.decisions
            assert S_lib.sod2_run_plan_dump(bnd) == A.dump(A.bind(po, sym, ref.decisions))
            for t, o in zip(g.outputs(), outs):
                got = to_host(o)
                assert got.shape == ref.values[t].shape and np.isfinite(got).all()
                err = rel_err(got, ref.values[t])
                worst = max(worst, err)
                assert err <= (1e-4 if dtype == "f32" else 2e-2), (seed, sym, g.tensors[t].name, err)
    print("gated random graphs", dtype, ": ran", ran, "switch decisions", switches, "worst rel err", worst)
    assert ran >= 80 and switches >= 150


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_random_graphs_with_compaction_against_the_oracle(S_lib, dtype):
    """Random graphs with NonZero / Gather / ScatterRows compaction (row masks are graph inputs: no rows, all rows,
    some rows): the counts a run reads back, the plan it ends with (made in mid-run with each count) and every
    output against the oracle."""
    import torch
    from tests.test_random_graphs import random_graph, make_inputs
    from paper_2403_00176_amd.session import Session, to_host
    ran = counts = 0
    worst = 0.0
    for seed in range(30):
        g, weights, shapes = random_graph(seed, dtype, compact=True)
        if g is None or not any(op.kind == "NonZero" for op in g.ops):
            continue
        po = P.build_plan(g, R.RDP(g).analyse())
        ses = Session(g)
        rs = np.random.RandomState(seed)
        W = {t: rs.randn(*d) * 0.3 for t, d in weights.items()}
        ses.upload_weights(W)
        for sym in ({"A": 3, "B": 5}, {"A": 9, "B": 12}, {"A": 1, "B": 1}, {"A": 4, "B": 7}):
            ins = make_inputs(g, shapes, sym, rs)
            ref = execute.run(g, po.order, W, ins)
            print(f"case compacting random graph {dtype} seed {seed} {sym} counts {ref.exec_values}", flush=True)
            bnd = ses.bind(sym)
            outs = ses.alloc_outputs(ses.output_shapes(bnd))
            ses.run(bnd, ses.upload_inputs(ins), outs)
            torch.cuda.synchronize()
            ran += 1
            counts += len(ref.exec_values)
            assert S_lib.sod2_run_exec_values(bnd) == ref.exec_values
            assert S_lib.sod2_run_plan_dump(bnd) == A.dump(A.bind(po, sym, exec_values=ref.exec_values))
            for t, o in zip(g.outputs(), outs):
                got = to_host(o)
                assert got.shape == ref.values[t].shape and np.isfinite(got).all()
                err = rel_err(got, ref.values[t])
                worst = max(worst, err)
                assert err <= (1e-4 if dtype == "f32" else 2e-2), (seed, sym, g.tensors[t].name, err)
    print("compacting random graphs", dtype, ": ran", ran, "counts read back", counts, "worst rel err", worst)
    assert ran >= 60 and counts >= 100


@pytest.mark.parametrize("wide", [False, True], ids=["narrow", "wide"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_random_graphs_with_gates_and_compaction_against_the_oracle(S_lib, dtype, wide):
    """<Switch, Combine> pairs and NonZero compaction in one random graph: decisions, counts, the plan made in mid-run
    with both kinds of read-back, and every output against the oracle."""
    import torch
    from tests.test_random_graphs import random_graph, make_inputs
    from paper_2403_00176_amd.session import Session, to_host
    ran = 0
    worst = 0.0
    for seed in range(40 if wide else 80):
        g, weights, shapes = random_graph(seed, dtype, wide=wide, gates=True, compact=True)
        if g is None or not (any(op.kind == "NonZero" for op in g.ops) and any(op.kind == "Switch" for op in g.ops)):
            continue
        po = P.build_plan(g, R.RDP(g).analyse())
        narrowing = any(op.kind == "Cast" and g.tensors[op.outputs[0]].dtype == "bf16" for op in g.ops)
        ses = Session(g)
        rs = np.random.RandomState(seed)
        W = {t: rs.randn(*d) * (0.5 / np.sqrt(d[-1]) if wide else 0.3) for t, d in weights.items()}
        ses.upload_weights(W)
        for sym in (({"A": 3, "B": 33}, {"A": 40, "B": 100}, {"A": 1, "B": 1}) if wide else ({"A": 3, "B": 5}, {"A": 9, "B": 12}, {"A": 1, "B": 1})):
            ins = make_inputs(g, shapes, sym, rs)
            ref = execute.run(g, po.order, W, ins)
            print(f"case mixed random graph {dtype} seed {seed} {sym} decisions {ref.decisions} counts {ref.exec_values}", flush=True)
            bnd = ses.bind(sym)
            outs = ses.alloc_outputs(ses.output_shapes(bnd))
            ses.run(bnd, ses.upload_inputs(ins), outs)
            torch.cuda.synchronize()
            ran += 1
            assert [bool(d) for d in S_lib.sod2_run_decisions(bnd)] == ref.decisions
            assert S_lib.sod2_run_exec_values(bnd) == ref.exec_values
            assert S_lib.sod2_run_plan_dump(bnd) == A.dump(A.bind(po, sym, ref.decisions, ref.exec_values))
            for t, o in zip(g.outputs(), outs):
                got = to_host(o)
                assert got.shape == ref.values[t].shape and np.isfinite(got).all()
                err = rel_err(got, ref.values[t])
                worst = max(worst, err)
                assert err <= (2e-4 if dtype == "f32" and not (wide and narrowing) else 2e-2), (seed, sym, g.tensors[t].name, err)
    print("mixed random graphs", dtype, "wide" if wide else "narrow", ": ran", ran, "worst rel err", worst)
    assert ran >= (25 if wide else 60)
