"""Pins for the value oracle: each operator against brute force or a closed form, and
whole-graph special cases that reduce to something known."""
import math

import numpy as np
import pytest

from oracle import ops as O
from oracle import execute
from oracle import rdp as R
from workloads import configs, rng


def order_of(g):
    return R.RDP(g).sorted_nodes()


def test_bf16_rounding_is_nearest_even():
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: even mantissa wins; 1 + 3*2^-8 ties upward to even
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -0.3, 3.0e38])
    r = O.round_to(x, "bf16")
    assert r[0] == 1.0 and r[1] == 1.0 + 2.0 ** -6 and r[2] == 1.0 + 2.0 ** -7
    assert abs(r[3] + 0.3) <= 0.3 * 2.0 ** -8
    assert np.array_equal(rng.bf16_bits_to_f32(rng.to_bf16_bits(x)).astype(np.float64), r)
    assert O.round_to(np.array([0.1]), "f32")[0] == float(np.float32(0.1))


def test_conv_matches_seven_loops_and_matmul():
    rs = np.random.RandomState(1)
    for (h, w, c, o, k, s, p) in ((7, 6, 3, 4, 3, 2, 1), (9, 9, 2, 3, 7, 2, 3), (5, 4, 3, 2, 1, 2, 0)):
        x = rs.randn(2, h, w, c)
        wt = rs.randn(o, k, k, c)
        got = O.conv2d_nhwc(x, wt, s, p)
        oh, ow = (h + 2 * p - k) // s + 1, (w + 2 * p - k) // s + 1
        ref = np.zeros((2, oh, ow, o))
        for n in range(2):
            for i in range(oh):
                for j in range(ow):
                    for q in range(o):
                        acc = 0.0
                        for a in range(k):
                            for b in range(k):
                                yy, xx = i * s + a - p, j * s + b - p
                                if 0 <= yy < h and 0 <= xx < w:
                                    for ch in range(c):
                                        acc += x[n, yy, xx, ch] * wt[q, a, b, ch]
                        ref[n, i, j, q] = acc
        assert got.shape == ref.shape and np.allclose(got, ref, rtol=1e-12, atol=1e-12)
    x = rs.randn(1, 5, 5, 8)
    wt = rs.randn(6, 1, 1, 8)
    assert np.allclose(O.conv2d_nhwc(x, wt, 1, 0).reshape(25, 6), x.reshape(25, 8) @ wt.reshape(6, 8).T)


def test_maxpool_brute_force():
    rs = np.random.RandomState(2)
    x = rs.randn(1, 7, 8, 3) - 5.0            # all negative: zero padding would be wrong
    got = O.maxpool_nhwc(x, 3, 2, 1)
    for i in range(got.shape[1]):
        for j in range(got.shape[2]):
            win = [x[0, yy, xx] for yy in range(2 * i - 1, 2 * i + 2) for xx in range(2 * j - 1, 2 * j + 2)
                   if 0 <= yy < 7 and 0 <= xx < 8]
            assert np.array_equal(got[0, i, j], np.max(win, axis=0))


def test_row_operators_closed_forms():
    rs = np.random.RandomState(3)
    g, b = rs.randn(16), rs.randn(16)
    assert np.allclose(O.layernorm(np.full((3, 16), 2.5), g, b, 1e-5), np.tile(b, (3, 1)))
    x = rs.randn(4, 16) * 3 + 1
    y = O.layernorm(x, np.ones(16), np.zeros(16), 0.0)
    assert np.allclose(y.mean(-1), 0, atol=1e-12) and np.allclose((y ** 2).mean(-1), 1)
    assert np.allclose(O.softmax(np.full((2, 7), 3.3), 0), 1 / 7)
    s = O.softmax(rs.randn(5, 9) * 30, 0)
    assert np.allclose(s.sum(-1), 1) and (s >= 0).all()
    x = rs.randn(2, 4, 6)
    c = O.softmax(x, 1)                          # Lq=4, Lk=6: row i sees j <= i + 2
    for i in range(4):
        assert np.all(c[:, i, i + 3:] == 0) and np.allclose(c[:, i, :i + 3].sum(-1), 1)
        ref = np.exp(x[:, i, :i + 3]); ref /= ref.sum(-1, keepdims=True)
        assert np.allclose(c[:, i, :i + 3], ref)
    xs = np.linspace(-6, 6, 49)
    assert np.allclose(O.gelu(xs), [0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in xs], atol=1e-15)
    assert np.allclose(O.sigmoid(xs) + O.sigmoid(-xs), 1)
    # values, not only the symmetry (1 / (1 + exp(-2x)) is symmetric too): sigma(ln 3) = 3/4, sigma(-ln 3) = 1/4,
    # sigma(ln 9) = 9/10, sigma(0) = 1/2
    assert np.allclose(O.sigmoid(np.array([math.log(3.0), -math.log(3.0), math.log(9.0), 0.0])), [0.75, 0.25, 0.9, 0.5],
                       rtol=0, atol=1e-15)


def test_layernorm_epsilon_sits_inside_the_root():
    """Rows of +-a have mean 0 and variance a^2; with eps = 3 a^2 the denominator is sqrt(a^2 + 3 a^2) = 2a, so the
    result is +-gamma/2 + beta.  sqrt(var) + eps would give a / (a + 3 a^2), eps left out +-gamma, eps added
    after the division something else again: each fails here."""
    a = 0.25
    x = np.tile(np.array([a, -a]), (3, 4))                       # [3, 8]
    gamma = np.linspace(0.5, 2.0, 8)
    beta = np.linspace(-1.0, 1.0, 8)
    got = O.layernorm(x, gamma, beta, 3 * a * a)
    ref = np.tile(np.array([0.5, -0.5]), (3, 4)) * gamma + beta
    assert np.allclose(got, ref, rtol=0, atol=1e-15)
    # a shifted row: the mean is removed before the variance is taken (biased, divisor n)
    got = O.layernorm(x + 7.0, gamma, beta, 3 * a * a)
    assert np.allclose(got, ref, rtol=0, atol=1e-12)
    # n = 4 values 0, 0, 0, 4: mean 1, biased variance 3 (the unbiased one would be 4); eps = 1 -> root 2
    got = O.layernorm(np.array([[0.0, 0.0, 0.0, 4.0]]), np.ones(4), np.zeros(4), 1.0)
    assert np.allclose(got, [[-0.5, -0.5, -0.5, 1.5]], rtol=0, atol=1e-15)


def _run(w, sym, call=0, weights=None, **kw):
    W = w.make_weights() if weights is None else weights
    return execute.run(w.graph, order_of(w.graph), W, w.make_inputs(call, sym), **kw), W


def test_zero_and_identity_weights_reduce_the_block():
    w = configs.config1()
    g = w.graph
    W = w.make_weights()
    # zero the two projections that feed the residual adds: the block is the identity
    for name in ("l0.o.w", "l0.o.b", "l0.ffn2.w", "l0.ffn2.b"):
        W[g.tensor_id(name)] = np.zeros_like(W[g.tensor_id(name)])
    res, _ = _run(w, {"L": 19}, weights=W)
    x = O.round_to(w.make_inputs(0, {"L": 19})[g.tensor_id("x")], "f32")
    assert np.array_equal(res.values[g.outputs()[0]], x)
    # identity FFN1 weight + zero bias: pre-GELU tensor equals LayerNorm output zero-extended
    W = w.make_weights()
    eye = np.zeros((1024, 256)); eye[:256] = np.eye(256)
    W[g.tensor_id("l0.ffn1.w")] = eye
    W[g.tensor_id("l0.ffn1.b")] = np.zeros(1024)
    res, _ = _run(w, {"L": 19}, weights=W)
    ln2 = [i for i, t in enumerate(g.tensors) if t.name.startswith("l0.ln2_")][0]
    ffn1 = [i for i, t in enumerate(g.tensors) if t.name.startswith("l0.ffn1_b")][0]
    assert np.array_equal(res.values[ffn1][..., :256], res.values[ln2])
    assert not res.values[ffn1][..., 256:].any()


def test_attention_matches_per_head_loops():
    """The Reshape/Transpose/Gather plumbing of the encoder equals explicit per-head attention."""
    w = configs.config1()
    g = w.graph
    res, W = _run(w, {"L": 23})
    v = res.values
    name = lambda p: [i for i, t in enumerate(g.tensors) if t.name.startswith(p)][0]
    qkv = v[name("l0.qkv_b")][0]                   # [L, 768]
    ctx = v[name("ctx_")][0]                       # [L, 256]
    for h in range(4):
        q = qkv[:, 0 * 256 + h * 64: 0 * 256 + (h + 1) * 64]
        k = qkv[:, 1 * 256 + h * 64: 1 * 256 + (h + 1) * 64]
        vv = qkv[:, 2 * 256 + h * 64: 2 * 256 + (h + 1) * 64]
        s = q @ k.T / 8.0
        p = np.exp(s - s.max(-1, keepdims=True)); p /= p.sum(-1, keepdims=True)
        assert np.allclose(ctx[:, h * 64:(h + 1) * 64], p @ vv, atol=2e-6)


def test_float64_run_bounds_the_rounded_oracle():
    w = configs.config1()
    g = w.graph
    res, W = _run(w, {"L": 40})
    g64 = configs.config1().graph
    for t in g64.tensors:
        if t.dtype == "f32":
            t.dtype = "f64x"
    # run with no rounding at all by bypassing round_to for the made-up dtype
    orig = O.round_to
    try:
        O.round_to = lambda x, d: x if d == "f64x" else orig(x, d)
        execute.O.round_to = O.round_to
        exact = execute.run(g64, order_of(g64), W, w.make_inputs(0, {"L": 40}))
    finally:
        O.round_to = orig
        execute.O.round_to = orig
    a, b = res.values[g.outputs()[0]], exact.values[g64.outputs()[0]]
    assert np.abs(a - b).max() / np.abs(b).max() < 1e-5


def test_gate_closed_forms():
    """Config 4: a gate bias of +10 skips every layer (output = final LayerNorm of the input);
    -10 runs every layer (same values as the ungated stack with the same layer weights)."""
    lay = 2
    skip = configs.config4(1, layers=lay, gate_bias=10.0)
    run_ = configs.config4(1, layers=lay, gate_bias=-10.0)
    sym = {"L": 128}
    rs, Ws = _run(skip, sym)
    assert rs.decisions == [True] * lay
    g = skip.graph
    x = O.round_to(skip.make_inputs(0, sym)[g.tensor_id("x")], "bf16")
    ref = O.round_to(O.layernorm(x, O.round_to(Ws[g.tensor_id("lnf.g")], "bf16"),
                                 O.round_to(Ws[g.tensor_id("lnf.beta")], "bf16"), 1e-5), "bf16")
    assert np.array_equal(rs.values[g.outputs()[0]], ref)
    rr, Wr = _run(run_, sym)
    assert rr.decisions == [False] * lay
    # the ungated encoder fed the same layer weights gives the same output
    plain = configs.encoder(4, lay, 768, 12, 3072, "bf16", 4, (128, 384), 1, final_ln=True)
    Wp = {plain.graph.tensor_id(run_.graph.tensors[t].name): v for t, v in Wr.items()
          if not run_.graph.tensors[t].name.startswith("g")}
    rp = execute.run(plain.graph, order_of(plain.graph), Wp, {plain.graph.tensor_id("x"): run_.make_inputs(0, sym)[run_.graph.tensor_id("x")]})
    assert np.array_equal(rp.values[plain.graph.outputs()[0]], rr.values[run_.graph.outputs()[0]])
    # forcing decisions overrides the predicate
    rf = execute.run(run_.graph, order_of(run_.graph), Wr, run_.make_inputs(0, sym), forced=[True] * lay)
    assert rf.decisions == [True] * lay


def test_input_generators_follow_the_stated_distributions():
    z = rng.normal(11, (200000,), 0.0, 0.02)
    assert abs(z.mean()) < 2e-4 and abs(z.std() - 0.02) < 2e-4
    u = rng.uniform(12, (100000,))
    assert 0 < u.min() and u.max() < 1 and abs(u.mean() - 0.5) < 5e-3
    k = rng.randint(13, (50000,), 32, 512)
    assert k.min() == 32 and k.max() == 512
    assert np.array_equal(rng.normal(5, (10,)), rng.normal(5, (20,))[:10])      # counter based
    for cfg in (1, 2, 3, 4):
        w = configs.BUILDERS[cfg]()
        for c in w.calls:
            for n, lo, hi in w.graph.symbols:
                assert lo <= c[n] <= hi
    assert all(c["H"] % 32 == 0 and c["H"] == c["W"] for c in configs.config3().calls)
