"""The five synthetic dynamic workloads and their seeded data.

They stand in for the trained models and public datasets of the paper's
evaluation (Section 5.1: images 224-640 in multiples of 32, sequences 32-512),
none of which is available: same operator mix, shape ranges and dynamism
(shape dynamism, control-flow dynamism, both), random-initialised weights.

Every builder returns a ``Workload``: the graph description, a function that
materialises the weights (``seed = 1000 * config + weight index``), the list
of per-call symbol draws and a function producing the inputs of a call.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, Dict, List

import numpy as np

from . import rng
from .graphdesc import GraphBuilder, GraphDesc, WEIGHT, INPUT

INT_MAX = 2 ** 31 - 1


@dataclass
class Workload:
    name: str
    config: int
    graph: GraphDesc
    dtype: str                                   # float storage type of the graph
    calls: List[Dict[str, int]]                  # symbol values per call
    make_weights: Callable[[], Dict[int, np.ndarray]]          # tensor id -> float64 array
    make_inputs: Callable[[int, Dict[str, int]], Dict[int, np.ndarray]]
    weight_spec: Dict[int, tuple] = None


class _Weights:
    """Records (kind, params) per weight tensor; values are generated on demand."""

    def __init__(self, config: int):
        self.config = config
        self.spec: Dict[int, tuple] = {}

    def add(self, tid, kind, *params):
        self.spec[tid] = (kind,) + params

    def make(self, graph: GraphDesc) -> Dict[int, np.ndarray]:
        out = {}
        for k, (tid, spec) in enumerate(sorted(self.spec.items())):
            shape = tuple(graph.tensors[tid].dims)
            seed = 1000 * self.config + k
            kind = spec[0]
            if kind == "normal":
                out[tid] = rng.normal(seed, shape, spec[1], spec[2])
            elif kind == "const":
                out[tid] = np.full(shape, spec[1], dtype=np.float64)
            else:
                raise ValueError(kind)
        return out


def _linear(b: GraphBuilder, w: _Weights, x, n_in, n_out, name, dtype, std=0.02, bias_std=0.02):
    """x @ W^T + bias with W stored [out, in] (the layout a Linear layer keeps)."""
    W = b.weight(f"{name}.w", dtype, [n_out, n_in]); w.add(W, "normal", 0.0, std)
    B = b.weight(f"{name}.b", dtype, [n_out]); w.add(B, "normal", 0.0, bias_std)
    y = b.op("MatMul", [x, W], transB=1, hint=name)
    return b.op("Add", [y, B], hint=name + "_b")


def _layernorm(b, w, x, n, name, dtype):
    g = b.weight(f"{name}.g", dtype, [n]); w.add(g, "normal", 1.0, 0.02)
    be = b.weight(f"{name}.beta", dtype, [n]); w.add(be, "normal", 0.0, 0.02)
    return b.op("LayerNorm", [x, g, be], eps=1e-5, hint=name)


def _encoder_layer(b, w, x, hidden, heads, ffn, name, dtype, lead):
    """Pre-LN block.  ``lead`` = tensor ids of the 1-element int tensors holding the leading dims."""
    d = hidden // heads
    h1 = _layernorm(b, w, x, hidden, f"{name}.ln1", dtype)
    qkv = _linear(b, w, h1, hidden, 3 * hidden, f"{name}.qkv", dtype)
    tgt = b.op("Concat", lead + [b.const(f"{name}.c3hd", [3, heads, d])], axis=0, dtype="i64")
    qkv5 = b.op("Reshape", [qkv, tgt], hint="qkv5")                    # [B, L, 3, h, d]
    qkvT = b.op("Transpose", [qkv5], perm=(2, 0, 3, 1, 4), hint="qkvT")  # [3, B, h, L, d]
    q = b.op("Gather", [qkvT, b.const(f"{name}.i0", 0)], axis=0, hint="q")
    k = b.op("Gather", [qkvT, b.const(f"{name}.i1", 1)], axis=0, hint="k")
    v = b.op("Gather", [qkvT, b.const(f"{name}.i2", 2)], axis=0, hint="v")
    kT = b.op("Transpose", [k], perm=(0, 1, 3, 2), hint="kT")
    s = b.op("MatMul", [q, kT], transB=0, hint="qk")
    s = b.op("Mul", [s, b.const(f"{name}.scale", 1.0 / np.sqrt(d), "f32")], hint="scaled")
    p = b.op("Softmax", [s], causal=0, hint="probs")
    c = b.op("MatMul", [p, v], transB=0, hint="pv")                    # [B, h, L, d]
    cT = b.op("Transpose", [c], perm=(0, 2, 1, 3), hint="ctxT")        # [B, L, h, d]
    tgt2 = b.op("Concat", lead + [b.const(f"{name}.chid", [hidden])], axis=0, dtype="i64")
    c2 = b.op("Reshape", [cT, tgt2], hint="ctx")
    o = _linear(b, w, c2, hidden, hidden, f"{name}.o", dtype)
    x1 = b.op("Add", [o, x], hint="res1")
    h2 = _layernorm(b, w, x1, hidden, f"{name}.ln2", dtype)
    f = _linear(b, w, h2, hidden, ffn, f"{name}.ffn1", dtype)
    f = b.op("Gelu", [f], hint="gelu")
    f2 = _linear(b, w, f, ffn, hidden, f"{name}.ffn2", dtype)
    return b.op("Add", [f2, x1], hint="res2")


def _lead_dims(b, x, n, tag):
    """Shape(x) -> n one-element tensors (the pattern an exporter emits for dynamic reshapes)."""
    shp = b.op("Shape", [x], dtype="i64", hint=f"{tag}.shape")
    return [b.op("Gather", [shp, b.const(f"{tag}.ax{i}", [i])], axis=0, dtype="i64", hint=f"{tag}.dim{i}")
            for i in range(n)]


def _draws(seed, spec, n_calls):
    """spec: list of (symbol, lo, hi, step); one independent stream per symbol."""
    calls = [dict() for _ in range(n_calls)]
    for j, (name, lo, hi, step) in enumerate(spec):
        vals = rng.randint(seed + 17 * j, (n_calls,), 0, (hi - lo) // step)
        for c, v in zip(calls, vals):
            c[name] = int(lo + step * v)
    return calls


def encoder(config: int, layers: int, hidden: int, heads: int, ffn: int, dtype: str,
            batch, seq_range, n_calls: int, final_ln: bool, gated=False,
            gate_bias: float = None, taps: bool = False) -> Workload:
    """Configs 1, 2, 4 and 6: a stack of pre-LN encoder blocks on x[B, L, hidden].

    ``gated=True``: one skip decision per layer and call (<Switch, Combine>, config 4).
    ``gated="sample"``: one decision per layer and *sequence*; the sequences that run the layer are
    compacted with NonZero + Gather (an execution-determined batch size), the block runs on the
    compacted batch, ScatterRows writes its rows back (config 6).
    ``taps=True``: the residual stream after every layer is a graph output as well (same operators, same
    weights, same values; a test can then say in which layer a difference starts)."""
    syms = [("L", seq_range[0], seq_range[1])]
    if isinstance(batch, tuple):
        syms = [("B", batch[0], batch[1])] + syms
        bdim = "B"
    else:
        bdim = int(batch)
    b = GraphBuilder(syms)
    w = _Weights(config)
    x = b.input("x", dtype, [bdim, "L", hidden])
    lead = _lead_dims(b, x, 2, "x")
    for l in range(layers):
        if gated == "sample":
            # per-sequence gate: mean over the tokens of a sequence -> Linear -> ReLU -> Linear -> ReLU;
            # a sequence runs the layer when its gate value is non-zero (logit > 0)
            m = b.op("ReduceMean", [x], axes=(1,), keepdims=0, dtype="f32", hint=f"g{l}.pool")
            g1 = b.op("Relu", [_linear(b, w, m, hidden, 64, f"g{l}.fc1", "f32", std=0.5)], hint=f"g{l}.relu")
            if gate_bias is None:
                z = _linear(b, w, g1, 64, 1, f"g{l}.fc2", "f32", std=0.25, bias_std=1.0)
            else:
                z = _linear(b, w, g1, 64, 1, f"g{l}.fc2", "f32")
                w.spec[b.g.tensor_id(f"g{l}.fc2.b")] = ("const", float(gate_bias))
            keep = b.op("Relu", [z], hint=f"g{l}.keep")                          # [B, 1]
            kv = b.op("Reshape", [keep, b.const(f"g{l}.flat", [-1])], hint=f"g{l}.keepv")   # [B]
            nz = b.op("NonZero", [kv], dtype="i64", hint=f"g{l}.nz")             # [1, B'] execution determined
            idx = b.op("Gather", [nz, b.const(f"g{l}.row0", 0)], axis=0, dtype="i64", hint=f"g{l}.idx")   # [B']
            xs = b.op("Gather", [x, idx], axis=0, hint=f"g{l}.xs")               # [B', L, hidden]
            lead_s = _lead_dims(b, xs, 2, f"xs{l}")
            ys = _encoder_layer(b, w, xs, hidden, heads, ffn, f"l{l}", dtype, lead_s)
            x = b.op("ScatterRows", [x, idx, ys], hint=f"g{l}.merge")
        elif gated:
            # gate: mean over all token rows -> Linear(hidden,64) -> ReLU -> Linear(64,1) -> sigmoid
            m = b.op("ReduceMean", [x], axes=(0, 1), keepdims=1, dtype="f32", hint=f"g{l}.pool")
            g1 = b.op("Relu", [_linear(b, w, m, hidden, 64, f"g{l}.fc1", "f32")], hint=f"g{l}.relu")
            if gate_bias is None:
                g2 = _linear(b, w, g1, 64, 1, f"g{l}.fc2", "f32", bias_std=1.0)
            else:
                g2 = _linear(b, w, g1, 64, 1, f"g{l}.fc2", "f32")
                w.spec[b.g.tensor_id(f"g{l}.fc2.b")] = ("const", float(gate_bias))
            pred = b.op("Sigmoid", [g2], hint=f"g{l}.sig")
            run, skip = b.op("Switch", [x, pred], n_out=2, threshold=0.5, hint=f"sw{l}")
            y = _encoder_layer(b, w, run, hidden, heads, ffn, f"l{l}", dtype, lead)
            x = b.op("Combine", [y, skip], hint=f"cmb{l}")
        else:
            x = _encoder_layer(b, w, x, hidden, heads, ffn, f"l{l}", dtype, lead)
        if taps:
            b.mark_output(x)
    if final_ln:
        x = _layernorm(b, w, x, hidden, "lnf", dtype)
    b.mark_output(x, "y")
    g = b.build()
    spec = ([("B", batch[0], batch[1], 1)] if isinstance(batch, tuple) else []) + \
           [("L", seq_range[0], seq_range[1], 1)]
    calls = _draws(7000 + config, spec, n_calls)

    def make_inputs(call_idx, sym):
        B = sym.get("B", bdim)
        return {g.tensor_id("x"): rng.normal(100000 * config + call_idx, (B, sym["L"], hidden))}

    return Workload(f"cfg{config}", config, g, dtype, calls, lambda: w.make(g), make_inputs, w.spec)


def config1(n_calls=8):
    return encoder(1, 1, 256, 4, 1024, "f32", 1, (16, 128), n_calls, final_ln=False)


def config2(n_calls=64, layers=12, taps=False):
    return encoder(2, layers, 768, 12, 3072, "bf16", (1, 8), (32, 512), n_calls, final_ln=True, taps=taps)


def config4(n_calls=64, layers=12, gate_bias=None):
    return encoder(4, layers, 768, 12, 3072, "bf16", 4, (128, 384), n_calls, final_ln=True,
                   gated=True, gate_bias=gate_bias)


def config6(n_calls=32, layers=12, gate_bias=None):
    """Config 4 with the decision taken per sequence and the batch compacted: control-flow dynamism
    that turns into shape dynamism through an execution-determined operator (NonZero).  Not one of
    the five benchmark configurations; it exercises the EDO class of Table 2 end to end."""
    return encoder(6, layers, 768, 12, 3072, "bf16", (2, 8), (128, 384), n_calls, final_ln=True,
                   gated="sample", gate_bias=gate_bias)


# ---------------------------------------------------------------------------
# config 3: ResNet-50 layout, NHWC
# ---------------------------------------------------------------------------

def _conv(b, w, x, cin, cout, k, stride, pad, name, dtype, relu):
    W = b.weight(f"{name}.w", dtype, [cout, k, k, cin])
    w.add(W, "normal", 0.0, float(np.sqrt(2.0 / (k * k * cin))))
    B = b.weight(f"{name}.b", dtype, [cout]); w.add(B, "normal", 0.0, 0.02)
    y = b.op("Conv", [x, W], stride=stride, pad=pad, hint=name)
    y = b.op("Add", [y, B], hint=name + "_b")
    return b.op("Relu", [y], hint=name + "_r") if relu else y


def _bottleneck(b, w, x, cin, mid, cout, stride, project, name, dtype):
    y = _conv(b, w, x, cin, mid, 1, 1, 0, f"{name}.c1", dtype, True)
    y = _conv(b, w, y, mid, mid, 3, stride, 1, f"{name}.c2", dtype, True)
    y = _conv(b, w, y, mid, cout, 1, 1, 0, f"{name}.c3", dtype, False)
    sc = _conv(b, w, x, cin, cout, 1, stride, 0, f"{name}.sc", dtype, False) if project else x
    return b.op("Relu", [b.op("Add", [y, sc], hint=name + "_add")], hint=name + "_out")


def resnet50(config=3, n_calls=32, sizes=tuple(range(224, 641, 32)), stages=(3, 4, 6, 3),
             classes=1000, dtype="bf16", taps=False) -> Workload:
    """``taps=True``: the feature map after every stage is a graph output as well (same operators and values)."""
    b = GraphBuilder([("H", min(sizes), max(sizes)), ("W", min(sizes), max(sizes))])
    w = _Weights(config)
    x = b.input("x", dtype, [1, "H", "W", 3])
    y = _conv(b, w, x, 3, 64, 7, 2, 3, "stem", dtype, True)
    y = b.op("MaxPool", [y], kernel=3, stride=2, pad=1, hint="pool")
    cin = 64
    for s, n in enumerate(stages):
        mid, cout = 64 << s, 256 << s
        for i in range(n):
            stride = 2 if (i == 0 and s > 0) else 1
            y = _bottleneck(b, w, y, cin, mid, cout, stride, i == 0, f"s{s}b{i}", dtype)
            cin = cout
        if taps:
            b.mark_output(y)
    y = b.op("ReduceMean", [y], axes=(1, 2), keepdims=0, hint="gap")
    y = _linear(b, w, y, cin, classes, "fc", dtype)
    b.mark_output(y, "logits")
    g = b.build()
    idx = rng.randint(7000 + config, (n_calls,), 0, len(sizes) - 1)
    calls = [{"H": int(sizes[i]), "W": int(sizes[i])} for i in idx]

    def make_inputs(call_idx, sym):
        return {g.tensor_id("x"): rng.uniform(100000 * config + call_idx, (1, sym["H"], sym["W"], 3))}

    return Workload(f"cfg{config}", config, g, dtype, calls, lambda: w.make(g), make_inputs, w.spec)


def config3(n_calls=32):
    return resnet50(3, n_calls)


def fpn(config=7, n_calls=16, sizes=tuple(range(224, 641, 32)), stages=(3, 4, 6, 3), width=256, dtype="bf16") -> Workload:
    """A detection-style neck on the ResNet backbone (after the paper's YOLO-V6 experiment: images in
    multiples of 32): features of stride 8 / 16 / 32, a top-down path that enlarges the coarser map to
    the size of the finer one (Resize whose target shape is *computed* from Shape of the other tensor:
    an ISVDOS operator, Table 2), Concat along the channels, 3x3 convolutions; three output maps."""
    b = GraphBuilder([("H", min(sizes), max(sizes)), ("W", min(sizes), max(sizes))])
    w = _Weights(config)
    x = b.input("x", dtype, [1, "H", "W", 3])
    y = _conv(b, w, x, 3, 64, 7, 2, 3, "stem", dtype, True)
    y = b.op("MaxPool", [y], kernel=3, stride=2, pad=1, hint="pool")
    cin, feats = 64, []
    for s, n in enumerate(stages):
        mid, cout = 64 << s, 256 << s
        for i in range(n):
            stride = 2 if (i == 0 and s > 0) else 1
            y = _bottleneck(b, w, y, cin, mid, cout, stride, i == 0, f"s{s}b{i}", dtype)
            cin = cout
        feats.append((y, cout))
    (c3, n3), (c4, n4), (c5, n5) = feats[1], feats[2], feats[3]
    zero, one, three, four = (b.const(f"k{v}", [v]) for v in (0, 1, 3, 4))
    axis0 = b.const("ax0", [0])

    def part(t, lo, hi, tag):        # Shape(t)[lo:hi] as an exporter writes it
        shp = b.op("Shape", [t], dtype="i64", hint=tag + ".shape")
        return b.op("Slice", [shp, lo, hi, axis0], dtype="i64", hint=tag + ".part")

    def enlarge(small, like, tag):   # nearest-neighbour Resize of `small` to the spatial size of `like`
        sizes_t = b.op("Concat", [part(small, zero, one, tag + ".n"), part(like, one, three, tag + ".hw"),
                                  part(small, three, four, tag + ".c")], axis=0, dtype="i64", hint=tag + ".sizes")
        return b.op("Resize", [small, sizes_t], hint=tag)

    p5 = _conv(b, w, c5, n5, width, 1, 1, 0, "lat5", dtype, False)
    p4 = _conv(b, w, c4, n4, width, 1, 1, 0, "lat4", dtype, False)
    m4 = b.op("Concat", [enlarge(p5, p4, "up5"), p4], axis=3, hint="cat4")
    m4 = _conv(b, w, m4, 2 * width, width, 3, 1, 1, "fuse4", dtype, True)
    p3 = _conv(b, w, c3, n3, width, 1, 1, 0, "lat3", dtype, False)
    m3 = b.op("Concat", [enlarge(m4, p3, "up4"), p3], axis=3, hint="cat3")
    m3 = _conv(b, w, m3, 2 * width, width, 3, 1, 1, "fuse3", dtype, True)
    b.mark_output(_conv(b, w, m3, width, width, 1, 1, 0, "head3", dtype, False), "out8")
    b.mark_output(_conv(b, w, m4, width, width, 1, 1, 0, "head4", dtype, False), "out16")
    b.mark_output(_conv(b, w, p5, width, width, 1, 1, 0, "head5", dtype, False), "out32")
    g = b.build()
    idx = rng.randint(7000 + config, (n_calls,), 0, len(sizes) - 1)
    calls = [{"H": int(sizes[i]), "W": int(sizes[i])} for i in idx]

    def make_inputs(call_idx, sym):
        return {g.tensor_id("x"): rng.uniform(100000 * config + call_idx, (1, sym["H"], sym["W"], 3))}

    return Workload(f"cfg{config}", config, g, dtype, calls, lambda: w.make(g), make_inputs, w.spec)


def config7(n_calls=16):
    return fpn(7, n_calls)


# ---------------------------------------------------------------------------
# config 5: autoregressive decoder with a KV cache in the arena (two graphs, one set of weights)
# ---------------------------------------------------------------------------

@dataclass
class DecoderWorkload:
    name: str
    config: int
    prefill: GraphDesc                           # symbols P; ids/pos [P]
    decode: GraphDesc                            # symbols P, t; ids/pos [1]; caches hold P+t rows
    dtype: str
    prompts: List[int]                           # prompt length per sequence
    t_max: int                                   # generated tokens per sequence
    vocab: int
    weight_spec: Dict[str, tuple]                # weight name -> (kind, params, seed index)
    make_prompt: Callable[[int], np.ndarray] = None

    def make_weights_by_name(self, threads: int = 8) -> Dict[str, np.ndarray]:
        from concurrent.futures import ThreadPoolExecutor
        by_name = {t.name: t for t in self.prefill.tensors if t.role == WEIGHT}

        def one(item):
            name, (kind, a, b_, k) = item
            return name, rng.normal(1000 * self.config + k, tuple(by_name[name].dims), a, b_)
        with ThreadPoolExecutor(max_workers=threads) as ex:      # the generator is counter based: order free
            return dict(ex.map(one, self.weight_spec.items()))

    @staticmethod
    def weights_for(graph: GraphDesc, by_name: Dict[str, np.ndarray]) -> Dict[int, np.ndarray]:
        return {i: by_name[t.name] for i, t in enumerate(graph.tensors) if t.role == WEIGHT}


def _decoder_graph(mode, layers, hidden, heads, ffn, vocab, max_pos, p_range, t_max, dtype, w: _Weights):
    """Pre-LN decoder blocks on x[n, hidden] (batch 1): n = P rows for the prompt, 1 row per generated
    token.  K and V of every layer are appended to session tensors holding ``past`` rows."""
    d = hidden // heads
    if mode == "prefill":
        b = GraphBuilder([("P", p_range[0], p_range[1])])
        n, past = "P", 0
    else:
        b = GraphBuilder([("P", p_range[0], p_range[1]), ("t", 0, t_max - 1)])
        n, past = 1, "P+t"
    ids = b.input("ids", "i64", [n])
    pos = b.input("pos", "i64", [n])
    tok = b.weight("tok_emb", dtype, [vocab, hidden]); w.add(tok, "normal", 0.0, 0.02)
    pw = b.weight("pos_emb", dtype, [max_pos, hidden]); w.add(pw, "normal", 0.0, 0.02)
    caches = [(b.session_input(f"l{l}.kc", dtype, [past, hidden], [f"P+{t_max}", hidden]),
               b.session_input(f"l{l}.vc", dtype, [past, hidden], [f"P+{t_max}", hidden])) for l in range(layers)]
    e_pos = b.op("Gather", [pw, pos], axis=0, hint="e_pos")
    x = b.op("Add", [b.op("Gather", [tok, ids], axis=0, hint="e_tok"), e_pos], hint="embed")
    split = b.const("c.split", [0, 3, heads, d])
    flat = b.const("c.flat", [0, hidden])
    heads3 = b.const("c.heads", [0, heads, d])
    sel = [b.const(f"c.i{i}", i) for i in range(3)]
    scale = b.const("c.scale", 1.0 / np.sqrt(d), "f32")
    for l in range(layers):
        name = f"l{l}"
        h1 = _layernorm(b, w, x, hidden, f"{name}.ln1", dtype)
        qkv = _linear(b, w, h1, hidden, 3 * hidden, f"{name}.qkv", dtype)
        qkv4 = b.op("Reshape", [qkv, split], hint="qkv4")                            # [n, 3, h, d]
        q = b.op("Gather", [qkv4, sel[0]], axis=1, hint="q")                         # [n, h, d]
        k_new = b.op("Reshape", [b.op("Gather", [qkv4, sel[1]], axis=1, hint="k")    , flat], hint="k_new")
        v_new = b.op("Reshape", [b.op("Gather", [qkv4, sel[2]], axis=1, hint="v"), flat], hint="v_new")
        kc = b.op("CacheAppend", [caches[l][0], k_new], hint=f"{name}.kc_out")      # [past + n, hidden]
        vc = b.op("CacheAppend", [caches[l][1], v_new], hint=f"{name}.vc_out")
        qT = b.op("Transpose", [q], perm=(1, 0, 2), hint="qT")                       # [h, n, d]
        kT = b.op("Transpose", [b.op("Reshape", [kc, heads3], hint="k3")], perm=(1, 2, 0), hint="kT")   # [h, d, T]
        s = b.op("MatMul", [qT, kT], transB=0, hint="qk")                            # [h, n, T]
        s = b.op("Mul", [s, scale], hint="scaled")
        p = b.op("Softmax", [s], causal=1, hint="probs")
        vT = b.op("Transpose", [b.op("Reshape", [vc, heads3], hint="v3")], perm=(1, 0, 2), hint="vT")   # [h, T, d]
        c = b.op("MatMul", [p, vT], transB=0, hint="pv")                             # [h, n, d]
        c = b.op("Reshape", [b.op("Transpose", [c], perm=(1, 0, 2), hint="ctxT"), flat], hint="ctx")
        x1 = b.op("Add", [_linear(b, w, c, hidden, hidden, f"{name}.o", dtype), x], hint="res1")
        h2 = _layernorm(b, w, x1, hidden, f"{name}.ln2", dtype)
        f = b.op("Gelu", [_linear(b, w, h2, hidden, ffn, f"{name}.ffn1", dtype)], hint="gelu")
        x = b.op("Add", [_linear(b, w, f, ffn, hidden, f"{name}.ffn2", dtype), x1], hint="res2")
    last = b.op("Slice", [x, b.const("c.m1", [-1]), b.const("c.end", [INT_MAX]), b.const("c.ax0", [0])], hint="last")
    hN = _layernorm(b, w, last, hidden, "lnf", dtype)
    lm = b.weight("lm_head", dtype, [vocab, hidden]); w.add(lm, "normal", 0.0, 0.02)
    logits = b.mark_output(b.op("MatMul", [hN, lm], transB=1, hint="lm"), "logits")   # [1, vocab]
    b.mark_output(b.op("ArgMax", [logits], dtype="i64", hint="argmax"), "next")        # [1]
    return b.build()


def decoder(config=5, layers=24, hidden=1024, heads=16, ffn=4096, vocab=32000, p_range=(64, 512), t_max=256,
            n_prompts=8, dtype="bf16") -> DecoderWorkload:
    """Config 5.  Architecture details the config leaves open: pre-LN blocks with erf GELU, a final
    LayerNorm, learned absolute positions, an untied LM head without bias, softmax scale 1/sqrt(d)."""
    graphs, specs = {}, {}
    for mode in ("prefill", "decode"):
        w = _Weights(config)
        graphs[mode] = _decoder_graph(mode, layers, hidden, heads, ffn, vocab, p_range[1] + t_max, p_range, t_max, dtype, w)
        specs[mode] = {graphs[mode].tensors[tid].name: spec + (k,) for k, (tid, spec) in enumerate(sorted(w.spec.items()))}
    assert specs["prefill"] == specs["decode"], "the two graphs must declare the same weights in the same order"
    prompts = [int(v) for v in rng.randint(7000 + config, (n_prompts,), p_range[0], p_range[1])]

    def make_prompt(i):
        return rng.randint(100000 * config + i, (prompts[i],), 0, vocab - 1)

    return DecoderWorkload(f"cfg{config}", config, graphs["prefill"], graphs["decode"], dtype, prompts, t_max, vocab,
                           specs["prefill"], make_prompt)


def config5(n_prompts=8, layers=24):
    return decoder(5, layers=layers, n_prompts=n_prompts)


BUILDERS = {1: config1, 2: config2, 3: config3, 4: config4, 6: config6, 7: config7}
