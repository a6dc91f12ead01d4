#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: dynamic-shape inference latency, peak arena MB and
roofline fraction on synthetic config 2 (12-layer bf16 encoder, B in [1,8], L in [32,512] redrawn
per call).  One step = sod2_bind + sod2_run + stream synchronise for one call, inputs already on
the device.  Prints one JSON line."""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_FP32_VECTOR_TFLOPS = 157.3   # vector ALUs: 256 CUs x 128 lanes x 2 flop x 2.4 GHz
PEAK_HBM_GBS = 8000.0


def bench_ablation(args, S, dev):
    """The paper's optimisation breakdown (Figs. 5 and 6: latency and memory as RDP-enabled fusion, static
    execution planning, dynamic memory planning and multi-version kernels are switched on one after the
    other) on the synthetic workload: same calls, same weights, one Session per setting."""
    import torch
    from paper_2403_00176_amd.session import Session
    from workloads import configs
    w = configs.BUILDERS[args.config](n_calls=args.steps + args.warmup)
    W = w.make_weights()
    # (in-place reuse of a dying operand's storage belongs to the memory plan: on from the DMP stage)
    stages = [("none", dict(fusion=0, sep=0, dmp=0, mvc=0, inplace=0)), ("+fusion", dict(fusion=1, sep=0, dmp=0, mvc=0, inplace=0)),
              ("+sep", dict(fusion=1, sep=1, dmp=0, mvc=0, inplace=0)), ("+dmp", dict(fusion=1, sep=1, dmp=1, mvc=0, inplace=1)),
              ("+mvc", dict(fusion=1, sep=1, dmp=1, mvc=1, inplace=1))]
    rows = {}
    for name, opts in stages:
        ses = Session(w.graph, device=dev, **opts)
        ses.upload_weights(W)
        calls, max_arena = [], 0
        for ci in range(args.steps + args.warmup):
            sym = w.calls[ci]
            b = ses.bind(sym)
            max_arena = max(max_arena, S.sod2_binding_arena_bytes(b)[0])
            calls.append((sym, ses.upload_inputs(w.make_inputs(ci, sym)), ses.alloc_outputs(ses.output_shapes(b))))
        ses.ensure_arena(max_arena)
        lat, arena, steps = [], [], []
        for k, (sym, ins, outs) in enumerate(calls):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            b = ses.bind(sym)
            ses.run(b, ins, outs)
            ses.stream.synchronize()
            if k >= args.warmup:
                lat.append((time.perf_counter() - t0) * 1e3)
                arena.append(S.sod2_run_arena_bytes(b)[0] / 2 ** 20)
                steps.append(sum(1 for line in S.sod2_run_plan_dump(b).splitlines() if line.startswith("step ")))
        rows[name] = dict(latency_ms=round(sum(lat) / len(lat), 4), peak_arena_mb_mean=round(sum(arena) / len(arena), 3),
                          peak_arena_mb_max=round(max(arena), 3), steps_per_call=round(sum(steps) / len(steps), 1))
        del ses
        torch.cuda.empty_cache()
    base = rows["none"]
    for r in rows.values():
        r["speedup_vs_none"] = round(base["latency_ms"] / r["latency_ms"], 3)
        r["arena_vs_none"] = round(r["peak_arena_mb_mean"] / base["peak_arena_mb_mean"], 3)
    print(json.dumps({"metric": "optimisation breakdown (latency ms per call, peak arena MB)", "unit": "ms", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup, "data": "synthetic", "dtype": w.dtype,
                      "config": {"workload": f"config {args.config}", "calls": args.steps}, "stages": rows,
                      "paper_context": "Figs. 5-6: each optimisation switched on after the previous one"}))


def bench_decoder(args, S, dev):
    """Config 5 (not the headline workload): per sequence one prompt pass and `t_max` greedy decode steps, the
    next token read on the device; reports ms per generated token (steps replayed from one captured HIP
    graph, and bound and launched one by one) and the prompt-pass latency."""
    import numpy as np
    import torch
    from paper_2403_00176_amd.session import DecoderSession
    from workloads import configs
    w = configs.config5(n_prompts=max(1, min(args.steps, 8)))
    ses = DecoderSession(w.prefill, w.decode, w.t_max, device=dev)
    ses.upload_weights(w.make_weights_by_name())
    rows = []
    for i, P in enumerate(w.prompts):
        prompt = torch.from_numpy(np.asarray(w.make_prompt(i), dtype=np.int64)).to(dev)
        ses.start(P, w.vocab)
        for rep in range(2):                       # first repetition warms up
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ses.prefill(prompt)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for t in range(w.t_max):
                ses.decode(t)
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            ses.prefill(prompt)
            torch.cuda.synchronize()
            t3 = time.perf_counter()
            ses.decode_replay(0, w.t_max)
            torch.cuda.synchronize()
            t4 = time.perf_counter()
        pre = []                                   # the prompt pass again, five times: the median is reported
        for _ in range(5):
            torch.cuda.synchronize()
            tp = time.perf_counter()
            ses.prefill(prompt)
            torch.cuda.synchronize()
            pre.append((time.perf_counter() - tp) * 1e3)
        b = ses.dec.bind({"P": P, "t": w.t_max - 1})
        S.sod2_binding_set_profiling(b, True)
        ses.decode(w.t_max - 1, b)
        torch.cuda.synchronize()
        per = {}
        for r in S.sod2_binding_launch_records(b):
            if r["group"] < 0:
                continue
            k = per.setdefault(r["kernel"], [0, 0.0, 0.0])
            k[0] += 1; k[1] += r["ms"]; k[2] += r["bytes"]
        rows.append(dict(P=P, prefill_ms=round(sorted(pre)[2], 3), decode_ms_per_token=round((t4 - t3) * 1e3 / w.t_max, 4),
                         decode_ms_per_token_step_by_step=round((t2 - t1) * 1e3 / w.t_max, 4),
                         arena_mb=round(ses.arena.numel() / 2 ** 20, 2),
                         last_step_kernels={k: dict(n=v[0], us=round(v[1] * 1e3, 1), gbs=round(v[2] / max(v[1], 1e-9) / 1e6, 1))
                                            for k, v in per.items()}))
        print(json.dumps(rows[-1]), file=sys.stderr, flush=True)
    # a decode step must stream every weight once (the embedding rows aside) and the keys / values cached so far
    d = w.decode
    emb = {d.tensor_id("tok_emb"), d.tensor_id("pos_emb")}
    hidden = d.tensors[d.tensor_id("tok_emb")].dims[1]
    wbytes = sum(x.numel() * x.element_size() for t, x in zip(d.weights(), ses.dec.weights) if t not in emb) + 2 * hidden * 2
    kv_row_bytes = sum(d.tensors[t].dims[1] * 2 for t in d.session_inputs())     # one cached row of every layer's K and V
    for r in rows:
        kv = kv_row_bytes * (r["P"] + w.t_max / 2)                         # mean over the generated tokens
        gbs = (wbytes + kv) / (r["decode_ms_per_token"] * 1e-3) / 1e9
        r["roofline"] = dict(bound="hbm", achieved=round(gbs, 1), peak=PEAK_HBM_GBS, unit="GB/s", frac=round(gbs / PEAK_HBM_GBS, 4),
                             algorithmic_bytes_per_token=int(wbytes + kv))
    out = {"metric": "decode latency per generated token", "unit": "ms",
           "value": round(sum(r["decode_ms_per_token"] for r in rows) / len(rows), 4), "n_gpus": 1,
           "roofline": dict(bound="hbm", unit="GB/s", peak=PEAK_HBM_GBS,
                            achieved=round(sum(r["roofline"]["achieved"] for r in rows) / len(rows), 1),
                            frac=round(sum(r["roofline"]["frac"] for r in rows) / len(rows), 4), traffic=None),
           "config": {"workload": "config 5: 24-layer decoder, hidden 1024, KV cache in the arena, greedy 256 tokens"},
           "dtype": "bf16", "data": "synthetic", "sequences": rows}
    print(json.dumps(out))


def bench_gemm_table(args, S, dev):
    """The four weight contractions of config 2's layer as graphs of their own (MatMul + bias through the same C ABI),
    at M = 1024, 2048, 4096: kernel version the shape rule picks, duration (HIP events on the launch stream, net of
    the event overhead measured in the same run) and TFLOP/s against the bf16 MFMA peak.  Not a bench line of the
    driver: the table behind profiles/config2_contraction_shapes.txt."""
    import numpy as np
    import torch
    from paper_2403_00176_amd.session import Session
    from workloads import GraphBuilder
    rows = []
    for name, N, K in (("QKV", 2304, 768), ("attention output", 768, 768), ("FFN1", 3072, 768), ("FFN2", 768, 3072)):
        gb = GraphBuilder([("M", 1, 8192)])
        x = gb.input("x", "bf16", ["M", K])
        wt = gb.weight("w", "bf16", [N, K])
        bias = gb.weight("b", "bf16", [N])
        gb.mark_output(gb.op("Add", [gb.op("MatMul", [x, wt], transB=1), bias]), "y")
        g = gb.build()
        ses = Session(g, device=dev)
        rs = np.random.RandomState(N + K)
        ses.upload_weights({wt: rs.randn(N, K) * 0.02, bias: rs.randn(N) * 0.02})
        for M in (1024, 2048, 4096):
            b = ses.bind({"M": M})
            ins = ses.upload_inputs({x: rs.randn(M, K)})
            outs = ses.alloc_outputs(ses.output_shapes(b))
            for _ in range(5):
                ses.run(b, ins, outs)
            torch.cuda.synchronize()
            S.sod2_binding_set_profiling(b, True)
            us, ovh, variant = [], [], None
            for _ in range(args.steps):
                ses.run(b, ins, outs)
                torch.cuda.synchronize()
                recs = S.sod2_binding_launch_records(b)
                # (the first two records are one and two empty launches between the same kind of event pair)
                ovh.append(max(2 * recs[0]["ms"] - recs[1]["ms"], 0.0) * 1e3 if len(recs) > 1 and recs[1]["group"] == -2 else 0.0)
                for r in recs:
                    if r["group"] >= 0 and r["kernel"] == "gemm":
                        us.append(r["ms"] * 1e3)
                        variant = r["variant"]
            raw = float(np.median(us))
            over = float(np.median(ovh))
            net = raw - over
            flops = 2.0 * M * N * K
            rows.append(dict(contraction=name, M=M, N=N, K=K, variant=variant, us_events=round(raw, 2), event_overhead_us=round(over, 2),
                             us_net=round(net, 2), tflops_events=round(flops / raw / 1e6, 1), tflops_net=round(flops / net / 1e6, 1),
                             frac_of_mfma_peak_net=round(flops / net / 1e6 / PEAK_BF16_TFLOPS, 4)))
            print(json.dumps(rows[-1]), file=sys.stderr, flush=True)
        del ses
    print(json.dumps({"metric": "contraction shapes of config 2", "unit": "TFLOP/s", "peak": PEAK_BF16_TFLOPS, "rows": rows}))


def measured_traffic(family, config=2):
    """HBM bytes per launch of a kernel family, from the committed rocprofv3 --pmc summaries of this same
    command (FETCH_SIZE and WRITE_SIZE, each scaled by a plain copy of known size): counters cannot be read
    from inside the process, so the number comes from profiles/ and is None when no summary is there."""
    total = 0.0
    if family == "conv":                  # the implicit-GEMM convolutions run the contraction kernels: the summaries list them there
        family = "gemm"
    for name in (f"config{config}_fetch_size.txt", f"config{config}_write_size.txt"):
        path = os.path.join(ROOT, "profiles", name)
        if not os.path.exists(path):
            return None
        val = None
        for line in open(path):
            if line.startswith(f"ALL {family} kernels"):
                parts = [p.strip() for p in line.split("|")]
                if len(parts) >= 4:
                    val = float(parts[3])
        if val is None:
            return None
        total += val
    return total


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--cpu-seconds", type=float, default=25.0, help="budget of the oracle timing leg (0 = skip)")
    ap.add_argument("--ablation", action="store_true",
                    help="optimisation breakdown: the same calls with fusion, execution planning, memory planning and "
                         "kernel versions switched on one after the other")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="the default line (config 2) also carries a short run of configs 1, 3, 4, 5, 6 and 7 (field "
                         "other_configs), each in a child process started before this one touches the GPU; this switches it off")
    ap.add_argument("--gemm-table", action="store_true",
                    help="the four weight contractions of config 2 at M = 1024, 2048, 4096, each a graph of its own")
    ap.add_argument("--calibration-copy-mb", type=int, default=0,
                    help="before the timed region, run a plain device copy of this many MiB three times: under "
                         "rocprofv3 --pmc it gives the scale of FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (each call is an independent request; "
              "more GPUs would each serve their own calls) -- use --gpus 1", file=sys.stderr)
        sys.exit(2)

    # the other configurations, briefly, each in a process of its own (run to the end before this process
    # initialises the GPU; a failure there is recorded, it does not stop the headline run)
    other = None
    if args.config == 2 and not (args.ablation or args.gemm_table or args.no_other_configs or args.calibration_copy_mb):
        import subprocess
        other = {}
        for c, extra in ((1, ["--steps", "16"]), (3, ["--steps", "16"]), (4, ["--steps", "16"]), (5, ["--steps", "2"]),
                         (6, ["--steps", "16"]), (7, ["--steps", "16"])):
            cmd = [sys.executable, os.path.abspath(__file__), "--config", str(c), "--warmup", "2", "--cpu-seconds", "0",
                   "--no-other-configs"] + extra
            try:
                r = subprocess.run(cmd, capture_output=True, text=True, timeout=240)
                d = json.loads(r.stdout.strip().splitlines()[-1])
                keep = {k: d[k] for k in ("metric", "value", "unit", "steps", "pipelined_ms_per_step", "roofline", "roofline_by_class")
                        if k in d}
                if "peak_arena_mb" in d:
                    keep["peak_arena_mb_mean"] = d["peak_arena_mb"]["mean"]
                if "sequences" in d:
                    keep["prefill_ms"] = [q["prefill_ms"] for q in d["sequences"]]
                keep["workload"] = d["config"]["workload"]
                other[f"config{c}"] = keep
            except Exception as e:                                   # noqa: BLE001 -- reported, not fatal
                other[f"config{c}"] = {"error": f"{type(e).__name__}: {e}"[:300]}

    import numpy as np
    import torch
    if not os.path.exists(os.path.join(ROOT, "paper_2403_00176_amd", "libsod2.so")):
        import __graft_entry__
        __graft_entry__.build()
    import paper_2403_00176_amd as S
    from paper_2403_00176_amd.session import Session
    from workloads import configs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    if args.ablation:
        return bench_ablation(args, S, dev)
    if args.gemm_table:
        return bench_gemm_table(args, S, dev)
    if args.config == 5:
        return bench_decoder(args, S, dev)
    n_calls = args.steps + args.warmup
    w = configs.BUILDERS[args.config](n_calls=max(n_calls, 64)) if args.config != 2 else configs.config2(max(n_calls, 64))
    t0 = time.perf_counter()
    ses = Session(w.graph, device=dev)
    compile_ms = (time.perf_counter() - t0) * 1e3       # graph build + RDP + plan, once
    W = w.make_weights()
    ses.upload_weights(W)
    weight_bytes = sum(x.numel() * x.element_size() for x in ses.weights)

    # all inputs and outputs resident in HBM before any timing; warm-up calls come first, the timed
    # calls are the first `steps` draws of the seeded list
    order = list(range(args.steps, args.steps + args.warmup)) + list(range(args.steps))
    calls = []
    max_arena = 0
    for ci in order:
        sym = w.calls[ci]
        b = ses.bind(sym)
        max_arena = max(max_arena, S.sod2_binding_arena_bytes(b)[0])
        ins = ses.upload_inputs(w.make_inputs(ci, sym))
        outs = ses.alloc_outputs(ses.output_shapes(b))
        calls.append((ci, sym, ins, outs))
    ses.ensure_arena(max_arena)
    torch.cuda.synchronize()
    stream = ses.stream

    enqueue_ms = []

    def one_call(sym, ins, outs, sync=True):
        b = ses.bind(sym)
        t_run = time.perf_counter()
        ses.run(b, ins, outs)
        enqueue_ms.append((time.perf_counter() - t_run) * 1e3)   # launch table + enqueue, host side
        if sync:
            stream.synchronize()
        return b

    if args.calibration_copy_mb:
        src = torch.ones(args.calibration_copy_mb << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    one_call(*calls[0][1:])
    first_call_ms = (time.perf_counter() - t0) * 1e3
    for c in calls[1:args.warmup]:
        one_call(*c[1:])
    timed = calls[args.warmup:]

    # ---- timed region: exactly `steps` calls, each synchronised (a latency, not a pipelined rate)
    torch.cuda.synchronize()
    lat, arena_mb, kept = [], [], []
    del enqueue_ms[:]
    t_begin = time.perf_counter()
    for ci, sym, ins, outs in timed:
        t1 = time.perf_counter()
        b = one_call(sym, ins, outs)
        lat.append((time.perf_counter() - t1) * 1e3)
        arena_mb.append(S.sod2_run_arena_bytes(b)[0] / 2 ** 20)       # the executed plan (== the bound one without control flow)
        kept.append(S.sod2_run_exec_values(b))
    torch.cuda.synchronize()
    total_s = time.perf_counter() - t_begin
    ms_per_step = total_s * 1e3 / len(timed)
    run_enqueue_ms = sum(enqueue_ms) / len(enqueue_ms)

    # ---- same calls without the per-call synchronise (host planning overlaps the GPU)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for ci, sym, ins, outs in timed:
        one_call(sym, ins, outs, sync=False)
    torch.cuda.synchronize()
    pipelined_ms = (time.perf_counter() - t1) * 1e3 / len(timed)

    # ---- host-only cost of bind
    t1 = time.perf_counter()
    for ci, sym, ins, outs in timed:
        ses.bind(sym)
    bind_ms = (time.perf_counter() - t1) * 1e3 / len(timed)

    # ---- per-kernel durations with HIP events on the launch stream, same calls
    # (every duration is event-to-event and is used as measured; the first two records of a run are one and two
    # empty launches timed the same way: 2 * t1 - t2 estimates what the pair of events adds to each duration,
    # reported as event_overhead_us and in the *_net_of_event_overhead figures, for information only)
    # sub-graph classes of the plan (all-constant shapes / symbolic-and-constant / execution-determined):
    # their share of the sub-graphs and of the kernel time, the two panels of the paper's Fig. 8
    sg_of_group, sg_count, sg_ms, seen_sg, versions = {}, {}, {}, set(), {}
    for gi in range(S.sod2_plan_counts(ses.plan)[0]):
        gr = S.sod2_plan_query_group(ses.plan, gi)
        sg_of_group[gr["gid"]] = gr["sg_class"]
        if gr["subgraph"] not in seen_sg:
            seen_sg.add(gr["subgraph"])
            sg_count[gr["sg_class"]] = sg_count.get(gr["sg_class"], 0) + 1
        if gr["kind"] == "ELTWISE":
            versions[gr["versions"]] = versions.get(gr["versions"], 0) + 1
    per = {}
    tokens = 0
    empty_ms = []
    t_roof_ms = 0.0          # per launch max(flops / MFMA peak, bytes / HBM peak), summed over the timed calls
    # which roofline binds a launch: the matrix cores when 2MNK / peak >= algorithmic bytes / HBM peak, else HBM
    # (a contraction against a [K, N] weight is weight-bandwidth bound below ~300 rows); per class the summed
    # algorithmic work over the summed event durations, against that class's own peak
    cls = {}
    big = sorted((c[1].get("B", 1) * c[1].get("L", c[1].get("H", 1)) for c in timed))[(3 * len(timed)) // 4]
    chains_big = {}          # memory-bound chains on the largest quarter of the calls (bandwidth-bound sizes)
    for ci, sym, ins, outs in timed:
        b = ses.bind(sym)
        S.sod2_binding_set_profiling(b, True)
        ses.run(b, ins, outs)
        stream.synchronize()
        n_tok = sym.get("B", 1) * sym.get("L", sym.get("H", 1))
        tokens += n_tok
        recs = S.sod2_binding_launch_records(b)
        base = max(2 * recs[0]["ms"] - recs[1]["ms"], 0.0) if len(recs) > 1 and recs[1]["group"] == -2 else 0.0
        empty_ms.append(base)
        for r in recs:
            if r["group"] < 0:
                continue
            c_ = sg_of_group.get(r["group"], "known")
            sg_ms[c_] = sg_ms.get(c_, 0.0) + r["ms"]
            k = per.setdefault(r["kernel"], dict(launches=0, ms=0.0, flops=0.0, bytes=0.0, raw_ms=0.0))
            k["launches"] += 1
            k["ms"] += r["ms"]
            k["raw_ms"] += max(r["ms"] - base, 1e-4)
            k["flops"] += r["flops"]
            k["bytes"] += r["bytes"]
            t_mfma, t_hbm = r["flops"] / (PEAK_BF16_TFLOPS * 1e12), r["bytes"] / (PEAK_HBM_GBS * 1e9)
            t_roof_ms += max(t_mfma, t_hbm) * 1e3
            fam = "contraction" if r["kernel"] in ("gemm", "conv") else r["kernel"]
            name = f"{fam}:{'mfma' if t_mfma >= t_hbm else 'hbm'}"
            q = cls.setdefault(name, dict(launches=0, ms=0.0, raw_ms=0.0, flops=0.0, bytes=0.0))
            q["launches"] += 1; q["ms"] += r["ms"]; q["raw_ms"] += max(r["ms"] - base, 1e-4)
            q["flops"] += r["flops"]; q["bytes"] += r["bytes"]
            if n_tok >= big and fam not in ("contraction", "attention"):
                q = chains_big.setdefault(fam, dict(launches=0, ms=0.0, raw_ms=0.0, bytes=0.0))
                q["launches"] += 1; q["ms"] += r["ms"]; q["raw_ms"] += max(r["ms"] - base, 1e-4); q["bytes"] += r["bytes"]
    kernels = {}
    for name, k in per.items():
        kernels[name] = dict(launches=k["launches"], total_ms=round(k["ms"], 3),
                             avg_us=round(1e3 * k["ms"] / k["launches"], 2),
                             avg_us_net_of_event_overhead=round(1e3 * k["raw_ms"] / k["launches"], 2),
                             tflops=round(k["flops"] / (k["ms"] * 1e-3) / 1e12, 2) if k["ms"] else 0.0,
                             gbs=round(k["bytes"] / (k["ms"] * 1e-3) / 1e9, 1) if k["ms"] else 0.0)
    roofline_by_class = {}
    for name, q in sorted(cls.items()):
        bound = name.split(":")[1]
        if bound == "mfma":
            a = q["flops"] / (q["ms"] * 1e-3) / 1e12
            a_net = q["flops"] / (q["raw_ms"] * 1e-3) / 1e12
            roofline_by_class[name] = dict(bound="mfma", launches=q["launches"], avg_us=round(1e3 * q["ms"] / q["launches"], 2),
                                           achieved=round(a, 1), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s", frac=round(a / PEAK_BF16_TFLOPS, 4),
                                           frac_net_of_event_overhead=round(a_net / PEAK_BF16_TFLOPS, 4))
        else:
            a = q["bytes"] / (q["ms"] * 1e-3) / 1e9
            a_net = q["bytes"] / (q["raw_ms"] * 1e-3) / 1e9
            roofline_by_class[name] = dict(bound="hbm", launches=q["launches"], avg_us=round(1e3 * q["ms"] / q["launches"], 2),
                                           achieved=round(a, 1), peak=PEAK_HBM_GBS, unit="GB/s", frac=round(a / PEAK_HBM_GBS, 4),
                                           frac_net_of_event_overhead=round(a_net / PEAK_HBM_GBS, 4))
    chains_on_largest_calls = {
        fam: dict(launches=q["launches"], avg_us=round(1e3 * q["ms"] / q["launches"], 2),
                  mb_per_launch=round(q["bytes"] / q["launches"] / 1e6, 3),
                  achieved_gbs=round(q["bytes"] / (q["ms"] * 1e-3) / 1e9, 1),
                  frac_of_hbm=round(q["bytes"] / (q["ms"] * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                  frac_of_hbm_net_of_event_overhead=round(q["bytes"] / (q["raw_ms"] * 1e-3) / 1e9 / PEAK_HBM_GBS, 4))
        for fam, q in sorted(chains_big.items())}
    n_sg, all_ms = max(sum(sg_count.values()), 1), max(sum(sg_ms.values()), 1e-9)
    subgraph_classes = {c: dict(subgraphs=sg_count.get(c, 0), share=round(sg_count.get(c, 0) / n_sg, 3),
                                kernel_time_share=round(sg_ms.get(c, 0.0) / all_ms, 3))
                        for c in ("known", "mixed", "nac")}
    dom = max(per, key=lambda n: per[n]["ms"])
    d = per[dom]
    traffic = measured_traffic(dom, args.config) if args.config in (2, 3) else None
    traffic_source = (f"profiles/config{args.config}_fetch_size.txt + profiles/config{args.config}_write_size.txt: rocprofv3 --pmc FETCH_SIZE / "
                      "WRITE_SIZE of this command, committed summaries (counters cannot be read inside the run); per launch of every "
                      "contraction kernel of the run") if traffic is not None else None
    if dom in ("gemm", "conv"):
        achieved = d["flops"] / (d["ms"] * 1e-3) / 1e12
        # bf16 contractions run on the matrix cores; an fp32 graph (config 1) runs plain FMA kernels on the vector ALUs
        peak, bound = (PEAK_BF16_TFLOPS, "mfma") if w.dtype == "bf16" else (PEAK_FP32_VECTOR_TFLOPS, "alu")
        roofline = dict(bound=bound, kernel=dom, achieved=round(achieved, 2), peak=peak, unit="TFLOP/s",
                        frac=round(achieved / peak, 4), traffic=traffic, traffic_source=traffic_source,
                        algorithmic_bytes_per_launch=d["bytes"] / d["launches"],
                        avg_launch_us=round(1e3 * d["ms"] / d["launches"], 2),
                        flops_per_launch=d["flops"] / d["launches"],
                        note="all contraction launches against the MFMA peak, the weight-bandwidth-bound ones included; "
                             "roofline_by_class separates them")
    else:
        achieved = d["bytes"] / (d["ms"] * 1e-3) / 1e9
        roofline = dict(bound="hbm", kernel=dom, achieved=round(achieved, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                        frac=round(achieved / PEAK_HBM_GBS, 4), traffic=traffic, traffic_source=traffic_source,
                        avg_launch_us=round(1e3 * d["ms"] / d["launches"], 2),
                        bytes_per_launch=d["bytes"] / d["launches"])

    # ---- CPU baseline: the oracle as it stands, on a bounded sample of the same calls
    cpu = None
    if args.cpu_seconds > 0:
        from oracle import rdp as R, plan as P, execute
        try:
            from threadpoolctl import threadpool_info
            cores = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        ro = R.RDP(w.graph).analyse()
        po = P.build_plan(w.graph, ro)
        # a stratified sample of the timed calls: median size first, then the quartiles, the octiles, ... until the
        # time budget is used up (the largest calls alone would take minutes), so the sample keeps the size mix
        by_size = sorted(timed, key=lambda c: c[1].get("B", 1) * c[1].get("L", c[1].get("H", 1)))
        order_, seen_, frac_ = [], set(), [0.5, 0.25, 0.75, 0.125, 0.375, 0.625, 0.875] + [(2 * i + 1) / 32 for i in range(16)]
        for f in frac_:
            i = min(int(f * len(by_size)), len(by_size) - 1)
            if i not in seen_:
                seen_.add(i); order_.append(by_size[i])
        spent, times, gpu_same, desc, toks = 0.0, [], [], [], 0
        for ci, sym, ins, outs in order_:
            if spent >= args.cpu_seconds:
                break
            host_in = w.make_inputs(ci, sym)
            t1 = time.perf_counter()
            execute.run(w.graph, po.order, W, host_in)
            dt = time.perf_counter() - t1
            spent += dt
            times.append(dt * 1e3)
            gpu_same.append(lat[[c[0] for c in timed].index(ci)])
            desc.append("x".join(str(v) for v in sym.values()))
            toks += sym.get("B", 1) * sym.get("L", sym.get("H", 1))
        cpu = dict(value=round(sum(times) / len(times), 2), unit="ms", cores=int(cores), kind="oracle",
                   sample=f"{len(times)} of the {len(timed)} timed calls, drawn at the median, quartiles, octiles, ... of the call "
                          f"sizes until {args.cpu_seconds:.0f} s of CPU time were used (symbol values {', '.join(desc)}; "
                          f"{toks} tokens / pixels rows against {tokens} in all timed calls); float64 numpy, unfused",
                   gpu_ms_same_calls=round(sum(gpu_same) / len(gpu_same), 3))

    out = {
        "metric": "dynamic-shape inference latency",
        "value": round(ms_per_step, 4),
        "unit": "ms",
        "n_gpus": 1,
        "steps": len(timed),
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else w.dtype,
        "data": "synthetic",
        "config": {"workload": f"config {args.config}: " + {
            1: "one pre-LN encoder block fp32, hidden 256, L in [16,128]",
            2: "12-layer pre-LN encoder, hidden 768, 12 heads, FFN 3072 GELU, bf16 storage / fp32 accumulate, "
               "B in [1,8] and L in [32,512] redrawn per call",
            3: "ResNet-50 layout NHWC bf16, batch 1, H=W in {224..640 step 32}",
            4: "config 2 with per-layer skip gates, batch 4, L in [128,384]",
            7: "ResNet-50 backbone + detection-style neck (Resize to a computed shape, Concat, 3x3 convs), bf16 NHWC, "
               "batch 1, H=W in {224..640 step 32}",
            6: "config 2's encoder with a skip gate per layer and sequence: kept sequences compacted by "
               "NonZero + Gather (execution-determined batch), ScatterRows back; B in [2,8], L in [128,384]"}[args.config],
            "calls": len(timed), "tokens": tokens},
        "latency_ms": {"mean": round(sum(lat) / len(lat), 4), "min": round(min(lat), 4), "max": round(max(lat), 4)},
        "pipelined_ms_per_step": round(pipelined_ms, 4),
        "bind_ms": round(bind_ms, 4),
        "run_enqueue_ms": round(run_enqueue_ms, 4),
        "first_call_ms": round(first_call_ms, 3),
        "compile_once_ms": round(compile_ms, 2),
        "peak_arena_mb": {"min": round(min(arena_mb), 3), "max": round(max(arena_mb), 3),
                          "mean": round(sum(arena_mb) / len(arena_mb), 3)},
        # device memory the session holds beyond weights, inputs and outputs: the largest planned arena plus the
        # optional split-K workspace behind it (not part of the plan, not in peak_arena_mb)
        "workspace_mb": round(ses.workspace_bytes / 2 ** 20, 3),
        "arena_allocation_mb": round(ses.arena.numel() / 2 ** 20, 3),
        "weight_mb": round(weight_bytes / 2 ** 20, 1),
        **({"kept_fraction": round(sum(sum(k) for k in kept) / max(sum(len(k) * c[1]["B"] for k, c in zip(kept, timed)), 1), 3)}
           if any(kept) else {}),
        "tokens_per_s": round(tokens / total_s, 1),
        "roofline": roofline,
        "roofline_by_class": roofline_by_class,
        "chains_on_largest_calls": chains_on_largest_calls,
        # whole call against the roofline: what the launches of a call would take at the peak that binds each
        # of them, over the measured latency of the call (launch gaps, planning and the synchronise included)
        "call_roofline": {"t_roof_ms_per_call": round(t_roof_ms / len(timed), 4),
                          "frac_of_latency": round(t_roof_ms / len(timed) / (sum(lat) / len(lat)), 4)},
        "kernels": kernels,
        "subgraph_classes": subgraph_classes,
        # fused elementwise groups by the number of code versions they need (Fig. 8's 1 / 2-4 / 5-8 buckets)
        "eltwise_group_versions": {"1": versions.get(1, 0), "2-4": sum(v for k, v in versions.items() if 2 <= k <= 4),
                                   "5-8": sum(v for k, v in versions.items() if 5 <= k <= 8)},
        "event_overhead_us": round(1e3 * sum(empty_ms) / max(len(empty_ms), 1), 2),
        "cpu_baseline": cpu,
        **({"other_configs": other} if other is not None else {}),
        "paper_context": "SoD2 reports up to 3.9x speed-up (vs ONNX Runtime, Adreno 660 GPU, fp16) and up to 88% less "
                         "peak memory (Snapdragon 888 CPU); other hardware, not comparable",
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
