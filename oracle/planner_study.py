"""Planner quality study (Section 4.4.1, last paragraph: the paper scores its peak-first planner at 1.05x of the
optimum and the greedy "smallest free slot" comparison at 1.16x).  For the synthetic configurations, per call: the
arena the peak-first placement needs, what best fit in execution order needs, and the optimum -- the peak of live
bytes when a placement reaches that lower bound, else the result of a branch and bound over all arena tensors of
the call (node-limited: "proven" says whether it finished).  And the same on random lifetime sets of 12-20 tensors,
the sizes an exhaustive search cannot reach.

Test infrastructure (it calls only the oracle and the seeded workloads): run as
    python -m oracle.planner_study > profiles/planner_quality_configs.txt
"""
from __future__ import annotations

import random
import sys

from . import arena as A, plan as P, rdp as R
from workloads import configs


def study(name, workload, calls, exec_values=None, out=sys.stdout, node_limit=400_000):
    g = workload.graph
    po_peak = P.build_plan(g, R.RDP(g).analyse())
    po_best = P.build_plan(g, R.RDP(g).analyse(), P.Opts(dmp=False))
    n_sw = sum(1 for op in g.ops if op.kind == "Switch")
    rnd = random.Random(17)
    tot = dict(peak=0, best=0, opt=0, proven=0, at_bound=0, n=[])
    for sym in calls:
        dec = [rnd.random() < 0.5 for _ in range(n_sw)]
        ev = exec_values(sym) if exec_values else ()
        bp, bb = A.bind(po_peak, sym, dec, ev), A.bind(po_best, sym, dec, ev)
        peak, best = bp.arena_bytes - bp.session_bytes, bb.arena_bytes - bb.session_bytes
        lower = bp.peak_live - bp.session_bytes
        if min(peak, best) == lower:
            opt, proven = lower, True
            tot["at_bound"] += 1
        else:
            ts = [A.ArenaTensor(a.tid, a.bytes, a.start, a.end) for a in bp.tensors.values()]
            opt, proven = A.optimal_arena_bytes_bnb(ts, node_limit=node_limit, incumbent=min(peak, best))
        tot["peak"] += peak; tot["best"] += best; tot["opt"] += opt; tot["proven"] += proven
        tot["n"].append(len(bp.tensors))
    n = tot["n"]
    print(f"{name}: {len(calls)} calls of {min(n)}-{max(n)} arena tensors | peak-first / optimum = {tot['peak'] / tot['opt']:.4f}, "
          f"best fit / optimum = {tot['best'] / tot['opt']:.4f} | optimum proven for {tot['proven']} calls "
          f"({tot['at_bound']} by a placement that equals the peak of live bytes)", file=out)
    return tot


def main(out=sys.stdout):
    print("# planner quality on the synthetic configurations (python -m oracle.planner_study); the paper reports 1.05x of the",
          file=out)
    print("# optimum for its planner and 1.16x for the greedy comparison (Section 4.4.1) on its own models", file=out)
    w2 = configs.config2(16)
    study("config 2 (12-layer encoder)", w2, w2.calls[:8], out=out)
    w3 = configs.config3(8)
    study("config 3 (ResNet-50 layout)", w3, w3.calls[:6], out=out)
    w4 = configs.config4(8)
    study("config 4 (layer skipping, random decisions)", w4, w4.calls[:6], out=out)
    w6 = configs.config6(8, layers=4)
    study("config 6 (per-sequence gates, counts known)", w6, w6.calls[:4],
          exec_values=lambda sym: [max(sym["B"] // 2, 1)] * 4, out=out)
    w7 = configs.config7(6)
    study("config 7 (detection neck)", w7, w7.calls[:4], out=out)
    # random lifetime sets of the sizes the exhaustive search cannot reach
    rnd = random.Random(23)
    r_peak = r_best = r_opt = 0
    proven = 0
    for trial in range(40):
        n = rnd.randint(12, 20)
        ts = []
        for i in range(n):
            s = rnd.randint(0, 14)
            ts.append(A.ArenaTensor(i, 256 * rnd.randint(1, 16), s, s + rnd.randint(0, 5)))
        live = [sum(t.bytes for t in ts if t.start <= k <= t.end) for k in range(22)]
        mine = [A.ArenaTensor(t.tid, t.bytes, t.start, t.end) for t in ts]
        placed = []
        A.place_region(mine, list(range(22)), live, placed)
        peak = max(c.offset + c.bytes for c in placed)
        placed = []
        for c in sorted((A.ArenaTensor(t.tid, t.bytes, t.start, t.end) for t in ts), key=lambda a: (a.start, a.tid)):
            c.offset = A.best_fit(c, placed)
            placed.append(c)
        best = max(c.offset + c.bytes for c in placed)
        # the search starts from the better of the two (a node-limited search that ends unproven then never
        # reports more than a placement already in hand)
        opt, ok = A.optimal_arena_bytes_bnb(ts, incumbent=min(peak, best))
        proven += ok
        r_peak += peak
        r_best += best
        r_opt += opt
    print(f"random lifetimes, 40 sets of 12-20 tensors (optimum proven for {proven}): peak-first / optimum = {r_peak / r_opt:.4f}, "
          f"best fit / optimum = {r_best / r_opt:.4f}", file=out)


if __name__ == "__main__":
    main()
