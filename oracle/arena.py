"""Run-time half of the plan: concrete sizes, lifetimes and arena offsets once
the symbols (and, with control flow, the Switch decisions) are known
(Section 4.4.1).

Reading of the two-sentence description in the paper.  Executed sub-graphs are
taken in execution order; consecutive ones with resolved sizes and no control
operator are planned together as one region (a stack of blocks has a peak in
every block, and a tensor that lives from one block into the next must not be
placed before the next peak is known).  Within a region:
  1. live bytes per step; the steps are visited from the one with the most live
     bytes down (earlier step first on ties): the peak first, as in the paper,
     then the next highest step, and so on;
  2. at each visited step the tensors live there that have no offset yet, by
     (start step, id),
  are placed one by one at the lowest offset where they overlap no tensor
  already placed (in this or an earlier region) whose lifetime intersects.
Sizes are element count x element size rounded up to 256 bytes.  Control flow
follows dead-token propagation: the Switch output that is not taken is dead,
an operator with a dead input does not run, Combine forwards its live input.

Session tensors (a KV cache: tensors that persist across calls) take a region of
their own at the bottom of the arena: one slot per session input, in tensor-id
order, sized for its declared capacity at the bound symbols; every other offset
starts above that region.  CacheAppend writes into the slot of its first input.

Execution-determined extents (Section 4.3): ``exec_values`` holds the counts of
the NonZero operators that have executed so far, in execution order.  A NonZero
that has not run yet is planned at its upper bound (the element count of its
input); binding again with the count known gives the plan for what follows
(offsets of what has already run do not change: a cut follows every NonZero and
sub-graphs are placed in execution order).  The greedy placement is not
monotone in the sizes, so the exact plan can need more bytes than the
upper-bound one; whoever runs the plan must check before going on.  The
result of a NonZero is allocated before its extent is known: its storage is
always rank x upper bound indices plus one 8-byte slot that receives the count.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from itertools import permutations
from typing import Dict, List, Sequence, Tuple

from . import rdp as R
from .expr import Expr
from .plan import Plan, DT_BYTES, align_up, arena_candidate, COUNTING_GROUPS


class SymbolOutOfRange(Exception):
    pass


class UnresolvedShape(Exception):
    pass


class CapacityExceeded(Exception):
    pass


@dataclass
class ArenaTensor:
    tid: int
    bytes: int
    start: int
    end: int
    offset: int = -1


@dataclass
class Binding:
    plan: Plan
    env: Dict[str, int]
    steps: List[int] = field(default_factory=list)            # executed item indices
    step_sg: List[int] = field(default_factory=list)          # sub-graph of each step
    decisions: Dict[int, bool] = field(default_factory=dict)  # Switch op id -> skip?
    tensors: Dict[int, ArenaTensor] = field(default_factory=dict)
    dims: Dict[int, List[int]] = field(default_factory=dict)
    arena_bytes: int = 0
    peak_live: int = 0
    dead_ops: set = field(default_factory=set)
    dyn_base: Dict[int, int] = field(default_factory=dict)
    session: Dict[int, Tuple[int, int]] = field(default_factory=dict)   # session input -> (offset, bytes)
    session_root: Dict[int, int] = field(default_factory=dict)          # session tensor -> its session input
    session_bytes: int = 0
    exec: List[Tuple[int, int, bool]] = field(default_factory=list)     # executed NonZero: (op id, extent used, known?)
    versions: Dict[int, str] = field(default_factory=dict)   # multi-version group -> the version the bound symbols select


def concrete_dims(plan: Plan, t: int, env) -> List[int]:
    s = plan.rdp.S[t]
    if not isinstance(s, list) or any(not R.is_expr(d) for d in s):
        raise UnresolvedShape(f"tensor {t} ({plan.graph.tensors[t].name})")
    return [d.eval(env) for d in s]


def select_version(plan: Plan, gr, env) -> str:
    """Section 4.2: of the code versions of a fused group with unproven broadcast pairs, the one that holds for the
    bound symbols.  One letter per unproven pair, in the plan's order: 'e' the two extents are equal, 'a' the first
    operand's is 1 (it is broadcast), 'b' the second's.  (Anything else does not broadcast: evaluating the result's
    extent has already failed.)"""
    out = []
    for a, b, k in gr.unproven:
        da, db = concrete_dims(plan, a, env), concrete_dims(plan, b, env)
        x = da[-k] if k <= len(da) else 1
        y = db[-k] if k <= len(db) else 1
        out.append("e" if x == y else ("a" if x == 1 else "b"))
    return "".join(out)


def intersects(a: ArenaTensor, b: ArenaTensor) -> bool:
    return a.start <= b.end and b.start <= a.end


def first_fit(t: ArenaTensor, placed: Sequence[ArenaTensor]) -> int:
    busy = sorted((p.offset, p.offset + p.bytes) for p in placed if intersects(t, p))
    off = 0
    for lo, hi in busy:
        if off + t.bytes <= lo:
            break
        off = max(off, hi)
    return off


def last_fit(t: ArenaTensor, placed: Sequence[ArenaTensor], ceiling: int) -> int:
    """The highest offset that fits below ``ceiling``; the lowest offset that fits when there is none."""
    busy = sorted(((p.offset, p.offset + p.bytes) for p in placed if intersects(t, p)), key=lambda r: (-r[1], -r[0]))
    end = ceiling
    for lo, hi in busy:
        if end - t.bytes >= hi:
            break
        end = min(end, lo)
    return end - t.bytes if end - t.bytes >= 0 else first_fit(t, placed)


def bind(plan: Plan, sym: Dict[str, int], decisions: Sequence[bool] = (),
         exec_values: Sequence[int] = ()) -> Binding:
    g = plan.graph
    for name, lo, hi in g.symbols:
        if name not in sym or not (lo <= sym[name] <= hi):
            raise SymbolOutOfRange(name)
    env = {name: int(sym[name]) for name, _, _ in g.symbols}
    b = Binding(plan, env)
    prod = plan.rdp.producer
    cap_elems = {}
    for t, d in enumerate(g.tensors):
        if d.role == "input" and d.session:
            n = 1
            for c in d.capacity:
                n *= Expr.parse(c).eval(env)
            cap_elems[t] = n
            nbytes = align_up(n * DT_BYTES[d.dtype])
            b.session[t] = (b.session_bytes, nbytes)
            b.session_root[t] = t
            b.session_bytes += nbytes
    group_dead: Dict[int, bool] = {}
    memo: Dict[int, Tuple[bool, int]] = {}
    dec = list(decisions)
    counts = list(exec_values)

    def info(t: int) -> Tuple[bool, int]:
        """(dead?, tensor whose storage t occupies)."""
        if t in memo:
            return memo[t]
        p = prod[t]
        if p < 0 or plan.folded[p]:
            r = (False, t)
        else:
            op = g.ops[p]
            if op.kind == "Switch":
                d, base = info(op.inputs[0])
                skip = b.decisions.get(p)
                taken = (op.outputs.index(t) == 1) == bool(skip)
                r = (d or skip is None or not taken, base)
            elif op.kind == "Combine":
                r = (True, t)
                for i in op.inputs:
                    d, base = info(i)
                    if not d:
                        r = (False, base)
                        break
            elif plan.view[p]:
                r = info(op.inputs[0])
            elif t in plan.inplace:                    # the result took over an operand's storage
                r = (group_dead[plan.group_of_op[p]], info(plan.inplace[t])[1])
            else:
                r = (group_dead[plan.group_of_op[p]], t)
        memo[t] = r
        return r

    reads_at: Dict[int, int] = {}          # base tensor -> last step reading it
    for s, sg in enumerate(plan.subgraphs):
        for i in sg:
            it = plan.items[i]
            step = len(b.steps)
            if it.is_group:
                gr = plan.groups[it.ref]
                inside = {o for n in gr.ops for o in g.ops[n].outputs}
                ext = [t for n in gr.ops for t in g.ops[n].inputs
                       if t not in inside and plan.sbase[t] not in inside]     # a view of a member's result is internal
                dead = any(info(t)[0] for t in ext)
                group_dead[gr.gid] = dead
                if dead:
                    b.dead_ops.update(gr.ops)
                    continue
                for t in ext:
                    reads_at[info(t)[1]] = step
                t = gr.out
                nz_bytes = None
                if gr.kind in COUNTING_GROUPS:
                    n_op = gr.ops[0]
                    src = concrete_dims(plan, g.ops[n_op].inputs[0], env)
                    ub = 1
                    for d in src:
                        ub *= d
                    known = bool(counts)
                    v = int(counts.pop(0)) if known else ub
                    if not 0 <= v <= ub:
                        raise ValueError("a NonZero count outside [0, element count of its input]")
                    env[R.exec_symbol(n_op)] = v
                    b.exec.append((n_op, v, known))
                    nz_bytes = align_up((len(src) * ub + 1) * DT_BYTES[g.tensors[t].dtype])
                b.dims[t] = concrete_dims(plan, t, env)
                if gr.versions > 1:
                    b.versions[gr.gid] = select_version(plan, gr, env)
                for n_op in gr.ops:                       # a CACHEAPPEND group, or appends inside an attention group
                    if g.ops[n_op].kind != "CacheAppend":
                        continue
                    tc = g.ops[n_op].outputs[0]
                    src = g.ops[n_op].inputs[0]
                    if src not in b.session_root:
                        raise ValueError("CacheAppend must extend a session tensor")
                    b.dims[tc] = concrete_dims(plan, tc, env)
                    b.session_root[tc] = b.session_root[src]
                    n = 1
                    for d in b.dims[tc]:
                        n *= d
                    if n > cap_elems[b.session_root[tc]]:
                        raise CapacityExceeded(g.tensors[tc].name)
                if arena_candidate(plan, t) and t not in plan.inplace:
                    n = DT_BYTES[g.tensors[t].dtype]
                    for d in b.dims[t]:
                        n *= d
                    b.tensors[t] = ArenaTensor(t, nz_bytes if nz_bytes is not None else align_up(n), step, step)
                for t in gr.also:                         # the operator's further results
                    b.dims[t] = concrete_dims(plan, t, env)
                    if arena_candidate(plan, t):
                        n = DT_BYTES[g.tensors[t].dtype]
                        for d in b.dims[t]:
                            n *= d
                        if t in plan.fold_y:              # R9: rows plus their partial sums (8 bytes per 32 columns)
                            n = n * 9 // 8
                        b.tensors[t] = ArenaTensor(t, align_up(n), step, step)
            else:
                op = g.ops[it.ref]
                if op.kind == "Switch":
                    if info(op.inputs[0])[0]:
                        b.dead_ops.add(it.ref)
                        continue
                    if not dec:
                        raise ValueError("a Switch decision is missing")
                    b.decisions[it.ref] = bool(dec.pop(0))
                    for t in op.inputs:
                        reads_at[info(t)[1]] = step
                else:
                    live = [t for t in op.inputs if not info(t)[0]]
                    if not live:
                        b.dead_ops.add(it.ref)
                        continue
                    reads_at[info(live[0])[1]] = step
            b.steps.append(i)
            b.step_sg.append(s)
    for t, at in b.tensors.items():
        at.end = max(at.start, reads_at.get(t, at.start))
    for t in range(len(g.tensors)):
        if prod[t] >= 0 and not plan.folded[prod[t]] and prod[t] not in b.dead_ops:
            d, base = info(t)
            if not d:
                b.dyn_base[t] = base

    nsteps = len(b.steps)
    live_bytes = [0] * nsteps
    for at in b.tensors.values():
        for k in range(at.start, at.end + 1):
            live_bytes[k] += at.bytes
    b.peak_live = max(live_bytes, default=0) + b.session_bytes

    placed: List[ArenaTensor] = []
    if plan.opts.dmp:
        for ks in planning_regions(plan, b):
            place_region([at for at in b.tensors.values() if ks[0] <= at.start <= ks[-1]], ks, live_bytes, placed)
    else:
        for a in sorted(b.tensors.values(), key=lambda a: (a.start, a.tid)):
            a.offset = best_fit(a, placed)
            placed.append(a)
    for a in placed:
        a.offset += b.session_bytes
    b.arena_bytes = max((a.offset + a.bytes for a in placed), default=b.session_bytes)
    return b


def place_region(mine: Sequence[ArenaTensor], ks: Sequence[int], live_bytes: Sequence[int], placed: List[ArenaTensor]):
    """Peak-first placement of the tensors that start in the steps ``ks``: the steps are visited from the
    one with the most live bytes down (earlier first on ties); at each, the tensors live there that have
    no offset yet are placed one by one.  The region cannot end below ``ceiling``, the larger of its own
    peak of live bytes and what is already placed.  Four variants of the pass are tried in a fixed order
    and the first one that ends lowest is kept (the search stops at the first that ends at the ceiling):
    tensors of a step by (start, id) or by (size descending, start, id), each at the lowest offset that
    fits or at the highest offset below the ceiling that fits."""
    mine = list(mine)
    if not mine:
        return
    ceiling = max(max(live_bytes[k] for k in ks), max((p.offset + p.bytes for p in placed), default=0))
    by_need = sorted(ks, key=lambda k: (-live_bytes[k], k))
    best = None
    for by_size, high in ((False, False), (True, False), (False, True), (True, True)):
        for a in mine:
            a.offset = -1
        cur = list(placed)
        key = (lambda a: (-a.bytes, a.start, a.tid)) if by_size else (lambda a: (a.start, a.tid))
        for p in by_need:
            for a in sorted((a for a in mine if a.offset < 0 and a.start <= p <= a.end), key=key):
                a.offset = last_fit(a, cur, ceiling) if high else first_fit(a, cur)
                cur.append(a)
        top = max(a.offset + a.bytes for a in mine)
        if best is None or top < best[0]:
            best = (top, [a.offset for a in mine])
        if best[0] <= ceiling:
            break
    for a, o in zip(mine, best[1]):
        a.offset = o
    placed.extend(mine)


def planning_regions(plan: Plan, b: Binding) -> List[List[int]]:
    """Executed steps grouped into the stretches that are planned together: consecutive sub-graphs with
    known sizes and no control operator form one region.  A sub-graph holding a Switch, a Combine or a
    NonZero is a region of its own (what follows it is planned when it has executed, and nothing placed
    before may depend on it); so is a sub-graph with execution-determined sizes as long as a NonZero
    that ran before it still has no known count (it is then planned at the upper bound and planned
    again, together with its neighbours, once the count is there: Section 4.3)."""
    known = sum(1 for _, _, k in b.exec if k)
    seen = 0                                   # NonZero groups executed before the current step
    alone = []
    for k in range(len(b.steps)):
        it = plan.items[b.steps[k]]
        nz = it.is_group and plan.groups[it.ref].kind in COUNTING_GROUPS
        alone.append((not it.is_group) or nz or (plan.sg_class[b.step_sg[k]] == "nac" and seen > known))
        seen += nz
    regions: List[List[int]] = []
    for k in range(len(b.steps)):
        new_sg = k == 0 or b.step_sg[k] != b.step_sg[k - 1]
        if not regions or (new_sg and (alone[k] or alone[k - 1])):
            regions.append([])
        regions[-1].append(k)
    return regions


def best_fit(t: ArenaTensor, placed: Sequence[ArenaTensor]) -> int:
    """The comparison strategy named in Section 4.4.1: the smallest free slot that holds the tensor."""
    busy = sorted((p.offset, p.offset + p.bytes) for p in placed if intersects(t, p))
    top = max((p.offset + p.bytes for p in placed), default=0)
    gaps, cur = [], 0
    for lo, hi in busy:
        if lo > cur:
            gaps.append((lo - cur, cur))
        cur = max(cur, hi)
    if top > cur:
        gaps.append((top - cur, cur))
    fits = sorted(gp for gp in gaps if gp[0] >= t.bytes)
    return fits[0][1] if fits else cur


def optimal_arena_bytes(tensors: Sequence[ArenaTensor]) -> int:
    """Exhaustive optimum (used in Section 4.4.1 to score the planner): the best placement is
    reached by first-fit in *some* order (sort an optimal layout by offset), so try every order."""
    assert len(tensors) <= 9
    best = None
    for perm in permutations(tensors):
        placed = []
        for a in perm:
            c = ArenaTensor(a.tid, a.bytes, a.start, a.end)
            c.offset = first_fit(c, placed)
            placed.append(c)
        top = max((c.offset + c.bytes for c in placed), default=0)
        best = top if best is None else min(best, top)
    return best or 0


def optimal_arena_bytes_bnb(tensors: Sequence[ArenaTensor], node_limit: int = 3_000_000, incumbent: int = None):
    """Optimum of the offset assignment (dynamic storage allocation) by branch and bound, for the mid-size lifetime
    sets the exhaustive search cannot reach.  As in ``optimal_arena_bytes`` the optimum is reached by first fit in
    *some* order (sort an optimal layout by offset: by induction first fit puts every tensor at or below its offset
    there), so the search runs over orders, extending a partial order by one tensor at its first-fit offset.  Cuts: a
    tensor that would end at or above the best layout found; a partial layout already seen with the same set of
    placed tensors and offsets no better (memo on the frozen layout).  It stops as soon as a layout reaches the lower
    bound (the largest sum of bytes alive at one step).  Returns (bytes, proven): proven is False when the node limit
    ended the search; the value is then the best layout found, an upper bound of the optimum.  ``incumbent``: the
    bytes of a layout already known (a planner's), used as the first bound."""
    ts = sorted(tensors, key=lambda a: (-a.bytes * (a.end - a.start + 1), a.tid))
    n = len(ts)
    if n == 0:
        return 0, True
    steps = sorted({k for a in ts for k in range(a.start, a.end + 1)})
    lower = max(sum(a.bytes for a in ts if a.start <= k <= a.end) for k in steps)
    conflicts = [[j for j in range(n) if j != i and intersects(ts[i], ts[j])] for i in range(n)]
    off = [-1] * n

    def fit(i: int) -> int:
        busy = sorted((off[j], off[j] + ts[j].bytes) for j in conflicts[i] if off[j] >= 0)
        o = 0
        for lo, hi in busy:
            if o + ts[i].bytes <= lo:
                break
            o = max(o, hi)
        return o

    best = 0
    for i in range(n):                         # a first incumbent: first fit, largest first
        off[i] = fit(i)
        best = max(best, off[i] + ts[i].bytes)
    off = [-1] * n
    if incumbent is not None:
        best = min(best, incumbent)
    state = {"best": best, "nodes": 0, "stop": best == lower, "out_of_nodes": False}
    seen = set()

    def rec(placed: int, top: int):
        if state["stop"]:
            return
        if placed == n:
            if top < state["best"]:
                state["best"] = top
                state["stop"] = top == lower
            return
        state["nodes"] += 1
        if state["nodes"] > node_limit:
            state["stop"] = state["out_of_nodes"] = True
            return
        key = tuple(off)
        if key in seen:
            return
        seen.add(key)
        # every tensor still to come must fit below the incumbent wherever it lands: cheap look-ahead
        cand = []
        for i in range(n):
            if off[i] >= 0:
                continue
            o = fit(i)
            if o + ts[i].bytes >= state["best"]:
                return                          # it only moves up as more tensors are placed
            cand.append((o, i))
        for o, i in sorted(cand):
            off[i] = o
            rec(placed + 1, max(top, o + ts[i].bytes))
            off[i] = -1
            if state["stop"]:
                return

    rec(0, 0)
    return state["best"], not state["out_of_nodes"]


def check_no_overlap(b: Binding):
    ts = list(b.tensors.values())
    slots = sorted(b.session.values())
    for (o1, n1), (o2, n2) in zip(slots, slots[1:]):
        assert o1 + n1 <= o2
    assert not slots or slots[-1][0] + slots[-1][1] == b.session_bytes
    for i, x in enumerate(ts):
        assert x.offset >= b.session_bytes and x.offset % 256 == 0
        for y in ts[i + 1:]:
            if intersects(x, y):
                assert x.offset + x.bytes <= y.offset or y.offset + y.bytes <= x.offset, (x, y)


def dump(b: Binding) -> str:
    plan = b.plan
    lines = ["sym " + " ".join(f"{name}={b.env[name]}" for name, _, _ in plan.graph.symbols)]
    for n_op, v, known in b.exec:
        lines.append(f"exec {R.exec_symbol(n_op)}={v} {'known' if known else 'bound'}")
    for t in sorted(b.session):
        lines.append(f"session t{t} off={b.session[t][0]} bytes={b.session[t][1]}")
    for k, i in enumerate(b.steps):
        it = plan.items[i]
        lines.append(f"step {k} {'g' if it.is_group else 'c'}{it.ref}")
    for gid in sorted(b.versions):
        lines.append(f"version g{gid} {b.versions[gid]} of {plan.groups[gid].versions}")
    for t in sorted(b.dims):
        dims = " ".join(map(str, b.dims[t]))
        if t in b.tensors:
            a = b.tensors[t]
            lines.append(f"t{t} dims=[{dims}] off={a.offset} bytes={a.bytes} life={a.start}..{a.end}")
        elif t in b.session_root:
            lines.append(f"t{t} dims=[{dims}] session=t{b.session_root[t]}")
        elif t in plan.inplace:
            lines.append(f"t{t} dims=[{dims}] inplace=t{b.dyn_base[t]}")
        else:
            lines.append(f"t{t} dims=[{dims}] external")
    lines.append(f"arena_bytes={b.arena_bytes}")
    lines.append(f"peak_live={b.peak_live}")
    return "\n".join(lines) + "\n"
