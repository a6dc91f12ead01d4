// Run-time half of the plan (Section 4.4.1): evaluate the symbols, derive the executed steps,
// tensor lifetimes and arena offsets.
//
// Executed sub-graphs in execution order; consecutive ones with resolved sizes and no control operator
// are planned together as one region (a tensor that lives from one block into the next must not be
// placed before the next block's peak is known).  Within a region the steps are visited from the one
// with the most live bytes down (earlier first on ties): the peak first, then the next highest step,
// ...; at each the tensors live there that have no offset yet, by (start, id), are placed at the lowest
// offset that overlaps no already placed tensor with an intersecting lifetime.  Sizes are rounded up
// to 256 bytes.  Control flow uses dead tokens: the Switch output not taken is dead, an
// item with a dead input does not run, Combine forwards its live input.
//
// Session tensors (a KV cache) persist across calls: one slot per session input at the bottom of
// the arena, in tensor-id order, sized for the declared capacity at the bound symbols; every other
// offset starts above that region.  CacheAppend writes into the slot of its first input.
//
// Execution-determined extents (Section 4.3): a NonZero (or NMS) whose count is not known yet is planned at
// its upper bound (the element count of its first input); binding again with the count gives the plan for
// what follows, and nothing that already ran moves (a cut follows every NonZero, sub-graphs are
// placed in execution order).  Its result is allocated before the extent is known: always rank x
// upper bound indices plus one 8-byte slot for the count.  First fit is not monotone in the sizes:
// the exact plan may need more bytes than the upper-bound plan, the caller must check.
#include <algorithm>
#include <functional>

#include "internal.hpp"

namespace sod2 {

static const int64_t kMaxTensorBytes = (int64_t)1 << 44;   // far beyond any device memory; keeps the byte arithmetic in range

namespace {
bool intersects(const ArenaTensor& a, const ArenaTensor& b) { return a.start <= b.end && b.start <= a.end; }

typedef std::vector<std::pair<int64_t, int64_t>> Ranges;
// (busy: scratch of the caller, so that placing a tensor allocates nothing)
int64_t first_fit(const ArenaTensor& t, const std::vector<const ArenaTensor*>& placed, Ranges& busy) {
  busy.clear();
  for (const ArenaTensor* p : placed) if (intersects(t, *p)) busy.push_back({p->offset, p->offset + p->bytes});
  std::sort(busy.begin(), busy.end());
  int64_t off = 0;
  for (const auto& b : busy) {
    if (off + t.bytes <= b.first) break;
    off = std::max(off, b.second);
  }
  return off;
}
// the highest offset that fits below the ceiling; the lowest offset that fits when there is none
int64_t last_fit(const ArenaTensor& t, const std::vector<const ArenaTensor*>& placed, Ranges& busy, int64_t ceiling) {
  busy.clear();
  for (const ArenaTensor* p : placed) if (intersects(t, *p)) busy.push_back({p->offset + p->bytes, p->offset});   // (hi, lo)
  std::sort(busy.begin(), busy.end(), [](const std::pair<int64_t, int64_t>& x, const std::pair<int64_t, int64_t>& y) { return x > y; });
  int64_t end = ceiling;
  for (const auto& b : busy) {
    if (end - t.bytes >= b.first) break;
    end = std::min(end, b.second);
  }
  return end - t.bytes >= 0 ? end - t.bytes : first_fit(t, placed, busy);
}
// comparison strategy of Section 4.4.1: the smallest free slot that can hold the tensor
int64_t best_fit(const ArenaTensor& t, const std::vector<const ArenaTensor*>& placed) {
  std::vector<std::pair<int64_t, int64_t>> busy;
  int64_t top = 0;
  for (const ArenaTensor* p : placed) {
    top = std::max(top, p->offset + p->bytes);
    if (intersects(t, *p)) busy.push_back({p->offset, p->offset + p->bytes});
  }
  std::sort(busy.begin(), busy.end());
  std::vector<std::pair<int64_t, int64_t>> gaps;   // (size, offset)
  int64_t cur = 0;
  for (const auto& b : busy) {
    if (b.first > cur) gaps.push_back({b.first - cur, cur});
    cur = std::max(cur, b.second);
  }
  if (top > cur) gaps.push_back({top - cur, cur});
  std::sort(gaps.begin(), gaps.end());
  for (const auto& gp : gaps) if (gp.first >= t.bytes) return gp.second;
  return cur;
}
}  // namespace

BindResult bind_plan(const Plan& p, const std::vector<int64_t>& symbols, const std::vector<int>& decisions,
                     bool allow_undecided, const std::vector<int64_t>& exec_values) {
  const Graph& G = *p.g;
  BindResult b;
  if (symbols.size() != G.symbols.size()) throw Error(SOD2_ERR_INVALID_ARG, "wrong number of symbol values");
  for (size_t i = 0; i < symbols.size(); ++i) {
    const Symbol& s = G.symbols[i];
    if (symbols[i] < s.lo || symbols[i] > s.hi)
      throw Error(SOD2_ERR_SYMBOL_OUT_OF_RANGE, "symbol " + s.name + " = " + std::to_string(symbols[i]) +
                                                    " outside [" + std::to_string(s.lo) + ", " + std::to_string(s.hi) + "]");
    b.env[s.name] = symbols[i];
  }
  std::map<int, int64_t> cap_elems;
  for (int t : G.session_ids) {
    int64_t n = 1;
    for (const auto& c : G.tensors[t].capacity) n *= Expr::parse(c).eval(b.env);
    cap_elems[t] = n;
    int64_t nbytes = (n * dtype_bytes(G.tensors[t].dtype) + 255) / 256 * 256;
    b.session[t] = {b.session_bytes, nbytes};
    b.session_root[t] = t;
    b.session_bytes += nbytes;
  }
  std::vector<int64_t> sv = symbols;                  // graph symbols, then one slot per execution symbol
  sv.resize(p.xc.symbols.size(), 0);
  p.xc.atom_values(sv, &b.atom_vals);
  size_t next_exec = 0;
  const int nt = (int)G.tensors.size();
  std::vector<char> group_dead(G.ops.size(), 0);   // by group id (= an operator id)
  std::vector<signed char> memo_dead(nt, -1);       // tensor -> dead?  (-1: not computed yet)
  std::vector<int> memo_base(nt, -1);               // tensor -> storage tensor
  size_t next_dec = 0;

  struct Info {
    const Plan& p; const Graph& G; BindResult& b;
    std::vector<char>& group_dead; std::vector<signed char>& memo_dead; std::vector<int>& memo_base;
    std::pair<bool, int> operator()(int t) {
      if (memo_dead[t] >= 0) return {memo_dead[t] != 0, memo_base[t]};
      std::pair<bool, int> r(false, t);
      int pr = G.producer[t];
      if (pr >= 0 && !p.folded[pr]) {
        const Op& op = G.ops[pr];
        if (op.kind == SOD2_OP_SWITCH) {
          auto d = (*this)(op.in[0]);
          auto dec = b.decisions.find(pr);
          bool is_skip_out = op.out.size() > 1 && op.out[1] == t;
          bool taken = dec != b.decisions.end() && (is_skip_out == (dec->second != 0));
          r = {d.first || dec == b.decisions.end() || !taken, d.second};
        } else if (op.kind == SOD2_OP_COMBINE) {
          r = {true, t};
          for (int i : op.in) {
            auto d = (*this)(i);
            if (!d.first) { r = {false, d.second}; break; }
          }
        } else if (p.view[pr]) {
          r = (*this)(op.in[0]);
        } else if (p.inplace[t] >= 0) {             // the result took over an operand's storage
          r = {group_dead[p.group_of_op[pr]] != 0, (*this)(p.inplace[t]).second};
        } else {
          r = {group_dead[p.group_of_op[pr]] != 0, t};
        }
      }
      memo_dead[t] = r.first ? 1 : 0;
      memo_base[t] = r.second;
      return r;
    }
  } info{p, G, b, group_dead, memo_dead, memo_base};

  std::vector<int> reads_at(nt, -1);
  b.tensors.reserve(p.items.size() + 8);
  b.dims.reserve(p.items.size() + 8);
  b.steps.reserve(p.items.size());
  b.step_sg.reserve(p.items.size());
  for (size_t s = 0; s < p.subgraphs.size(); ++s) {
    for (int i : p.subgraphs[s]) {
      const Item& it = p.items[i];
      int step = (int)b.steps.size();
      if (it.is_group) {
        const Group& gr = p.groups.at(it.ref);
        const std::vector<int>& ext = p.item_ext[i];
        bool dead = false;
        for (int t : ext) if (info(t).first) dead = true;
        group_dead[gr.gid] = dead;
        if (dead) { b.dead_ops.insert(gr.ops.begin(), gr.ops.end()); continue; }
        for (int t : ext) reads_at[info(t).second] = step;
        int t = gr.out;
        int64_t nz_bytes = -1;
        if (gr.kind == G_NONZERO || gr.kind == G_NMS) {
          int n_op = gr.ops[0], src = G.ops[n_op].in[0];
          if (p.cshape[src].empty() && !p.rdp->S[src].resolved())
            throw Error(SOD2_ERR_UNRESOLVED_SHAPE, "shape of " + G.tensors[src].name + " is not resolved");
          int64_t ub = 1;
          for (const CompiledExpr& d : p.cshape[src]) ub *= d.eval(b.atom_vals);
          bool known = next_exec < exec_values.size();
          int64_t v = known ? exec_values[next_exec++] : ub;
          if (v < 0 || v > ub) throw Error(SOD2_ERR_INVALID_ARG, "a NonZero count outside [0, element count of its input]");
          size_t slot = G.symbols.size() + (std::find(p.exec_ops.begin(), p.exec_ops.end(), n_op) - p.exec_ops.begin());
          sv[slot] = v;
          p.xc.atom_values(sv, &b.atom_vals);
          b.exec.push_back({n_op, v, known});
          nz_bytes = ((int64_t)p.cshape[src].size() * ub + 1) * dtype_bytes(G.tensors[t].dtype);
        }
        const LS& sh = p.rdp->S[t];
        if (!sh.resolved())
          throw Error(SOD2_ERR_UNRESOLVED_SHAPE, "shape of " + G.tensors[t].name + " is not resolved: " + sh.str());
        int64_t n = dtype_bytes(G.tensors[t].dtype);
        {
          DimList& dims = b.dims[t];
          dims.n = 0;
          for (const CompiledExpr& d : p.cshape[t]) {
            dims.push_back(d.eval(b.atom_vals));
            // (a window larger than its input, symbols at extreme values: refuse instead of planning with garbage)
            if (dims.back() < 0 || (dims.back() > 0 && n > kMaxTensorBytes / dims.back()))
              throw Error(SOD2_ERR_SHAPE_MISMATCH, "extent of " + G.tensors[t].name + " at the bound symbols is negative or the tensor exceeds 2^44 bytes");
            n *= dims.back();
          }
        }
        if (gr.versions > 1) {
          // Section 4.2: of the code versions of a fused group with unproven broadcast pairs, the one that holds for
          // the bound symbols; per pair 'e' equal extents, 'a' the first operand's is 1 (broadcast), 'b' the second's
          std::string v;
          for (const Group::Pair& pr : gr.unproven) {
            const auto &ca = p.cshape[pr.a], &cb = p.cshape[pr.b];
            const int64_t x = pr.k <= (int)ca.size() ? ca[ca.size() - pr.k].eval(b.atom_vals) : 1;
            const int64_t y = pr.k <= (int)cb.size() ? cb[cb.size() - pr.k].eval(b.atom_vals) : 1;
            v += x == y ? 'e' : (x == 1 ? 'a' : 'b');
          }
          b.versions[gr.gid] = v;
        }
        for (int n_op : gr.ops) {                       // a CACHEAPPEND group, or appends inside an attention group
          if (G.ops[n_op].kind != SOD2_OP_CACHEAPPEND) continue;
          int tc = G.ops[n_op].out[0];
          auto root = b.session_root.find(G.ops[n_op].in[0]);
          if (root == b.session_root.end()) throw Error(SOD2_ERR_UNSUPPORTED, "CacheAppend must extend a session tensor");
          DimList cd;
          int64_t elems = 1;
          for (const CompiledExpr& d : p.cshape[tc]) { cd.push_back(d.eval(b.atom_vals)); elems *= cd.back(); }
          if (p.cshape[tc].empty() && !p.rdp->S[tc].resolved())
            throw Error(SOD2_ERR_UNRESOLVED_SHAPE, "shape of " + G.tensors[tc].name + " is not resolved");
          b.dims[tc] = cd;
          int root_id = root->second;
          b.session_root[tc] = root_id;
          if (elems > cap_elems.at(root_id))
            throw Error(SOD2_ERR_INVALID_ARG, "session tensor " + G.tensors[tc].name + " would outgrow its capacity");
        }
        if (nz_bytes >= 0) n = nz_bytes;
        if (p.arena_candidate(t) && p.inplace[t] < 0) b.tensors[t] = ArenaTensor{t, (n + 255) / 256 * 256, step, step, -1};
        for (int t2 : gr.also) {                        // the operator's further results
          if (!p.rdp->S[t2].resolved())
            throw Error(SOD2_ERR_UNRESOLVED_SHAPE, "shape of " + G.tensors[t2].name + " is not resolved: " + p.rdp->S[t2].str());
          DimList d2;
          int64_t n2 = dtype_bytes(G.tensors[t2].dtype);
          for (const CompiledExpr& d : p.cshape[t2]) { d2.push_back(d.eval(b.atom_vals)); n2 *= d2.back(); }
          b.dims[t2] = d2;
          if (p.fold_y[t2] >= 0) n2 = n2 * 9 / 8;       // R9: rows plus their partial sums (8 bytes per 32 columns)
          if (p.arena_candidate(t2)) b.tensors[t2] = ArenaTensor{t2, (n2 + 255) / 256 * 256, step, step, -1};
        }
      } else {
        const Op& op = G.ops[it.ref];
        if (op.kind == SOD2_OP_SWITCH) {
          if (info(op.in[0]).first) { b.dead_ops.insert(it.ref); continue; }
          int dec = 0;
          if (next_dec < decisions.size()) dec = decisions[next_dec++] ? 1 : 0;
          else if (allow_undecided) ++b.undecided;
          else throw Error(SOD2_ERR_INVALID_ARG, "a Switch decision is missing");
          b.decisions[it.ref] = dec;
          b.switch_order.push_back(it.ref);
          for (int t : op.in) reads_at[info(t).second] = step;
        } else {
          int live = -1;
          for (int t : op.in) if (!info(t).first) { live = t; break; }
          if (live < 0) { b.dead_ops.insert(it.ref); continue; }
          reads_at[info(live).second] = step;
        }
      }
      b.steps.push_back(i);
      b.step_sg.push_back((int)s);
    }
  }
  for (auto& kv : b.tensors) {
    kv.second.end = std::max(kv.second.start, reads_at[kv.first]);
  }
  b.dyn_base.assign(nt, -1);
  for (int t = 0; t < nt; ++t) {
    int pr = G.producer[t];
    if (pr < 0 || p.folded[pr] || (!b.dead_ops.empty() && b.dead_ops.count(pr))) continue;
    auto d = info(t);
    if (!d.first) b.dyn_base[t] = d.second;
  }

  int nsteps = (int)b.steps.size();
  std::vector<int64_t> live_bytes(nsteps, 0);
  for (const auto& kv : b.tensors)
    for (int k = kv.second.start; k <= kv.second.end; ++k) live_bytes[k] += kv.second.bytes;
  for (int64_t v : live_bytes) b.peak_live = std::max(b.peak_live, v);
  b.peak_live += b.session_bytes;

  std::vector<const ArenaTensor*> placed;
  Ranges busy;
  int64_t top = 0;                                     // highest byte of anything placed so far
  if (p.opts.dmp) {
    std::vector<ArenaTensor*> by_start;                // every region takes its tensors from the front
    for (auto& kv : b.tensors) by_start.push_back(&kv.second);
    std::stable_sort(by_start.begin(), by_start.end(), [](const ArenaTensor* x, const ArenaTensor* y) { return x->start < y->start; });
    size_t next_t = 0;
    // a sub-graph with a control operator or a NonZero is planned alone; so is one with execution-
    // determined sizes as long as a NonZero that ran before it has no known count yet
    std::vector<char> alone_v(nsteps, 0);
    {
      int known = 0, seen = 0;
      for (const auto& e : b.exec) known += e.known ? 1 : 0;
      for (int k = 0; k < nsteps; ++k) {
        const Item& it = p.items[b.steps[k]];
        bool nz = it.is_group && (p.groups.at(it.ref).kind == G_NONZERO || p.groups.at(it.ref).kind == G_NMS);
        alone_v[k] = !it.is_group || nz || (p.sg_class[b.step_sg[k]] == "nac" && seen > known);
        seen += nz ? 1 : 0;
      }
    }
    auto alone = [&](int k) { return alone_v[k] != 0; };
    int k0 = 0;
    while (k0 < nsteps) {
      // region: consecutive sub-graphs with resolved sizes and no control operator are planned together
      int k1 = k0;
      while (k1 + 1 < nsteps) {
        bool new_sg = b.step_sg[k1 + 1] != b.step_sg[k1];
        if (new_sg && (alone(k1 + 1) || alone(k1))) break;
        ++k1;
      }
      // a tensor that ended before this region starts can no longer intersect anything placed from here on
      placed.erase(std::remove_if(placed.begin(), placed.end(), [k0](const ArenaTensor* a) { return a->end < k0; }), placed.end());
      std::vector<ArenaTensor*> mine;
      while (next_t < by_start.size() && by_start[next_t]->start <= k1) mine.push_back(by_start[next_t++]);
      if (!mine.empty()) {
        // the peak first, then the next highest step, and so on; at each step the tensors live there
        // that have no offset yet are placed one by one.  The region cannot end below the ceiling (its
        // own peak of live bytes, or what is already placed).  Four variants of the pass, in a fixed
        // order, the first that ends lowest is kept and the search stops at one that ends at the
        // ceiling: tensors of a step by (start, id) or by (size descending, start, id), each at the
        // lowest offset that fits or at the highest one below the ceiling that fits.
        std::vector<int> steps_by_need;
        int64_t ceiling = top;
        for (int k = k0; k <= k1; ++k) { steps_by_need.push_back(k); ceiling = std::max(ceiling, live_bytes[k]); }
        std::stable_sort(steps_by_need.begin(), steps_by_need.end(), [&](int x, int y) { return live_bytes[x] > live_bytes[y]; });
        std::sort(mine.begin(), mine.end(), [](const ArenaTensor* x, const ArenaTensor* y) {
          return x->start != y->start ? x->start < y->start : x->tid < y->tid;
        });
        std::vector<ArenaTensor*> by_size = mine;
        std::stable_sort(by_size.begin(), by_size.end(), [](const ArenaTensor* x, const ArenaTensor* y) { return x->bytes > y->bytes; });
        const size_t n_before = placed.size();
        int64_t best_top = -1;
        std::vector<int64_t> best_off(mine.size());
        for (int variant = 0; variant < 4; ++variant) {
          const std::vector<ArenaTensor*>& order = (variant & 1) ? by_size : mine;
          const bool high = variant >= 2;
          for (ArenaTensor* a : mine) a->offset = -1;
          placed.resize(n_before);
          size_t left = mine.size();
          int64_t region_top = 0;
          for (int pk : steps_by_need) {
            if (left == 0) break;
            for (ArenaTensor* a : order) {
              if (a->offset >= 0 || a->start > pk || a->end < pk) continue;
              a->offset = high ? last_fit(*a, placed, busy, ceiling) : first_fit(*a, placed, busy);
              region_top = std::max(region_top, a->offset + a->bytes);
              placed.push_back(a);
              --left;
            }
          }
          if (best_top < 0 || region_top < best_top) {
            best_top = region_top;
            for (size_t i = 0; i < mine.size(); ++i) best_off[i] = mine[i]->offset;
          }
          if (best_top <= ceiling) break;
        }
        for (size_t i = 0; i < mine.size(); ++i) mine[i]->offset = best_off[i];
        top = std::max(top, best_top);
      }
      k0 = k1 + 1;
    }
  } else {
    std::vector<ArenaTensor*> all;
    for (auto& kv : b.tensors) all.push_back(&kv.second);
    std::sort(all.begin(), all.end(), [](const ArenaTensor* x, const ArenaTensor* y) {
      return x->start != y->start ? x->start < y->start : x->tid < y->tid;
    });
    for (ArenaTensor* a : all) { a->offset = best_fit(*a, placed); placed.push_back(a); }
  }
  b.arena_bytes = b.session_bytes;
  for (auto& kv : b.tensors) {
    kv.second.offset += b.session_bytes;
    b.arena_bytes = std::max(b.arena_bytes, kv.second.offset + kv.second.bytes);
  }
  return b;
}

std::string BindResult::dump(const Plan& p) const {
  std::string out = "sym";
  for (const auto& s : p.g->symbols) out += " " + s.name + "=" + std::to_string(env.at(s.name));
  out += "\n";
  for (const Exec& e : exec)
    out += "exec " + exec_symbol(e.op) + "=" + std::to_string(e.value) + (e.known ? " known\n" : " bound\n");
  for (const auto& kv : session)
    out += "session t" + std::to_string(kv.first) + " off=" + std::to_string(kv.second.first) + " bytes=" +
           std::to_string(kv.second.second) + "\n";
  for (size_t k = 0; k < steps.size(); ++k) {
    const Item& it = p.items[steps[k]];
    out += "step " + std::to_string(k) + " " + (it.is_group ? "g" : "c") + std::to_string(it.ref) + "\n";
  }
  for (const auto& kv : versions)
    out += "version g" + std::to_string(kv.first) + " " + kv.second + " of " + std::to_string(p.groups.at(kv.first).versions) + "\n";
  for (const auto& kv : dims) {
    out += "t" + std::to_string(kv.first) + " dims=[";
    for (size_t i = 0; i < kv.second.size(); ++i) { if (i) out += " "; out += std::to_string(kv.second[i]); }
    out += "]";
    auto at = tensors.find(kv.first);
    if (at != tensors.end())
      out += " off=" + std::to_string(at->second.offset) + " bytes=" + std::to_string(at->second.bytes) + " life=" +
             std::to_string(at->second.start) + ".." + std::to_string(at->second.end) + "\n";
    else if (session_root.count(kv.first))
      out += " session=t" + std::to_string(session_root.at(kv.first)) + "\n";
    else if (p.inplace[kv.first] >= 0)
      out += " inplace=t" + std::to_string(dyn_base[kv.first]) + "\n";
    else
      out += " external\n";
  }
  out += "arena_bytes=" + std::to_string(arena_bytes) + "\npeak_live=" + std::to_string(peak_live) + "\n";
  return out;
}
}  // namespace sod2
