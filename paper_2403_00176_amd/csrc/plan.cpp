// Static planning on the RDP result: fusion groups (Section 4.2), sub-graph partition and
// execution order (Section 4.3).
//
// Rules (the paper leaves them to an earlier fusion system and to "exhaustive search"):
//  R0 an operator whose outputs are integer tensors with a fully resolved value map is folded;
//  R1 Reshape / Slice / Transpose / Expand / Gather-with-scalar-host-index are views (no kernel); one whose result is a
//     graph output is a COPY group (the view written out densely into the caller's buffer), and an operator with a
//     known value map is not folded when its result is a graph output; a strided view (a permutation, a slice or index
//     of a dim other than the first, an Expand, or a view of one) read by an operator whose kernel wants dense operands,
//     and a permuted view read by LayerNorm, Softmax or Reshape, is a COPY group as well (its result an arena tensor);
//  R2 MatMul / Conv absorbs, in order and each at most once: Mul by a host scalar, Add of a rank-1
//     weight equal to the last dim, an activation, Add of a non-constant tensor of proven-equal
//     shape, an activation, a Transpose (stored permuted); each absorbed operator must be the sole
//     consumer of the chain so far;
//  R3 LayerNorm, GroupNorm, MaxUnpool, Softmax, MaxPool, AveragePool, ReduceMean, ArgMax, CacheAppend, NonZero, NMS, ScatterRows, Resize, Upsample,
//     OneHot, TopK (one group, two results), and a Concat, Range, ConstantOfShape or EyeLike that is not folded stand alone; a
//     non-view Gather absorbs one Add of proven-equal shape;
//  R4 other elementwise operators chain (up to 8; a Round joins only behind an fp32 value, else it starts a chain).  A dim pair of the two operands of a binary member is proven when
//     RDP shows the extents equal or one of them 1: one form of the fused loop nest.  A pair of two resolved but
//     unrelated extents doubles the number of code versions (Fig. 4), one of which is selected at bind; the chain
//     stops before the member that would need more than max_versions (8) and at an unresolved extent;
//  R5 group id = smallest member id; groups are ordered by the node-order position of their
//     last member;
//  R6 attention: a GEMM group of MatMul [+ Mul by a host scalar] read by one Softmax alone, whose
//     result is the first operand of one MatMul alone leading a GEMM group of MatMul [+ Transpose]:
//     the three become one ATTENTION group (scores and probabilities never reach memory); bf16
//     tensors and the known head size the options state (64: what the fused kernel is written for).
//  R8 cache append inside attention: when the key and the value operand of an ATTENTION group are,
//     through views only and with no other reader, the results of two CacheAppend operators that
//     each append a known number of at most append_max_rows (4) bf16 rows (the decode step), their CACHEAPPEND groups
//     join the ATTENTION group: its kernel writes the new rows into the session slots itself.
// Partition: cut around control operators, NonZero and NMS, after a group with a nac output, wherever
// at most one arena tensor is live, and every 14 items.  Order inside a sub-graph: the sequence
// with the smallest peak of live bytes at the symbols' upper bounds, ties to smaller group ids.
//
// Execution-determined extents (Section 4.3): with a NonZero or an NMS in the graph the plan is built on the
// analysis with named EDO extents; a tensor that is unresolved or sized by an execution symbol
// counts as nac: a cut follows every item that writes one and such sub-graphs keep the node order.
#include <algorithm>
#include <set>
#include <limits>

#include "internal.hpp"

namespace sod2 {

static const char* kGroupNames[] = {"GEMM", "CONV", "LAYERNORM", "SOFTMAX", "MAXPOOL", "REDUCEMEAN", "ARGMAX",
                                    "CACHEAPPEND", "NONZERO", "GATHER", "ELTWISE", "ATTENTION", "SCATTER", "RESIZE", "CONCAT", "RANGE", "FILL", "ONEHOT", "TOPK", "GROUPNORM", "MAXUNPOOL", "AVGPOOL", "NMS", "COPY"};
const char* group_kind_name(int k) { return kGroupNames[k]; }

namespace {
const int kMaxSubgraph = 14;

bool is_act(int k) { return k == SOD2_OP_RELU || k == SOD2_OP_GELU || k == SOD2_OP_SIGMOID; }
bool is_eltwise(int k) { return k == SOD2_OP_ADD || k == SOD2_OP_MUL || is_act(k) || k == SOD2_OP_CAST || k == SOD2_OP_ROUND; }
bool is_view_kind(int k) { return k == SOD2_OP_RESHAPE || k == SOD2_OP_SLICE || k == SOD2_OP_TRANSPOSE || k == SOD2_OP_EXPAND; }
bool scalar_gather(const Graph& G, const Op& op) {     // Gather with a scalar host index: a view
  const Tensor& idx = G.tensors[op.in[1]];
  return idx.has_data && idx.host_rank == 0;
}
bool is_dense_only(int k) {                          // operators whose kernels want dense operands
  switch (k) {
    case SOD2_OP_CONCAT: case SOD2_OP_REDUCEMEAN: case SOD2_OP_MAXPOOL: case SOD2_OP_AVERAGEPOOL: case SOD2_OP_GROUPNORM:
    case SOD2_OP_CONV: case SOD2_OP_MAXUNPOOL: case SOD2_OP_RESIZE: case SOD2_OP_UPSAMPLE: case SOD2_OP_SCATTERROWS:
    case SOD2_OP_TOPK: case SOD2_OP_ARGMAX: case SOD2_OP_NONZERO: case SOD2_OP_NMS: return true;
    default: return false;
  }
}
bool is_control(int k) { return k == SOD2_OP_SWITCH || k == SOD2_OP_COMBINE; }
bool is_counting(int k) { return k == SOD2_OP_NONZERO || k == SOD2_OP_NMS; }   // a result whose length is found by running

bool shape_equal(const LS& a, const LS& b) {
  if (!a.resolved() || !b.resolved() || a.d.size() != b.d.size()) return false;
  for (size_t i = 0; i < a.d.size(); ++i) if (a.d[i].e != b.d[i].e) return false;
  return true;
}
bool pair_proven(const LV& a, const LV& b) {
  return a.val() && b.val() && (a.e == b.e || a.is_c(1) || b.is_c(1));
}
// Dim pairs of the two operands of a binary elementwise operator that RDP cannot prove equal or 1, the dim counted
// from the last; none for a unary operator; false when an extent is unresolved
bool unproven_pairs(const Rdp& R, const Op& op, std::vector<Group::Pair>* out) {
  out->clear();
  if (op.in.size() != 2) return true;
  const LS &sa = R.S[op.in[0]], &sb = R.S[op.in[1]];
  if (!sa.is_list() || !sb.is_list()) return false;
  const size_t r = std::max(sa.d.size(), sb.d.size());
  for (size_t k = 1; k <= r; ++k) {
    const LV x = k <= sa.d.size() ? sa.d[sa.d.size() - k] : LV::c(1);
    const LV y = k <= sb.d.size() ? sb.d[sb.d.size() - k] : LV::c(1);
    if (pair_proven(x, y)) continue;
    if (!x.val() || !y.val()) return false;
    out->push_back({op.in[0], op.in[1], (int)k});
  }
  return true;
}
int64_t align_up(int64_t n) { return (n + 255) / 256 * 256; }
}  // namespace

bool Plan::arena_candidate(int t) const {
  const Tensor& d = g->tensors[t];
  return d.role == SOD2_INTER && !d.is_output && !d.session;
}

bool Plan::execution_determined(int t) const {
  const LS& s = rdp->S[t];
  if (!s.resolved()) return true;
  for (const auto& d : s.d) if (mentions_exec(d.e)) return true;
  return false;
}

// size used by the order search; an execution-determined tensor counts as 0 (unknown)
static int64_t bytes_at(const Plan& p, int t, const std::map<std::string, int64_t>& env) {
  const LS& s = p.rdp->S[t];
  if (p.execution_determined(t)) return 0;
  int64_t n = dtype_bytes(p.g->tensors[t].dtype);
  for (const auto& d : s.d) n *= d.e.eval(env);
  if (p.fold_y[t] >= 0) n = n * 9 / 8;             // R9: per row and 32 columns an 8-byte pair of partial sums behind the rows
  return align_up(n);
}

void Plan::build() {
  const Graph& G = *g;
  paper_rdp = rdp;
  for (const Op& op : G.ops)
    if (is_counting(op.kind) && !named) {
      // Section 4.3: what follows an EDO is planned when it has executed.  With its extent named,
      // the sizes that follow are expressions evaluated at that moment instead of re-inferred.
      named = std::make_shared<Rdp>();
      named->g = g;
      named->named_edo = true;
      named->analyse(nullptr);
      rdp = named.get();
    }
  const Rdp& R = *rdp;
  int nops = (int)G.ops.size();
  order = G.sorted_nodes();
  std::vector<int> pos(nops, -1);
  for (int i = 0; i < (int)order.size(); ++i) pos[order[i]] = i;
  for (int i = 0; i < nops; ++i)
    if (pos[i] < 0) throw Error(SOD2_ERR_INVALID_ARG, "operator unreachable from the graph inputs");

  // R0 / R1
  folded.assign(nops, 0);
  view.assign(nops, 0);
  for (int i = 0; i < nops; ++i) {
    const Op& op = G.ops[i];
    if (is_control(op.kind)) {
      for (int o : op.out)
        if (G.tensors[o].is_output)            // control operators forward storage, they write none
          throw Error(SOD2_ERR_UNSUPPORTED, "a graph output must not be the direct result of a Switch or Combine "
                                            "(put an operator behind it: a Cast to its own type copies it)");
      if (op.kind == SOD2_OP_SWITCH) ++n_switches;
      continue;
    }
    bool ints = true, known = true, to_caller = false;   // to_caller: its result must reach the caller's buffer
    for (int o : op.out) {
      if (!is_int(G.tensors[o].dtype)) ints = false;
      if (!R.V[o].resolved()) known = false;
      if (G.tensors[o].is_output) to_caller = true;
    }
    if (ints && known && !to_caller) folded[i] = 1;
    else if (is_view_kind(op.kind)) view[i] = !to_caller;
    else if (op.kind == SOD2_OP_GATHER) view[i] = scalar_gather(G, op) && !to_caller;
  }
  // R1, second half: a view that a kernel could not walk is written out.  In the node order, so that a view of a view
  // inherits: strided = permutes dims, slices or indexes a dim other than the first, or repeats elements; permuted =
  // a Transpose is involved.
  {
    const int nten = (int)G.tensors.size();
    std::vector<char> strided(nten, 0), permuted(nten, 0);   // per tensor: it is such a view (control operators pass it on)
    // the operators that get to read tensor t, with the tensor they read it as: consumers, looking through Switch / Combine
    auto readers = [&](int t) {
        std::vector<std::pair<int, int>> out;
        std::vector<int> stack{t};
        std::set<std::pair<int, int>> seen;
        while (!stack.empty()) {
          const int u = stack.back();
          stack.pop_back();
          for (int c : G.consumers[u]) {
            if (folded[c] || !seen.insert({c, u}).second) continue;
            if (is_control(G.ops[c].kind)) stack.insert(stack.end(), G.ops[c].out.begin(), G.ops[c].out.end());
            else out.push_back({c, u});
          }
        }
        std::sort(out.begin(), out.end());
        return out;
    };
    for (int n : order) {
      const Op& op = G.ops[n];
      if (op.kind == SOD2_OP_SWITCH) {
        for (int o : op.out) { strided[o] = strided[op.in[0]]; permuted[o] = permuted[op.in[0]]; }
        continue;
      }
      if (op.kind == SOD2_OP_COMBINE) {
        for (int t : op.in) { strided[op.out[0]] |= strided[t]; permuted[op.out[0]] |= permuted[t]; }
        continue;
      }
      if (!view[n]) continue;
      const int src = op.in[0], res = op.out[0];
      const LS& ss = R.S[src];
      const int64_t rank = ss.is_list() ? (int64_t)ss.d.size() : -1;
      bool s = false, pm = false;
      if (op.kind == SOD2_OP_TRANSPOSE) {
        for (size_t i = 0; i < op.ia.size(); ++i) if (op.ia[i] != (int64_t)i) s = pm = true;
      } else if (op.kind == SOD2_OP_SLICE) {
        const LS& ax = R.V[op.in[3]];
        bool known = rank > 0 && ax.is_list();
        if (known) for (const auto& e : ax.d) if (!(e.val() && e.e.is_const())) known = false;
        s = !known;
        if (known) for (const auto& e : ax.d) if (((e.e.const_value() % rank) + rank) % rank != 0) s = true;
      } else if (op.kind == SOD2_OP_EXPAND) {
        s = true;
      } else if (op.kind == SOD2_OP_GATHER) {
        s = rank <= 0 || ((op.ia.at(0) % rank) + rank) % rank != 0;
      }
      strided[res] = s || strided[src];
      permuted[res] = pm || permuted[src];
      for (const auto& cu : readers(res)) {
        const int c2 = cu.first, k = G.ops[c2].kind;
        const bool table = k == SOD2_OP_GATHER && !view[c2] && G.ops[c2].in[0] == cu.second;   // rows picked by an index tensor
        if (((is_dense_only(k) || table) && strided[res]) ||
            ((k == SOD2_OP_LAYERNORM || k == SOD2_OP_SOFTMAX || k == SOD2_OP_RESHAPE) && permuted[res])) {
          view[n] = 0;                               // a COPY group: its result is dense
          strided[res] = permuted[res] = 0;
          break;
        }
      }
    }
  }

  auto sole_consumer = [&](int t) -> int {
    if (G.tensors[t].is_output || G.consumers[t].size() != 1) return -1;
    return G.consumers[t][0];
  };
  auto other = [&](const Op& op, int cur) { return op.in[0] == cur ? op.in[1] : op.in[0]; };
  auto host_scalar = [&](int t) {
    const Tensor& d = G.tensors[t];
    return d.has_data && (d.idata.size() + d.fdata.size()) == 1;
  };

  // R2 - R4
  group_of_op.assign(nops, -1);
  std::set<int> absorbed_transpose;
  auto new_group = [&](int kind, const std::vector<int>& chain) {
    Group gr;
    gr.kind = kind;
    gr.chain = chain;
    gr.ops = chain;
    std::sort(gr.ops.begin(), gr.ops.end());
    gr.gid = gr.ops.front();
    int last = chain[0];
    for (int n : chain) if (pos[n] > pos[last]) last = n;
    gr.out = G.ops[last].out[0];
    gr.also.assign(G.ops[last].out.begin() + 1, G.ops[last].out.end());
    for (int n : chain) group_of_op[n] = gr.gid;
    groups[gr.gid] = gr;
  };
  for (int n : order) {
    const Op& op = G.ops[n];
    if (folded[n] || group_of_op[n] >= 0 || is_control(op.kind)) continue;
    if (view[n] && !absorbed_transpose.count(n)) continue;
    if (op.kind == SOD2_OP_MATMUL || op.kind == SOD2_OP_CONV) {
      std::vector<int> chain{n};
      int cur = op.out[0], state = 0;
      while (true) {
        int c = sole_consumer(cur);
        if (c < 0 || folded[c] || group_of_op[c] >= 0) break;
        const Op& cop = G.ops[c];
        // with fusion off only the permuted store remains: it is a layout choice of the contraction
        // (no arithmetic is merged), and without it the Reshape that follows would need a copy
        if (!opts.fusion && cop.kind != SOD2_OP_TRANSPOSE) break;
        int nxt = -1;
        if (cop.kind == SOD2_OP_MUL && state < 1 && host_scalar(other(cop, cur))) nxt = 1;
        else if (cop.kind == SOD2_OP_ADD) {
          int o = other(cop, cur);
          const LS &so = R.S[o], &sc = R.S[cur];
          int role = G.tensors[o].role;
          if (state < 2 && role == SOD2_WEIGHT && so.is_list() && so.d.size() == 1 && sc.is_list() &&
              sc.d.back().val() && so.d[0].val() && so.d[0].e == sc.d.back().e) nxt = 2;
          else if (state < 4 && role != SOD2_WEIGHT && role != SOD2_HOSTCONST && shape_equal(so, sc)) nxt = 4;
        } else if (is_act(cop.kind)) {
          nxt = state < 3 ? 3 : (state == 4 ? 5 : -1);
        } else if (cop.kind == SOD2_OP_TRANSPOSE && state < 6) {
          nxt = 6;
          absorbed_transpose.insert(c);
        }
        if (nxt < 0) break;
        chain.push_back(c);
        cur = cop.out[0];
        state = nxt;
        if (state == 6) break;
      }
      new_group(op.kind == SOD2_OP_MATMUL ? G_GEMM : G_CONV, chain);
    } else if (op.kind == SOD2_OP_LAYERNORM) new_group(G_LAYERNORM, {n});
    else if (op.kind == SOD2_OP_SOFTMAX) new_group(G_SOFTMAX, {n});
    else if (op.kind == SOD2_OP_MAXPOOL) new_group(G_MAXPOOL, {n});
    else if (op.kind == SOD2_OP_REDUCEMEAN) new_group(G_REDUCEMEAN, {n});
    else if (op.kind == SOD2_OP_ARGMAX) new_group(G_ARGMAX, {n});
    else if (op.kind == SOD2_OP_CACHEAPPEND) new_group(G_CACHEAPPEND, {n});
    else if (op.kind == SOD2_OP_NONZERO) new_group(G_NONZERO, {n});
    else if (op.kind == SOD2_OP_SCATTERROWS) new_group(G_SCATTER, {n});
    else if (op.kind == SOD2_OP_RESIZE) new_group(G_RESIZE, {n});
    else if (op.kind == SOD2_OP_CONCAT) new_group(G_CONCAT, {n});
    else if (op.kind == SOD2_OP_RANGE) new_group(G_RANGE, {n});
    else if (op.kind == SOD2_OP_UPSAMPLE) new_group(G_RESIZE, {n});
    else if (op.kind == SOD2_OP_CONSTANTOFSHAPE || op.kind == SOD2_OP_EYELIKE) new_group(G_FILL, {n});
    else if (op.kind == SOD2_OP_ONEHOT) new_group(G_ONEHOT, {n});
    else if (op.kind == SOD2_OP_TOPK) new_group(G_TOPK, {n});
    else if (op.kind == SOD2_OP_GROUPNORM) new_group(G_GROUPNORM, {n});
    else if (op.kind == SOD2_OP_MAXUNPOOL) new_group(G_MAXUNPOOL, {n});
    else if (op.kind == SOD2_OP_AVERAGEPOOL) new_group(G_AVGPOOL, {n});
    else if (op.kind == SOD2_OP_NMS) new_group(G_NMS, {n});
    else if (is_view_kind(op.kind) || (op.kind == SOD2_OP_GATHER && scalar_gather(G, op)))
      new_group(G_COPY, {n});          // a view whose result is a graph output: materialised in the caller's buffer
    else if (op.kind == SOD2_OP_GATHER) {
      std::vector<int> chain{n};
      int c = sole_consumer(op.out[0]);
      if (opts.fusion && c >= 0 && G.ops[c].kind == SOD2_OP_ADD && group_of_op[c] < 0 &&
          shape_equal(R.S[other(G.ops[c], op.out[0])], R.S[op.out[0]]))
        chain.push_back(c);
      new_group(G_GATHER, chain);
    } else if (is_eltwise(op.kind)) {
      std::vector<int> chain{n};
      int cur = op.out[0];
      std::vector<Group::Pair> pairs;
      if (!unproven_pairs(R, op, &pairs)) pairs.clear();    // of the seed itself: they count once it has company
      while (opts.fusion && chain.size() < 8) {
        int c = sole_consumer(cur);
        if (c < 0 || group_of_op[c] >= 0 || !is_eltwise(G.ops[c].kind)) break;
        const Op& cop = G.ops[c];
        if (cop.kind == SOD2_OP_ROUND && G.tensors[cur].dtype != SOD2_F32) break;   // Round must see the value as stored
        std::vector<Group::Pair> more;
        if (!unproven_pairs(R, cop, &more) || (1LL << (pairs.size() + more.size())) > std::max(max_versions(), 1)) break;
        pairs.insert(pairs.end(), more.begin(), more.end());
        chain.push_back(c);
        cur = cop.out[0];
      }
      new_group(G_ELTWISE, chain);
      if (chain.size() > 1 && !pairs.empty()) {
        Group& gr = groups[*std::min_element(chain.begin(), chain.end())];
        gr.versions = 1 << pairs.size();
        gr.unproven = pairs;
      }
    } else {
      throw Error(SOD2_ERR_UNSUPPORTED, std::string("no grouping rule for ") + op_name(op.kind));
    }
  }
  for (int c : absorbed_transpose) view[c] = 0;

  // R6: attention
  if (opts.fusion) {
    auto kinds_are = [&](const Group& gr, std::initializer_list<int> a, std::initializer_list<int> b) {
      std::vector<int> k;
      for (int m : gr.ops) k.push_back(G.ops[m].kind);
      return k == std::vector<int>(a) || k == std::vector<int>(b);
    };
    // R8 helper: the CacheAppend whose result reaches tensor t through views only, each link read by
    // nobody else, when it appends a known number of at most 4 bf16 rows; else -1
    auto append_behind = [&](int t) -> int {
      while (true) {
        int pr = G.producer[t];
        if (pr < 0 || G.tensors[t].is_output || G.consumers[t].size() != 1) return -1;
        if (view[pr]) { t = G.ops[pr].in[0]; continue; }
        const Op& ca = G.ops[pr];
        if (ca.kind != SOD2_OP_CACHEAPPEND || group_of_op[pr] < 0 || groups[group_of_op[pr]].kind != G_CACHEAPPEND) return -1;
        const LS& rows = R.S[ca.in[1]];
        if (G.tensors[t].dtype != SOD2_BF16 || !rows.is_list() || rows.d.empty() || !rows.d[0].val() ||
            !rows.d[0].e.is_const() || rows.d[0].e.const_value() > append_max_rows())
          return -1;
        return pr;
      }
    };
    for (int n : order) {
      const Op& op = G.ops[n];
      if (op.kind != SOD2_OP_SOFTMAX || group_of_op[n] < 0 || groups[group_of_op[n]].kind != G_SOFTMAX) continue;
      int x = op.in[0], y = op.out[0];
      int p1 = G.producer[x];
      if (p1 < 0 || group_of_op[p1] < 0 || sole_consumer(x) != n) continue;
      const Group g1 = groups[group_of_op[p1]];
      if (g1.kind != G_GEMM || g1.out != x || !kinds_are(g1, {SOD2_OP_MATMUL}, {SOD2_OP_MATMUL, SOD2_OP_MUL})) continue;
      int c2 = sole_consumer(y);
      if (c2 < 0 || G.ops[c2].kind != SOD2_OP_MATMUL || G.ops[c2].in[0] != y || G.ops[c2].in[1] == y) continue;
      const Group g2 = groups[group_of_op[c2]];
      if (g2.kind != G_GEMM || g2.ops.front() != c2 || !kinds_are(g2, {SOD2_OP_MATMUL}, {SOD2_OP_MATMUL, SOD2_OP_TRANSPOSE}))
        continue;
      const Op& mm1 = G.ops[g1.ops[0]];
      bool bf = true;
      for (int t : {mm1.in[0], mm1.in[1], G.ops[c2].in[1], x, y, g2.out}) if (G.tensors[t].dtype != SOD2_BF16) bf = false;
      const LS &sq = R.S[mm1.in[0]], &sv = R.S[G.ops[c2].in[1]];
      if (!bf || !sq.is_list() || !sv.is_list() || sq.d.empty() || sv.d.empty() || !sq.d.back().is_c(attn_head_dim()) || !sv.d.back().is_c(attn_head_dim()))
        continue;
      Group gr;
      gr.kind = G_ATTENTION;
      gr.chain = g1.chain;
      gr.chain.push_back(n);
      gr.chain.insert(gr.chain.end(), g2.chain.begin(), g2.chain.end());
      groups.erase(g1.gid);
      groups.erase(group_of_op[n]);
      groups.erase(g2.gid);
      // R8: the decode step's attention appends the new key / value rows itself
      int ca_k = append_behind(mm1.in[1]), ca_v = append_behind(G.ops[c2].in[1]);
      if (ca_k >= 0 && ca_v >= 0 && ca_k != ca_v) {
        groups.erase(group_of_op[ca_k]);
        groups.erase(group_of_op[ca_v]);
        gr.chain.insert(gr.chain.begin(), {ca_k, ca_v});
      }
      gr.ops = gr.chain;
      std::sort(gr.ops.begin(), gr.ops.end());
      gr.gid = gr.ops.front();
      gr.out = g2.out;
      for (int m : gr.ops) group_of_op[m] = gr.gid;
      groups[gr.gid] = gr;
    }
  }

  // R7: LayerNorm as the prologue of a contraction
  if (opts.fusion) {
    for (int n : order) {
      const Op& op = G.ops[n];
      if (op.kind != SOD2_OP_LAYERNORM || group_of_op[n] < 0 || groups[group_of_op[n]].kind != G_LAYERNORM) continue;
      int y = op.out[0];
      int c = sole_consumer(y);
      if (c < 0 || G.ops[c].kind != SOD2_OP_MATMUL || G.ops[c].in[0] != y || G.ops[c].in[1] == y) continue;
      const Group gm = groups[group_of_op[c]];
      if (gm.kind != G_GEMM || gm.ops.front() != c) continue;
      bool bf = true;
      for (int t : op.in) if (G.tensors[t].dtype != SOD2_BF16) bf = false;
      for (int t : {y, G.ops[c].in[1], gm.out}) if (G.tensors[t].dtype != SOD2_BF16) bf = false;
      const LS& sx = R.S[op.in[0]];
      if (!bf || !sx.is_list() || sx.d.empty()) continue;
      bool known = true;
      for (const auto& d : sx.d) if (!d.val() || !d.e.is_const()) known = false;
      if (!known) continue;
      int64_t kdim = sx.d.back().e.const_value(), rows = 1;
      for (size_t i = 0; i + 1 < sx.d.size(); ++i) rows *= sx.d[i].e.const_value();
      if (kdim > prologue_max_k() || kdim % prologue_k_multiple() != 0 || rows > prologue_max_rows()) continue;
      Group gr;
      gr.kind = G_GEMM;
      gr.chain = gm.chain;                       // the contraction stays the seed; the LayerNorm is its prologue
      gr.prologue = n;
      gr.ops = gm.ops;
      gr.ops.push_back(n);
      std::sort(gr.ops.begin(), gr.ops.end());
      gr.gid = gr.ops.front();
      gr.out = gm.out;
      groups.erase(group_of_op[n]);
      groups.erase(gm.gid);
      for (int m : gr.ops) group_of_op[m] = gr.gid;
      groups[gr.gid] = gr;
    }
  }

  // R9: a LayerNorm behind a contraction becomes that contraction's second result
  fold_y.assign(G.tensors.size(), -1);
  for (auto& kv : groups) {
    kv.second.key = 0;
    for (int m : kv.second.ops) kv.second.key = std::max(kv.second.key, pos[m]);
  }
  if (opts.fusion && opts.fold_ln) {
    for (int n : order) {
      const Op& op = G.ops[n];
      if (op.kind != SOD2_OP_LAYERNORM || group_of_op[n] < 0 || groups[group_of_op[n]].kind != G_LAYERNORM) continue;
      const int x = op.in[0], y = op.out[0];
      const int px = G.producer[x];
      if (px < 0 || group_of_op[px] < 0) continue;
      Group& gp = groups[group_of_op[px]];
      if (gp.kind != G_GEMM || gp.out != x || !gp.also.empty() || G.ops[gp.ops.front()].kind != SOD2_OP_MATMUL) continue;
      bool barred = false;
      for (int m : gp.ops) {
        const int k = G.ops[m].kind;
        if (k == SOD2_OP_TRANSPOSE || k == SOD2_OP_LAYERNORM || k == SOD2_OP_CACHEAPPEND) barred = true;
      }
      if (barred) continue;
      const int c = sole_consumer(y);
      if (c < 0 || G.ops[c].kind != SOD2_OP_MATMUL || G.ops[c].in[0] != y || G.ops[c].in[1] == y) continue;
      Group& gm = groups[group_of_op[c]];
      const int wt = G.ops[c].in[1];
      const LS &sw = R.S[wt], &sx = R.S[x];
      if (gm.kind != G_GEMM || gm.ops.front() != c || gm.lnfold >= 0 || G.ops[c].ia.empty() || !G.ops[c].ia[0] ||
          G.tensors[wt].role != SOD2_WEIGHT || !sw.is_list() || sw.d.size() != 2)
        continue;
      bool bf = true;
      for (int t : op.in) if (G.tensors[t].dtype != SOD2_BF16) bf = false;
      for (int t : {y, wt, gm.out}) if (G.tensors[t].dtype != SOD2_BF16) bf = false;
      if (!bf || !sx.resolved() || sx.d.empty() || !sx.d.back().e.is_const() || sx.d.back().e.const_value() <= 0 ||
          sx.d.back().e.const_value() % fold_k_multiple() != 0)
        continue;
      groups.erase(group_of_op[n]);
      gp.ops.push_back(n);
      std::sort(gp.ops.begin(), gp.ops.end());
      gp.also = {y};
      group_of_op[n] = gp.gid;
      gm.lnfold = n;
      fold_y[y] = n;
    }
  }
  // constants derived from the weights for the contractions that read a folded LayerNorm: two fp32 vectors over
  // the contraction's columns each, one block per group
  for (const auto& kv : groups) {
    if (kv.second.lnfold < 0) continue;
    const LS& sw = R.S[G.ops[kv.second.ops.front()].in[1]];
    if (!sw.d[0].e.is_const()) continue;
    const_off[kv.first] = const_bytes;
    const_bytes += (2 * sw.d[0].e.const_value() * 4 + 255) / 256 * 256;
  }

  // static storage bases: views and Switch outputs alias their (data) input
  int nt = (int)G.tensors.size();
  sbase.resize(nt);
  for (int t = 0; t < nt; ++t) sbase[t] = t;
  for (int n : order) {
    const Op& op = G.ops[n];
    if (view[n] || op.kind == SOD2_OP_SWITCH)
      for (int o : op.out) sbase[o] = sbase[op.in[0]];
  }
  for (auto& kv : groups) {
    Group& gr = kv.second;
    std::set<int> inside, seen;
    for (int n : gr.ops) for (int o : G.ops[n].out) inside.insert(o);
    for (int n : gr.ops)
      for (int t : G.ops[n].in) {
        int b = sbase[t];
        if (inside.count(t) || inside.count(b) || seen.count(b)) continue;
        seen.insert(b);
        gr.ins.push_back(b);
      }
  }

  // items in a topological order of groups and control operators (R5)
  struct Entry { int pos; bool is_group; int ref; };
  std::vector<Entry> entries;
  for (const auto& kv : groups) {
    entries.push_back({kv.second.key, true, kv.first});
  }
  for (int n = 0; n < nops; ++n) if (is_control(G.ops[n].kind)) entries.push_back({pos[n], false, n});
  std::sort(entries.begin(), entries.end(), [](const Entry& a, const Entry& b) { return a.pos < b.pos; });
  for (const auto& e : entries) {
    Item it;
    it.is_group = e.is_group;
    it.ref = e.ref;
    if (e.is_group) {
      it.reads = groups[e.ref].ins;
      it.writes = {groups[e.ref].out};
      it.writes.insert(it.writes.end(), groups[e.ref].also.begin(), groups[e.ref].also.end());
    } else {
      const Op& op = G.ops[e.ref];
      for (int t : op.in)
        if (std::find(it.reads.begin(), it.reads.end(), sbase[t]) == it.reads.end()) it.reads.push_back(sbase[t]);
      if (op.kind == SOD2_OP_COMBINE) it.writes = op.out;
    }
    items.push_back(it);
  }

  // partition ------------------------------------------------------------------------------------
  int n = (int)items.size();
  std::map<int, int> last_read;
  for (int i = 0; i < n; ++i) for (int t : items[i].reads) last_read[t] = i;
  auto lr = [&](int t) { auto it = last_read.find(t); return it == last_read.end() ? -1 : it->second; };
  auto has_nac = [&](const Item& it) {
    for (int t : it.writes) if (execution_determined(t)) return true;
    return false;
  };
  std::vector<char> cut_after(n, 0);
  std::set<int> live;
  for (int i = 0; i < n; ++i) {
    const Item& it = items[i];
    for (int t : it.writes) if (arena_candidate(t) && lr(t) > i) live.insert(t);
    for (auto p = live.begin(); p != live.end();) p = (lr(*p) > i) ? std::next(p) : live.erase(p);
    bool edo = !it.is_group || groups[it.ref].kind == G_NONZERO || groups[it.ref].kind == G_NMS;
    if (edo) {
      cut_after[i] = 1;
      if (i > 0) cut_after[i - 1] = 1;
    } else if (has_nac(it) || live.size() <= 1) {
      cut_after[i] = 1;
    }
  }
  std::vector<std::vector<int>> pieces;
  std::vector<int> cur;
  for (int i = 0; i < n; ++i) {
    cur.push_back(i);
    if (cut_after[i] || (int)cur.size() == kMaxSubgraph) { pieces.push_back(cur); cur.clear(); }
  }
  if (!cur.empty()) pieces.push_back(cur);

  std::map<std::string, int64_t> env_hi;
  for (const auto& s : G.symbols) env_hi[s.name] = s.hi;

  for (const auto& piece : pieces) {
    // class of the sub-graph (Section 4.3): all known / mixed / contains nac
    std::string cls = "known";
    for (int i : piece)
      for (int t : items[i].writes) {
        if (execution_determined(t)) { cls = "nac"; break; }
        for (const auto& d : R.S[t].d) if (!d.e.is_const() && cls != "nac") cls = "mixed";
      }
    sg_class.push_back(cls);
    int k = (int)piece.size();
    if (!opts.sep || k <= 2 || cls == "nac") { subgraphs.push_back(piece); continue; }

    // exhaustive search as a dynamic programme over the set of executed items
    int first = piece.front(), end = piece.back();
    std::map<int, int> idx, produced_in;
    for (int j = 0; j < k; ++j) idx[piece[j]] = j;
    std::vector<int> tensors;
    for (int i : piece)
      for (int t : items[i].writes)
        if (arena_candidate(t)) { produced_in[t] = idx[i]; tensors.push_back(t); }
    auto incoming = [&](int t) {
      if (!arena_candidate(t)) return false;
      for (int i = 0; i < first; ++i)
        if (std::find(items[i].writes.begin(), items[i].writes.end(), t) != items[i].writes.end()) return true;
      return false;
    };
    for (int i : piece)
      for (int t : items[i].reads)
        if (!produced_in.count(t) && std::find(tensors.begin(), tensors.end(), t) == tensors.end() && incoming(t))
          tensors.push_back(t);
    size_t nt2 = tensors.size();
    std::vector<int64_t> size(nt2);
    std::vector<int> prod(nt2, -1);
    std::vector<uint32_t> readers(nt2, 0);
    std::vector<char> live_out(nt2, 0);
    for (size_t a = 0; a < nt2; ++a) {
      int t = tensors[a];
      size[a] = bytes_at(*this, t, env_hi);
      if (produced_in.count(t)) prod[a] = produced_in[t];
      for (int i : piece)
        if (std::find(items[i].reads.begin(), items[i].reads.end(), t) != items[i].reads.end()) readers[a] |= 1u << idx[i];
      live_out[a] = lr(t) > end;
    }
    std::map<int, int> writer;                         // any tensor written in the piece, outputs included
    for (int i : piece) for (int t : items[i].writes) writer[t] = idx[i];
    std::vector<uint32_t> deps(k, 0);
    for (int i : piece)
      for (int t : items[i].reads)
        if (writer.count(t)) deps[idx[i]] |= 1u << writer[t];
    auto step_mem = [&](uint32_t S, int j) {
      int64_t mem = 0;
      for (size_t a = 0; a < nt2; ++a) {
        int p = prod[a];
        if (p >= 0 && p != j && !((S >> p) & 1)) continue;
        if (p == j || live_out[a] || (readers[a] & ~S)) mem += size[a];
      }
      return mem;
    };
    uint32_t full = (1u << k) - 1;
    const int64_t INF = std::numeric_limits<int64_t>::max();
    std::vector<int64_t> best(full + 1, INF);
    best[full] = 0;
    for (int64_t Sx = (int64_t)full - 1; Sx >= 0; --Sx) {
      uint32_t S = (uint32_t)Sx;
      int64_t b = INF;
      for (int j = 0; j < k; ++j) {
        if (((S >> j) & 1) || (deps[j] & ~S)) continue;
        int64_t nx = best[S | (1u << j)];
        if (nx == INF) continue;
        b = std::min(b, std::max(step_mem(S, j), nx));
      }
      best[S] = b;
    }
    std::vector<int> by_id(k);
    for (int j = 0; j < k; ++j) by_id[j] = j;
    std::stable_sort(by_id.begin(), by_id.end(), [&](int a, int b) {
      if (items[piece[a]].ref != items[piece[b]].ref) return items[piece[a]].ref < items[piece[b]].ref;
      return a < b;
    });
    std::vector<int> seq;
    uint32_t S = 0;
    int64_t target = best[0];
    while (S != full) {
      bool moved = false;
      for (int j : by_id) {
        if (((S >> j) & 1) || (deps[j] & ~S)) continue;
        int64_t nx = best[S | (1u << j)];
        if (nx == INF) continue;
        if (std::max(step_mem(S, j), nx) <= target) { seq.push_back(piece[j]); S |= 1u << j; moved = true; break; }
      }
      if (!moved) throw Error(SOD2_ERR_INVALID_ARG, "execution-order search found no valid order");
    }
    subgraphs.push_back(seq);
  }

  // In-place reuse (a refinement of the lifetime rule of Section 4.4.1): the result of a contraction
  // group with a residual operand, or of an elementwise group, takes over the storage of an operand r
  // when, on every path, (1) r is a group's result in the arena with the type and provably the shape
  // of the result, which lives in the arena too; (2) the group reads the storage of r through that
  // operand only (a kernel thread reads just the elements of r it is about to write) and stores
  // without a permutation; (3) the group is the last item in the planned order that reads the storage
  // of r and no Combine forwards r.
  inplace.assign(nt, -1);
  if (opts.inplace) {
    std::map<int, int> position;
    for (const auto& sg : subgraphs) for (int i : sg) { int k = (int)position.size(); position[i] = k; }
    std::set<int> combined, taken;
    std::map<int, std::vector<int>> readers;
    for (size_t i = 0; i < items.size(); ++i) {
      if (!items[i].is_group && G.ops[items[i].ref].kind == SOD2_OP_COMBINE) combined.insert(items[i].reads.begin(), items[i].reads.end());
      for (int t : items[i].reads) readers[t].push_back((int)i);
    }
    for (size_t i = 0; i < items.size(); ++i) {
      if (!items[i].is_group) continue;
      const Group& gr = groups.at(items[i].ref);
      if ((gr.kind != G_GEMM && gr.kind != G_CONV && gr.kind != G_ELTWISE) || !arena_candidate(gr.out)) continue;
      bool barred = false;
      for (int n : gr.ops) {
        int k = G.ops[n].kind;
        // (a LayerNorm that is the group's second result, R9, reads the finished rows: no bar)
        if (k == SOD2_OP_TRANSPOSE || (k == SOD2_OP_LAYERNORM && fold_y[G.ops[n].out[0]] != n) || k == SOD2_OP_CACHEAPPEND) barred = true;
      }
      if (barred) continue;
      std::set<int> inside;
      for (int n : gr.ops) for (int o : G.ops[n].out) inside.insert(o);
      std::vector<int> outer, cands;
      for (int n : gr.ops)
        for (int t : G.ops[n].in)
          if (!inside.count(t) && !inside.count(sbase[t])) {
            outer.push_back(t);
            if (gr.kind == G_ELTWISE || G.ops[n].kind == SOD2_OP_ADD) cands.push_back(t);
          }
      for (int r : cands) {
        const Tensor& d = G.tensors[r];
        if (d.role != SOD2_INTER || !arena_candidate(r) || combined.count(r) || taken.count(r)) continue;
        int pr = G.producer[r];
        if (pr < 0 || folded[pr] || view[pr] || is_control(G.ops[pr].kind) || is_counting(G.ops[pr].kind)) continue;
        if (groups.at(group_of_op[pr]).out != r) continue;
        if (d.dtype != G.tensors[gr.out].dtype || !shape_equal(R.S[r], R.S[gr.out])) continue;
        int through = 0;
        bool only_r = true;
        for (int t : outer) if (sbase[t] == r) { ++through; if (t != r) only_r = false; }
        if (through != 1 || !only_r) continue;
        bool last = true;
        for (int j : readers[r]) if (j != (int)i && position.at(j) > position.at((int)i)) last = false;
        if (!last) continue;
        inplace[gr.out] = r;
        taken.insert(r);
        break;
      }
    }
  }

  // flattened forms used by every bind
  for (const Symbol& sy : G.symbols) xc.symbols.push_back(sy.name);
  for (int n : order) if (is_counting(G.ops[n].kind)) exec_ops.push_back(n);
  for (int n : exec_ops) xc.symbols.push_back(exec_symbol(n));   // their values follow the graph symbols'
  cshape.assign(nt, {});
  for (int t = 0; t < nt; ++t) {
    if (!R.S[t].resolved()) continue;
    for (const LV& d : R.S[t].d) cshape[t].push_back(xc.compile(d.e));
  }
  item_ext.assign(items.size(), {});
  for (size_t i = 0; i < items.size(); ++i) {
    if (!items[i].is_group) continue;
    const Group& gr = groups.at(items[i].ref);
    std::set<int> inside;
    for (int n : gr.ops) for (int o : G.ops[n].out) inside.insert(o);
    for (int n : gr.ops)
      for (int t : G.ops[n].in)
        if (!inside.count(t) && !inside.count(sbase[t])) item_ext[i].push_back(t);     // a view of a member's result is internal
  }
}

std::string Plan::dump() const {
  std::string out = "order";
  for (int n : order) out += " " + std::to_string(n);
  out += "\nfolded";
  for (size_t i = 0; i < folded.size(); ++i) if (folded[i]) out += " " + std::to_string(i);
  out += "\nviews";
  for (size_t i = 0; i < view.size(); ++i) if (view[i]) out += " " + std::to_string(i);
  out += "\n";
  for (size_t t = 0; t < g->tensors.size(); ++t) {      // shapes that wait for an EDO to execute
    const LS& s = rdp->S[t];
    bool named_dim = false;
    if (s.is_list()) for (const auto& d : s.d) if (d.val() && mentions_exec(d.e)) named_dim = true;
    if (named_dim) out += "named t" + std::to_string(t) + " S=" + s.str() + "\n";
  }
  auto join = [](const std::vector<int>& v, const char* prefix) {
    std::string s;
    for (size_t i = 0; i < v.size(); ++i) { if (i) s += " "; s += prefix + std::to_string(v[i]); }
    return s;
  };
  for (const auto& it : items) {
    if (it.is_group) {
      const Group& gr = groups.at(it.ref);
      out += "g" + std::to_string(gr.gid) + " " + group_kind_name(gr.kind) + " ops=[" + join(gr.ops, "") + "] out=t" +
             std::to_string(gr.out);
      for (int t : gr.also) out += " also=t" + std::to_string(t);
      out += " ins=[" + join(gr.ins, "t") + "]";
      if (gr.versions > 1) {
        out += " versions=" + std::to_string(gr.versions) + " unproven=[";
        for (size_t k = 0; k < gr.unproven.size(); ++k)
          out += std::string(k ? " " : "") + "t" + std::to_string(gr.unproven[k].a) + "~t" + std::to_string(gr.unproven[k].b) + "@" +
                 std::to_string(gr.unproven[k].k);
        out += "]";
      }
      if (gr.lnfold >= 0) out += " lnfold=" + std::to_string(gr.lnfold);
      out += "\n";
    } else {
      out += "c" + std::to_string(it.ref) + " " + op_name(g->ops[it.ref].kind) + "\n";
    }
  }
  for (size_t t = 0; t < inplace.size(); ++t)
    if (inplace[t] >= 0) out += "inplace t" + std::to_string(t) + "=t" + std::to_string(inplace[t]) + "\n";
  for (size_t s = 0; s < subgraphs.size(); ++s) {
    out += "sg" + std::to_string(s) + " " + sg_class[s];
    for (int i : subgraphs[s]) out += std::string(" ") + (items[i].is_group ? "g" : "c") + std::to_string(items[i].ref);
    out += "\n";
  }
  return out;
}
}  // namespace sod2
