// Graph bookkeeping and Rank and Dimension Propagation (Section 4.1, Alg. 1).
//
// Every visit of an operator re-applies its transfer function and meets the result into the
// stored S-/V-map, so the fixed point is independent of the visiting order; the early return of
// Alg. 1 is the shortcut valid for the sorted order.  Switch forwards its data input's maps to
// all outputs, Combine takes the meet of its defined inputs, a backward transfer (of shapes, and of
// values through Shape and ConstantOfShape) assigns only
// what is unique, and whatever is still undef at the fixed point is lowered to nac.
#include <algorithm>
#include <functional>

#include "internal.hpp"

namespace sod2 {

static const char* kOpNames[SOD2_OP_COUNT] = {
    "Shape", "Gather", "Concat", "Reshape", "Slice", "Transpose", "MatMul", "Conv", "Add", "Mul", "Relu",
    "Gelu", "Sigmoid", "Cast", "Softmax", "LayerNorm", "ReduceMean", "MaxPool", "ArgMax", "CacheAppend",
    "NonZero", "Switch", "Combine", "ScatterRows", "Resize", "Range", "Expand", "Upsample", "ConstantOfShape",
    "EyeLike", "OneHot", "TopK", "GroupNorm", "MaxUnpool", "AveragePool", "Round", "NMS"};
const char* op_name(int kind) { return (kind >= 0 && kind < SOD2_OP_COUNT) ? kOpNames[kind] : "?"; }

int op_class(int kind) {   // Table 2
  switch (kind) {
    case SOD2_OP_SHAPE: case SOD2_OP_CONSTANTOFSHAPE: case SOD2_OP_EYELIKE: return 0;
    case SOD2_OP_RESHAPE: case SOD2_OP_SLICE: case SOD2_OP_RESIZE: case SOD2_OP_RANGE: case SOD2_OP_EXPAND:
    case SOD2_OP_ONEHOT: case SOD2_OP_UPSAMPLE: case SOD2_OP_TOPK: case SOD2_OP_GROUPNORM: case SOD2_OP_MAXUNPOOL: return 2;
    case SOD2_OP_NONZERO: case SOD2_OP_NMS: case SOD2_OP_SWITCH: case SOD2_OP_COMBINE: return 3;
    default: return 1;
  }
}
int dtype_bytes(int dtype) { return dtype == SOD2_BF16 ? 2 : (dtype == SOD2_I64 ? 8 : 4); }

void Graph::finish() {
  int nt = (int)tensors.size();
  producer.assign(nt, -1);
  consumers.assign(nt, {});
  for (int i = 0; i < (int)ops.size(); ++i) {
    for (int t : ops[i].out) {
      if (t < 0 || t >= nt) throw Error(SOD2_ERR_INVALID_ARG, "operator output id out of range");
      if (producer[t] >= 0) throw Error(SOD2_ERR_INVALID_ARG, "tensor written twice: " + tensors[t].name);
      producer[t] = i;
    }
    for (int t : ops[i].in) {
      if (t < 0 || t >= nt) throw Error(SOD2_ERR_INVALID_ARG, "operator input id out of range");
      consumers[t].push_back(i);
    }
  }
  weight_pos.assign(nt, -1);
  input_pos.assign(nt, -1);
  output_pos.assign(nt, -1);
  for (int t = 0; t < nt; ++t) {
    if (tensors[t].role == SOD2_WEIGHT) { weight_pos[t] = (int)weight_ids.size(); weight_ids.push_back(t); }
    if (tensors[t].role == SOD2_INPUT && !tensors[t].session) { input_pos[t] = (int)input_ids.size(); input_ids.push_back(t); }
    if (tensors[t].is_output) { output_pos[t] = (int)output_ids.size(); output_ids.push_back(t); }
    if (tensors[t].role == SOD2_INPUT && tensors[t].session) {
      // a session input lives in the arena; CacheAppend extends it in place, so nothing else may read it
      if (!tensors[t].declared || tensors[t].capacity.size() != tensors[t].dims.size())
        throw Error(SOD2_ERR_INVALID_ARG, "session input needs declared dims and capacity dims: " + tensors[t].name);
      for (int c : consumers[t])
        if (ops[c].kind != SOD2_OP_CACHEAPPEND || ops[c].in[0] != t || consumers[t].size() != 1)
          throw Error(SOD2_ERR_UNSUPPORTED, "a session input may only be extended by one CacheAppend: " + tensors[t].name);
      session_ids.push_back(t);
    }
  }
  for (const Op& op : ops)
    if (op.kind == SOD2_OP_CACHEAPPEND && !tensors[op.in[0]].session)
      throw Error(SOD2_ERR_UNSUPPORTED, "CacheAppend must extend a session tensor");
  for (int t = 0; t < nt; ++t)
    if (tensors[t].is_output && producer[t] < 0)
      throw Error(SOD2_ERR_INVALID_ARG, "graph output " + tensors[t].name + " is produced by no operator (an input, a weight or a "
                                        "dangling tensor cannot be an output: nothing would write the caller's buffer)");
  // the operators must form a directed acyclic graph: in the node order every input is produced earlier
  std::vector<int> order = sorted_nodes();
  std::vector<int> pos(ops.size(), -1);
  for (size_t i = 0; i < order.size(); ++i) pos[order[i]] = (int)i;
  for (size_t i = 0; i < ops.size(); ++i) {
    if (pos[i] < 0) throw Error(SOD2_ERR_INVALID_ARG, "operator unreachable from the graph inputs (or on a cycle)");
    for (int t : ops[i].in)
      if (producer[t] >= 0 && pos[producer[t]] >= pos[i])
        throw Error(SOD2_ERR_INVALID_ARG, "the graph has a cycle through " + tensors[t].name);
  }
}

std::vector<int> Graph::sorted_nodes() const {
  int n = (int)ops.size();
  std::vector<std::vector<int>> succ(n);
  for (int i = 0; i < n; ++i) {
    std::set<int> s;
    for (int t : ops[i].out) for (int c : consumers[t]) s.insert(c);
    succ[i].assign(s.begin(), s.end());
  }
  std::vector<char> seen(n, 0);
  std::vector<int> post;
  for (int r = 0; r < n; ++r) {
    bool root = true;
    for (int t : ops[r].in) if (producer[t] >= 0) root = false;
    if (!root || seen[r]) continue;
    seen[r] = 1;
    std::vector<std::pair<int, size_t>> stack{{r, 0}};
    while (!stack.empty()) {
      int u = stack.back().first;
      size_t k = stack.back().second;
      if (k < succ[u].size()) {
        stack.back().second = k + 1;
        int v = succ[u][k];
        if (!seen[v]) { seen[v] = 1; stack.push_back({v, 0}); }
      } else {
        post.push_back(u);
        stack.pop_back();
      }
    }
  }
  std::reverse(post.begin(), post.end());
  return post;
}

// ---- dim arithmetic on lattice values: nac absorbs, then undef ---------------------------------
namespace {
const int64_t kIntMax = 2147483647LL;

template <class F> LV arith(const LV& a, const LV& b, F f) {
  if (a.k == LV::NAC || b.k == LV::NAC) return LV::nac();
  if (a.k == LV::UNDEF || b.k == LV::UNDEF) return LV::undef();
  return f(a.e, b.e);
}
LV add(const LV& a, const LV& b) { return arith(a, b, [](const Expr& x, const Expr& y) { return LV::of(x + y); }); }
LV sub(const LV& a, const LV& b) { return arith(a, b, [](const Expr& x, const Expr& y) { return LV::of(x - y); }); }
LV mul(const LV& a, const LV& b) { return arith(a, b, [](const Expr& x, const Expr& y) { return LV::of(x * y); }); }
LV fdiv(const LV& a, int64_t c) { return a.val() ? LV::of(a.e.floordiv(c)) : a; }

LV bcast_dim(const LV& a, const LV& b) {
  if (a.val() && b.val()) {
    if (a.e == b.e) return a;
    if (a.is_c(1)) return b;
    if (b.is_c(1)) return a;
    if (a.e.is_const() && b.e.is_const())
      throw Error(SOD2_ERR_SHAPE_MISMATCH, "cannot broadcast " + a.e.str() + " with " + b.e.str());
    // unproven: equal, or one of them 1 (Fig. 4); the extent is still a function of the symbols -- an
    // operation-inferred constant, evaluated and checked when they are bound
    return LV::of(a.e.bcast(b.e));
  }
  // a known constant other than 1 fixes the output whatever the other side turns out to be
  if (a.val() && a.e.is_const() && a.e.const_value() != 1) return a;
  if (b.val() && b.e.is_const() && b.e.const_value() != 1) return b;
  if (a.k == LV::UNDEF || b.k == LV::UNDEF) return LV::undef();
  return LV::nac();
}
std::vector<LV> bcast(std::vector<LV> a, std::vector<LV> b) {
  size_t r = std::max(a.size(), b.size());
  a.insert(a.begin(), r - a.size(), LV::c(1));
  b.insert(b.begin(), r - b.size(), LV::c(1));
  std::vector<LV> o;
  for (size_t i = 0; i < r; ++i) o.push_back(bcast_dim(a[i], b[i]));
  return o;
}
LV window(const LV& d, int64_t k, int64_t stride, int64_t pad) {   // floor((d + 2p - k)/s) + 1
  return add(fdiv(add(d, LV::c(2 * pad - k)), stride), LV::c(1));
}
int64_t norm_axis(int64_t a, size_t rank) {         // an axis or an index in [-rank, rank)
  int64_t r = (int64_t)rank;
  if (a < -r || a >= r) throw Error(SOD2_ERR_SHAPE_MISMATCH, "axis or index " + std::to_string(a) + " outside a rank or length of " + std::to_string(r));
  return a < 0 ? a + r : a;
}

struct Out { bool ready = false; LS s, v; };     // result of one forward transfer
}  // namespace

// ---- the analysis ------------------------------------------------------------------------------
namespace {
struct Analyser {
  const Graph& g;
  std::vector<LS>& S;
  std::vector<LS>& V;
  bool named_edo;
  Analyser(const Graph& g_, std::vector<LS>& s, std::vector<LS>& v, bool named) : g(g_), S(s), V(v), named_edo(named) {}

  bool refine(std::vector<LS>& store, int t, const LS& nw) {
    if (nw.k == LS::UNDEF) return false;
    LS upd = meet(store[t], nw);
    if (upd.same(store[t])) return false;
    store[t] = upd;
    return true;
  }

  Out forward(const Op& op, int op_id) {
    Out r;
    auto in_s = [&](int k) -> const LS& { return S[op.in[k]]; };
    auto in_v = [&](int k) -> const LS& { return V[op.in[k]]; };
    auto done = [&](const LS& s, const LS& v = LS::undef()) { r.ready = true; r.s = s; r.v = v; return r; };
    switch (op.kind) {
      case SOD2_OP_SHAPE: {
        const LS& x = in_s(0);
        if (x.k == LS::UNDEF) return r;
        if (x.k == LS::NAC) return done(LS::nac(), LS::nac());
        return done(LS::list({LV::c((int64_t)x.d.size())}), LS::list(x.d));   // ISDO: value = input shape
      }
      case SOD2_OP_RELU: case SOD2_OP_GELU: case SOD2_OP_SIGMOID: case SOD2_OP_ROUND: case SOD2_OP_CAST:
      case SOD2_OP_SOFTMAX: case SOD2_OP_LAYERNORM: case SOD2_OP_GROUPNORM: {
        if (in_s(0).k == LS::UNDEF) return r;
        return done(in_s(0));
      }
      case SOD2_OP_TRANSPOSE: {
        const LS& x = in_s(0);
        if (x.k == LS::UNDEF) return r;
        if (x.k == LS::NAC) return done(LS::nac());
        if (op.ia.size() != x.d.size()) throw Error(SOD2_ERR_SHAPE_MISMATCH, "Transpose rank");
        LS o = LS::list({});
        for (int64_t p : op.ia) o.d.push_back(x.d[p]);
        return done(o);
      }
      case SOD2_OP_GATHER: {
        const LS &d = in_s(0), &i = in_s(1);
        if (d.k == LS::UNDEF || i.k == LS::UNDEF) return r;
        if (d.k == LS::NAC || i.k == LS::NAC) return done(LS::nac(), LS::nac());
        size_t ax = norm_axis(op.ia.at(0), d.d.size());
        LS o = LS::list({});
        o.d.insert(o.d.end(), d.d.begin(), d.d.begin() + ax);
        o.d.insert(o.d.end(), i.d.begin(), i.d.end());
        o.d.insert(o.d.end(), d.d.begin() + ax + 1, d.d.end());
        LS v;
        const LS &dv = in_v(0), &iv = in_v(1);
        if (dv.is_list() && iv.is_list() && d.d.size() == 1) {
          bool all_c = true;
          for (const auto& e : iv.d) if (!(e.val() && e.e.is_const())) all_c = false;
          if (all_c) {
            v = LS::list({});
            for (const auto& e : iv.d) v.d.push_back(dv.d[norm_axis(e.e.const_value(), dv.d.size())]);
          } else v = LS::nac();
        } else if (dv.k == LS::NAC || iv.k == LS::NAC) v = LS::nac();
        return done(o, v);
      }
      case SOD2_OP_CONCAT: {
        for (size_t k = 0; k < op.in.size(); ++k) if (in_s(k).k == LS::UNDEF) return r;
        for (size_t k = 0; k < op.in.size(); ++k) if (in_s(k).k == LS::NAC) return done(LS::nac(), LS::nac());
        size_t rank = in_s(0).d.size();
        for (size_t k = 0; k < op.in.size(); ++k)
          if (in_s(k).d.size() != rank) throw Error(SOD2_ERR_SHAPE_MISMATCH, "Concat rank");
        size_t ax = norm_axis(op.ia.at(0), rank);
        LS o = LS::list({});
        for (size_t j = 0; j < rank; ++j) {
          LV acc = (j == ax) ? LV::c(0) : LV::undef();
          for (size_t k = 0; k < op.in.size(); ++k)
            acc = (j == ax) ? add(acc, in_s(k).d[j]) : meet(acc, in_s(k).d[j]);
          o.d.push_back(acc);
        }
        LS v;
        bool all_list = rank == 1, any_nac = false;
        for (size_t k = 0; k < op.in.size(); ++k) {
          if (!in_v(k).is_list()) all_list = false;
          if (in_v(k).k == LS::NAC) any_nac = true;
        }
        if (all_list) {
          v = LS::list({});
          for (size_t k = 0; k < op.in.size(); ++k) v.d.insert(v.d.end(), in_v(k).d.begin(), in_v(k).d.end());
        } else if (any_nac) v = LS::nac();
        return done(o, v);
      }
      case SOD2_OP_RESHAPE: {
        const LS &x = in_s(0), &ts = in_s(1), &tv = in_v(1);
        if (x.k == LS::UNDEF || ts.k == LS::UNDEF || tv.k == LS::UNDEF) return r;
        if (tv.k == LS::NAC) {                       // only the rank may be known
          if (ts.is_list() && ts.d[0].val() && ts.d[0].e.is_const())
            return done(LS::list(std::vector<LV>((size_t)ts.d[0].e.const_value(), LV::nac())));
          return done(LS::nac());
        }
        LS o = LS::list({});
        int infer = -1;
        for (size_t k = 0; k < tv.d.size(); ++k) {
          const LV& e = tv.d[k];
          if (e.is_c(0)) o.d.push_back((x.is_list() && k < x.d.size()) ? x.d[k] : LV::nac());
          else if (e.is_c(-1)) { infer = (int)k; o.d.push_back(LV::undef()); }
          else o.d.push_back(e);
        }
        if (infer >= 0) {
          if (x.k == LS::NAC) o.d[infer] = LV::nac();
          else {
            LV total = LV::c(1), known = LV::c(1);
            for (const auto& d : x.d) total = mul(total, d);
            for (size_t k = 0; k < o.d.size(); ++k) if ((int)k != infer) known = mul(known, o.d[k]);
            if (total.k == LV::UNDEF || known.k == LV::UNDEF) return r;
            Expr q;
            if (total.k == LV::NAC || known.k == LV::NAC) o.d[infer] = LV::nac();
            else o.d[infer] = total.e.exact_div(known.e, &q) ? LV::of(q) : LV::nac();
          }
        }
        return done(o);
      }
      case SOD2_OP_SLICE: {
        const LS& x = in_s(0);
        const LS &st = in_v(1), &en = in_v(2), &ax = in_v(3);
        if (x.k == LS::UNDEF || st.k == LS::UNDEF || en.k == LS::UNDEF || ax.k == LS::UNDEF) return r;
        if (x.k == LS::NAC || !ax.is_list() || !st.is_list() || !en.is_list()) return done(LS::nac(), LS::nac());
        LS o = x;
        bool have0 = false, bad0 = false;
        LV lo0, hi0;
        for (size_t k = 0; k < ax.d.size(); ++k) {
          size_t a = norm_axis(ax.d[k].e.const_value(), x.d.size());
          const LV &s = st.d[k], &e = en.d[k];
          const LV& D = x.d[a];
          if (!(s.val() && e.val())) {
            o.d[a] = LV::nac();
            if (k == 0) bad0 = true;
            continue;
          }
          // a constant bound follows the usual conventions (negative: from the end; INT_MAX: the end); a computed one
          // (an expression from the value map) is a position as it stands, range-checked when it is bound
          LV lo = s, hi = e;
          if (s.e.is_const() && s.e.const_value() < 0) lo = add(D, s);
          if (e.e.is_const()) {
            const int64_t ev = e.e.const_value();
            hi = ev >= kIntMax ? D : (ev < 0 ? add(D, e) : e);
          }
          o.d[a] = sub(hi, lo);
          if (k == 0) { have0 = true; lo0 = lo; hi0 = hi; }
        }
        LS v;
        const LS& xv = in_v(0);
        if (xv.is_list() && x.d.size() == 1 && have0 && !bad0) {
          if (lo0.val() && hi0.val() && lo0.e.is_const() && hi0.e.is_const()) {
            v = LS::list({});
            for (int64_t k = lo0.e.const_value(); k < hi0.e.const_value() && k < (int64_t)xv.d.size(); ++k)
              v.d.push_back(xv.d[k]);
          } else v = LS::nac();
        }
        return done(o, v);
      }
      case SOD2_OP_MATMUL: {
        const LS &a = in_s(0), &b = in_s(1);
        if (a.k == LS::UNDEF || b.k == LS::UNDEF) return r;
        if (a.k == LS::NAC || b.k == LS::NAC) return done(LS::nac());
        if (a.d.size() < 2 || b.d.size() < 2) throw Error(SOD2_ERR_SHAPE_MISMATCH, "MatMul needs rank >= 2");
        bool tb = !op.ia.empty() && op.ia[0];
        const LV& n = tb ? b.d[b.d.size() - 2] : b.d.back();
        const LV& kb = tb ? b.d.back() : b.d[b.d.size() - 2];
        meet(a.d.back(), kb);                          // throws when two known constants differ
        std::vector<LV> o = bcast(std::vector<LV>(a.d.begin(), a.d.end() - 2), std::vector<LV>(b.d.begin(), b.d.end() - 2));
        o.push_back(a.d[a.d.size() - 2]);
        o.push_back(n);
        return done(LS::list(o));
      }
      case SOD2_OP_CONV: {
        const LS &x = in_s(0), &w = in_s(1);
        if (x.k == LS::UNDEF || w.k == LS::UNDEF) return r;
        if (x.k == LS::NAC || w.k == LS::NAC) return done(LS::nac());
        if (x.d.size() != 4 || w.d.size() != 4) throw Error(SOD2_ERR_SHAPE_MISMATCH, "Conv needs rank 4");
        meet(x.d[3], w.d[3]);
        int64_t s = op.ia.at(0), p = op.ia.at(1);
        if (!(w.d[1].val() && w.d[1].e.is_const() && w.d[2].val() && w.d[2].e.is_const()))
          throw Error(SOD2_ERR_UNSUPPORTED, "Conv kernel size must be a known constant");
        return done(LS::list({x.d[0], window(x.d[1], w.d[1].e.const_value(), s, p),
                              window(x.d[2], w.d[2].e.const_value(), s, p), w.d[0]}));
      }
      case SOD2_OP_MAXPOOL: case SOD2_OP_AVERAGEPOOL: {
        const LS& x = in_s(0);
        if (x.k == LS::UNDEF) return r;
        if (x.k == LS::NAC) return done(LS::nac());
        int64_t k = op.ia.at(0), s = op.ia.at(1), p = op.ia.at(2);
        return done(LS::list({x.d[0], window(x.d[1], k, s, p), window(x.d[2], k, s, p), x.d[3]}));
      }
      case SOD2_OP_ADD: case SOD2_OP_MUL: {
        const LS &a = in_s(0), &b = in_s(1);
        if (a.k == LS::NAC || b.k == LS::NAC) return done(LS::nac(), LS::nac());
        if (a.k == LS::UNDEF || b.k == LS::UNDEF) return r;
        LS v;
        const LS &av = in_v(0), &bv = in_v(1);
        if (av.is_list() && bv.is_list() && a.d.size() <= 1 && b.d.size() <= 1 && !av.d.empty() && !bv.d.empty()) {
          size_t n = std::max(av.d.size(), bv.d.size());
          if ((av.d.size() == 1 || av.d.size() == n) && (bv.d.size() == 1 || bv.d.size() == n)) {
            v = LS::list({});
            for (size_t i = 0; i < n; ++i) {
              const LV &x = av.d[i % av.d.size()], &y = bv.d[i % bv.d.size()];
              v.d.push_back(op.kind == SOD2_OP_ADD ? add(x, y) : mul(x, y));
            }
          }
        }
        return done(LS::list(bcast(a.d, b.d)), v);
      }
      case SOD2_OP_REDUCEMEAN: {
        const LS& x = in_s(0);
        if (x.k == LS::UNDEF) return r;
        if (x.k == LS::NAC) return done(LS::nac());
        std::set<size_t> axes;
        for (size_t k = 1; k < op.ia.size(); ++k) axes.insert(norm_axis(op.ia[k], x.d.size()));
        LS o = LS::list({});
        for (size_t k = 0; k < x.d.size(); ++k) {
          if (!axes.count(k)) o.d.push_back(x.d[k]);
          else if (op.ia.at(0)) o.d.push_back(LV::c(1));
        }
        return done(o);
      }
      case SOD2_OP_ARGMAX: {
        const LS& x = in_s(0);
        if (x.k == LS::UNDEF) return r;
        if (x.k == LS::NAC) return done(LS::nac());
        return done(LS::list(std::vector<LV>(x.d.begin(), x.d.end() - 1)));
      }
      case SOD2_OP_CACHEAPPEND: {
        const LS &p = in_s(0), &n = in_s(1);
        if (p.k == LS::UNDEF || n.k == LS::UNDEF) return r;
        if (p.k == LS::NAC || n.k == LS::NAC) return done(LS::nac());
        LS o = LS::list({add(p.d[0], n.d[0])});
        for (size_t k = 1; k < p.d.size() && k < n.d.size(); ++k) o.d.push_back(meet(p.d[k], n.d[k]));
        return done(o);
      }
      case SOD2_OP_NONZERO: {                            // execution determined
        if (!named_edo) return done(LS::nac(), LS::nac());
        // the extent is unknown until the operator has run and a constant afterwards: give it a name
        const LS& x = in_s(0);
        if (x.k == LS::UNDEF) return r;
        if (x.k == LS::NAC) return done(LS::nac(), LS::nac());
        return done(LS::list({LV::c((int64_t)x.d.size()), LV::of(Expr::symbol(exec_symbol(op_id)))}), LS::nac());
      }
      case SOD2_OP_NMS: {                                // execution determined: how many boxes are kept
        if (!named_edo) return done(LS::nac(), LS::nac());
        if (in_s(0).k == LS::UNDEF) return r;
        return done(LS::list({LV::of(Expr::symbol(exec_symbol(op_id)))}), LS::nac());
      }
      case SOD2_OP_RANGE: {          // length ceil((limit - start) / delta) for a known positive delta (limit >= start assumed)
        for (int k = 0; k < 3; ++k) if (in_v(k).k == LS::UNDEF) return r;
        bool ok = true;
        for (int k = 0; k < 3; ++k) if (!in_v(k).is_list() || in_v(k).d.size() != 1 || !in_v(k).d[0].val()) ok = false;
        if (!ok || !in_v(2).d[0].e.is_const() || in_v(2).d[0].e.const_value() <= 0)
          return done(LS::list({LV::nac()}), LS::nac());
        const Expr &start = in_v(0).d[0].e, &limit = in_v(1).d[0].e;
        const int64_t d = in_v(2).d[0].e.const_value();
        Expr n = (limit - start + Expr::constant(d - 1)).floordiv(d);
        if (n.is_const() && n.const_value() < 0) n = Expr::constant(0);
        LS v = LS::nac();
        if (n.is_const() && n.const_value() <= 16) {
          v = LS::list({});
          for (int64_t i = 0; i < n.const_value(); ++i) v.d.push_back(LV::of(start + Expr::constant(i * d)));
        }
        return done(LS::list({LV::of(n)}), v);
      }
      case SOD2_OP_EXPAND: {         // broadcast of input 0 against the shape held by the values of input 1
        const LS &x = in_s(0), &tv = in_v(1);
        if (x.k == LS::UNDEF || tv.k == LS::UNDEF) return r;
        if (!x.is_list() || !tv.is_list()) return done(LS::nac());
        return done(LS::list(bcast(x.d, tv.d)));
      }
      case SOD2_OP_RESIZE: {                             // output shape = the values of the sizes input (ISVDOS)
        const LS &x = in_s(0), &ts = in_s(1), &tv = in_v(1);
        if (x.k == LS::UNDEF || ts.k == LS::UNDEF || tv.k == LS::UNDEF) return r;
        if (tv.is_list()) {
          if (x.is_list() && x.d.size() != tv.d.size()) throw Error(SOD2_ERR_SHAPE_MISMATCH, "Resize rank");
          return done(LS::list(tv.d));
        }
        if (x.is_list()) return done(LS::list(std::vector<LV>(x.d.size(), LV::nac())));   // the rank survives
        return done(LS::nac());
      }
      case SOD2_OP_MAXUNPOOL: {                          // output shape = the values of the output_shape input (ISVDOS)
        const LS &x = in_s(0), &ts = in_s(2), &tv = in_v(2);
        if (x.k == LS::UNDEF || ts.k == LS::UNDEF || tv.k == LS::UNDEF) return r;
        if (tv.is_list()) {
          if (x.is_list() && x.d.size() != tv.d.size()) throw Error(SOD2_ERR_SHAPE_MISMATCH, "MaxUnpool rank");
          return done(LS::list(tv.d));
        }
        if (x.is_list()) return done(LS::list(std::vector<LV>(x.d.size(), LV::nac())));
        return done(LS::nac());
      }
      case SOD2_OP_CONSTANTOFSHAPE: {                    // shape = the values of the input, every element the attribute
        const LS &ts = in_s(0), &tv = in_v(0);
        if (ts.k == LS::UNDEF || tv.k == LS::UNDEF) return r;
        if (tv.is_list()) {
          LS v = LS::undef();
          bool consts = tv.d.size() <= 1;
          for (const LV& d : tv.d) if (!d.val() || !d.e.is_const()) consts = false;
          if (consts) {
            int64_t n = tv.d.empty() ? 1 : tv.d[0].e.const_value();
            if (n <= 16) v = LS::list(std::vector<LV>((size_t)std::max<int64_t>(n, 0), LV::c((int64_t)op.fa)));
          }
          return done(LS::list(tv.d), v);
        }
        if (ts.is_list() && ts.d.size() == 1 && ts.d[0].val() && ts.d[0].e.is_const())   // the rank is the shape tensor's length
          return done(LS::list(std::vector<LV>((size_t)ts.d[0].e.const_value(), LV::nac())));
        return done(LS::nac());
      }
      case SOD2_OP_EYELIKE: {
        const LS& x = in_s(0);
        if (x.k == LS::UNDEF) return r;
        if (x.is_list() && x.d.size() != 2) throw Error(SOD2_ERR_SHAPE_MISMATCH, "EyeLike needs a matrix");
        return done(x);
      }
      case SOD2_OP_ONEHOT: {                             // indices.shape + [depth], the depth from the value of input 1
        const LS &x = in_s(0), &dv = in_v(1);
        if (x.k == LS::UNDEF || dv.k == LS::UNDEF) return r;
        if (!x.is_list()) return done(LS::nac());
        std::vector<LV> d = x.d;
        d.push_back(dv.is_list() && dv.d.size() == 1 && dv.d[0].val() ? dv.d[0] : LV::nac());
        return done(LS::list(d));
      }
      case SOD2_OP_TOPK: {                               // both results: the input's shape, last extent = the value of input 1
        const LS &x = in_s(0), &kv = in_v(1);
        if (x.k == LS::UNDEF || kv.k == LS::UNDEF) return r;
        if (!x.is_list()) return done(LS::nac());
        if (x.d.empty()) throw Error(SOD2_ERR_SHAPE_MISMATCH, "TopK of a scalar");
        std::vector<LV> d(x.d.begin(), x.d.end() - 1);
        d.push_back(kv.is_list() && kv.d.size() == 1 && kv.d[0].val() ? kv.d[0] : LV::nac());
        return done(LS::list(d));
      }
      case SOD2_OP_UPSAMPLE: {                           // every extent times its whole-number factor (a host constant)
        const Tensor& sc = g.tensors[op.in[1]];
        if (!sc.has_data || sc.fdata.empty()) throw Error(SOD2_ERR_SHAPE_MISMATCH, "Upsample factors must be whole host constants >= 1");
        for (double f : sc.fdata) if (f != (double)(int64_t)f || f < 1) throw Error(SOD2_ERR_SHAPE_MISMATCH, "Upsample factors must be whole host constants >= 1");
        const LS& x = in_s(0);
        if (x.k == LS::UNDEF) return r;
        if (!x.is_list()) return done(LS::nac());
        if (x.d.size() != sc.fdata.size()) throw Error(SOD2_ERR_SHAPE_MISMATCH, "Upsample rank");
        std::vector<LV> d;
        for (size_t i = 0; i < x.d.size(); ++i) d.push_back(mul(x.d[i], LV::c((int64_t)sc.fdata[i])));
        return done(LS::list(d));
      }
      case SOD2_OP_SCATTERROWS: {                        // a copy of input 0 with some rows replaced
        if (in_s(0).k == LS::UNDEF) return r;
        return done(in_s(0));
      }
      default:
        throw Error(SOD2_ERR_UNSUPPORTED, std::string("no transfer function for ") + op_name(op.kind));
    }
  }

  // IV <- F^bv(OV): the values of input t, as many as it has elements (a vector or a scalar, known to RDP)
  bool backward_values(int t, LS vals) {
    const LS& s = S[t];
    if (!vals.is_list() || !s.is_list() || s.d.size() > 1) return false;
    if (s.d.size() == 1 && !(s.d[0].k == LV::VAL && s.d[0].e.is_const() && s.d[0].e.const_value() == (int64_t)vals.d.size())) return false;
    if (s.d.empty() && vals.d.size() != 1) return false;
    for (auto& d : vals.d) if (d.k == LV::NAC) d = LV::undef();
    return refine(V, t, vals);
  }

  // IS <- F^bs(OS), only where the answer is unique (Section 3: Add is ambiguous, so nothing)
  bool backward(const Op& op, int k) {
    const LS& out = S[op.out[0]];
    LS nw;
    bool ch0 = false;
    const Graph& G = g;
    switch (op.kind) {
      case SOD2_OP_SHAPE:                               // backward value transfer: the result's value is the input's shape
        if (k == 0 && V[op.out[0]].is_list()) nw = V[op.out[0]];
        break;
      case SOD2_OP_CONSTANTOFSHAPE: {                   // the result's shape is the value of the input
        if (k != 0 || !out.is_list()) return false;
        LS v = out;
        for (auto& d : v.d) if (d.k == LV::NAC) d = LV::undef();
        bool ch = refine(V, op.in[0], v);
        return refine(S, op.in[0], LS::list({LV::c((int64_t)out.d.size())})) || ch;
      }
      case SOD2_OP_RELU: case SOD2_OP_GELU: case SOD2_OP_SIGMOID: case SOD2_OP_ROUND: case SOD2_OP_CAST:
      case SOD2_OP_SOFTMAX: case SOD2_OP_LAYERNORM: case SOD2_OP_GROUPNORM:
        if (k == 0 && out.is_list()) nw = out;
        if (k == 0 && op.kind == SOD2_OP_CAST && is_int(G.tensors[op.in[0]].dtype) && is_int(G.tensors[op.out[0]].dtype))
          ch0 = backward_values(op.in[0], V[op.out[0]]);   // F^bv: an integer Cast changes no value
        break;
      case SOD2_OP_ADD: {
        // F^bv: with the other operand's values known, in = out - other (unique when this operand has as many
        // elements as the result: a broadcast one could not be told from its repeats)
        if (!is_int(G.tensors[op.in[k]].dtype)) return false;
        const LS &ov = V[op.out[0]], &other = V[op.in[1 - k]];
        if (!ov.is_list() || !other.is_list() || !(other.d.size() == 1 || other.d.size() == ov.d.size())) return false;
        for (const auto& d : other.d) if (d.k != LV::VAL) return false;
        LS vals = LS::list({});
        for (size_t i = 0; i < ov.d.size(); ++i) vals.d.push_back(sub(ov.d[i], other.d[i % other.d.size()]));
        return backward_values(op.in[k], vals);
      }
      case SOD2_OP_CONCAT: {
        // F^bv: input k of a Concat of vectors holds the elements behind those of the inputs before it
        if (!is_int(G.tensors[op.in[k]].dtype)) return false;
        const LS& ov = V[op.out[0]];
        if (!ov.is_list()) return false;
        std::vector<int64_t> n;
        for (int t : op.in) {
          const LS& x = S[t];
          if (!x.is_list() || x.d.size() != 1 || x.d[0].k != LV::VAL || !x.d[0].e.is_const()) return false;
          n.push_back(x.d[0].e.const_value());
        }
        int64_t before = 0, total = 0;
        for (size_t i = 0; i < n.size(); ++i) { if ((int)i < k) before += n[i]; total += n[i]; }
        if (total != (int64_t)ov.d.size()) return false;
        LS vals = LS::list(std::vector<LV>(ov.d.begin() + before, ov.d.begin() + before + n[k]));
        return backward_values(op.in[k], vals);
      }
      case SOD2_OP_TRANSPOSE:
        if (out.is_list()) {
          nw = LS::list(std::vector<LV>(op.ia.size()));
          for (size_t i = 0; i < op.ia.size(); ++i) nw.d[op.ia[i]] = out.d[i];
        }
        break;
      case SOD2_OP_MATMUL:
        if (k == 0) {
          const LS& b = S[op.in[1]];
          if (b.is_list() && b.d.size() == 2) {
            bool tb = !op.ia.empty() && op.ia[0];
            const LV& kd = tb ? b.d[1] : b.d[0];
            if (out.is_list()) {
              nw = LS::list(std::vector<LV>(out.d.begin(), out.d.end() - 1));
              nw.d.push_back(kd);
            } else if (S[op.in[0]].is_list()) {
              nw = LS::list(std::vector<LV>(S[op.in[0]].d.size() - 1));
              nw.d.push_back(kd);
            }
          }
        }
        break;
      case SOD2_OP_CONV:
        if (k == 0 && S[op.in[1]].is_list())
          nw = LS::list({out.is_list() ? out.d[0] : LV::undef(), LV::undef(), LV::undef(), S[op.in[1]].d[3]});
        break;
      default:
        break;
    }
    if (nw.k != LS::LIST) return ch0;
    for (auto& d : nw.d) if (d.k == LV::NAC) d = LV::undef();   // a nac carries no backward information
    return refine(S, op.in[k], nw) || ch0;
  }
};
}  // namespace

void Rdp::analyse(const std::vector<int>* order_in) {
  const Graph& gr = *g;
  size_t nt = gr.tensors.size();
  S.assign(nt, LS::undef());
  V.assign(nt, LS::undef());
  std::vector<int> order = order_in ? *order_in : gr.sorted_nodes();
  for (size_t i = 0; i < nt; ++i) {                   // set_model_input_shape
    const Tensor& t = gr.tensors[i];
    if (t.declared) {
      S[i] = LS::list({});
      for (const auto& d : t.dims) S[i].d.push_back(LV::of(Expr::parse(d)));
    }
    if (t.has_data && is_int(t.dtype) && t.idata.size() <= 16 && t.host_rank <= 1) {
      V[i] = LS::list({});
      for (int64_t v : t.idata) V[i].d.push_back(LV::c(v));
    }
  }
  Analyser A(gr, S, V, named_edo);
  bool changed = true;
  sweeps = 0;
  while (changed) {
    changed = false;
    ++sweeps;
    for (int n : order) {
      const Op& op = gr.ops[n];
      if (op.kind == SOD2_OP_COMBINE) {               // Merge
        LS s, v;
        for (int t : op.in) {
          s = meet(s, S[t]);
          if (V[t].k != LS::UNDEF) v = meet(v, V[t]);
        }
        for (int o : op.out) { changed |= A.refine(S, o, s); changed |= A.refine(V, o, v); }
        continue;
      }
      if (op.kind == SOD2_OP_SWITCH) {                // transit to all successors
        for (int o : op.out) { changed |= A.refine(S, o, S[op.in[0]]); changed |= A.refine(V, o, V[op.in[0]]); }
        for (int o : op.out) changed |= A.refine(S, op.in[0], S[o]);
        continue;
      }
      Out r = A.forward(op, n);
      if (r.ready) {
        for (int o : op.out) {
          changed |= A.refine(S, o, r.s);
          if (is_int(gr.tensors[o].dtype)) changed |= A.refine(V, o, r.v);
        }
      }
      for (size_t k = 0; k < op.in.size(); ++k)
        if (S[op.in[k]].has_undef() || (is_int(gr.tensors[op.in[k]].dtype) && V[op.in[k]].has_undef()))
          changed |= A.backward(op, (int)k);
    }
  }
  for (auto* store : {&S, &V})
    for (auto& x : *store) {
      if (x.k == LS::UNDEF) x = LS::nac();
      else if (x.k == LS::LIST) for (auto& e : x.d) if (e.k == LV::UNDEF) e = LV::nac();
    }
}

std::string Rdp::dump() const {
  std::string out;
  for (size_t i = 0; i < g->tensors.size(); ++i) {
    const Tensor& t = g->tensors[i];
    out += "t" + std::to_string(i) + " " + t.name + " S=" + S[i].str() + " V=" + (is_int(t.dtype) ? V[i].str() : "-") + "\n";
  }
  return out;
}
}  // namespace sod2
