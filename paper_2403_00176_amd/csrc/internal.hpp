// Host-side data structures of the SoD2 library: symbolic expressions, the RDP lattice,
// the graph, the static plan and a binding.  Device code lives in kernels.hip / run.hip.
#pragma once
#include <algorithm>
#include <cstdint>
#include <map>
#include <memory>
#include <set>
#include <stdexcept>
#include <string>
#include <vector>

#include "../../include/sod2.h"

namespace sod2 {

struct Error : std::runtime_error {
  int code;
  Error(int c, const std::string& m) : std::runtime_error(m), code(c) {}
};

// ---------------------------------------------------------------------------------------------
// Expressions: polynomials with integer coefficients over atoms (symbols, unsimplified floordiv /
// mod, and bcast(a, b): the extent two unrelated dims broadcast to, checked when the symbols are bound).  These are the "operation-inferred constants" of the RDP domain (Section 4.1, V').
// ---------------------------------------------------------------------------------------------
struct Expr {
  typedef std::vector<std::string> Mono;           // sorted atom names
  std::map<Mono, int64_t> terms;                   // no zero coefficients

  static Expr constant(int64_t c);
  static Expr symbol(const std::string& name);
  static Expr parse(const std::string& text);      // int | symbol | sum of those

  bool is_const() const;
  int64_t const_value() const;
  bool is_symbol() const;
  int cls() const;                                 // 0 known, 1 symbolic, 2 operation-inferred
  std::string str() const;                         // canonical text
  bool operator==(const Expr& o) const { return terms == o.terms; }
  bool operator!=(const Expr& o) const { return !(*this == o); }

  Expr operator+(const Expr& o) const;
  Expr operator-(const Expr& o) const;
  Expr operator*(const Expr& o) const;
  Expr floordiv(int64_t c) const;
  Expr mod(int64_t c) const;
  Expr bcast(const Expr& o) const;                 // extent of the broadcast of two aligned dims (Section 4.2, Fig. 4)
  bool exact_div(const Expr& o, Expr* q) const;    // o a single term dividing every term
  int64_t eval(const std::map<std::string, int64_t>& env) const;
};

// Expressions flattened for repeated evaluation at bind: atoms become indices into a table whose
// values are computed once per binding (inner expressions of floordiv / mod before their users).
struct CompiledExpr {
  struct Term { int64_t coef; std::vector<int> atoms; };
  std::vector<Term> terms;
  int64_t eval(const std::vector<int64_t>& atom_vals) const {
    int64_t total = 0;
    for (const Term& t : terms) {
      int64_t v = t.coef;
      for (int a : t.atoms) v *= atom_vals[a];
      total += v;
    }
    return total;
  }
};
struct ExprCompiler {
  struct Atom { int kind; int sym; int64_t c; CompiledExpr inner, inner2; std::string name; };   // 0 symbol, 1 floordiv, 2 mod, 3 bcast
  std::vector<std::string> symbols;                // position = index of the value handed to atom_values
  std::vector<Atom> atoms;
  std::map<std::string, int> index;
  CompiledExpr compile(const Expr& e);
  void atom_values(const std::vector<int64_t>& symbol_values, std::vector<int64_t>* out) const;
 private:
  int intern(const std::string& atom_name);
};

// ---------------------------------------------------------------------------------------------
// Lattice of Fig. 2: undef > {known, symbolic, operation-inferred constant} > nac
// ---------------------------------------------------------------------------------------------
struct LV {                                        // one component: a dim or an element
  enum K { UNDEF, NAC, VAL } k = UNDEF;
  Expr e;
  static LV undef() { return LV(); }
  static LV nac() { LV v; v.k = NAC; return v; }
  static LV of(const Expr& x) { LV v; v.k = VAL; v.e = x; return v; }
  static LV c(int64_t x) { return of(Expr::constant(x)); }
  bool val() const { return k == VAL; }
  bool is_c(int64_t x) const { return k == VAL && e.is_const() && e.const_value() == x; }
  bool same(const LV& o) const { return k == o.k && (k != VAL || e == o.e); }
};
struct LS {                                        // a shape or a value vector
  enum K { UNDEF, NAC, LIST } k = UNDEF;
  std::vector<LV> d;
  static LS undef() { return LS(); }
  static LS nac() { LS s; s.k = NAC; return s; }
  static LS list(const std::vector<LV>& v) { LS s; s.k = LIST; s.d = v; return s; }
  bool is_list() const { return k == LIST; }
  bool resolved() const;                           // a list with every component a value
  bool same(const LS& o) const;
  bool has_undef() const;
  std::string str() const;
};
LV meet(const LV& a, const LV& b);                 // throws Error(SHAPE_MISMATCH) on two constants
LS meet(const LS& a, const LS& b);

// ---------------------------------------------------------------------------------------------
// Graph
// ---------------------------------------------------------------------------------------------
struct Tensor {
  std::string name;
  int dtype = 0, role = 0;
  bool declared = false, is_output = false, session = false;
  std::vector<std::string> dims, capacity;
  std::vector<int64_t> idata;                      // HOSTCONST integer values
  std::vector<double> fdata;                       // HOSTCONST float values
  int host_rank = 0;
  bool has_data = false;
};
struct Op {
  int kind = 0;
  std::vector<int> in, out;
  std::vector<int64_t> ia;
  double fa = 0;
};
struct Symbol { std::string name; int64_t lo, hi; };

struct Graph {
  std::vector<Symbol> symbols;
  std::vector<Tensor> tensors;
  std::vector<Op> ops;
  std::vector<int> producer;                       // per tensor, -1 for graph inputs / constants
  std::vector<std::vector<int>> consumers;         // per tensor
  std::vector<int> weight_ids, input_ids, output_ids;   // input_ids: inputs passed by pointer
  std::vector<int> session_ids;                        // session inputs (stored in the arena)
  std::vector<int> weight_pos, input_pos, output_pos;  // per tensor: position in the lists above, or -1
  void finish();                                   // fills the derived fields, validates ids
  std::vector<int> sorted_nodes() const;           // reverse post-order of a depth-first walk
};
int op_class(int kind);                            // 0 ISDO, 1 ISDOS, 2 ISVDOS, 3 EDO
const char* op_name(int kind);
int dtype_bytes(int dtype);
inline bool is_int(int dtype) { return dtype == SOD2_I64 || dtype == SOD2_I32; }

// Name of the extent an execution-determined operator produces (known once it has run).
inline std::string exec_symbol(int op_id) { return "@nz" + std::to_string(op_id); }
bool mentions_exec(const Expr& e);                 // nested floordiv / mod atoms included

struct Rdp {
  const Graph* g = nullptr;
  std::vector<LS> S, V;
  int sweeps = 0;
  // false: Alg. 1 as printed (every EDO output nac).  true: the extent a NonZero produces is named
  // by an execution symbol, so what follows is an expression in it; this refines the first analysis
  // (same values where that one has values; nac there wherever this one has nac or such a symbol).
  bool named_edo = false;
  void analyse(const std::vector<int>* order);
  std::string dump() const;
};

// ---------------------------------------------------------------------------------------------
// Static plan
// ---------------------------------------------------------------------------------------------
enum GroupKind { G_GEMM, G_CONV, G_LAYERNORM, G_SOFTMAX, G_MAXPOOL, G_REDUCEMEAN, G_ARGMAX,
                 G_CACHEAPPEND, G_NONZERO, G_GATHER, G_ELTWISE, G_ATTENTION, G_SCATTER, G_RESIZE, G_CONCAT, G_RANGE, G_FILL, G_ONEHOT, G_TOPK, G_GROUPNORM, G_MAXUNPOOL, G_AVGPOOL, G_NMS, G_COPY };
const char* group_kind_name(int k);

struct Group {
  int gid = 0, kind = 0, out = -1;
  std::vector<int> ops;                            // sorted by operator id
  std::vector<int> chain;                          // members in absorption order (seed first)
  int prologue = -1;                               // LayerNorm operator applied to the contraction's first operand, or -1
  std::vector<int> ins;                            // static bases read from outside
  std::vector<int> also;                           // further results of the same operator (TopK: the indices)
  int versions = 1;                                // code versions of the fused loop nest (Fig. 4; 1: every pair proven)
  struct Pair { int a, b, k; };                    // operands of a binary member and the aligned dim, counted from the last
  std::vector<Pair> unproven;
  int lnfold = -1;                                 // the LayerNorm (a second result of the producing group) this contraction reads
  int key = -1;                                    // node-order position that places the group among the items
};
struct Item {
  bool is_group = true;
  int ref = 0;
  std::vector<int> reads, writes;
};
struct Plan {
  const Graph* g = nullptr;
  const Rdp* rdp = nullptr;                        // the analysis the plan is built on
  const Rdp* paper_rdp = nullptr;                  // Alg. 1 as printed; == rdp unless the graph holds a NonZero
  std::shared_ptr<Rdp> named;                      // analysis with named EDO extents, owned (see Rdp::named_edo)
  std::vector<int> exec_ops;                       // NonZero operators in the node order
  bool execution_determined(int t) const;          // nac in the paper's lattice: unresolved or in an execution symbol
  sod2_plan_opts opts{1, 1, 1, 1, 1, 0, 0, 0, 0, 0, 0, 1, 0};
  int fold_k_multiple() const { return opts.fold_k_multiple > 0 ? opts.fold_k_multiple : 64; }
  std::vector<int> fold_y;                         // per tensor: the LayerNorm that makes it a contraction's second result, or -1
  std::map<int, int64_t> const_off;                // group reading a folded LayerNorm -> byte offset of its derived constants
  int64_t const_bytes = 0;                         // size of the buffer that holds them all
  // the limits of R4 and R6-R8 with the defaults (what this library's kernels fuse) filled in
  int max_versions() const { return opts.max_versions > 0 ? opts.max_versions : 8; }
  int attn_head_dim() const { return opts.attn_head_dim > 0 ? opts.attn_head_dim : 64; }
  int append_max_rows() const { return opts.append_max_rows > 0 ? opts.append_max_rows : 4; }
  int prologue_max_rows() const { return opts.prologue_max_rows > 0 ? opts.prologue_max_rows : 8; }
  int prologue_max_k() const { return opts.prologue_max_k > 0 ? opts.prologue_max_k : 1024; }
  int prologue_k_multiple() const { return opts.prologue_k_multiple > 0 ? opts.prologue_k_multiple : 64; }
  std::vector<int> order;
  std::vector<char> folded, view;
  std::map<int, Group> groups;
  std::vector<int> group_of_op;                    // -1 when the operator is in no group
  std::vector<Item> items;
  std::vector<std::vector<int>> subgraphs;
  std::vector<std::string> sg_class;
  std::vector<int> sbase;
  int n_switches = 0;
  // flattened for bind: per tensor the compiled dims (empty when unresolved), per item the tensors a
  // group reads from outside itself
  ExprCompiler xc;
  std::vector<std::vector<CompiledExpr>> cshape;
  std::vector<std::vector<int>> item_ext;
  void build();
  std::string dump() const;
  bool arena_candidate(int t) const;
  std::vector<int> inplace;                        // group result -> the operand whose storage it takes over, or -1
};

// ---------------------------------------------------------------------------------------------
// Binding: concrete shapes, lifetimes, offsets (Section 4.4.1) and the launch table
// ---------------------------------------------------------------------------------------------
struct ArenaTensor { int tid; int64_t bytes; int start, end; int64_t offset; };

// The part of std::map<int, V> that a binding needs, over one sorted vector: a plan is bound on the
// critical path of every call (and again after every execution-determined fact), and a node
// allocation per tensor was a third of that time.  Iteration is in key order; references stay valid
// until the next insertion.
template <class V>
struct FlatMap {
  typedef std::pair<int, V> value_type;
  typedef typename std::vector<value_type>::iterator iterator;
  typedef typename std::vector<value_type>::const_iterator const_iterator;
  std::vector<value_type> v;
  iterator begin() { return v.begin(); }
  iterator end() { return v.end(); }
  const_iterator begin() const { return v.begin(); }
  const_iterator end() const { return v.end(); }
  size_t size() const { return v.size(); }
  bool empty() const { return v.empty(); }
  void reserve(size_t n) { v.reserve(n); }
  iterator lower(int k) {
    return std::lower_bound(v.begin(), v.end(), k, [](const value_type& a, int key) { return a.first < key; });
  }
  const_iterator lower(int k) const {
    return std::lower_bound(v.begin(), v.end(), k, [](const value_type& a, int key) { return a.first < key; });
  }
  iterator find(int k) { iterator it = lower(k); return (it != v.end() && it->first == k) ? it : v.end(); }
  const_iterator find(int k) const { const_iterator it = lower(k); return (it != v.end() && it->first == k) ? it : v.end(); }
  size_t count(int k) const { return find(k) != v.end() ? 1 : 0; }
  V& operator[](int k) {
    if (v.empty() || v.back().first < k) { v.push_back(value_type(k, V())); return v.back().second; }
    iterator it = lower(k);
    if (it == v.end() || it->first != k) it = v.insert(it, value_type(k, V()));
    return it->second;
  }
  const V& at(int k) const {
    const_iterator it = find(k);
    if (it == v.end()) throw std::out_of_range("FlatMap::at");
    return it->second;
  }
};

// extents of one tensor, stored inline (a rank is at most SOD2_MAX_RANK)
struct DimList {
  int n = 0;
  int64_t d[SOD2_MAX_RANK];
  size_t size() const { return (size_t)n; }
  const int64_t* begin() const { return d; }
  const int64_t* end() const { return d + n; }
  int64_t operator[](size_t i) const { return d[i]; }
  int64_t back() const { return d[n - 1]; }
  void push_back(int64_t x) {
    if (n >= SOD2_MAX_RANK) throw Error(SOD2_ERR_UNSUPPORTED, "tensor rank above SOD2_MAX_RANK");
    d[n++] = x;
  }
};

struct Layout {                                    // where an executed tensor lives
  int base = -1;                                   // tensor whose storage it occupies
  std::vector<int64_t> dims;
};

struct BindResult {
  std::map<std::string, int64_t> env;
  std::vector<int64_t> atom_vals;                  // values of Plan::xc's atoms at the bound symbols
  std::vector<int> steps, step_sg;                 // executed item indices
  std::map<int, int> decisions;                    // Switch op id -> 1 when the skip output is taken
  std::vector<int> switch_order;                   // executed Switch operators in order
  FlatMap<ArenaTensor> tensors;
  FlatMap<DimList> dims;                           // outputs of executed groups
  std::vector<int> dyn_base;                       // per tensor: the tensor providing its storage, -1 when not executed
  std::set<int> dead_ops;
  std::map<int, std::pair<int64_t, int64_t>> session;   // session input -> (offset, bytes) at the arena bottom
  std::map<int, int> session_root;                 // session tensor -> the session input whose slot it occupies
  std::map<int, std::string> versions;             // multi-version group -> the version the bound symbols select
  int64_t session_bytes = 0;
  int64_t arena_bytes = 0, peak_live = 0;
  int undecided = 0;                               // Switches met without a given decision
  struct Exec { int op; int64_t value; bool known; };   // an executed NonZero and the extent planned with
  std::vector<Exec> exec;                          // in execution order; !known: the upper bound was used
  std::string dump(const Plan& p) const;
};
// exec_values: extents found by the NonZero operators that have executed so far, in execution order;
// the ones still to run are planned at their upper bound (the element count of their input)
BindResult bind_plan(const Plan& p, const std::vector<int64_t>& symbols, const std::vector<int>& decisions,
                     bool allow_undecided, const std::vector<int64_t>& exec_values = {});

}  // namespace sod2
