// extern "C" surface for the host-side half of the library: graph construction, RDP, planning,
// binding queries.  sod2_run and the launch table live in run.hip.
#include <cstring>

#include "internal.hpp"
#include "handles.hpp"

using namespace sod2;

namespace {
thread_local std::string g_err;
}
namespace sod2 {
void set_error(const std::string& m) { g_err = m; }
}

#define SOD2_TRY try {
#define SOD2_CATCH                                                        \
  }                                                                       \
  catch (const sod2::Error& e) { g_err = e.what(); return e.code; }       \
  catch (const std::exception& e) { g_err = e.what(); return SOD2_ERR_INVALID_ARG; } \
  return SOD2_OK;

static sod2_status copy_text(const std::string& s, char* buf, size_t cap, size_t* needed) {
  if (needed) *needed = s.size() + 1;
  if (!buf || cap < s.size() + 1) {
    if (buf && cap) { std::memcpy(buf, s.data(), cap - 1); buf[cap - 1] = 0; }
    g_err = "text buffer too small";
    return SOD2_ERR_BUFFER_TOO_SMALL;
  }
  std::memcpy(buf, s.c_str(), s.size() + 1);
  return SOD2_OK;
}

extern "C" {

const char* sod2_last_error(void) { return g_err.c_str(); }
const char* sod2_version(void) { return "sod2-mi355x 0.1 (gfx950)"; }

// integer attributes that every later stage indexes or divides by: refused here, once
static void check_attrs(const Op& op) {
  auto bad = [&](const char* what) { throw Error(SOD2_ERR_INVALID_ARG, std::string(op_name(op.kind)) + ": " + what); };
  const std::vector<int64_t>& a = op.ia;
  switch (op.kind) {
    case SOD2_OP_TRANSPOSE: {
      std::vector<char> seen(a.size(), 0);
      for (int64_t p : a) {
        if (p < 0 || p >= (int64_t)a.size() || seen[p]) bad("the attribute must be a permutation of 0 .. rank-1");
        seen[p] = 1;
      }
      if (a.empty() || a.size() > SOD2_MAX_RANK) bad("a permutation of 1 .. SOD2_MAX_RANK axes");
      break;
    }
    case SOD2_OP_CONV:
      if (a.size() != 2 || a[0] < 1 || a[0] > 64 || a[1] < 0 || a[1] > 64) bad("attributes stride (1 .. 64) and pad (0 .. 64)");
      break;
    case SOD2_OP_MAXPOOL: case SOD2_OP_AVERAGEPOOL:
      if (a.size() != 3 || a[0] < 1 || a[0] > 64 || a[1] < 1 || a[1] > 64 || a[2] < 0 || a[2] >= a[0])
        bad("attributes kernel (1 .. 64), stride (1 .. 64) and pad (0 .. kernel-1)");
      break;
    case SOD2_OP_GATHER: case SOD2_OP_CONCAT:
      if (a.size() != 1 || a[0] < -SOD2_MAX_RANK || a[0] >= SOD2_MAX_RANK) bad("one axis attribute");
      break;
    case SOD2_OP_MATMUL: case SOD2_OP_SOFTMAX:
      if (a.size() > 1 || (a.size() == 1 && a[0] != 0 && a[0] != 1)) bad("the attribute is 0 or 1");
      break;
    case SOD2_OP_REDUCEMEAN:
      if (a.size() < 2 || a.size() > 1 + SOD2_MAX_RANK || (a[0] != 0 && a[0] != 1)) bad("attributes keepdims (0 or 1), then the axes");
      for (size_t i = 1; i < a.size(); ++i) if (a[i] < -SOD2_MAX_RANK || a[i] >= SOD2_MAX_RANK) bad("axis out of range");
      break;
    case SOD2_OP_GROUPNORM:
      if (a.size() != 1 || a[0] < 1) bad("the number of groups must be positive");
      break;
    case SOD2_OP_NMS:
      if (a.size() > 1 || (a.size() == 1 && (a[0] < 0 || a[0] > 0x7fffffff))) bad("max_out must not be negative");
      if (!(op.fa >= 0.0 && op.fa <= 1.0)) bad("the overlap threshold lies in [0, 1]");
      break;
    case SOD2_OP_LAYERNORM:
      if (!(op.fa >= 0.0)) bad("epsilon must not be negative");
      break;
    default: break;
  }
  if (op.in.size() > 64 || op.out.size() > 8) bad("too many inputs or outputs");
}

sod2_status sod2_graph_build(const sod2_graph_desc* d, sod2_graph_t** out) {
  SOD2_TRY
  if (!d || !out) throw Error(SOD2_ERR_INVALID_ARG, "null argument");
  std::unique_ptr<sod2_graph_s> h(new sod2_graph_s);
  Graph& g = h->g;
  for (int i = 0; i < d->n_symbols; ++i) {
    if (d->symbol_lo[i] > d->symbol_hi[i] || d->symbol_lo[i] < 0) throw Error(SOD2_ERR_INVALID_ARG, "bad symbol range");
    g.symbols.push_back({d->symbol_names[i], d->symbol_lo[i], d->symbol_hi[i]});
    Expr::symbol(d->symbol_names[i]);
  }
  for (int i = 0; i < d->n_tensors; ++i) {
    const sod2_tensor_desc& td = d->tensors[i];
    Tensor t;
    t.name = td.name ? td.name : ("t" + std::to_string(i));
    if (td.dtype < 0 || td.dtype > SOD2_I32 || td.role < 0 || td.role > SOD2_HOSTCONST)
      throw Error(SOD2_ERR_INVALID_ARG, "bad dtype or role for " + t.name);
    if (td.rank > SOD2_MAX_RANK) throw Error(SOD2_ERR_INVALID_ARG, "rank above SOD2_MAX_RANK for " + t.name);
    t.dtype = td.dtype;
    t.role = td.role;
    t.is_output = td.is_output != 0;
    t.session = td.session != 0;
    t.declared = td.rank >= 0;
    for (int k = 0; k < td.rank; ++k) {
      t.dims.push_back(td.dims[k]);
      Expr e = Expr::parse(t.dims.back());           // validates the text
      for (const auto& term : e.terms)
        for (const auto& a : term.first) {
          bool found = false;
          for (const auto& s : g.symbols) if (s.name == a) found = true;
          if (!found) throw Error(SOD2_ERR_INVALID_ARG, "dim of " + t.name + " uses undeclared symbol " + a);
        }
      if (td.capacity_dims) t.capacity.push_back(td.capacity_dims[k]);
    }
    if (td.role == SOD2_HOSTCONST) {
      if (!td.host_data || td.host_count < 1) throw Error(SOD2_ERR_INVALID_ARG, "host constant without data: " + t.name);
      t.has_data = true;
      t.host_rank = td.rank;
      for (int64_t k = 0; k < td.host_count; ++k) {
        if (td.dtype == SOD2_I64) t.idata.push_back(((const int64_t*)td.host_data)[k]);
        else if (td.dtype == SOD2_I32) t.idata.push_back(((const int32_t*)td.host_data)[k]);
        else if (td.dtype == SOD2_F32) t.fdata.push_back(((const float*)td.host_data)[k]);
        else throw Error(SOD2_ERR_INVALID_ARG, "host constants are i64, i32 or f32");
      }
    } else if ((td.role == SOD2_WEIGHT) && !t.declared) {
      throw Error(SOD2_ERR_INVALID_ARG, "weight without a declared shape: " + t.name);
    }
    g.tensors.push_back(t);
  }
  for (int i = 0; i < d->n_ops; ++i) {
    const sod2_op_desc& od = d->ops[i];
    if (od.kind < 0 || od.kind >= SOD2_OP_COUNT) throw Error(SOD2_ERR_UNSUPPORTED, "unknown operator kind");
    Op op;
    op.kind = od.kind;
    op.in.assign(od.inputs, od.inputs + od.n_inputs);
    op.out.assign(od.outputs, od.outputs + od.n_outputs);
    if (od.n_iattr) op.ia.assign(od.iattr, od.iattr + od.n_iattr);
    op.fa = od.fattr;
    static const int n_in[SOD2_OP_COUNT] = {1, 2, -1, 2, 4, 1, 2, 2, 2, 2, 1, 1, 1, 1, 1, 3, 1, 1, 1, 2, 1, 2, -1, 3, 2, 3, 2, 2, 1, 1, 3, 2, 3, 3, 1, 1, 2};
    if (n_in[op.kind] >= 0 && (int)op.in.size() != n_in[op.kind])
      throw Error(SOD2_ERR_INVALID_ARG, std::string("wrong input count for ") + op_name(op.kind));
    if (op.out.empty() || ((op.kind == SOD2_OP_SWITCH || op.kind == SOD2_OP_TOPK) && op.out.size() != 2))
      throw Error(SOD2_ERR_INVALID_ARG, std::string("wrong output count for ") + op_name(op.kind));
    check_attrs(op);
    g.ops.push_back(op);
  }
  g.finish();
  *out = h.release();
  SOD2_CATCH
}
void sod2_graph_destroy(sod2_graph_t* g) { delete g; }

sod2_status sod2_graph_op_class(const sod2_graph_t* g, int32_t op, int32_t* cls) {
  SOD2_TRY
  if (!g || !cls || op < 0 || op >= (int)g->g.ops.size()) throw Error(SOD2_ERR_INVALID_ARG, "bad argument");
  *cls = op_class(g->g.ops[op].kind);
  SOD2_CATCH
}

sod2_status sod2_op_kind_class(int32_t kind, int32_t* cls) {
  SOD2_TRY
  if (!cls || kind < 0 || kind >= SOD2_OP_COUNT) throw Error(SOD2_ERR_INVALID_ARG, "bad operator kind");
  *cls = op_class(kind);
  SOD2_CATCH
}

static sod2_status infer(const sod2_graph_t* g, const std::vector<int>* order, sod2_rdp_t** out) {
  SOD2_TRY
  if (!g || !out) throw Error(SOD2_ERR_INVALID_ARG, "null argument");
  std::unique_ptr<sod2_rdp_s> h(new sod2_rdp_s);
  h->r.g = &g->g;
  h->r.analyse(order);
  *out = h.release();
  SOD2_CATCH
}
sod2_status sod2_rdp_infer(const sod2_graph_t* g, sod2_rdp_t** out) { return infer(g, nullptr, out); }
sod2_status sod2_rdp_infer_ordered(const sod2_graph_t* g, const int32_t* order, int32_t n, sod2_rdp_t** out) {
  if (!g || !order || n != (int)g->g.ops.size()) { g_err = "order must list every operator once"; return SOD2_ERR_INVALID_ARG; }
  std::vector<int> o(order, order + n);
  std::vector<char> seen(n, 0);
  for (int v : o) {
    if (v < 0 || v >= n || seen[v]) { g_err = "order is not a permutation"; return SOD2_ERR_INVALID_ARG; }
    seen[v] = 1;
  }
  return infer(g, &o, out);
}
void sod2_rdp_destroy(sod2_rdp_t* r) { delete r; }

sod2_status sod2_rdp_query(const sod2_rdp_t* r, int32_t t, int32_t* rank, sod2_dim_info* dims) {
  SOD2_TRY
  if (!r || !rank || !dims || t < 0 || t >= (int)r->r.S.size()) throw Error(SOD2_ERR_INVALID_ARG, "bad argument");
  const LS& s = r->r.S[t];
  if (!s.is_list()) { *rank = -1; return SOD2_OK; }
  *rank = (int)s.d.size();
  for (size_t k = 0; k < s.d.size() && k < SOD2_MAX_RANK; ++k) {
    sod2_dim_info& di = dims[k];
    std::memset(&di, 0, sizeof(di));
    if (!s.d[k].val()) { di.cls = 3; std::strcpy(di.expr, "nac"); continue; }
    di.cls = s.d[k].e.cls();
    if (di.cls == 0) di.value = s.d[k].e.const_value();
    std::string txt = s.d[k].e.str();
    std::strncpy(di.expr, txt.c_str(), sizeof(di.expr) - 1);
  }
  SOD2_CATCH
}
sod2_status sod2_rdp_sweeps(const sod2_rdp_t* r, int32_t* sweeps) {
  if (!r || !sweeps) { g_err = "null argument"; return SOD2_ERR_INVALID_ARG; }
  *sweeps = r->r.sweeps;
  return SOD2_OK;
}
sod2_status sod2_rdp_dump(const sod2_rdp_t* r, char* buf, size_t cap, size_t* needed) {
  if (!r) { g_err = "null argument"; return SOD2_ERR_INVALID_ARG; }
  return copy_text(r->r.dump(), buf, cap, needed);
}

sod2_status sod2_plan(const sod2_graph_t* g, const sod2_rdp_t* r, const sod2_plan_opts* opts, sod2_plan_t** out) {
  SOD2_TRY
  if (!g || !r || !out || r->r.g != &g->g) throw Error(SOD2_ERR_INVALID_ARG, "null argument or RDP of another graph");
  std::unique_ptr<sod2_plan_s> h(new sod2_plan_s);
  h->p.g = &g->g;
  h->p.rdp = &r->r;
  if (opts) h->p.opts = *opts;
  h->p.build();
  *out = h.release();
  SOD2_CATCH
}
void sod2_plan_destroy(sod2_plan_t* p) { delete p; }
sod2_status sod2_plan_counts(const sod2_plan_t* p, int32_t* ng, int32_t* ns, int32_t* nsw) {
  if (!p) { g_err = "null argument"; return SOD2_ERR_INVALID_ARG; }
  if (ng) *ng = (int)p->p.groups.size();
  if (ns) *ns = (int)p->p.subgraphs.size();
  if (nsw) *nsw = p->p.n_switches;
  return SOD2_OK;
}
sod2_status sod2_plan_dump(const sod2_plan_t* p, char* buf, size_t cap, size_t* needed) {
  if (!p) { g_err = "null argument"; return SOD2_ERR_INVALID_ARG; }
  return copy_text(p->p.dump(), buf, cap, needed);
}

sod2_status sod2_plan_query_group(const sod2_plan_t* p, int32_t index, sod2_group_info* info, int32_t* ops, int32_t ops_cap,
                                  int32_t* ins, int32_t ins_cap) {
  if (!p || !info) { g_err = "null argument"; return SOD2_ERR_INVALID_ARG; }
  const Plan& pl = p->p;
  int seen = 0;
  for (size_t sg = 0; sg < pl.subgraphs.size(); ++sg) {
    for (int i : pl.subgraphs[sg]) {
      const Item& it = pl.items[i];
      if (!it.is_group) continue;
      if (seen++ != index) continue;
      const Group& gr = pl.groups.at(it.ref);
      info->gid = gr.gid; info->kind = gr.kind; info->out = gr.out; info->out2 = gr.also.empty() ? -1 : gr.also[0];
      info->n_ops = (int)gr.ops.size(); info->n_ins = (int)gr.ins.size();
      info->subgraph = (int)sg;
      info->sg_class = pl.sg_class[sg] == "known" ? 0 : (pl.sg_class[sg] == "mixed" ? 1 : 2);
      info->inplace_of = pl.inplace[gr.out];
      info->versions = gr.versions;
      for (int k = 0; k < info->n_ops && k < ops_cap && ops; ++k) ops[k] = gr.ops[k];
      for (int k = 0; k < info->n_ins && k < ins_cap && ins; ++k) ins[k] = gr.ins[k];
      return SOD2_OK;
    }
  }
  g_err = "group index outside 0 .. n_groups-1";
  return SOD2_ERR_INVALID_ARG;
}

static sod2_status query_tensor(const Plan& pl, const BindResult& b, int32_t t, sod2_tensor_info* info) {
  if (!info || t < 0 || t >= (int)pl.g->tensors.size()) { g_err = "null argument or tensor id out of range"; return SOD2_ERR_INVALID_ARG; }
  std::memset(info, 0, sizeof *info);
  info->base = -1;
  auto d = b.dims.find(t);
  if (d == b.dims.end()) return SOD2_OK;             // not written by an executed group
  info->executed = 1;
  info->rank = (int)d->second.size();
  for (int i = 0; i < info->rank; ++i) info->dims[i] = d->second[i];
  auto at = b.tensors.find(t);
  if (at != b.tensors.end()) {
    info->where = 0; info->base = t;
    info->offset = at->second.offset; info->bytes = at->second.bytes;
    info->life_start = at->second.start; info->life_end = at->second.end;
  } else if (b.session_root.count(t)) {
    info->where = 1; info->base = b.session_root.at(t);
    info->offset = b.session.at(info->base).first; info->bytes = b.session.at(info->base).second;
  } else if (pl.inplace[t] >= 0) {
    info->where = 2; info->base = b.dyn_base[t];
  } else {
    info->where = 3; info->base = t;
  }
  return SOD2_OK;
}
sod2_status sod2_binding_query_tensor(const sod2_binding_t* b, int32_t t, sod2_tensor_info* info) {
  if (!b) { g_err = "null argument"; return SOD2_ERR_INVALID_ARG; }
  return query_tensor(*b->plan, b->b, t, info);
}
sod2_status sod2_run_query_tensor(const sod2_binding_t* b, int32_t t, sod2_tensor_info* info) {
  if (!b) { g_err = "null argument"; return SOD2_ERR_INVALID_ARG; }
  return query_tensor(*b->plan, b->has_executed ? b->executed : b->b, t, info);
}
sod2_status sod2_run_trace(const sod2_binding_t* b, sod2_trace_entry* e, int32_t cap, int32_t* n) {
  if (!b || !n) { g_err = "null argument"; return SOD2_ERR_INVALID_ARG; }
  *n = (int)b->trace.size();
  for (int i = 0; i < *n && i < cap && e; ++i) e[i] = b->trace[i];
  return SOD2_OK;
}

static sod2_status do_bind(const sod2_plan_t* p, const int64_t* sym, int32_t n, const int32_t* dec, int32_t nd,
                           bool allow_undecided, sod2_binding_t** out, const int64_t* ev = nullptr, int32_t ne = 0) {
  SOD2_TRY
  if (!p || !out || (n > 0 && !sym) || (nd > 0 && !dec) || (ne > 0 && !ev)) throw Error(SOD2_ERR_INVALID_ARG, "null argument");
  std::unique_ptr<sod2_binding_s> h(new sod2_binding_s);
  h->plan = &p->p;
  h->symbols.assign(sym, sym + n);
  std::vector<int> d(dec, dec + nd);
  h->planned_exec.assign(ev, ev + ne);
  h->b = bind_plan(p->p, h->symbols, d, allow_undecided, h->planned_exec);
  h->planned_decisions = d;
  *out = h.release();
  SOD2_CATCH
}
sod2_status sod2_bind(const sod2_plan_t* p, const int64_t* sym, int32_t n, sod2_binding_t** out) {
  return do_bind(p, sym, n, nullptr, 0, true, out);
}
sod2_status sod2_bind_decided(const sod2_plan_t* p, const int64_t* sym, int32_t n, const int32_t* dec, int32_t nd,
                              sod2_binding_t** out) {
  return do_bind(p, sym, n, dec, nd, false, out);
}
sod2_status sod2_bind_executed(const sod2_plan_t* p, const int64_t* sym, int32_t n, const int32_t* dec, int32_t nd,
                               const int64_t* ev, int32_t ne, sod2_binding_t** out) {
  return do_bind(p, sym, n, dec, nd, false, out, ev, ne);
}
sod2_status sod2_binding_arena_bytes(const sod2_binding_t* b, size_t* arena, size_t* peak) {
  if (!b) { g_err = "null argument"; return SOD2_ERR_INVALID_ARG; }
  if (arena) *arena = (size_t)b->b.arena_bytes;
  if (peak) *peak = (size_t)b->b.peak_live;
  return SOD2_OK;
}
sod2_status sod2_binding_dump(const sod2_binding_t* b, char* buf, size_t cap, size_t* needed) {
  if (!b) { g_err = "null argument"; return SOD2_ERR_INVALID_ARG; }
  return copy_text(b->b.dump(*b->plan), buf, cap, needed);
}
sod2_status sod2_binding_force_decisions(sod2_binding_t* b, const int32_t* dec, int32_t n) {
  if (!b || (n > 0 && !dec)) { g_err = "null argument"; return SOD2_ERR_INVALID_ARG; }
  b->forced.assign(dec, dec + n);
  b->has_forced = n > 0;
  return SOD2_OK;
}
sod2_status sod2_binding_force_variant(sod2_binding_t* b, int32_t v) {
  if (!b || v < -1 || (v > 6 && v < sod2::V_DL0) || v >= sod2::V_DL0 + sod2::DL_TILES) {
    g_err = "variant must be -1 .. 6, or 10 + a tile of the direct-to-LDS kernel";
    return SOD2_ERR_INVALID_ARG;
  }
  b->force_variant = v;
  b->launches_valid = false;
  return SOD2_OK;
}
sod2_status sod2_binding_force_splits(sod2_binding_t* b, int32_t n) {
  if (!b || n < 0 || n > 16) { g_err = "splits must be 0 (automatic) .. 16"; return SOD2_ERR_INVALID_ARG; }
  b->force_splits = n;
  b->launches_valid = false;
  return SOD2_OK;
}
sod2_status sod2_binding_workspace_bytes(const sod2_binding_t* b, size_t* bytes) {
  if (!b || !bytes) { g_err = "null argument"; return SOD2_ERR_INVALID_ARG; }
  *bytes = (size_t)sod2::WS_BYTES;
  return SOD2_OK;
}
sod2_status sod2_run_decisions(const sod2_binding_t* b, int32_t* dec, int32_t cap, int32_t* n) {
  if (!b || !n) { g_err = "null argument"; return SOD2_ERR_INVALID_ARG; }
  *n = (int)b->last_decisions.size();
  for (int i = 0; i < *n && i < cap && dec; ++i) dec[i] = b->last_decisions[i];
  return SOD2_OK;
}
sod2_status sod2_run_exec_values(const sod2_binding_t* b, int64_t* vals, int32_t cap, int32_t* n) {
  if (!b || !n) { g_err = "null argument"; return SOD2_ERR_INVALID_ARG; }
  *n = (int)b->last_exec.size();
  for (int i = 0; i < *n && i < cap && vals; ++i) vals[i] = b->last_exec[i];
  return SOD2_OK;
}
sod2_status sod2_run_plan_dump(const sod2_binding_t* b, char* buf, size_t cap, size_t* needed) {
  if (!b) { g_err = "null argument"; return SOD2_ERR_INVALID_ARG; }
  return copy_text((b->has_executed ? b->executed : b->b).dump(*b->plan), buf, cap, needed);
}
sod2_status sod2_run_arena_bytes(const sod2_binding_t* b, size_t* arena, size_t* peak) {
  if (!b) { g_err = "null argument"; return SOD2_ERR_INVALID_ARG; }
  const BindResult& r = b->has_executed ? b->executed : b->b;
  if (arena) *arena = (size_t)r.arena_bytes;
  if (peak) *peak = (size_t)r.peak_live;
  return SOD2_OK;
}
sod2_status sod2_binding_set_profiling(sod2_binding_t* b, int32_t on) {
  if (!b) { g_err = "null argument"; return SOD2_ERR_INVALID_ARG; }
  b->profiling = on != 0;
  return SOD2_OK;
}
sod2_status sod2_binding_launch_records(const sod2_binding_t* b, sod2_launch_record* recs, int32_t cap, int32_t* n) {
  if (!b || !n) { g_err = "null argument"; return SOD2_ERR_INVALID_ARG; }
  *n = (int)b->records.size();
  for (int i = 0; i < *n && i < cap && recs; ++i) recs[i] = b->records[i];
  return SOD2_OK;
}

}  // extern "C"
