// Launch-table construction (views, strides, kernel versions) and sod2_run.
#include <hip/hip_runtime.h>
#include <chrono>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <functional>
#include <memory>

#include "handles.hpp"

namespace sod2 {
hipError_t launch_gemm(const Launch& L, const GemmArgs& g, hipStream_t s);
hipError_t launch_conv(const Launch& L, const ConvArgs& c, hipStream_t s);
hipError_t launch_row(const Launch& L, const RowArgs& a, hipStream_t s);
hipError_t launch_reduce(const Launch& L, const ReduceArgs& a, hipStream_t s);
hipError_t launch_pool(const Launch& L, const PoolArgs& p, hipStream_t s);
hipError_t launch_eltwise(const Launch& L, const EltArgs& a, hipStream_t s);
hipError_t launch_gather(const Launch& L, const GatherArgs& a, hipStream_t s);
hipError_t launch_append(const Launch& L, const AppendArgs& a, hipStream_t s);
hipError_t launch_argmax(const Launch& L, const ArgmaxArgs& a, hipStream_t s);
hipError_t launch_nonzero(const NonzeroArgs& a, hipStream_t s);
hipError_t launch_nms(const NmsArgs& a, hipStream_t s);
hipError_t launch_scatter(const Launch& L, const ScatterArgs& a, hipStream_t s);
hipError_t launch_resize(const Launch& L, const ResizeArgs& a, hipStream_t s);
hipError_t launch_concat(const Launch& L, const ConcatArgs& a, hipStream_t s);
hipError_t launch_range(const RangeArgs& a, hipStream_t s);
hipError_t launch_fill(const FillArgs& a, hipStream_t s);
hipError_t launch_onehot(const OneHotArgs& a, hipStream_t s);
hipError_t launch_topk(const TopKArgs& a, hipStream_t s);
hipError_t launch_groupnorm(const Launch& L, const GroupNormArgs& a, hipStream_t s);
hipError_t launch_unpool(const Launch& L, const UnpoolArgs& a, hipStream_t s);
hipError_t launch_attention(const AttnArgs& a, hipStream_t s);
hipError_t launch_null(hipStream_t s);
hipError_t launch_fold_constants(const void* W, const void* gamma, const void* beta, const void* bias, float scale, int N,
                                 int K, void* s_out, void* c_out, hipStream_t s);

void destroy_events(void* events, int n) {
  hipEvent_t* e = (hipEvent_t*)events;
  for (int i = 0; i < n; ++i) (void)hipEventDestroy(e[i]);
  delete[] e;
}
}  // namespace sod2

sod2_binding_s::~sod2_binding_s() {
  if (events) sod2::destroy_events(events, n_events);
}
extern "C" void sod2_binding_destroy(sod2_binding_t* b) { delete b; }

namespace sod2 {
namespace {

const int64_t kIntMax = 2147483647LL;

// A short list of extents, strides or axes kept inline (a rank is at most SOD2_MAX_RANK): building
// the launches of a call allocates nothing per tensor (it used to cost ~1.7 us per launch, on the
// critical path after every read-back).
struct Dims {
  int n = 0;
  int64_t d[SOD2_MAX_RANK];
  Dims() {}
  explicit Dims(size_t count, int64_t v = 0) {
    if (count > SOD2_MAX_RANK) throw Error(SOD2_ERR_UNSUPPORTED, "tensor rank above SOD2_MAX_RANK");
    n = (int)count;
    for (int i = 0; i < n; ++i) d[i] = v;
  }
  size_t size() const { return (size_t)n; }
  bool empty() const { return n == 0; }
  int64_t& operator[](size_t i) { return d[i]; }
  int64_t operator[](size_t i) const { return d[i]; }
  int64_t* begin() { return d; }
  int64_t* end() { return d + n; }
  const int64_t* begin() const { return d; }
  const int64_t* end() const { return d + n; }
  int64_t& back() { return d[n - 1]; }
  int64_t back() const { return d[n - 1]; }
  void push_back(int64_t x) {
    if (n >= SOD2_MAX_RANK) throw Error(SOD2_ERR_UNSUPPORTED, "tensor rank above SOD2_MAX_RANK");
    d[n++] = x;
  }
  void erase(int64_t* pos) {
    for (int64_t* q = pos; q + 1 < d + n; ++q) q[0] = q[1];
    --n;
  }
  void assign(size_t count, int64_t v) { *this = Dims(count, v); }
  int64_t front() const { return d[0]; }
  int64_t at(size_t i) const {
    if (i >= (size_t)n) throw Error(SOD2_ERR_INVALID_ARG, "dim index out of range");
    return d[i];
  }
  bool operator==(const Dims& o) const {
    if (n != o.n) return false;
    for (int i = 0; i < n; ++i) if (d[i] != o.d[i]) return false;
    return true;
  }
  bool operator!=(const Dims& o) const { return !(*this == o); }
};

struct View {                    // element units
  int base = -1;
  int64_t off = 0;
  Dims dims, strides;
  bool contiguous() const {
    int64_t s = 1;
    for (int i = (int)dims.size() - 1; i >= 0; --i) {
      if (dims[i] != 1 && strides[i] != s) return false;
      s *= dims[i];
    }
    return true;
  }
  int64_t numel() const { int64_t n = 1; for (auto d : dims) n *= d; return n; }
};

Dims contiguous_strides(const Dims& d) {
  Dims s(d.size(), 1);
  for (int i = (int)d.size() - 2; i >= 0; --i) s[i] = s[i + 1] * d[i + 1];
  return s;
}

// strides of a reshaped view, or false when the new shape would need a copy
bool reshape_strides(const View& in, const Dims& nd, Dims* ns) {
  struct Run { int64_t size, stride; };
  std::vector<Run> runs;                        // maximal blocks that are flat in memory
  for (size_t i = 0; i < in.dims.size(); ++i) {
    if (in.dims[i] == 1) continue;
    if (!runs.empty() && runs.back().stride == in.strides[i] * in.dims[i]) {
      runs.back().size *= in.dims[i];
      runs.back().stride = in.strides[i];
    } else {
      runs.push_back({in.dims[i], in.strides[i]});
    }
  }
  ns->assign(nd.size(), 1);
  size_t r = 0, i = 0;
  while (i < nd.size()) {
    if (nd[i] == 1) { (*ns)[i] = 1; ++i; continue; }
    if (r >= runs.size()) return false;
    size_t j = i;
    int64_t prod = 1;
    while (j < nd.size() && prod < runs[r].size) { prod *= nd[j]; ++j; }
    if (prod != runs[r].size) return false;
    int64_t st = runs[r].stride;
    for (size_t k = j; k-- > i;) { (*ns)[k] = st; st *= nd[k]; }
    i = j;
    ++r;
  }
  return r == runs.size();
}

struct Builder {
  const Plan& p;
  const Graph& G;
  const BindResult& b;
  int force_variant;
  int force_splits = 0;
  bool folding = false;                            // the caller has handed over the constants folded LayerNorms need
  std::vector<int> memo_at;                        // tensor -> position in memo, or -1
  std::vector<View> memo;                          // reserved for every tensor up front: references stay valid

  Builder(const Plan& p_, const BindResult& b_, int fv) : p(p_), G(*p_.g), b(b_), force_variant(fv) {
    memo_at.assign(G.tensors.size(), -1);
    memo.reserve(G.tensors.size());
  }

  Dims eval_dims(int t) const {
    const LS& s = p.rdp->S[t];
    if (!s.resolved()) throw Error(SOD2_ERR_UNRESOLVED_SHAPE, "shape of " + G.tensors[t].name + " is not resolved");
    Dims d;
    for (const CompiledExpr& x : p.cshape[t]) d.push_back(x.eval(b.atom_vals));
    return d;
  }
  // a per-column parameter (bias, LayerNorm scale / shift): a dense vector of exactly n elements
  void need_vector(int t, int64_t n, const char* what) {
    const View& v = view_of(t);
    if (!v.contiguous() || v.numel() != n)
      throw Error(SOD2_ERR_SHAPE_MISMATCH, std::string(what) + " " + G.tensors[t].name + " must be a dense vector of " + std::to_string(n) + " elements");
  }
  bool live(int t) const {
    int pr = G.producer[t];
    return pr < 0 || p.folded[pr] || b.dyn_base[t] >= 0;
  }

  const View& view_of(int t) {
    if (memo_at[t] >= 0) return memo[memo_at[t]];
    View v;
    int pr = G.producer[t];
    auto sr = b.session_root.find(t);
    if (sr != b.session_root.end()) {               // a session tensor: dense rows in its root's arena slot
      v.base = sr->second;
      v.dims = eval_dims(t);
      v.strides = contiguous_strides(v.dims);
    } else if (pr < 0 || (!p.view[pr] && G.ops[pr].kind != SOD2_OP_SWITCH && G.ops[pr].kind != SOD2_OP_COMBINE)) {
      const Group* owner = pr >= 0 ? &p.groups.at(p.group_of_op[pr]) : nullptr;
      if (owner && owner->out != t && std::find(owner->also.begin(), owner->also.end(), t) == owner->also.end())
        throw Error(SOD2_ERR_UNSUPPORTED, "tensor inside a fused group is read from outside: " + G.tensors[t].name);
      v.base = (pr >= 0 && p.inplace[t] >= 0 && b.dyn_base[t] >= 0) ? b.dyn_base[t] : t;   // in place: the operand's storage
      v.dims = eval_dims(t);
      v.strides = contiguous_strides(v.dims);
    } else {
      const Op& op = G.ops[pr];
      if (op.kind == SOD2_OP_SWITCH) v = view_of(op.in[0]);
      else if (op.kind == SOD2_OP_COMBINE) {
        int src = -1;
        for (int i : op.in) if (live(i)) { src = i; break; }
        if (src < 0) throw Error(SOD2_ERR_INVALID_ARG, "Combine without a live input");
        v = view_of(src);
      } else {
        v = derived_view(op, t);
      }
    }
    memo_at[t] = (int)memo.size();
    memo.push_back(v);
    return memo.back();
  }

  // the view a Reshape / Slice / Transpose / Expand / scalar-index Gather makes of its first operand; t = its result
  View derived_view(const Op& op, int t) {
    const View in = view_of(op.in[0]);
    View v = in;
    if (op.kind == SOD2_OP_TRANSPOSE) {
      for (size_t i = 0; i < op.ia.size(); ++i) { v.dims[i] = in.dims[op.ia[i]]; v.strides[i] = in.strides[op.ia[i]]; }
    } else if (op.kind == SOD2_OP_GATHER) {
      int64_t r = (int64_t)in.dims.size();
      int64_t ax = ((op.ia.at(0) % r) + r) % r;
      int64_t idx = G.tensors[op.in[1]].idata.at(0);
      if (idx < 0) idx += in.dims[ax];
      if (idx < 0 || idx >= in.dims[ax]) throw Error(SOD2_ERR_INVALID_ARG, "Gather index out of range");
      v.off += idx * in.strides[ax];
      v.dims.erase(v.dims.begin() + ax);
      v.strides.erase(v.strides.begin() + ax);
    } else if (op.kind == SOD2_OP_SLICE) {
      // bounds and axes as RDP carries them: host constants, or expressions computed from shapes (value maps),
      // evaluated at the bound symbols
      const LS &st = p.rdp->V[op.in[1]], &en = p.rdp->V[op.in[2]], &ax = p.rdp->V[op.in[3]];
      if (!st.resolved() || !en.resolved() || !ax.resolved() || st.d.size() != ax.d.size() || en.d.size() != ax.d.size())
        throw Error(SOD2_ERR_UNSUPPORTED, "Slice bounds must be known to RDP (host constants or values computed from shapes)");
      for (size_t k = 0; k < ax.d.size(); ++k) {
        int64_t r = (int64_t)in.dims.size();
        int64_t a = ((ax.d[k].e.eval(b.env) % r) + r) % r, D = in.dims[a];
        const int64_t sv = st.d[k].e.eval(b.env), ev = en.d[k].e.eval(b.env);
        const bool sc = st.d[k].e.is_const(), ec = en.d[k].e.is_const();
        int64_t s = (sc && sv < 0) ? D + sv : sv;
        int64_t e = (ec && ev >= kIntMax) ? D : ((ec && ev < 0) ? D + ev : ev);
        if (s < 0 || e > D || s > e) throw Error(SOD2_ERR_INVALID_ARG, "Slice bounds outside the tensor");
        v.off += s * in.strides[a];
        v.dims[a] = e - s;
      }
    } else if (op.kind == SOD2_OP_EXPAND) {         // broadcast dims get stride 0
      Dims nd = eval_dims(t), ns(nd.size(), 0);
      if (nd.size() < in.dims.size()) throw Error(SOD2_ERR_SHAPE_MISMATCH, "Expand lowers the rank");
      size_t pad = nd.size() - in.dims.size();
      for (size_t i = 0; i < in.dims.size(); ++i) {
        if (in.dims[i] == nd[pad + i]) ns[pad + i] = in.strides[i];
        else if (in.dims[i] != 1) throw Error(SOD2_ERR_SHAPE_MISMATCH, "Expand of a dim that is neither 1 nor the target");
      }
      v.dims = nd;
      v.strides = ns;
    } else if (op.kind == SOD2_OP_RESHAPE) {
      Dims nd = eval_dims(t), ns;
      if (View{0, 0, nd, {}}.numel() != in.numel()) throw Error(SOD2_ERR_SHAPE_MISMATCH, "Reshape changes the element count");
      if (!reshape_strides(in, nd, &ns))
        throw Error(SOD2_ERR_UNSUPPORTED, "Reshape of a strided view needs a copy: " + G.tensors[t].name);
      v.dims = nd;
      v.strides = ns;
    }
    return v;
  }

  Ref ref_of(const View& v, int dtype) const {
    Ref r;
    int t = v.base;
    int64_t eb = dtype_bytes(dtype);
    auto at = b.tensors.find(t);
    if (at != b.tensors.end()) { r.space = SP_ARENA; r.byte_off = at->second.offset + v.off * eb; return r; }
    auto ss = b.session.find(t);
    if (ss != b.session.end()) { r.space = SP_ARENA; r.byte_off = ss->second.first + v.off * eb; return r; }
    r.byte_off = v.off * eb;
    if (G.weight_pos[t] >= 0) { r.space = SP_WEIGHT; r.index = G.weight_pos[t]; }
    else if (G.output_pos[t] >= 0) { r.space = SP_OUTPUT; r.index = G.output_pos[t]; }
    else if (G.input_pos[t] >= 0) { r.space = SP_INPUT; r.index = G.input_pos[t]; }
    else throw Error(SOD2_ERR_INVALID_ARG, "tensor has no storage: " + G.tensors[t].name);
    return r;
  }
  Ref ref_t(int t) { return ref_of(view_of(t), G.tensors[t].dtype); }

  static int act_of(int kind) {
    return kind == SOD2_OP_RELU ? ACT_RELU : (kind == SOD2_OP_GELU ? ACT_GELU : ACT_SIGMOID);
  }
  int other(const Op& op, int cur) const { return op.in[0] == cur ? op.in[1] : op.in[0]; }

  // epilogue description shared by MatMul and Conv groups
  struct Epi { float scale = 1.f; int bias = -1, res = -1, act1 = ACT_NONE, act2 = ACT_NONE, transpose = -1; };
  Epi epilogue(const Group& gr) const {
    Epi e;
    int cur = G.ops[gr.chain[0]].out[0];
    for (size_t k = 1; k < gr.chain.size(); ++k) {
      const Op& op = G.ops[gr.chain[k]];
      if (op.kind == SOD2_OP_MUL) e.scale *= (float)G.tensors[other(op, cur)].fdata.at(0);
      else if (op.kind == SOD2_OP_ADD) {
        int o = other(op, cur);
        if (G.tensors[o].role == SOD2_WEIGHT && e.bias < 0 && e.res < 0 && e.act1 == ACT_NONE) e.bias = o;
        else e.res = o;
      } else if (op.kind == SOD2_OP_TRANSPOSE) e.transpose = gr.chain[k];
      else (e.res >= 0 ? e.act2 : e.act1) = act_of(op.kind);
      cur = op.out[0];
    }
    return e;
  }

  // Kernel version (Section 4.4.2: fat / regular / skinny versions chosen at run time by shape), a
  // pure function of the contraction's shape.  Measured on MI355X: from ~1024 tiles of 128 x 128 on, the
  // 256-row tiles win (half the operand bytes per flop; 8192 x 8192 x 4096 runs at 0.99 PFLOP/s); with at least ~160 tiles of
  // 128 x 128 the 8-wave 128 x 128 x 64 kernel wins (three ring stages when k is long, two stages
  // and two workgroups per CU otherwise); below that the 64 x 64 x 64 tile with a four-stage ring
  // puts more workgroups (more loads in flight) on the chip.
  int pick_variant(int dtype, int64_t M, int64_t N, int64_t K, int64_t batch) const {
    if (dtype != SOD2_BF16) return (M <= 8 && force_variant != V_SIMPLE && p.opts.mvc) ? V_GEMV : V_SIMPLE;   // fp32: plain FMA kernels
    if (force_variant >= 0) return force_variant;
    // multi-version kernels off (the breakdown study of Section 5.3): one version of the same kernel for every
    // shape -- the 128 x 128 x 64 tile, no skinny version, no k groups, no split-K
    if (!p.opts.mvc) return V_DL0 + DL_128x128x64_S2_W8T;
    if (M <= 8) return V_GEMV;                     // decode shape: weight streaming, one wave per column
    const int64_t t128 = ((M + 127) / 128) * ((N + 127) / 128) * batch;
    const int64_t t64 = ((M + 63) / 64) * ((N + 63) / 64) * batch;
    if (t128 >= 1024) return V_DL0 + (K >= 2048 ? DL_256x256x64_S2_W8 : DL_256x128x32_S3_W8);   // fat versions
    // the 64x64 tile runs two workgroups per CU: as long as all its tiles are resident at once
    // (512 on 256 CUs) it finishes first; one tile more and a second round starts, then 128x128 wins
    // (128 x 128 tiles: 4 x 2 waves, so that a wave stores whole 128-byte lines; with at most one tile per CU the
    // three-stage ring with one workgroup per CU beats two stages and two per CU, k short or long)
    if (t64 > 512)
      return V_DL0 + (t128 <= 256 ? (K >= 2048 ? DL_128x128x64_S2_W8G2 : DL_128x128x64_S3_W8T)
                                  : (K >= 2048 ? DL_128x128x64_S3_W8T : DL_128x128x64_S2_W8T));
    // with at most one tile per CU a workgroup's walk over k is the whole duration: two wave groups
    // share the tile and split k between them (0.5 - 4 us less per launch on config 2's shapes)
    if (t64 <= 256) return V_DL0 + DL_64x64x64_S3_G2;
    return V_DL0 + (K >= 2048 ? DL_64x64x64_S2_G2 : DL_64x64x64_S4_W4);   // two per CU; the groups pay off on a long k (9 % at k = 3072)
  }

  // Split-K (only with the direct-to-LDS kernel; costs a second launch that sums the partials): for a
  // long k with few tiles, where one workgroup per tile would walk k alone while most CUs idle.
  int pick_splits(int variant, int64_t M, int64_t N, int64_t K, int64_t batch) const {
    if (variant < V_DL0 || force_splits == 1 || (!p.opts.mvc && force_splits == 0)) return 1;
    const bool grouped = variant == V_DL0 + DL_64x64x64_S3_G2;
    const bool small = grouped || variant == V_DL0 + DL_64x64x64_S4_W4 || variant == V_DL0 + DL_64x64x64_S2_G2;
    const int64_t bm = small ? 64 : 128, bn = small ? 64 : 128;
    const int64_t tiles = ((M + bm - 1) / bm) * ((N + bn - 1) / bn) * batch;
    int64_t s = force_splits;
    if (force_splits == 0) {
      if (!small || K < 2048 || tiles > 256) return 1;
      // measured: two wave groups walk k about twice as fast and one such workgroup fills a CU
      s = grouped ? std::min<int64_t>(256 / std::max<int64_t>(tiles, 1), K / 512)
                  : std::min<int64_t>(512 / std::max<int64_t>(tiles, 1), K / 384);
    }
    int64_t pow2 = 1;
    while (pow2 * 2 <= s && pow2 < (force_splits > 1 ? 16 : 8)) pow2 *= 2;
    s = pow2;
    while (s > 1 && (double)s * M * N * 4.0 * batch > (double)WS_PARTIAL_BYTES) s /= 2;
    return (int)std::max<int64_t>(s, 1);
  }

  Launch gemm_core(const Group& gr) {
    Launch L;
    L.group = gr.gid;
    L.kernel = K_GEMM;
    const Op& mm = G.ops[gr.chain[0]];
    Epi e = epilogue(gr);
    int dt = G.tensors[mm.in[0]].dtype;
    if (G.tensors[mm.in[1]].dtype != dt || G.tensors[gr.out].dtype != dt)
      throw Error(SOD2_ERR_UNSUPPORTED, "MatMul operands and result must share one float type");
    L.in_dtype = L.out_dtype = dt;
    // with a LayerNorm prologue the first operand is the LayerNorm's input: its result has no storage
    const Op* ln = gr.prologue >= 0 ? &G.ops[gr.prologue] : nullptr;
    const View &va = view_of(ln ? ln->in[0] : mm.in[0]), &vb = view_of(mm.in[1]);
    bool tb = !mm.ia.empty() && mm.ia[0];
    size_t ra = va.dims.size(), rb = vb.dims.size();
    GemmArgs g{};
    g.M = (int)va.dims[ra - 2];
    g.K = (int)va.dims[ra - 1];
    g.N = (int)(tb ? vb.dims[rb - 2] : vb.dims[rb - 1]);
    if ((tb ? vb.dims[rb - 1] : vb.dims[rb - 2]) != g.K) throw Error(SOD2_ERR_SHAPE_MISMATCH, "MatMul inner dims differ");
    g.a_sm = va.strides[ra - 2]; g.a_sk = va.strides[ra - 1];
    g.b_sn = tb ? vb.strides[rb - 2] : vb.strides[rb - 1];
    g.b_sk = tb ? vb.strides[rb - 1] : vb.strides[rb - 2];

    Dims logical = eval_dims(mm.out[0]);
    size_t nbatch = logical.size() - 2;
    // strides of C (and the residual) per logical dim
    Dims cs;
    if (e.transpose >= 0) {
      const Op& tp = G.ops[e.transpose];
      Dims od(logical.size());
      for (size_t i = 0; i < tp.ia.size(); ++i) od[i] = logical[tp.ia[i]];
      Dims os = contiguous_strides(od);
      cs.assign(logical.size(), 0);
      for (size_t i = 0; i < tp.ia.size(); ++i) cs[tp.ia[i]] = os[i];
    } else {
      cs = contiguous_strides(logical);
    }
    Dims rs(logical.size(), 0);
    if (e.res >= 0) {
      const View& vr = view_of(e.res);
      if (vr.dims != logical) throw Error(SOD2_ERR_SHAPE_MISMATCH, "residual shape differs from the MatMul result");
      rs = vr.strides;
    }
    auto bstride = [&](const View& v, size_t j) -> int64_t {       // stride of logical batch dim j in operand v
      size_t r = v.dims.size() - 2;
      if (j + r < nbatch) return 0;
      size_t k = j - (nbatch - r);
      return v.dims[k] == 1 ? 0 : v.strides[k];
    };
    struct BD { int64_t n, a, b, c, r; };
    std::vector<BD> bd;
    for (size_t j = 0; j < nbatch; ++j)
      if (logical[j] != 1) bd.push_back({logical[j], bstride(va, j), bstride(vb, j), cs[j], rs[j]});
    g.c_sm = cs[nbatch]; g.c_sn = cs[nbatch + 1];
    g.r_sm = rs[nbatch]; g.r_sn = rs[nbatch + 1];
    int64_t M = g.M;
    // fold the innermost batch dims into M while every operand stays a plain row walk
    while (!bd.empty()) {
      const BD& x = bd.back();
      bool ok = x.b == 0 && x.a == g.a_sm * M && x.c == g.c_sm * M && (e.res < 0 || x.r == g.r_sm * M);
      if (!ok) break;
      M *= x.n;
      bd.pop_back();
    }
    // merge adjacent batch dims
    for (size_t j = bd.size(); j-- > 1;) {
      BD &hi = bd[j - 1], &lo = bd[j];
      if (hi.a == lo.a * lo.n && hi.b == lo.b * lo.n && hi.c == lo.c * lo.n && hi.r == lo.r * lo.n) {
        hi = {hi.n * lo.n, lo.a, lo.b, lo.c, lo.r};
        bd.erase(bd.begin() + j);
      }
    }
    if (bd.size() > 2) throw Error(SOD2_ERR_UNSUPPORTED, "MatMul with more than two independent batch dims");
    while (bd.size() < 2) bd.insert(bd.begin(), {1, 0, 0, 0, 0});
    if (M > 0x7fffffffLL) throw Error(SOD2_ERR_UNSUPPORTED, "MatMul M too large");
    g.M = (int)M;
    g.nb0 = (int)bd[0].n; g.nb1 = (int)bd[1].n;
    g.a_sb0 = bd[0].a; g.a_sb1 = bd[1].a; g.b_sb0 = bd[0].b; g.b_sb1 = bd[1].b;
    g.c_sb0 = bd[0].c; g.c_sb1 = bd[1].c; g.r_sb0 = bd[0].r; g.r_sb1 = bd[1].r;
    g.scale = e.scale; g.act1 = e.act1; g.act2 = e.act2;
    L.r[0] = ref_of(va, dt);
    L.r[1] = ref_of(vb, dt);
    L.r[2] = ref_t(gr.out);
    if (e.bias >= 0) { need_vector(e.bias, g.N, "bias"); L.r[3] = ref_t(e.bias); }
    if (e.res >= 0) L.r[4] = ref_of(view_of(e.res), dt);
    int64_t batch = (int64_t)g.nb0 * g.nb1;
    L.variant = pick_variant(dt, g.M, g.N, g.K, batch);
    // the one tile of the shape rule that cannot write or read a folded LayerNorm gives way to its neighbour
    if (folding && force_variant < 0 && L.variant == V_DL0 + DL_128x128x64_S2_W8G2 &&
        ((!gr.also.empty() && p.fold_y[gr.also[0]] >= 0) || gr.lnfold >= 0))
      L.variant = V_DL0 + DL_128x128x64_S3_W8T;
    g.splits = pick_splits(L.variant, g.M, g.N, g.K, batch);
    if (ln) {
      if (g.a_sk != 1 || g.K % 64 != 0 || g.K > 1024 || (g.M > 1 && g.a_sm % 8 != 0) || !tb || g.b_sk != 1)
        throw Error(SOD2_ERR_UNSUPPORTED, "LayerNorm prologue needs dense k-contiguous operands and K a multiple of 64 up to 1024");
      if (g.M > 8 || batch != 1) throw Error(SOD2_ERR_UNSUPPORTED, "LayerNorm prologue is for at most 8 rows");
      need_vector(ln->in[1], g.K, "LayerNorm scale");
      need_vector(ln->in[2], g.K, "LayerNorm shift");
      L.r[5] = ref_t(ln->in[1]);
      L.r[6] = ref_t(ln->in[2]);
      g.ln_eps = (float)ln->fa;
      g.splits = 1;
    }
    L.u.gemm = g;
    double eb = dtype_bytes(dt);
    L.flops = 2.0 * g.M * g.N * g.K * batch;
    double bcount = (bd[0].b || bd[1].b) ? (double)batch : ((bd[1].b || g.nb0 == 1) ? 1.0 : 1.0);
    L.bytes = eb * ((double)g.M * g.K * batch + (double)g.N * g.K * bcount + (double)g.M * g.N * batch * (e.res >= 0 ? 2 : 1) +
                    (e.bias >= 0 ? g.N : 0));
    if (ln) {
      L.flops += 8.0 * g.M * g.K * batch;
      L.bytes += eb * 2.0 * g.K;
    }
    return L;
  }

  // A contraction that takes part in the folding of a LayerNorm (the LayerNorm behind it is its second result, or its
  // first operand is such a second result).  Whether the pair of kernels can do it is decided here, from both launches,
  // so that the two sides always agree; otherwise the LayerNorm's row kernel runs right behind the producing contraction.
  static bool dl_can_fold(int variant) {
    switch (variant - V_DL0) {
      case DL_256x256x64_S2_W8: case DL_256x128x32_S3_W8: case DL_128x128x64_S3_W8T:
      case DL_128x128x64_S2_W8T: case DL_64x64x64_S3_G2: case DL_64x64x64_S2_G2: case DL_64x64x64_S4_W4: return true;
      default: return false;
    }
  }
  std::map<int, bool> pair_memo;
  bool pair_ok(int ln) {
    if (!folding) return false;
    auto it = pair_memo.find(ln);
    if (it != pair_memo.end()) return it->second;
    bool ok = false;
    const Group& gp = p.groups.at(p.group_of_op[ln]);
    const Group* gc = nullptr;
    for (const auto& kv : p.groups) if (kv.second.lnfold == ln) gc = &kv.second;
    if (gc && gp.lnfold < 0 && gc->also.empty() && gc->prologue < 0 && G.tensors[gp.out].dtype == SOD2_BF16 &&
        G.tensors[G.ops[ln].in[1]].role == SOD2_WEIGHT && G.tensors[G.ops[ln].in[2]].role == SOD2_WEIGHT) {
      Launch lp, lc;
      try {
        lp = gemm_core(gp);
        lc = gemm_core(*gc);
      } catch (const Error&) {                                  // (the consumer sits in a branch this binding skips)
        pair_memo[ln] = false;
        return false;
      }
      const GemmArgs &a = lp.u.gemm, &c = lc.u.gemm;
      const Epi ep = epilogue(gp), ec = epilogue(*gc);
      const bool prod = dl_can_fold(lp.variant) && a.nb0 * a.nb1 == 1 && a.c_sn == 1 && a.c_sm == a.N && a.N % 32 == 0 &&
                        a.a_sk == 1 && a.K % 8 == 0 && a.a_sm % 8 == 0 && a.b_sk == 1 && a.b_sn % 8 == 0 &&
                        (ep.res < 0 || (a.r_sn == 1 && a.r_sm % 8 == 0));
      const bool cons = dl_can_fold(lc.variant) && c.splits == 1 && c.nb0 * c.nb1 == 1 && c.a_sk == 1 && c.a_sm == c.K &&
                        c.b_sk == 1 && c.b_sn % 8 == 0 && c.c_sn == 1 && c.c_sm % 8 == 0 && c.N % 8 == 0 &&
                        (ec.res < 0 || (c.r_sn == 1 && c.r_sm % 8 == 0)) && c.M == a.M && c.K == a.N &&
                        (ec.bias < 0 || G.tensors[ec.bias].role == SOD2_WEIGHT) && p.const_off.count(gc->gid);
      ok = prod && cons;
    }
    pair_memo[ln] = ok;
    return ok;
  }
  Launch gemm(const Group& gr) {
    Launch L = gemm_core(gr);
    const int y = (!gr.also.empty() && p.fold_y[gr.also[0]] >= 0) ? gr.also[0] : -1;
    if (y >= 0) {
      const Op& ln = G.ops[p.fold_y[y]];
      const View& vx = view_of(gr.out);
      if (!vx.contiguous()) throw Error(SOD2_ERR_UNSUPPORTED, "LayerNorm behind a contraction needs a dense result");
      RowArgs a{};
      a.cols = (int)vx.dims.back();
      a.rows = vx.numel() / std::max<int64_t>(a.cols, 1);
      a.x_stride = a.y_stride = a.cols;
      a.eps = (float)ln.fa;
      L.post = a;
      L.post_ln = true;
      need_vector(ln.in[1], a.cols, "LayerNorm scale");
      need_vector(ln.in[2], a.cols, "LayerNorm shift");
      L.r[7] = ref_t(y);
      L.r[8] = ref_t(ln.in[1]);
      L.r[9] = ref_t(ln.in[2]);
      L.fold_pair = pair_ok(p.fold_y[y]);
      double eb = dtype_bytes(L.out_dtype);
      L.flops += 8.0 * a.rows * a.cols;
      L.bytes += eb * a.rows * a.cols + (L.fold_pair ? 0.25 * a.rows * a.cols : eb * a.rows * a.cols);
    }
    if (gr.lnfold >= 0 && pair_ok(gr.lnfold)) {
      L.fold_read = true;
      L.const_off = p.const_off.at(gr.gid);
      L.u.gemm.ln_eps = (float)G.ops[gr.lnfold].fa;
      L.bytes += 0.25 * L.u.gemm.M * L.u.gemm.K + 8.0 * L.u.gemm.N;
    }
    return L;
  }

  Launch conv(const Group& gr) {
    Launch L;
    L.group = gr.gid;
    L.kernel = K_CONV;
    const Op& cv = G.ops[gr.chain[0]];
    Epi e = epilogue(gr);
    if (e.transpose >= 0 || e.scale != 1.f) throw Error(SOD2_ERR_UNSUPPORTED, "Conv epilogue with scale or transpose");
    int dt = G.tensors[cv.in[0]].dtype;
    L.in_dtype = L.out_dtype = dt;
    const View &vx = view_of(cv.in[0]), &vw = view_of(cv.in[1]);
    if (!vx.contiguous() || !vw.contiguous()) throw Error(SOD2_ERR_UNSUPPORTED, "Conv needs contiguous NHWC operands");
    Dims od = eval_dims(cv.out[0]);
    ConvArgs c{};
    c.NB = (int)vx.dims[0]; c.H = (int)vx.dims[1]; c.W = (int)vx.dims[2]; c.C = (int)vx.dims[3];
    c.O = (int)vw.dims[0]; c.KH = (int)vw.dims[1]; c.KW = (int)vw.dims[2];
    c.stride = (int)cv.ia.at(0); c.pad = (int)cv.ia.at(1);
    c.OH = (int)od[1]; c.OW = (int)od[2];
    c.act1 = e.act1; c.act2 = e.act2;
    c.vec = c.C % 8 == 0;
    if ((int64_t)c.NB * c.OH * c.OW > 0x7fffffffLL) throw Error(SOD2_ERR_UNSUPPORTED, "Conv output too large");
    L.r[0] = ref_of(vx, dt);
    L.r[1] = ref_of(vw, dt);
    L.r[2] = ref_t(gr.out);
    if (e.bias >= 0) { need_vector(e.bias, c.O, "bias"); L.r[3] = ref_t(e.bias); }
    if (e.res >= 0) {
      const View& vr = view_of(e.res);
      if (!vr.contiguous() || vr.dims != od) throw Error(SOD2_ERR_UNSUPPORTED, "Conv residual must be contiguous and of the output shape");
      L.r[4] = ref_of(vr, dt);
    }
    int64_t M = (int64_t)c.NB * c.OH * c.OW;
    L.variant = pick_variant(dt, M, c.O, (int64_t)c.KH * c.KW * c.C, 1);
    c.splits = (c.vec && c.C % 64 == 0) ? pick_splits(L.variant, M, c.O, (int64_t)c.KH * c.KW * c.C, 1) : 1;
    L.u.conv = c;
    double eb = dtype_bytes(dt), K = (double)c.KH * c.KW * c.C;
    L.flops = 2.0 * M * c.O * K;
    L.bytes = eb * ((double)vx.numel() + (double)c.O * K + (double)M * c.O * (e.res >= 0 ? 2 : 1) + c.O);
    return L;
  }

  // rows x cols walk of a view whose last dim is dense
  void rows_of(const View& v, int64_t* rows, int64_t* stride) const {
    size_t r = v.dims.size();
    if (r == 0 || (v.dims[r - 1] != 1 && v.strides[r - 1] != 1)) throw Error(SOD2_ERR_UNSUPPORTED, "row kernel needs a dense last dim");
    int64_t n = 1, st = r >= 2 ? v.strides[r - 2] : v.dims[r - 1];
    for (size_t i = 0; i + 1 < r; ++i) n *= v.dims[i];
    int64_t expect = st;
    for (int i = (int)r - 2; i >= 0; --i) {
      if (v.dims[i] != 1 && v.strides[i] != expect) throw Error(SOD2_ERR_UNSUPPORTED, "row kernel needs evenly spaced rows");
      expect *= v.dims[i];
    }
    *rows = n;
    *stride = st;
  }

  Launch row(const Group& gr, bool layernorm) {
    Launch L;
    L.group = gr.gid;
    L.kernel = layernorm ? K_LAYERNORM : K_SOFTMAX;
    L.is_layernorm = layernorm;
    const Op& op = G.ops[gr.chain[0]];
    int dt = G.tensors[op.in[0]].dtype;
    if (G.tensors[gr.out].dtype != dt) throw Error(SOD2_ERR_UNSUPPORTED, "row kernel changes the dtype");
    L.in_dtype = L.out_dtype = dt;
    const View& vx = view_of(op.in[0]);
    RowArgs a{};
    int64_t rows, xs;
    rows_of(vx, &rows, &xs);
    a.rows = rows;
    a.cols = (int)vx.dims.back();
    a.x_stride = xs;
    a.y_stride = a.cols;
    a.eps = (float)op.fa;
    L.r[0] = ref_of(vx, dt);
    L.r[1] = ref_t(gr.out);
    if (layernorm) {
      need_vector(op.in[1], a.cols, "LayerNorm scale");
      need_vector(op.in[2], a.cols, "LayerNorm shift");
      L.r[2] = ref_t(op.in[1]);
      L.r[3] = ref_t(op.in[2]);
    } else {
      a.causal = !op.ia.empty() && op.ia[0];
      a.lq = vx.dims.size() >= 2 ? (int)vx.dims[vx.dims.size() - 2] : 1;
    }
    L.u.row = a;
    double eb = dtype_bytes(dt);
    L.flops = (layernorm ? 8.0 : 5.0) * rows * a.cols;
    L.bytes = eb * (2.0 * rows * a.cols + (layernorm ? 2.0 * a.cols : 0));
    return L;
  }

  Launch reduce(const Group& gr) {
    Launch L;
    L.group = gr.gid;
    L.kernel = K_REDUCE;
    const Op& op = G.ops[gr.chain[0]];
    const View& vx = view_of(op.in[0]);
    if (!vx.contiguous()) throw Error(SOD2_ERR_UNSUPPORTED, "ReduceMean needs a contiguous input");
    int64_t r = (int64_t)vx.dims.size();
    Dims axes;
    for (size_t k = 1; k < op.ia.size(); ++k) axes.push_back(((op.ia[k] % r) + r) % r);
    std::sort(axes.begin(), axes.end());
    for (size_t k = 1; k < axes.size(); ++k)
      if (axes[k] != axes[k - 1] + 1) throw Error(SOD2_ERR_UNSUPPORTED, "ReduceMean axes must be adjacent");
    ReduceArgs a{};
    int64_t batch = 1, R = 1, C = 1;
    for (int64_t i = 0; i < r; ++i) {
      if (i < axes.front()) batch *= vx.dims[i];
      else if (i <= axes.back()) R *= vx.dims[i];
      else C *= vx.dims[i];
    }
    a.batch = (int)batch; a.R = R; a.C = (int)C;
    L.in_dtype = G.tensors[op.in[0]].dtype;
    L.out_dtype = G.tensors[gr.out].dtype;
    L.r[0] = ref_of(vx, L.in_dtype);
    L.r[1] = ref_t(gr.out);
    L.u.red = a;
    L.flops = (double)batch * R * C;
    L.bytes = (double)batch * R * C * dtype_bytes(L.in_dtype) + (double)batch * C * dtype_bytes(L.out_dtype);
    return L;
  }

  Launch pool(const Group& gr) {
    Launch L;
    L.group = gr.gid;
    L.kernel = K_POOL;
    const Op& op = G.ops[gr.chain[0]];
    const View& vx = view_of(op.in[0]);
    if (!vx.contiguous()) throw Error(SOD2_ERR_UNSUPPORTED, "a pooling operator needs a contiguous input");
    Dims od = eval_dims(gr.out);
    PoolArgs a{};
    a.NB = (int)vx.dims[0]; a.H = (int)vx.dims[1]; a.W = (int)vx.dims[2]; a.C = (int)vx.dims[3];
    a.OH = (int)od[1]; a.OW = (int)od[2];
    a.k = (int)op.ia.at(0); a.stride = (int)op.ia.at(1); a.pad = (int)op.ia.at(2);
    a.avg = op.kind == SOD2_OP_AVERAGEPOOL;
    if (a.k < 1 || a.stride < 1 || a.pad < 0 || a.pad >= a.k) throw Error(SOD2_ERR_UNSUPPORTED, "pooling window: kernel >= 1, stride >= 1, 0 <= pad < kernel");
    L.in_dtype = L.out_dtype = G.tensors[op.in[0]].dtype;
    L.r[0] = ref_of(vx, L.in_dtype);
    L.r[1] = ref_t(gr.out);
    L.u.pool = a;
    double n_out = (double)a.NB * a.OH * a.OW * a.C;
    L.flops = n_out * a.k * a.k;
    L.bytes = dtype_bytes(L.in_dtype) * ((double)vx.numel() + n_out);
    return L;
  }

  Launch eltwise(const Group& gr) {
    Launch L;
    L.group = gr.gid;
    L.kernel = K_ELTWISE;
    EltArgs a{};
    Dims od = eval_dims(gr.out);
    if (od.size() > 6) throw Error(SOD2_ERR_UNSUPPORTED, "elementwise group above rank 6");
    a.rank = (int)od.size();
    a.total = 1;
    for (size_t i = 0; i < od.size(); ++i) { a.dims[i] = od[i]; a.total *= od[i]; }
    L.out_dtype = G.tensors[gr.out].dtype;
    if (L.out_dtype != SOD2_BF16 && L.out_dtype != SOD2_F32) throw Error(SOD2_ERR_UNSUPPORTED, "elementwise output dtype");
    auto add_input = [&](int t) -> int {
      const View& v = view_of(t);
      int dt = G.tensors[t].dtype;
      if (dt != SOD2_BF16 && dt != SOD2_F32) throw Error(SOD2_ERR_UNSUPPORTED, "elementwise operand dtype");
      if (a.n_in >= 5) throw Error(SOD2_ERR_UNSUPPORTED, "elementwise group with more than 5 operands");
      if (v.dims.size() > od.size()) throw Error(SOD2_ERR_SHAPE_MISMATCH, "operand rank above the output rank");
      int k = a.n_in++;
      size_t pad = od.size() - v.dims.size();
      for (size_t i = 0; i < od.size(); ++i) {
        int64_t d = i < pad ? 1 : v.dims[i - pad];
        if (d != 1 && d != od[i]) throw Error(SOD2_ERR_SHAPE_MISMATCH, "operand does not broadcast to the output");
        a.stride[k][i] = d == 1 ? 0 : v.strides[i - pad];
      }
      a.in_bf16[k] = dt == SOD2_BF16;
      L.r[k] = ref_of(v, dt);
      L.bytes += (double)v.numel() * dtype_bytes(dt);
      return k;
    };
    int cur = -1;
    for (size_t k = 0; k < gr.chain.size(); ++k) {
      const Op& op = G.ops[gr.chain[k]];
      int primary = op.in[0];
      if (k == 0) { add_input(primary); }
      else if (op.in.size() == 2 && op.in[1] == cur) primary = op.in[1];
      else primary = cur;
      int o = a.n_ops++;
      a.src[o] = -1;
      switch (op.kind) {
        case SOD2_OP_ADD: a.op[o] = E_ADD; break;
        case SOD2_OP_MUL: a.op[o] = E_MUL; break;
        case SOD2_OP_RELU: a.op[o] = E_RELU; break;
        case SOD2_OP_GELU: a.op[o] = E_GELU; break;
        case SOD2_OP_SIGMOID: a.op[o] = E_SIGMOID; break;
        case SOD2_OP_ROUND: a.op[o] = E_ROUND; break;
        default: {                                     // Cast: what it rounds to is part of the value, also inside a chain
          const int to = G.tensors[op.out[0]].dtype;
          if (is_int(to)) throw Error(SOD2_ERR_UNSUPPORTED, "Cast to an integer type in an elementwise group");
          a.op[o] = to == SOD2_BF16 ? E_CAST_BF16 : E_CAST;
          break;
        }
      }
      if (op.in.size() == 2) {
        int ot = (k == 0) ? op.in[1] : other(op, cur);
        const Tensor& td = G.tensors[ot];
        if (td.has_data && td.fdata.size() == 1) { a.src[o] = 5; a.imm[o] = (float)td.fdata[0]; }
        else a.src[o] = add_input(ot);
      }
      (void)primary;
      cur = op.out[0];
    }
    L.r[5] = ref_t(gr.out);
    L.in_dtype = L.out_dtype;
    L.u.elt = a;
    L.flops = (double)a.total * a.n_ops;
    L.bytes += (double)a.total * dtype_bytes(L.out_dtype);
    return L;
  }

  // COPY: a view operator whose result is a graph output; the view of its operand, read through its strides by the
  // elementwise kernel (one identity operation) and written densely
  Launch copy(const Group& gr) {
    Launch L;
    L.group = gr.gid;
    L.kernel = K_ELTWISE;
    const Op& op = G.ops[gr.ops[0]];
    const int dt = G.tensors[op.in[0]].dtype;
    if ((dt != SOD2_BF16 && dt != SOD2_F32) || G.tensors[gr.out].dtype != dt)
      throw Error(SOD2_ERR_UNSUPPORTED, "a view that is a graph output is copied by the elementwise kernel: bf16 or f32 only");
    const View src = derived_view(op, gr.out);
    if (src.dims.size() > 6) throw Error(SOD2_ERR_UNSUPPORTED, "elementwise group above rank 6");
    EltArgs a{};
    a.rank = (int)src.dims.size();
    a.total = 1;
    for (size_t i = 0; i < src.dims.size(); ++i) { a.dims[i] = src.dims[i]; a.total *= src.dims[i]; a.stride[0][i] = src.strides[i]; }
    if (a.rank == 0) { a.rank = 1; a.dims[0] = 1; a.stride[0][0] = 0; }
    a.n_in = 1;
    a.in_bf16[0] = dt == SOD2_BF16;
    a.n_ops = 1;
    a.op[0] = E_CAST;
    a.src[0] = -1;
    L.in_dtype = L.out_dtype = dt;
    L.r[0] = ref_of(src, dt);
    L.r[5] = ref_t(gr.out);
    L.u.elt = a;
    L.bytes = 2.0 * (double)a.total * dtype_bytes(dt);
    return L;
  }

  Launch gather(const Group& gr) {
    Launch L;
    L.group = gr.gid;
    L.kernel = K_GATHER;
    const Op& op = G.ops[gr.chain[0]];
    const View &vt = view_of(op.in[0]), &vi = view_of(op.in[1]);
    int dt = G.tensors[op.in[0]].dtype, it = G.tensors[op.in[1]].dtype;
    if (vt.dims.size() < 1 || !vt.contiguous() || vi.dims.size() != 1 || !vi.contiguous() || !is_int(it) ||
        (!op.ia.empty() && op.ia[0] != 0) || (dt != SOD2_BF16 && dt != SOD2_F32) || G.tensors[gr.out].dtype != dt)
      throw Error(SOD2_ERR_UNSUPPORTED, "Gather kernel: leading-dim slices of a contiguous float tensor by a rank-1 index tensor");
    GatherArgs a{};
    int64_t slice = 1;                                 // elements of one slice table[i, ...]
    for (size_t k = 1; k < vt.dims.size(); ++k) slice *= vt.dims[k];
    if (slice > 0x7fffffff) throw Error(SOD2_ERR_UNSUPPORTED, "Gather kernel: slice too large");
    a.rows = vi.dims[0];
    a.cols = (int)slice;
    a.table_rows = vt.dims[0];
    a.idx_i32 = it == SOD2_I32;
    L.in_dtype = L.out_dtype = dt;
    L.r[0] = ref_of(vt, dt);
    L.r[1] = ref_of(vi, it);
    L.r[2] = ref_t(gr.out);
    if (gr.chain.size() > 1) {
      const Op& add = G.ops[gr.chain[1]];
      int o = other(add, op.out[0]);
      const View& va = view_of(o);
      if (G.tensors[o].dtype != dt || va.dims.size() != 2 || va.dims[0] != a.rows || va.dims[1] != a.cols ||
          va.strides[1] != 1)
        throw Error(SOD2_ERR_UNSUPPORTED, "Gather kernel: the added operand must be a [rows, cols] tensor of the same type");
      a.add_stride = va.strides[0];
      L.r[3] = ref_of(va, dt);
    }
    L.u.gather = a;
    L.flops = gr.chain.size() > 1 ? (double)a.rows * a.cols : 0;
    L.bytes = dtype_bytes(dt) * (double)a.rows * a.cols * (gr.chain.size() > 1 ? 3 : 2) + dtype_bytes(it) * (double)a.rows;
    return L;
  }

  Launch append(const Group& gr) {
    Launch L;
    L.group = gr.gid;
    L.kernel = K_APPEND;
    const Op& op = G.ops[gr.chain[0]];
    const View &vc = view_of(op.in[0]), &vx = view_of(op.in[1]), &vo = view_of(gr.out);
    int dt = G.tensors[op.in[0]].dtype;
    if (G.tensors[op.in[1]].dtype != dt || vx.dims.size() != 2 || vc.dims.size() != 2 || vx.dims[1] != vc.dims[1] ||
        (vx.dims[1] != 1 && vx.strides[1] != 1) || vo.dims[0] != vc.dims[0] + vx.dims[0])
      throw Error(SOD2_ERR_UNSUPPORTED, "CacheAppend kernel: [past, cols] extended by [rows, cols] with a dense last dim");
    AppendArgs a{};
    a.rows = vx.dims[0];
    a.cols = (int)vx.dims[1];
    a.past = vc.dims[0];
    a.x_stride = vx.strides[0];
    L.in_dtype = L.out_dtype = dt;
    L.r[0] = ref_of(vx, dt);
    L.r[1] = ref_of(vo, dt);
    L.u.append = a;
    L.bytes = 2.0 * dtype_bytes(dt) * a.rows * a.cols;
    return L;
  }

  Launch argmax(const Group& gr) {
    Launch L;
    L.group = gr.gid;
    L.kernel = K_ARGMAX;
    const Op& op = G.ops[gr.chain[0]];
    const View& vx = view_of(op.in[0]);
    int dt = G.tensors[op.in[0]].dtype, ot = G.tensors[gr.out].dtype;
    if ((dt != SOD2_BF16 && dt != SOD2_F32) || !is_int(ot)) throw Error(SOD2_ERR_UNSUPPORTED, "ArgMax kernel: float rows to an integer index");
    ArgmaxArgs a{};
    int64_t nrows, xs;
    rows_of(vx, &nrows, &xs);
    a.rows = nrows;
    a.x_stride = xs;
    a.cols = (int)vx.dims.back();
    a.out_i32 = ot == SOD2_I32;
    L.in_dtype = dt;
    L.out_dtype = ot;
    L.r[0] = ref_of(vx, dt);
    L.r[1] = ref_t(gr.out);
    L.u.argmax = a;
    L.flops = (double)a.rows * a.cols;
    L.bytes = dtype_bytes(dt) * (double)a.rows * a.cols + dtype_bytes(ot) * (double)a.rows;
    return L;
  }

  // fused attention group: MatMul(q, k^T) [* scale] -> Softmax -> MatMul(p, v) [-> Transpose]
  Launch attention(const Group& gr) {
    Launch L;
    L.group = gr.gid;
    L.kernel = K_ATTENTION;
    const Op *mm1 = nullptr, *mm2 = nullptr, *sm = nullptr, *tp = nullptr;
    std::vector<const Op*> appends;                 // CacheAppend members: the kernel writes the new rows
    float scale = 1.f;
    int cur = -1;
    for (int n : gr.chain) {
      const Op& op = G.ops[n];
      if (op.kind == SOD2_OP_CACHEAPPEND) { appends.push_back(&op); continue; }
      if (op.kind == SOD2_OP_MATMUL) { (mm1 ? mm2 : mm1) = &op; }
      else if (op.kind == SOD2_OP_MUL) scale *= (float)G.tensors[other(op, cur)].fdata.at(0);
      else if (op.kind == SOD2_OP_SOFTMAX) sm = &op;
      else if (op.kind == SOD2_OP_TRANSPOSE) tp = &op;
      cur = op.out[0];
    }
    if (!mm1 || !mm2 || !sm) throw Error(SOD2_ERR_UNSUPPORTED, "malformed attention group");
    const int dt = SOD2_BF16;
    L.in_dtype = L.out_dtype = dt;
    const View &vq = view_of(mm1->in[0]), &vk = view_of(mm1->in[1]), &vv = view_of(mm2->in[1]);
    bool tb1 = !mm1->ia.empty() && mm1->ia[0], tb2 = !mm2->ia.empty() && mm2->ia[0];
    size_t r = vq.dims.size();
    if (r < 2 || vk.dims.size() != r || vv.dims.size() != r || r > 4)
      throw Error(SOD2_ERR_UNSUPPORTED, "attention operands must share one rank of 2 to 4");
    // logical [batch..., Lq, d] x [batch..., Lk, d] -> [batch..., Lq, Lk]; the second operand of a MatMul without
    // transB is [.., d, Lk]
    auto dim = [](const View& v, size_t i) { return v.dims[i]; };
    auto str = [](const View& v, size_t i) { return v.strides[i]; };
    const size_t kd = tb1 ? r - 1 : r - 2, kn = tb1 ? r - 2 : r - 1;      // d axis / key axis of k
    const size_t vn = tb2 ? r - 1 : r - 2, vd = tb2 ? r - 2 : r - 1;      // key axis / d axis of v
    AttnArgs a{};
    a.Lq = (int)dim(vq, r - 2);
    a.Lk = (int)dim(vk, kn);
    if (dim(vq, r - 1) != 64 || dim(vk, kd) != 64 || dim(vv, vd) != 64 || dim(vv, vn) != a.Lk)
      throw Error(SOD2_ERR_SHAPE_MISMATCH, "attention needs head size 64 and matching key counts");
    if ((dim(vq, r - 1) != 1 && str(vq, r - 1) != 1) || str(vk, kd) != 1 || str(vv, vd) != 1)
      throw Error(SOD2_ERR_UNSUPPORTED, "attention operands need a dense head dim");
    a.causal = !sm->ia.empty() && sm->ia[0];
    if (a.causal && a.Lk < a.Lq) throw Error(SOD2_ERR_UNSUPPORTED, "causal attention with fewer keys than queries");
    if (!(scale > 0.f)) throw Error(SOD2_ERR_UNSUPPORTED, "fused attention kernel: the score scale must be positive");
    a.scale = scale;
    a.q_sm = a.Lq == 1 ? 0 : str(vq, r - 2);            // the stride of a dim of size 1 carries no meaning
    a.k_sn = a.Lk == 1 ? 0 : str(vk, kn);
    a.v_sn = a.Lk == 1 ? 0 : str(vv, vn);
    // output strides per logical dim of mm2's result [batch..., Lq, d], through the absorbed Transpose
    Dims logical = eval_dims(mm2->out[0]), cs;
    if (tp) {
      Dims od(logical.size());
      for (size_t i = 0; i < tp->ia.size(); ++i) od[i] = logical[tp->ia[i]];
      Dims os = contiguous_strides(od);
      cs.assign(logical.size(), 0);
      for (size_t i = 0; i < tp->ia.size(); ++i) cs[tp->ia[i]] = os[i];
    } else {
      cs = contiguous_strides(logical);
    }
    if (cs[r - 1] != 1) throw Error(SOD2_ERR_UNSUPPORTED, "attention output needs a dense head dim");
    a.o_sm = a.Lq == 1 ? 0 : cs[r - 2];
    size_t nbatch = r - 2;
    if (nbatch > 2) throw Error(SOD2_ERR_UNSUPPORTED, "attention with more than two batch dims");
    int64_t nb[2] = {1, 1}, qs[2] = {0, 0}, ks[2] = {0, 0}, vs[2] = {0, 0}, os[2] = {0, 0};
    for (size_t j = 0; j < nbatch; ++j) {
      size_t slot = 2 - nbatch + j;
      nb[slot] = logical[j];
      auto bs = [&](const View& v) { return v.dims[j] == 1 ? 0 : v.strides[j]; };
      if ((vq.dims[j] != 1 && vq.dims[j] != logical[j]) || (vk.dims[j] != 1 && vk.dims[j] != logical[j]) ||
          (vv.dims[j] != 1 && vv.dims[j] != logical[j]))
        throw Error(SOD2_ERR_SHAPE_MISMATCH, "attention batch dims do not broadcast");
      qs[slot] = bs(vq); ks[slot] = bs(vk); vs[slot] = bs(vv); os[slot] = cs[j];
    }
    a.nb0 = (int)nb[0]; a.nb1 = (int)nb[1];
    a.q_sb0 = qs[0]; a.q_sb1 = qs[1]; a.k_sb0 = ks[0]; a.k_sb1 = ks[1];
    a.v_sb0 = vs[0]; a.v_sb1 = vs[1]; a.o_sb0 = os[0]; a.o_sb1 = os[1];
    for (int64_t s8 : {a.q_sm, a.k_sn, a.v_sn, a.q_sb0, a.q_sb1, a.k_sb0, a.k_sb1, a.v_sb0, a.v_sb1})
      if (s8 % 8 != 0) throw Error(SOD2_ERR_UNSUPPORTED, "attention operand strides must be multiples of 8 elements");
    for (int64_t s4 : {a.o_sm, a.o_sb0, a.o_sb1})
      if (s4 % 4 != 0) throw Error(SOD2_ERR_UNSUPPORTED, "attention output strides must be multiples of 4 elements");
    L.r[0] = ref_of(vq, dt);
    L.r[1] = ref_of(vk, dt);
    L.r[2] = ref_of(vv, dt);
    L.r[3] = ref_t(gr.out);
    if (!appends.empty()) {
      // which append feeds the keys, which the values: by the session slot the operand views live in
      const Op *ak = nullptr, *av = nullptr;
      for (const Op* ca : appends) {
        int root = b.session_root.at(ca->out[0]);
        if (root == vk.base) ak = ca;
        if (root == vv.base) av = ca;
      }
      if (appends.size() != 2 || !ak || !av || ak == av) throw Error(SOD2_ERR_UNSUPPORTED, "attention with cache appends: one for the keys, one for the values");
      const View &nk = view_of(ak->in[1]), &nv = view_of(av->in[1]);
      const View &ck = view_of(ak->out[0]), &cv = view_of(av->out[0]);
      const int64_t row = ck.dims.size() == 2 ? ck.dims[1] : -1;
      bool ok = nk.dims.size() == 2 && nv.dims.size() == 2 && cv.dims.size() == 2 && nk.dims[0] == nv.dims[0] &&
                nk.dims[1] == row && nv.dims[1] == row && cv.dims[1] == row && nk.strides[1] == 1 && nv.strides[1] == 1 &&
                ck.dims[0] == a.Lk && cv.dims[0] == a.Lk && nk.dims[0] <= 4 && a.Lq <= 4 && a.Lk <= 4096 && a.nb0 == 1 &&
                a.k_sb1 == 64 && a.v_sb1 == 64 && (int64_t)a.nb1 * 64 == row && (a.Lk == 1 || (a.k_sn == row && a.v_sn == row)) &&
                G.tensors[ak->in[1]].dtype == dt && G.tensors[av->in[1]].dtype == dt;
      if (!ok) throw Error(SOD2_ERR_UNSUPPORTED, "attention with cache appends: at most 4 new bf16 rows [n, heads * 64], at most 4 queries, at most 4096 keys");
      a.n_new = (int)nk.dims[0];
      a.new_k_sn = a.n_new == 1 ? 0 : nk.strides[0];
      a.new_v_sn = a.n_new == 1 ? 0 : nv.strides[0];
      if (a.new_k_sn % 8 != 0 || a.new_v_sn % 8 != 0) throw Error(SOD2_ERR_UNSUPPORTED, "attention operand strides must be multiples of 8 elements");
      L.r[4] = ref_of(nk, dt);
      L.r[5] = ref_of(nv, dt);
    }
    for (int i = 0; i < 6; ++i)
      if (L.r[i].byte_off % 16 != 0) throw Error(SOD2_ERR_UNSUPPORTED, "attention operands must be 16-byte aligned");
    L.u.attn = a;
    double batch = (double)a.nb0 * a.nb1;
    L.flops = 4.0 * batch * a.Lq * a.Lk * 64 * (a.causal ? 0.5 : 1.0);
    L.bytes = 2.0 * batch * 64 * (2.0 * a.Lq + 2.0 * a.Lk);
    return L;
  }

  // NonZero: indices [rank, count] into the upper-bound storage, the count behind them
  Launch nonzero(const Group& gr) {
    Launch L;
    L.group = gr.gid;
    L.kernel = K_NONZERO;
    const Op& op = G.ops[gr.ops[0]];
    const View& vx = view_of(op.in[0]);
    int dt = G.tensors[op.in[0]].dtype;
    if (!vx.contiguous() || vx.dims.size() > 4 || G.tensors[gr.out].dtype != SOD2_I64)
      throw Error(SOD2_ERR_UNSUPPORTED, "NonZero kernel: a contiguous tensor of rank <= 4, int64 result");
    if (!b.tensors.count(gr.out))                      // a caller buffer has no room for the count
      throw Error(SOD2_ERR_UNSUPPORTED, "the result of NonZero must be an intermediate tensor (read it through a Gather or Cast)");
    NonzeroArgs a{};
    a.rank = (int)vx.dims.size();
    a.n = 1;
    for (int k = 0; k < a.rank; ++k) { a.dims[k] = vx.dims[k]; a.n *= vx.dims[k]; }
    a.x_kind = dt == SOD2_F32 ? 0 : (dt == SOD2_BF16 ? 1 : (dt == SOD2_I64 ? 2 : 3));
    L.in_dtype = dt;
    L.out_dtype = SOD2_I64;
    L.r[0] = ref_of(vx, dt);
    L.r[1] = ref_t(gr.out);
    L.r[2] = L.r[1];                                   // the count: behind rank x upper bound indices
    L.r[2].byte_off += (int64_t)a.rank * a.n * 8;
    L.u.nz = a;
    L.bytes = (double)a.n * dtype_bytes(dt);
    return L;
  }

  // NMS: the kept boxes' indices into the upper-bound storage (one per box), the count behind them
  Launch nms(const Group& gr) {
    Launch L;
    L.group = gr.gid;
    L.kernel = K_NMS;
    const Op& op = G.ops[gr.ops[0]];
    const View &vs = view_of(op.in[0]), &vb = view_of(op.in[1]);
    if (G.tensors[op.in[0]].dtype != SOD2_F32 || G.tensors[op.in[1]].dtype != SOD2_F32 || G.tensors[gr.out].dtype != SOD2_I64 ||
        !vs.contiguous() || !vb.contiguous() || vs.dims.size() != 1 || vb.dims.size() != 2 || vb.dims[1] != 4)
      throw Error(SOD2_ERR_UNSUPPORTED, "NMS kernel: dense f32 scores [N] and boxes [N, 4], int64 result");
    if (vb.dims[0] != vs.dims[0]) throw Error(SOD2_ERR_SHAPE_MISMATCH, "NMS: one score per box");
    if (vs.dims[0] > NMS_MAX_BOXES) throw Error(SOD2_ERR_UNSUPPORTED, "NMS kernel: at most " + std::to_string(NMS_MAX_BOXES) + " boxes");
    if (!b.tensors.count(gr.out))                      // a caller buffer has no room for the count
      throw Error(SOD2_ERR_UNSUPPORTED, "the result of NMS must be an intermediate tensor (read it through a Gather or Cast)");
    NmsArgs a{};
    a.n = (int)vs.dims[0];
    a.max_out = op.ia.empty() ? 0 : (int)op.ia[0];
    a.iou = (float)op.fa;
    if (a.max_out < 0) throw Error(SOD2_ERR_INVALID_ARG, "NMS: max_out must not be negative");
    L.in_dtype = SOD2_F32;
    L.out_dtype = SOD2_I64;
    L.r[0] = ref_of(vs, SOD2_F32);
    L.r[1] = ref_of(vb, SOD2_F32);
    L.r[2] = ref_t(gr.out);
    L.r[3] = L.r[2];                                   // the count: behind the upper bound of n indices
    L.r[3].byte_off += (int64_t)a.n * 8;
    L.u.nms = a;
    L.bytes = 20.0 * a.n;
    return L;
  }

  Launch scatter(const Group& gr) {
    Launch L;
    L.group = gr.gid;
    L.kernel = K_SCATTER;
    const Op& op = G.ops[gr.ops[0]];
    const View &vx = view_of(op.in[0]), &vi = view_of(op.in[1]), &vy = view_of(op.in[2]);
    int dt = G.tensors[op.in[0]].dtype, it = G.tensors[op.in[1]].dtype;
    bool same_tail = vx.dims.size() == vy.dims.size() && vx.dims.size() >= 1;
    for (size_t k = 1; same_tail && k < vx.dims.size(); ++k) same_tail = vx.dims[k] == vy.dims[k];
    if (!same_tail || !vx.contiguous() || !vy.contiguous() || vi.dims.size() != 1 || !vi.contiguous() || !is_int(it) ||
        vy.dims[0] != vi.dims[0] || (dt != SOD2_BF16 && dt != SOD2_F32) || G.tensors[op.in[2]].dtype != dt ||
        G.tensors[gr.out].dtype != dt)
      throw Error(SOD2_ERR_UNSUPPORTED, "ScatterRows kernel: contiguous float tensors x[rows, ...], y[n, ...] and a rank-1 index tensor of n entries");
    ScatterArgs a{};
    a.rows = vx.dims[0];
    a.n = vi.dims[0];
    a.cols = 1;
    for (size_t k = 1; k < vx.dims.size(); ++k) a.cols *= vx.dims[k];
    a.idx_i32 = it == SOD2_I32;
    L.in_dtype = L.out_dtype = dt;
    L.r[0] = ref_of(vx, dt);
    L.r[1] = ref_of(vi, it);
    L.r[2] = ref_of(vy, dt);
    L.r[3] = ref_t(gr.out);
    L.u.scatter = a;
    L.bytes = 2.0 * a.rows * a.cols * dtype_bytes(dt);
    return L;
  }

  // copy unit of a dense row of `elems` elements: 16 bytes when every pointer offset and row allows it
  static int copy_unit(int64_t eb, std::initializer_list<int64_t> row_elems, std::initializer_list<int64_t> byte_offs) {
    bool v16 = true;
    for (int64_t e : row_elems) if ((e * eb) % 16 != 0) v16 = false;
    for (int64_t o : byte_offs) if (o % 16 != 0) v16 = false;
    return v16 ? 16 : (int)eb;
  }

  Launch resize(const Group& gr) {
    Launch L;
    L.group = gr.gid;
    L.kernel = K_RESIZE;
    const Op& op = G.ops[gr.ops[0]];
    const View &vx = view_of(op.in[0]), &vo = view_of(gr.out);
    int dt = G.tensors[op.in[0]].dtype;
    size_t r = vx.dims.size();
    if (!vx.contiguous() || r < 1 || r > 4 || vo.dims.size() != r || vo.dims[r - 1] != vx.dims[r - 1] ||
        (dt != SOD2_BF16 && dt != SOD2_F32) || G.tensors[gr.out].dtype != dt)
      throw Error(SOD2_ERR_UNSUPPORTED, "Resize kernel: nearest neighbour on a dense float tensor of rank <= 4 whose last dim is kept");
    ResizeArgs a{};
    for (int k = 0; k < 3; ++k) a.in[k] = a.out[k] = 1;
    for (size_t k = 0; k + 1 < r; ++k) { a.in[3 - (r - 1) + k] = vx.dims[k]; a.out[3 - (r - 1) + k] = vo.dims[k]; }
    for (int k = 0; k < 3; ++k) if (a.in[k] <= 0 && a.out[k] > 0) throw Error(SOD2_ERR_SHAPE_MISMATCH, "Resize from an empty dim");
    L.in_dtype = L.out_dtype = dt;
    L.r[0] = ref_of(vx, dt);
    L.r[1] = ref_t(gr.out);
    int64_t eb = dtype_bytes(dt), c = vx.dims[r - 1];
    L.unit_bytes = copy_unit(eb, {c}, {L.r[0].byte_off, L.r[1].byte_off});
    a.row_units = c * eb / L.unit_bytes;
    L.u.resize = a;
    L.bytes = (double)eb * ((double)vx.numel() + (double)vo.numel());
    return L;
  }

  Launch concat(const Group& gr) {
    Launch L;
    L.group = gr.gid;
    L.kernel = K_CONCAT;
    const Op& op = G.ops[gr.ops[0]];
    const View& vo = view_of(gr.out);
    int dt = G.tensors[gr.out].dtype;
    size_t r = vo.dims.size(), n = op.in.size();
    int64_t ax = op.ia.empty() ? 0 : ((op.ia[0] % (int64_t)r) + (int64_t)r) % (int64_t)r;
    if (n < 1 || n > 4 || r < 1 || (dt != SOD2_BF16 && dt != SOD2_F32))
      throw Error(SOD2_ERR_UNSUPPORTED, "Concat kernel: up to 4 dense float tensors");
    // dense operands joined along axis ax: for every index of the dims before ax, operand k contributes one run of
    // (its extent along ax) x (the dims behind ax) elements -- rows of runs, whatever the axis
    ConcatArgs a{};
    a.n_in = (int)n;
    a.rows = 1;
    for (int64_t k = 0; k < ax; ++k) a.rows *= vo.dims[k];
    int64_t inner = 1;
    for (size_t k = (size_t)ax + 1; k < r; ++k) inner *= vo.dims[k];
    int64_t eb = dtype_bytes(dt);
    int64_t cols[4] = {0, 0, 0, 0};
    bool v16 = true;
    for (size_t k = 0; k < n; ++k) {
      const View& vi = view_of(op.in[k]);
      if (!vi.contiguous() || vi.dims.size() != r || G.tensors[op.in[k]].dtype != dt)
        throw Error(SOD2_ERR_UNSUPPORTED, "Concat kernel: operands must be dense and of the result's type and rank");
      for (size_t j = 0; j < r; ++j)
        if ((int64_t)j != ax && vi.dims[j] != vo.dims[j]) throw Error(SOD2_ERR_SHAPE_MISMATCH, "Concat operands differ outside the axis");
      cols[k] = vi.dims[ax] * inner;
      L.r[k] = ref_of(vi, dt);
      if ((cols[k] * eb) % 16 != 0 || L.r[k].byte_off % 16 != 0) v16 = false;
    }
    L.r[4] = ref_t(gr.out);
    if (L.r[4].byte_off % 16 != 0) v16 = false;
    L.unit_bytes = v16 ? 16 : (int)eb;
    for (size_t k = 0; k < n; ++k) a.units[k] = cols[k] * eb / L.unit_bytes;
    L.in_dtype = L.out_dtype = dt;
    L.u.concat = a;
    L.bytes = 2.0 * eb * (double)vo.numel();
    return L;
  }

  Launch range(const Group& gr) {
    Launch L;
    L.group = gr.gid;
    L.kernel = K_RANGE;
    const Op& op = G.ops[gr.ops[0]];
    int dt = G.tensors[gr.out].dtype;
    const LS &vs = p.rdp->V[op.in[0]], &vd = p.rdp->V[op.in[2]];
    if (!is_int(dt) || !vs.is_list() || vs.d.size() != 1 || !vs.d[0].val() || !vd.is_list() || vd.d.size() != 1 ||
        !vd.d[0].val() || !vd.d[0].e.is_const())
      throw Error(SOD2_ERR_UNSUPPORTED, "Range kernel: start and delta must be known from the value maps");
    RangeArgs a{};
    a.start = vs.d[0].e.eval(b.env);
    a.delta = vd.d[0].e.const_value();
    a.n = eval_dims(gr.out).at(0);
    a.out_i32 = dt == SOD2_I32;
    L.in_dtype = L.out_dtype = dt;
    L.r[0] = ref_t(gr.out);
    L.u.range = a;
    L.bytes = (double)a.n * dtype_bytes(dt);
    return L;
  }

  Launch fill(const Group& gr) {
    Launch L;
    L.group = gr.gid;
    L.kernel = K_FILL;
    const Op& op = G.ops[gr.ops[0]];
    int dt = G.tensors[gr.out].dtype;
    Dims od = eval_dims(gr.out);
    FillArgs a{};
    a.n = 1;
    for (int64_t d : od) a.n *= d;
    a.dtype = dt;
    if (op.kind == SOD2_OP_EYELIKE) {
      if (od.size() != 2) throw Error(SOD2_ERR_SHAPE_MISMATCH, "EyeLike needs a matrix");
      a.cols = od[1];
      a.diag = op.ia.empty() ? 0 : op.ia[0];
      if (a.cols == 0) a.n = 0;
    } else {
      a.value = (float)op.fa;
    }
    L.in_dtype = L.out_dtype = dt;
    L.r[0] = ref_t(gr.out);
    L.u.fill = a;
    L.bytes = (double)a.n * dtype_bytes(dt);
    return L;
  }

  Launch onehot(const Group& gr) {
    Launch L;
    L.group = gr.gid;
    L.kernel = K_ONEHOT;
    const Op& op = G.ops[gr.ops[0]];
    const View& vi = view_of(op.in[0]);
    int it = G.tensors[op.in[0]].dtype, dt = G.tensors[gr.out].dtype;
    const Tensor& vals = G.tensors[op.in[2]];
    if (!is_int(it) || !vi.contiguous() || (dt != SOD2_BF16 && dt != SOD2_F32) || !vals.has_data || vals.fdata.size() != 2)
      throw Error(SOD2_ERR_UNSUPPORTED, "OneHot kernel: dense integer indices, a float result, values = host constant [off, on]");
    Dims od = eval_dims(gr.out);
    OneHotArgs a{};
    a.n = vi.numel();
    a.depth = od.back();
    if (a.depth < 0) throw Error(SOD2_ERR_INVALID_ARG, "OneHot with a negative depth");
    a.off = (float)vals.fdata[0];
    a.on = (float)vals.fdata[1];
    a.idx_i32 = it == SOD2_I32;
    a.out_bf16 = dt == SOD2_BF16;
    L.in_dtype = L.out_dtype = dt;
    L.r[0] = ref_of(vi, it);
    L.r[1] = ref_t(gr.out);
    L.u.onehot = a;
    L.bytes = (double)a.n * dtype_bytes(it) + (double)a.n * a.depth * dtype_bytes(dt);
    return L;
  }

  Launch topk(const Group& gr) {
    Launch L;
    L.group = gr.gid;
    L.kernel = K_TOPK;
    const Op& op = G.ops[gr.ops[0]];
    const View& vx = view_of(op.in[0]);
    int dt = G.tensors[op.in[0]].dtype, it = G.tensors[op.out[1]].dtype;
    if (!vx.contiguous() || vx.dims.empty() || (dt != SOD2_BF16 && dt != SOD2_F32) || G.tensors[gr.out].dtype != dt || !is_int(it))
      throw Error(SOD2_ERR_UNSUPPORTED, "TopK kernel: last axis of a dense float tensor, integer positions");
    Dims od = eval_dims(gr.out);
    TopKArgs a{};
    a.n = vx.dims.back();
    a.k = od.back();
    a.rows = a.n > 0 ? vx.numel() / a.n : 0;
    if (a.k < 0 || a.k > a.n) throw Error(SOD2_ERR_INVALID_ARG, "TopK: k outside [0, extent of the last axis]");
    a.x_bf16 = dt == SOD2_BF16;
    a.idx_i32 = it == SOD2_I32;
    L.in_dtype = L.out_dtype = dt;
    L.r[0] = ref_of(vx, dt);
    L.r[1] = ref_t(gr.out);
    L.r[2] = ref_t(op.out[1]);
    L.u.topk = a;
    L.bytes = (double)a.rows * (a.n * dtype_bytes(dt) + a.k * (dtype_bytes(dt) + dtype_bytes(it)));
    return L;
  }

  Launch groupnorm(const Group& gr) {
    Launch L;
    L.group = gr.gid;
    L.kernel = K_GROUPNORM;
    const Op& op = G.ops[gr.ops[0]];
    const View& vx = view_of(op.in[0]);
    int dt = G.tensors[op.in[0]].dtype;
    if (!vx.contiguous() || vx.dims.size() < 2 || (dt != SOD2_BF16 && dt != SOD2_F32) || G.tensors[gr.out].dtype != dt ||
        G.tensors[op.in[1]].dtype != dt || G.tensors[op.in[2]].dtype != dt)
      throw Error(SOD2_ERR_UNSUPPORTED, "GroupNorm kernel: a dense float tensor [N, ..., C] with scale and bias of its type");
    GroupNormArgs a{};
    const int64_t C = vx.dims.back(), groups = op.ia.empty() ? 0 : op.ia[0];
    if (groups <= 0 || C % groups != 0) throw Error(SOD2_ERR_SHAPE_MISMATCH, "GroupNorm: the channel count must be a multiple of the group count");
    const View &vg = view_of(op.in[1]), &vb = view_of(op.in[2]);
    if (vg.numel() != C || vb.numel() != C || !vg.contiguous() || !vb.contiguous())
      throw Error(SOD2_ERR_SHAPE_MISMATCH, "GroupNorm: scale and bias must hold one value per channel");
    a.n = vx.dims[0];
    a.s = 1;
    for (size_t k = 1; k + 1 < vx.dims.size(); ++k) a.s *= vx.dims[k];
    a.groups = (int)groups;
    a.cpg = (int)(C / groups);
    a.eps = (float)op.fa;
    L.in_dtype = L.out_dtype = dt;
    L.r[0] = ref_of(vx, dt);
    L.r[1] = ref_t(gr.out);
    L.r[2] = ref_of(vg, dt);
    L.r[3] = ref_of(vb, dt);
    L.u.gn = a;
    L.flops = 8.0 * (double)vx.numel();
    L.bytes = dtype_bytes(dt) * (2.0 * (double)vx.numel() + 2.0 * C);
    return L;
  }

  Launch maxunpool(const Group& gr) {
    Launch L;
    L.group = gr.gid;
    L.kernel = K_MAXUNPOOL;
    const Op& op = G.ops[gr.ops[0]];
    const View &vx = view_of(op.in[0]), &vi = view_of(op.in[1]);
    const int dt = G.tensors[op.in[0]].dtype;
    if (!vx.contiguous() || !vi.contiguous() || (dt != SOD2_BF16 && dt != SOD2_F32) || G.tensors[gr.out].dtype != dt ||
        G.tensors[op.in[1]].dtype != SOD2_I64)
      throw Error(SOD2_ERR_UNSUPPORTED, "MaxUnpool kernel: dense float data, dense int64 positions, a result of the data's type");
    if (vi.dims != vx.dims) throw Error(SOD2_ERR_SHAPE_MISMATCH, "MaxUnpool: data and positions differ in shape");
    UnpoolArgs a{};
    a.n_in = vx.numel();
    a.n_out = 1;
    for (int64_t d : eval_dims(gr.out)) a.n_out *= d;
    L.in_dtype = L.out_dtype = dt;
    L.r[0] = ref_of(vx, dt);
    L.r[1] = ref_of(vi, SOD2_I64);
    L.r[2] = ref_t(gr.out);
    L.u.unpool = a;
    L.bytes = (double)dtype_bytes(dt) * ((double)a.n_in + (double)a.n_out) + 8.0 * (double)a.n_in;
    return L;
  }

  Launch make(const Group& gr) {
    // a result without elements (an empty compacted batch): nothing to compute
    auto od = b.dims.find(gr.out);
    if (od != b.dims.end()) {
      int64_t n = 1;
      for (int64_t d : od->second) n *= d;
      if (n == 0 && gr.kind != G_NONZERO && gr.kind != G_NMS) { Launch L; L.group = gr.gid; L.kernel = K_OTHER; L.empty = true; return L; }
    }
    // The kernels of these groups read every float operand in the group's one storage type: a description that
    // mixes types there would make them read beyond a buffer, so it is refused here (host constants are not read
    // by kernels; elementwise chains, Cast, ReduceMean and the generators convert per operand).
    switch (gr.kind) {
      case G_GEMM: case G_CONV: case G_LAYERNORM: case G_SOFTMAX: case G_GROUPNORM: case G_ATTENTION: case G_MAXPOOL:
      case G_AVGPOOL: case G_CACHEAPPEND: case G_SCATTER: case G_CONCAT: case G_RESIZE: case G_MAXUNPOOL: case G_GATHER: {
        const int dt = G.tensors[gr.out].dtype;
        for (int n : gr.ops)
          for (int t : G.ops[n].in) {
            const Tensor& td = G.tensors[t];
            if (!td.has_data && !is_int(td.dtype) && td.dtype != dt)
              throw Error(SOD2_ERR_UNSUPPORTED, std::string(group_kind_name(gr.kind)) + " group: operand " + td.name +
                                                    " is not of the result's float type");
          }
        break;
      }
      default: break;
    }
    switch (gr.kind) {
      case G_NONZERO: return nonzero(gr);
      case G_NMS: return nms(gr);
      case G_SCATTER: return scatter(gr);
      case G_RANGE: return range(gr);
      case G_FILL: return fill(gr);
      case G_ONEHOT: return onehot(gr);
      case G_TOPK: return topk(gr);
      case G_GROUPNORM: return groupnorm(gr);
      case G_MAXUNPOOL: return maxunpool(gr);
      case G_RESIZE: return resize(gr);
      case G_CONCAT: return concat(gr);
      case G_ATTENTION: return attention(gr);
      case G_GATHER: return gather(gr);
      case G_CACHEAPPEND: return append(gr);
      case G_ARGMAX: return argmax(gr);
      case G_GEMM: return gemm(gr);
      case G_CONV: return conv(gr);
      case G_LAYERNORM: return row(gr, true);
      case G_SOFTMAX: return row(gr, false);
      case G_REDUCEMEAN: return reduce(gr);
      case G_MAXPOOL: case G_AVGPOOL: return pool(gr);
      case G_ELTWISE: return eltwise(gr);
      case G_COPY: return copy(gr);
      default:
        throw Error(SOD2_ERR_UNSUPPORTED, std::string("no kernel for group kind ") + group_kind_name(gr.kind));
    }
  }
};

struct Pointers {
  char* ws = nullptr;        // optional workspace behind the planned arena, or null
  const int* step = nullptr;             // replay: device step counter and the bytes by which each
  const int64_t* in_step = nullptr;      // input / output pointer advances per step
  const int64_t* out_step = nullptr;
  char* arena = nullptr; size_t arena_bytes = 0;
  const void* const* w = nullptr; int nw = 0;
  const void* const* in = nullptr; int nin = 0;
  void* const* out = nullptr; int nout = 0;
  const char* constants = nullptr; size_t constants_bytes = 0;   // constants derived from the weights for folded LayerNorms, or null
  Pointers(void* arena_, size_t bytes, const void* const* w_, int nw_, const void* const* in_, int nin_, void* const* out_, int nout_)
      : arena((char*)arena_), arena_bytes(bytes), w(w_), nw(nw_), in(in_), nin(nin_), out(out_), nout(nout_) {}
  void* at(const Ref& r) const {
    switch (r.space) {
      case SP_ARENA: return arena + r.byte_off;
      case SP_WEIGHT: return (char*)w[r.index] + r.byte_off;
      case SP_INPUT: return (char*)in[r.index] + r.byte_off;
      case SP_OUTPUT: return (char*)out[r.index] + r.byte_off;
      default: return nullptr;
    }
  }
};

bool al16(const void* p) { return ((uintptr_t)p & 15) == 0; }

int tune_group_m() {
  static int v = [] { const char* e = getenv("SOD2_GROUP_M"); int x = e ? atoi(e) : 8; return x > 0 ? x : 8; }();
  return v;
}

hipError_t dispatch(Launch L, const Pointers& P, hipStream_t s) {
  if (L.empty) return hipSuccess;
  switch (L.kernel) {
    case K_NONZERO: {
      NonzeroArgs a = L.u.nz;
      a.x = P.at(L.r[0]); a.out = (long long*)P.at(L.r[1]); a.count = (long long*)P.at(L.r[2]);
      return launch_nonzero(a, s);
    }
    case K_NMS: {
      NmsArgs a = L.u.nms;
      a.scores = (const float*)P.at(L.r[0]); a.boxes = (const float*)P.at(L.r[1]);
      a.out = (long long*)P.at(L.r[2]); a.count = (long long*)P.at(L.r[3]);
      a.ws = P.ws;
      return launch_nms(a, s);
    }
    case K_RANGE: {
      RangeArgs a = L.u.range;
      a.y = P.at(L.r[0]);
      return launch_range(a, s);
    }
    case K_FILL: {
      FillArgs a = L.u.fill;
      a.y = P.at(L.r[0]);
      return launch_fill(a, s);
    }
    case K_TOPK: {
      TopKArgs a = L.u.topk;
      a.x = P.at(L.r[0]); a.values = P.at(L.r[1]); a.indices = P.at(L.r[2]);
      return launch_topk(a, s);
    }
    case K_MAXUNPOOL: {
      UnpoolArgs a = L.u.unpool;
      a.x = P.at(L.r[0]); a.idx = P.at(L.r[1]); a.y = P.at(L.r[2]);
      if (((uintptr_t)a.idx & 7) != 0) return hipErrorInvalidValue;
      return launch_unpool(L, a, s);
    }
    case K_GROUPNORM: {
      GroupNormArgs a = L.u.gn;
      a.x = P.at(L.r[0]); a.y = P.at(L.r[1]); a.gamma = P.at(L.r[2]); a.beta = P.at(L.r[3]);
      return launch_groupnorm(L, a, s);
    }
    case K_ONEHOT: {
      OneHotArgs a = L.u.onehot;
      a.idx = P.at(L.r[0]); a.y = P.at(L.r[1]);
      return launch_onehot(a, s);
    }
    case K_RESIZE: {
      ResizeArgs a = L.u.resize;
      a.x = P.at(L.r[0]); a.y = P.at(L.r[1]);
      if (L.unit_bytes == 16 && (!al16(a.x) || !al16(a.y))) return hipErrorInvalidValue;
      return launch_resize(L, a, s);
    }
    case K_CONCAT: {
      ConcatArgs a = L.u.concat;
      for (int k = 0; k < a.n_in; ++k) {
        a.x[k] = P.at(L.r[k]);
        if (L.unit_bytes == 16 && !al16(a.x[k])) return hipErrorInvalidValue;
      }
      a.y = P.at(L.r[4]);
      if (L.unit_bytes == 16 && !al16(a.y)) return hipErrorInvalidValue;
      return launch_concat(L, a, s);
    }
    case K_SCATTER: {
      ScatterArgs a = L.u.scatter;
      a.x = P.at(L.r[0]); a.idx = P.at(L.r[1]); a.y = P.at(L.r[2]); a.out = P.at(L.r[3]);
      return launch_scatter(L, a, s);
    }
    case K_GEMM: {
      GemmArgs g = L.u.gemm;
      g.A = P.at(L.r[0]); g.B = P.at(L.r[1]); g.C = P.at(L.r[2]);
      g.bias = P.at(L.r[3]); g.res = P.at(L.r[4]);
      g.ln_gamma = P.at(L.r[5]); g.ln_beta = P.at(L.r[6]);
      if (g.ln_gamma && (!al16(g.ln_gamma) || !al16(g.ln_beta))) return hipErrorInvalidValue;
      if (g.M == 1) { g.a_sm = g.K; g.c_sm = g.N; g.r_sm = g.N; }     // the stride of a single row carries no meaning
      g.a_vec = g.a_sk == 1 && g.K % 8 == 0 && g.a_sm % 8 == 0 && g.a_sb0 % 8 == 0 && g.a_sb1 % 8 == 0 && al16(g.A);
      bool bal = g.b_sb0 % 8 == 0 && g.b_sb1 % 8 == 0 && al16(g.B);
      if (g.b_sk == 1 && g.K % 8 == 0 && g.b_sn % 8 == 0 && bal) g.b_mode = 0;
      else if (g.b_sn == 1 && g.N % 8 == 0 && g.b_sk % 8 == 0 && bal) g.b_mode = 1;
      else g.b_mode = 2;
      g.c_vec = g.c_sn == 1 && g.c_sm % 8 == 0 && g.c_sb0 % 8 == 0 && g.c_sb1 % 8 == 0 && al16(g.C) &&
                (!g.bias || al16(g.bias)) &&
                (!g.res || (g.r_sn == 1 && g.r_sm % 8 == 0 && g.r_sb0 % 8 == 0 && g.r_sb1 % 8 == 0 && al16(g.res)));
      g.group_m = tune_group_m();
      if (P.step && L.r[2].space == SP_OUTPUT && P.out_step[L.r[2].index]) {
        g.step = P.step;
        g.c_step = P.out_step[L.r[2].index] / dtype_bytes(L.out_dtype);
      }
      if (g.splits > 1 && P.ws) {
        g.ws = P.ws;
      } else {
        g.splits = 1;
      }
      const bool folding = P.constants != nullptr;             // both sides of every pair see the same answer
      if (L.fold_read && folding) {
        if (L.const_off < 0 || (size_t)L.const_off + 8u * (size_t)g.N > P.constants_bytes) return hipErrorInvalidValue;
        g.fold = 2;
        g.fold_s = P.constants + L.const_off;
        g.fold_c = P.constants + L.const_off + 4ll * g.N;
        g.bias = nullptr;                                      // part of fold_c
      }
      if (L.post_ln && L.fold_pair && folding) {
        g.fold = 1;
        g.fold_y = P.at(L.r[7]);
        g.fold_gamma = P.at(L.r[8]);
      }
      if (g.fold && !(L.variant >= V_DL0 && g.a_vec && g.b_mode == 0 && g.c_vec && al16(g.fold_y) && al16(g.fold_gamma)))
        return hipErrorInvalidValue;                           // the pair was promised a kernel that cannot run here
      hipError_t e = launch_gemm(L, g, s);
      if (e != hipSuccess || !L.post_ln || g.fold == 1) return e;
      RowArgs a = L.post;
      a.x = g.C; a.y = P.at(L.r[7]); a.gamma = P.at(L.r[8]); a.beta = P.at(L.r[9]);
      Launch row;
      row.kernel = K_LAYERNORM;
      row.is_layernorm = true;
      row.in_dtype = row.out_dtype = L.out_dtype;
      return launch_row(row, a, s);
    }
    case K_CONV: {
      ConvArgs c = L.u.conv;
      c.x = P.at(L.r[0]); c.w = P.at(L.r[1]); c.y = P.at(L.r[2]);
      c.bias = P.at(L.r[3]); c.res = P.at(L.r[4]);
      c.vec = c.vec && al16(c.x);
      if (c.splits > 1 && P.ws) c.ws = P.ws;
      else c.splits = 1;
      return launch_conv(L, c, s);
    }
    case K_LAYERNORM: case K_SOFTMAX: {
      RowArgs a = L.u.row;
      a.x = P.at(L.r[0]); a.y = P.at(L.r[1]); a.gamma = P.at(L.r[2]); a.beta = P.at(L.r[3]);
      return launch_row(L, a, s);
    }
    case K_REDUCE: {
      ReduceArgs a = L.u.red;
      a.x = P.at(L.r[0]); a.y = P.at(L.r[1]);
      return launch_reduce(L, a, s);
    }
    case K_POOL: {
      PoolArgs a = L.u.pool;
      a.x = P.at(L.r[0]); a.y = P.at(L.r[1]);
      return launch_pool(L, a, s);
    }
    case K_ELTWISE: {
      EltArgs a = L.u.elt;
      for (int k = 0; k < a.n_in; ++k) a.in[k] = P.at(L.r[k]);
      a.out = P.at(L.r[5]);
      return launch_eltwise(L, a, s);
    }
    case K_ATTENTION: {
      AttnArgs a = L.u.attn;
      a.q = P.at(L.r[0]); a.k = P.at(L.r[1]); a.v = P.at(L.r[2]); a.o = P.at(L.r[3]);
      if (a.n_new > 0) { a.new_k = P.at(L.r[4]); a.new_v = P.at(L.r[5]); }
      if (P.step && L.d_lk) { a.step = P.step; a.lk_step = L.d_lk; }
      if (!al16(a.q) || !al16(a.k) || !al16(a.v) || ((uintptr_t)a.o & 7) || !al16(a.new_k) || !al16(a.new_v)) return hipErrorInvalidValue;
      return launch_attention(a, s);
    }
    case K_GATHER: {
      GatherArgs a = L.u.gather;
      a.table = P.at(L.r[0]); a.idx = P.at(L.r[1]); a.y = P.at(L.r[2]); a.add = P.at(L.r[3]);
      if (P.step && L.r[1].space == SP_INPUT && P.in_step[L.r[1].index]) { a.step = P.step; a.idx_step = P.in_step[L.r[1].index]; }
      return launch_gather(L, a, s);
    }
    case K_APPEND: {
      AppendArgs a = L.u.append;
      a.x = P.at(L.r[0]); a.cache = P.at(L.r[1]);
      if (P.step && L.d_past) { a.step = P.step; a.past_step = L.d_past; }
      return launch_append(L, a, s);
    }
    case K_ARGMAX: {
      ArgmaxArgs a = L.u.argmax;
      a.x = P.at(L.r[0]); a.y = P.at(L.r[1]);
      if (P.step) {
        a.step = P.step;
        a.x_step = L.r[0].space == SP_OUTPUT ? P.out_step[L.r[0].index] : 0;
        a.y_step = L.r[1].space == SP_OUTPUT ? P.out_step[L.r[1].index] : 0;
      }
      return launch_argmax(L, a, s);
    }
    default:
      return hipErrorInvalidValue;
  }
}

// launch table for every executed group step of `b`, indexed by step (-1 kernel for control steps);
// steps before `first_step` (already run when a plan is rebuilt in mid-run) are left unbuilt (-2)
std::vector<Launch> build_launches(const Plan& p, const BindResult& b, int force_variant, int force_splits,
                                   size_t first_step = 0, bool folding = false) {
  Builder B(p, b, force_variant);
  B.force_splits = force_splits;
  B.folding = folding;
  std::vector<Launch> out;
  for (size_t k = 0; k < b.steps.size(); ++k) {
    const Item& it = p.items[b.steps[k]];
    if (k < first_step) { Launch L; L.kernel = -2; L.group = it.ref; out.push_back(L); continue; }
    if (!it.is_group) { Launch L; L.kernel = -1; L.group = it.ref; out.push_back(L); continue; }
    out.push_back(B.make(p.groups.at(it.ref)));
  }
  return out;
}

}  // namespace
}  // namespace sod2

using namespace sod2;

// ---------------------------------------------------------------------------------------------
// Scratch of sod2_run_static: the fp32 partial tiles of split-K contractions, for callers that cannot
// hand over a workspace because they cannot allocate one.  One copy per GPU, held until the process
// ends.  In host code the array's name is only a handle: the address the kernels get comes from
// hipGetSymbolAddress, asked once per device with that device current.
// ---------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[SOD2_STATIC_SCRATCH_BYTES];
namespace {
const int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];          // per device, null until the first call on that device
bool g_scratch_known[kMaxDevices];

// device address of `scratch` on the current device
char* static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
    throw Error(SOD2_ERR_HIP, "current device could not be determined");
  if (!g_scratch_known[dev]) {
    void* ptr = nullptr;
    hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr)
      throw Error(SOD2_ERR_HIP, std::string("address of the static scratch buffer: ") + hipGetErrorString(e));
    g_scratch_ptr[dev] = ptr;
    g_scratch_known[dev] = true;
  }
  return (char*)g_scratch_ptr[dev];
}
}  // namespace

// kernels that must be in flight for sod2_run to plan a Switch's other outcome while it waits for the predicate
static const int SPECULATE_MIN_QUEUED = 8;

// Read-back of the few bytes a run needs on the host (a Switch predicate, a NonZero count).  A one-thread
// kernel, enqueued behind the kernel that produced them, stores the bytes and then a sequence number
// into coherent pinned host memory; the host polls the sequence number.  Against a device-to-host copy
// followed by a stream synchronise this leaves out the copy engine's set-up and the wake-up of a
// blocked thread (config 4: 12 read-backs per call).  One slot per host thread, allocated on first use
// and kept until the process ends.  If the number has not arrived after 20 ms the stream is
// synchronised instead, so an error on the stream is reported rather than waited for.
__global__ void publish_kernel(const unsigned char* src, int nbytes, volatile unsigned long long* host,
                               unsigned long long seq) {
  unsigned long long v = 0;
  for (int i = 0; i < nbytes; ++i) v |= (unsigned long long)src[i] << (8 * i);
  host[0] = v;
  __threadfence_system();
  host[1] = seq;
}
namespace {
struct ReadbackSlot {
  unsigned long long* host = nullptr;
  unsigned long long* dev = nullptr;
  unsigned long long seq = 0;
};
ReadbackSlot& readback_slot() {
  static thread_local ReadbackSlot sl;
  if (!sl.host) {
    void* mem = nullptr;
    if (hipHostMalloc(&mem, 64, hipHostMallocCoherent | hipHostMallocMapped) != hipSuccess)
      throw Error(SOD2_ERR_HIP, "pinned host memory for read-backs could not be allocated");
    void* dev = nullptr;
    if (hipHostGetDevicePointer(&dev, mem, 0) != hipSuccess)
      throw Error(SOD2_ERR_HIP, "pinned host memory for read-backs is not visible to the device");
    std::memset(mem, 0, 64);
    sl.host = (unsigned long long*)mem;
    sl.dev = (unsigned long long*)dev;
  }
  return sl;
}
// enqueue the read-back of nbytes (<= 8) at src
void begin_read_back(const void* src, int nbytes, hipStream_t s) {
  ReadbackSlot& sl = readback_slot();
  ++sl.seq;
  hipLaunchKernelGGL(publish_kernel, dim3(1), dim3(1), 0, s, (const unsigned char*)src, nbytes, sl.dev, sl.seq);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) throw Error(SOD2_ERR_HIP, std::string("read-back launch failed: ") + hipGetErrorString(e));
}
// wait for it; returns the bytes, zero-extended
unsigned long long finish_read_back(hipStream_t s) {
  ReadbackSlot& sl = readback_slot();
  const auto t0 = std::chrono::steady_clock::now();
  int spins = 0;
  while (__atomic_load_n(&sl.host[1], __ATOMIC_ACQUIRE) != sl.seq) {
    __builtin_ia32_pause();
    if ((++spins & 1023) == 0 && std::chrono::steady_clock::now() - t0 > std::chrono::milliseconds(20)) {
      hipError_t e = hipStreamSynchronize(s);
      if (e != hipSuccess) throw Error(SOD2_ERR_HIP, std::string("read-back failed: ") + hipGetErrorString(e));
      if (__atomic_load_n(&sl.host[1], __ATOMIC_ACQUIRE) != sl.seq)
        throw Error(SOD2_ERR_HIP, "the read-back kernel finished without reporting");
      break;
    }
  }
  return __atomic_load_n(&sl.host[0], __ATOMIC_ACQUIRE);
}
}  // namespace

// ---------------------------------------------------------------------------------------------
// Replay: the launch sequence of one step captured in a HIP graph; the quantities that change from
// step to step are read by the kernels from a step counter in device memory
// ---------------------------------------------------------------------------------------------
namespace sod2 {
hipError_t launch_step_set(int* step, int value, hipStream_t s);
hipError_t launch_step_advance(int* step, hipStream_t s);
}
struct sod2_replay_s {
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
  int* step = nullptr;
  int max_steps = 0;
  ~sod2_replay_s() {
    if (exec) (void)hipGraphExecDestroy(exec);
    if (graph) (void)hipGraphDestroy(graph);
  }
};

namespace {
bool same_ref(const Ref& a, const Ref& b) { return a.space == b.space && a.index == b.index && a.byte_off == b.byte_off; }

// Launch b must equal launch a except for the fields a step may move; those are returned as deltas
bool step_delta(const Launch& a, const Launch& b, long long* d_past, int* d_lk) {
  *d_past = 0;
  *d_lk = 0;
  if (a.kernel != b.kernel || a.group != b.group || a.variant != b.variant || a.in_dtype != b.in_dtype ||
      a.out_dtype != b.out_dtype || a.is_layernorm != b.is_layernorm)
    return false;
  for (int i = 0; i < 7; ++i) if (!same_ref(a.r[i], b.r[i])) return false;
  Launch c = b;
  if (a.kernel == K_APPEND) {
    *d_past = b.u.append.past - a.u.append.past;
    c.u.append.past = a.u.append.past;
  } else if (a.kernel == K_ATTENTION) {
    *d_lk = b.u.attn.Lk - a.u.attn.Lk;
    c.u.attn.Lk = a.u.attn.Lk;
  }
  return std::memcmp(&a.u, &c.u, sizeof a.u) == 0;
}
}  // namespace

extern "C" sod2_status sod2_replay_create(const sod2_plan_t* ph, const int64_t* symbols, int32_t n_symbols, int32_t step_symbol,
                                          int32_t max_steps, void* arena, size_t arena_bytes, const void* const* weights,
                                          int32_t n_weights, const void* const* inputs, const int64_t* input_step_bytes,
                                          int32_t n_inputs, void* const* outputs, const int64_t* output_step_bytes,
                                          int32_t n_outputs, int32_t* step_counter, void* stream, sod2_replay_t** out) {
  try {
    if (!ph || !symbols || !out || !step_counter || !stream) throw Error(SOD2_ERR_INVALID_ARG, "null argument (a replay needs a stream of its own, not the null stream)");
    const Plan& p = ph->p;
    const Graph& G = *p.g;
    if (step_symbol < 0 || step_symbol >= n_symbols || max_steps < 1) throw Error(SOD2_ERR_INVALID_ARG, "bad step symbol or step count");
    if (p.n_switches) throw Error(SOD2_ERR_UNSUPPORTED, "a graph with Switch operators cannot be replayed");
    if (n_weights != (int)G.weight_ids.size() || n_inputs != (int)G.input_ids.size() || n_outputs != (int)G.output_ids.size())
      throw Error(SOD2_ERR_INVALID_ARG, "wrong number of weight, input or output pointers");
    if (((uintptr_t)arena & 255) != 0) throw Error(SOD2_ERR_INVALID_ARG, "arena must be 256-byte aligned");
    std::vector<int64_t> s0(symbols, symbols + n_symbols), s1 = s0, sN = s0;
    s1[step_symbol] += max_steps > 1 ? 1 : 0;
    sN[step_symbol] += max_steps - 1;
    BindResult b0 = bind_plan(p, s0, {}, false), b1 = bind_plan(p, s1, {}, false), bN = bind_plan(p, sN, {}, false);
    int64_t need = std::max(b0.arena_bytes, std::max(b1.arena_bytes, bN.arena_bytes));
    if ((size_t)need > arena_bytes) throw Error(SOD2_ERR_ARENA_TOO_SMALL, "arena of " + std::to_string(arena_bytes) + " bytes, the last step needs " + std::to_string(need));
    std::vector<Launch> L0 = build_launches(p, b0, -1, 1), L1 = build_launches(p, b1, -1, 1), LN = build_launches(p, bN, -1, 1);
    if (L0.size() != L1.size() || L0.size() != LN.size()) throw Error(SOD2_ERR_UNSUPPORTED, "the executed steps change with the step symbol");
    for (size_t i = 0; i < L0.size(); ++i) {
      long long dp, dpn;
      int dl, dln;
      if (!step_delta(L0[i], L1[i], &dp, &dl) || !step_delta(L0[i], LN[i], &dpn, &dln) ||
          dpn != dp * (max_steps - 1) || dln != dl * (max_steps - 1))
        throw Error(SOD2_ERR_UNSUPPORTED, "launch " + std::to_string(i) + " (group " + std::to_string(L0[i].group) +
                                              ") depends on the step symbol in a way the kernels cannot follow");
      L0[i].d_past = dp;
      L0[i].d_lk = dl;
      const Launch& L = L0[i];
      if (L.kernel == K_ATTENTION && dl && (L.u.attn.Lq > 4 || LN[i].u.attn.Lk > 4096))
        throw Error(SOD2_ERR_UNSUPPORTED, "only the few-query attention kernel follows a growing key count");
      // operands in caller memory that move with the step must belong to a kernel that follows them
      for (int k = 0; k < 7; ++k) {
        const Ref& r = L.r[k];
        bool moves = (r.space == SP_INPUT && input_step_bytes && input_step_bytes[r.index]) ||
                     (r.space == SP_OUTPUT && output_step_bytes && output_step_bytes[r.index]);
        if (!moves) continue;
        bool ok = (L.kernel == K_GATHER && k == 1) || (L.kernel == K_ARGMAX && k <= 1) ||
                  (L.kernel == K_GEMM && k == 2 && L.variant == V_GEMV);
        if (!ok) throw Error(SOD2_ERR_UNSUPPORTED, "launch " + std::to_string(i) + " reads or writes a stepping pointer it cannot follow");
      }
    }
    std::vector<int64_t> zin(std::max(n_inputs, 1), 0), zout(std::max(n_outputs, 1), 0);
    Pointers P(arena, arena_bytes, weights, n_weights, inputs, n_inputs, outputs, n_outputs);
    P.step = step_counter;
    P.in_step = input_step_bytes ? input_step_bytes : zin.data();
    P.out_step = output_step_bytes ? output_step_bytes : zout.data();
    std::unique_ptr<sod2_replay_s> r(new sod2_replay_s);
    r->step = step_counter;
    r->max_steps = max_steps;
    hipStream_t s = (hipStream_t)stream;
    if (hipStreamBeginCapture(s, hipStreamCaptureModeRelaxed) != hipSuccess) throw Error(SOD2_ERR_HIP, "stream capture could not start");
    hipError_t e = hipSuccess;
    for (const Launch& L : L0) {
      if (L.kernel < 0) continue;
      e = dispatch(L, P, s);
      if (e != hipSuccess) break;
    }
    if (e == hipSuccess) e = launch_step_advance(step_counter, s);
    hipError_t e2 = hipStreamEndCapture(s, &r->graph);
    if (e != hipSuccess || e2 != hipSuccess) throw Error(SOD2_ERR_HIP, std::string("capture failed: ") + hipGetErrorString(e != hipSuccess ? e : e2));
    if (hipGraphInstantiate(&r->exec, r->graph, nullptr, nullptr, 0) != hipSuccess) throw Error(SOD2_ERR_HIP, "graph instantiation failed");
    *out = r.release();
  } catch (const sod2::Error& e) {
    sod2::set_error(e.what());
    return e.code;
  } catch (const std::exception& e) {
    sod2::set_error(e.what());
    return SOD2_ERR_INVALID_ARG;
  }
  return SOD2_OK;
}

extern "C" sod2_status sod2_replay_launch(sod2_replay_t* r, int32_t first_step, int32_t n_steps, void* stream) {
  if (!r || first_step < 0 || n_steps < 0 || first_step + n_steps > r->max_steps) {
    sod2::set_error("steps outside the range the replay was created for");
    return SOD2_ERR_INVALID_ARG;
  }
  hipStream_t s = (hipStream_t)stream;
  if (launch_step_set(r->step, first_step, s) != hipSuccess) { sod2::set_error("step counter could not be set"); return SOD2_ERR_HIP; }
  for (int i = 0; i < n_steps; ++i)
    if (hipGraphLaunch(r->exec, s) != hipSuccess) { sod2::set_error("graph launch failed"); return SOD2_ERR_HIP; }
  return SOD2_OK;
}
extern "C" void sod2_replay_destroy(sod2_replay_t* r) { delete r; }

// sod2_run and sod2_run_static.  static_ws: split-K partials go to the library's static scratch buffer,
// and nothing may be allocated (no pinned read-back slot, no events).
static sod2_status run_impl(sod2_binding_t* h, void* arena, size_t arena_bytes, const void* const* weights,
                            int32_t n_weights, const void* const* inputs, int32_t n_inputs, void* const* outputs,
                            int32_t n_outputs, void* stream, bool static_ws) {
  try {
    if (!h) throw Error(SOD2_ERR_INVALID_ARG, "null binding");
    const Plan& p = *h->plan;
    const Graph& G = *p.g;
    if (static_ws) {
      if (p.n_switches > 0 || !p.exec_ops.empty())
        throw Error(SOD2_ERR_UNSUPPORTED, "sod2_run_static: a graph with Switch, NonZero or NMS operators reads values back through "
                                          "pinned host memory, which this entry point may not allocate; use sod2_run");
      if (h->profiling)
        throw Error(SOD2_ERR_UNSUPPORTED, "sod2_run_static: launch records need events, which this entry point may not create; "
                                          "switch profiling off or use sod2_run");
    }
    if (n_weights != (int)G.weight_ids.size() || n_inputs != (int)G.input_ids.size() || n_outputs != (int)G.output_ids.size())
      throw Error(SOD2_ERR_INVALID_ARG, "wrong number of weight, input or output pointers");
    for (int i = 0; i < n_weights; ++i) if (!weights[i]) throw Error(SOD2_ERR_INVALID_ARG, "null weight pointer");
    auto has_elements = [&](int t) {                   // (a tensor without elements may come with a null pointer)
      if (!p.rdp->S[t].resolved()) return true;
      for (const CompiledExpr& x : p.cshape[t]) if (x.eval(h->b.atom_vals) == 0) return false;
      return true;
    };
    for (int i = 0; i < n_inputs; ++i)
      if (!inputs[i] && has_elements(G.input_ids[i])) throw Error(SOD2_ERR_INVALID_ARG, "null input pointer");
    for (int i = 0; i < n_outputs; ++i)
      if (!outputs[i] && has_elements(G.output_ids[i])) throw Error(SOD2_ERR_INVALID_ARG, "null output pointer");
    if ((size_t)h->b.arena_bytes > arena_bytes || (h->b.arena_bytes > 0 && !arena))
      throw Error(SOD2_ERR_ARENA_TOO_SMALL, "arena of " + std::to_string(arena_bytes) + " bytes, plan needs " +
                                                std::to_string(h->b.arena_bytes));
    if (((uintptr_t)arena & 255) != 0) throw Error(SOD2_ERR_INVALID_ARG, "arena must be 256-byte aligned");
    hipStream_t s = (hipStream_t)stream;
    Pointers P(arena, arena_bytes, weights, n_weights, inputs, n_inputs, outputs, n_outputs);
    if (h->constants && h->constants_bytes < (size_t)p.const_bytes)
      throw Error(SOD2_ERR_INVALID_ARG, "constants buffer of " + std::to_string(h->constants_bytes) + " bytes, plan needs " +
                                            std::to_string(p.const_bytes));
    if (h->constants && p.const_bytes > 0) {
      P.constants = (const char*)h->constants;
      P.constants_bytes = h->constants_bytes;
    }
    // an arena longer than the plan by WS_BYTES carries the optional workspace at its end
    auto workspace_for = [&](int64_t plan_bytes) -> char* {
      size_t end = arena_bytes & ~(size_t)255;
      if (end < (size_t)WS_BYTES || end - (size_t)WS_BYTES < (size_t)((plan_bytes + 255) / 256 * 256)) return nullptr;
      return (char*)arena + end - WS_BYTES;
    };
    P.ws = static_ws ? static_scratch() : workspace_for(h->b.arena_bytes);

    // The launch table of a new binding is filled step by step as the run reaches each step, so the
    // first kernels are already executing while the later launches are still being prepared (an
    // unsupported group is therefore reported after the groups before it were launched).
    std::unique_ptr<Builder> first;
    if (!h->launches_valid) {
      h->launches.clear();
      for (size_t j = 0; j < h->b.steps.size(); ++j) {
        const Item& it = p.items[h->b.steps[j]];
        Launch L;
        L.kernel = it.is_group ? -2 : -1;
        L.group = it.ref;
        h->launches.push_back(L);
      }
      first.reset(new Builder(p, h->b, h->force_variant));
      first->force_splits = h->force_splits;
      first->folding = P.constants != nullptr;
    }
    if (static_ws) {
      // every launch is prepared before the first one is enqueued, so that a contraction whose partial
      // tiles do not fit the static buffer is refused with nothing launched
      for (size_t j = 0; j < h->b.steps.size(); ++j) {
        const Item& it = p.items[h->b.steps[j]];
        if (it.is_group && h->launches[j].kernel == -2) h->launches[j] = first->make(p.groups.at(it.ref));
        const Launch& L = h->launches[j];
        double need = 0;
        if (L.kernel == K_GEMM && L.u.gemm.splits > 1)
          need = 4.0 * L.u.gemm.splits * L.u.gemm.nb0 * L.u.gemm.nb1 * (double)L.u.gemm.M * L.u.gemm.N;
        else if (L.kernel == K_CONV && L.u.conv.splits > 1)
          need = 4.0 * L.u.conv.splits * (double)L.u.conv.NB * L.u.conv.OH * L.u.conv.OW * L.u.conv.O;
        if (need > (double)SOD2_STATIC_SCRATCH_BYTES)
          throw Error(SOD2_ERR_SCRATCH_TOO_SMALL, "sod2_run_static: group " + std::to_string(L.group) + " splits k into " +
                          std::to_string(L.kernel == K_GEMM ? L.u.gemm.splits : L.u.conv.splits) + " ranges and needs " +
                          std::to_string((long long)need) + " bytes of partial sums, the static buffer holds " +
                          std::to_string((long long)SOD2_STATIC_SCRATCH_BYTES) +
                          "; use sod2_run with a workspace behind the arena, or sod2_binding_force_splits(b, 1)");
      }
    }
    h->records.clear();
    h->trace.clear();
    h->last_decisions.clear();
    hipEvent_t* ev = nullptr;
    if (h->profiling) {
      int need = 2 * (int)h->b.steps.size() + 2 * (int)p.items.size() + 4;
      if (h->n_events < need) {
        if (h->events) destroy_events(h->events, h->n_events);
        ev = new hipEvent_t[need];
        for (int i = 0; i < need; ++i)
          if (hipEventCreate(&ev[i]) != hipSuccess) throw Error(SOD2_ERR_HIP, "hipEventCreate failed");
        h->events = ev;
        h->n_events = need;
      }
      ev = (hipEvent_t*)h->events;
    }
    int n_ev = 0;
    std::vector<std::pair<int, Launch>> timed;
    if (ev) {                  // first two records (kernel 7, groups -1 and -2): one and two empty launches
      Launch L;
      L.kernel = K_OTHER;
      for (int n = 1; n <= 2; ++n) {
        (void)hipEventRecord(ev[n_ev], s);
        for (int i = 0; i < n; ++i) (void)launch_null(s);
        (void)hipEventRecord(ev[n_ev + 1], s);
        L.group = -n;
        timed.push_back({n_ev, L});
        n_ev += 2;
      }
    }

    const BindResult* cur = &h->b;
    const std::vector<Launch>* launches = &h->launches;
    BindResult replanned;
    std::vector<Launch> relaunch;
    std::vector<int> decisions = h->planned_decisions;
    std::vector<int64_t> exec_values = h->planned_exec;
    h->last_exec.clear();
    FlatMap<int64_t> used_offset;                   // arena tensor -> offset used by an executed kernel
    used_offset.reserve(h->b.steps.size() + 8);
    std::unique_ptr<Builder> lazy;                  // builds the launches of `replanned` on demand
    // an execution-determined fact (a Switch decision, a NonZero count) has just become known at
    // step k: plan what follows with it (Section 4.3) and build the launches of the remaining steps
    auto replan = [&](size_t k, const char* what, BindResult* ready = nullptr) {
      if (ready) replanned = std::move(*ready);
      else replanned = bind_plan(p, h->symbols, decisions, true, exec_values);
      if ((size_t)replanned.arena_bytes > arena_bytes) {
        h->executed = replanned;               // sod2_run_arena_bytes now reports what this path needs
        h->has_executed = true;
        throw Error(SOD2_ERR_ARENA_TOO_SMALL, "arena of " + std::to_string(arena_bytes) + " bytes, the path taken needs " +
                                                  std::to_string(replanned.arena_bytes) + "; nothing after the " + what + " was launched");
      }
      // launches of the new plan are built one by one as the run reaches them (another fact may
      // arrive before most of them are needed)
      relaunch.clear();
      for (size_t j = 0; j < replanned.steps.size(); ++j) {
        const Item& it = p.items[replanned.steps[j]];
        Launch L;
        L.kernel = it.is_group ? -2 : -1;
        L.group = it.ref;
        relaunch.push_back(L);
      }
      lazy.reset(new Builder(p, replanned, h->force_variant));
      lazy->force_splits = h->force_splits;
      lazy->folding = P.constants != nullptr;
      P.ws = static_ws ? static_scratch() : workspace_for(replanned.arena_bytes);
      cur = &replanned;
      launches = &relaunch;
    };
    size_t k = 0, n_nz = 0;
    int queued = 0;                                 // kernels enqueued since the stream was last synchronised
    bool assumed = false;                           // a fact confirmed what the plan in use had assumed
    while (k < cur->steps.size()) {
      const Item& it = p.items[cur->steps[k]];
      if (it.is_group && (*launches)[k].kernel == -2) {
        if (launches == &relaunch) relaunch[k] = lazy->make(p.groups.at(it.ref));
        else h->launches[k] = first->make(p.groups.at(it.ref));
      }
      const Launch L = (*launches)[k];                // a copy: a re-plan below rebuilds the table
      if (it.is_group) {
        auto at = cur->tensors.find(p.groups.at(it.ref).out);
        if (at != cur->tensors.end()) used_offset[at->first] = at->second.offset;
        if (ev) (void)hipEventRecord(ev[n_ev], s);
        hipError_t e = dispatch(L, P, s);
        if (e != hipSuccess) throw Error(SOD2_ERR_HIP, std::string("kernel launch failed: ") + hipGetErrorString(e));
        if (ev) { (void)hipEventRecord(ev[n_ev + 1], s); timed.push_back({n_ev, L}); n_ev += 2; }
        if (!L.empty) ++queued;
        {
          int splits = 1;
          if (L.kernel == K_GEMM && P.ws) splits = std::max(L.u.gemm.splits, 1);
          else if (L.kernel == K_CONV && P.ws) splits = std::max(L.u.conv.splits, 1);
          int fold = 0;
          if (L.kernel == K_GEMM && !L.empty) {
            if (L.post_ln) fold = (L.fold_pair && P.constants) ? 1 : 3;
            if (L.fold_read && P.constants) fold = 2;
          }
          h->trace.push_back(sod2_trace_entry{1, it.ref, L.empty ? -1 : L.kernel, L.variant, splits, -1, fold});
        }
        if (L.kernel == K_NONZERO || L.kernel == K_NMS) {
          // the extent is execution determined: read the count back, then size and plan what follows
          const bool is_nms = L.kernel == K_NMS;
          begin_read_back(P.at(L.r[is_nms ? 3 : 2]), 8, s);
          const long long count = (long long)finish_read_back(s);
          queued = 0;
          if (count < 0 || count > (is_nms ? (long long)L.u.nms.n : L.u.nz.n))
            throw Error(SOD2_ERR_HIP, "a NonZero or NMS kernel reported an impossible count");
          h->last_exec.push_back(count);
          if (n_nz >= exec_values.size()) {
            exec_values.push_back(count);
            // (also when the count equals the assumed upper bound: with the count known the sub-graphs
            //  that follow are planned together instead of one by one)
            replan(k, is_nms ? "NMS" : "NonZero");
          } else if (exec_values[n_nz] != count) {
            throw Error(SOD2_ERR_INVALID_ARG, "the binding was planned for a NonZero / NMS count of " + std::to_string(exec_values[n_nz]) +
                                                  ", the run found " + std::to_string(count));
          }
          ++n_nz;
        }
      } else if (G.ops[it.ref].kind == SOD2_OP_SWITCH) {
        // position of this Switch among the executed ones
        size_t which = std::find(cur->switch_order.begin(), cur->switch_order.end(), it.ref) - cur->switch_order.begin();
        if (which >= decisions.size()) {
          // the predicate is execution determined: read it back, decide, plan what follows (Section 4.3)
          int dec;
          BindResult other;                        // the plan for the outcome the plan in use does not assume
          bool have_other = false;
          if (h->has_forced && which < h->forced.size()) {
            dec = h->forced[which] ? 1 : 0;
          } else {
            const Op& op = G.ops[it.ref];
            Builder B(p, *cur, h->force_variant);
            Ref r = B.ref_t(op.in[1]);
            float hv = 0.f;
            int dt = G.tensors[op.in[1]].dtype;
            begin_read_back(P.at(r), dt == SOD2_BF16 ? 2 : 4, s);
            // While the GPU still works through the kernels enqueued since the last synchronise (a layer that
            // ran: ~100 us), this thread would only wait: it plans the other outcome meanwhile, so that a
            // decision against the assumed one finds its plan ready.  With little work queued (the previous
            // layer was skipped too) the plan is computed after the decision, as before.
            if (queued >= SPECULATE_MIN_QUEUED) {
              std::vector<int> d2 = decisions;
              d2.push_back(1);
              other = bind_plan(p, h->symbols, d2, true, exec_values);
              have_other = true;
            }
            const uint32_t bits = (uint32_t)finish_read_back(s);
            queued = 0;
            const uint32_t u = dt == SOD2_BF16 ? bits << 16 : bits;
            std::memcpy(&hv, &u, 4);
            dec = hv > (float)op.fa ? 1 : 0;
          }
          decisions.push_back(dec);
          // the current plan assumed that the layer runs: only the other outcome changes it
          if (dec != 0) replan(k, "Switch", have_other ? &other : nullptr);
          else assumed = true;
        }
        h->trace.push_back(sod2_trace_entry{0, it.ref, -1, 0, 1, decisions[which], 0});
      } else {
        h->trace.push_back(sod2_trace_entry{0, it.ref, -1, 0, 1, -1, 0});      // Combine: forwards the taken path's tensor
      }
      ++k;
    }
    if (launches == &h->launches) h->launches_valid = true;      // complete: a second run of this binding reuses it
    if (assumed) {
      // same steps and offsets as the plan in use; computed again only so that the executed plan
      // reports every fact as known (the kernels are already enqueued: this overlaps their execution)
      replanned = bind_plan(p, h->symbols, decisions, true, exec_values);
      cur = &replanned;
    }
    for (int sw : cur->switch_order) h->last_decisions.push_back(cur->decisions.at(sw));
    for (const auto& kv : used_offset) {
      auto at = cur->tensors.find(kv.first);
      if (at == cur->tensors.end() || at->second.offset != kv.second)
        throw Error(SOD2_ERR_NONCAUSAL_PLAN, "an offset used before a Switch differs from the final plan");
    }
    if (ev) {
      if (hipStreamSynchronize(s) != hipSuccess) throw Error(SOD2_ERR_HIP, "stream synchronise failed");
      for (const auto& t : timed) {
        sod2_launch_record r{};
        r.group = t.second.group; r.kernel = t.second.kernel; r.variant = t.second.variant;
        (void)hipEventElapsedTime(&r.ms, ev[t.first], ev[t.first + 1]);
        r.flops = t.second.flops; r.bytes = t.second.bytes;
        h->records.push_back(r);
      }
    }
    if (cur == &replanned) {          // keep the executed plan for queries
      h->executed = replanned;
      h->has_executed = true;
    }
  } catch (const sod2::Error& e) {
    sod2::set_error(e.what());
    return e.code;
  } catch (const std::exception& e) {
    sod2::set_error(e.what());
    return SOD2_ERR_INVALID_ARG;
  }
  return SOD2_OK;
}

extern "C" sod2_status sod2_run(sod2_binding_t* h, void* arena, size_t arena_bytes, const void* const* weights,
                                int32_t n_weights, const void* const* inputs, int32_t n_inputs, void* const* outputs,
                                int32_t n_outputs, void* stream) {
  return run_impl(h, arena, arena_bytes, weights, n_weights, inputs, n_inputs, outputs, n_outputs, stream, false);
}

extern "C" sod2_status sod2_plan_constants_bytes(const sod2_plan_t* h, size_t* bytes) {
  if (!h || !bytes) { set_error("null argument"); return SOD2_ERR_INVALID_ARG; }
  *bytes = (size_t)h->p.const_bytes;
  return SOD2_OK;
}

extern "C" sod2_status sod2_plan_prepare_constants(const sod2_plan_t* h, const void* const* weights, int32_t n_weights,
                                                   void* constants, size_t bytes, void* stream) {
  try {
    if (!h || !weights) throw Error(SOD2_ERR_INVALID_ARG, "null argument");
    const Plan& p = h->p;
    const Graph& G = *p.g;
    if (n_weights != (int)G.weight_ids.size()) throw Error(SOD2_ERR_INVALID_ARG, "wrong number of weight pointers");
    if (p.const_bytes == 0) return SOD2_OK;
    if (!constants || bytes < (size_t)p.const_bytes || ((uintptr_t)constants & 255))
      throw Error(SOD2_ERR_INVALID_ARG, "constants buffer must be 256-byte aligned and hold " + std::to_string(p.const_bytes) + " bytes");
    for (const auto& kv : p.const_off) {
      const Group& gr = p.groups.at(kv.first);
      const Op& mm = G.ops[gr.chain[0]];
      const Op& ln = G.ops[gr.lnfold];
      // scale and bias of the contraction's epilogue, as the run reads them
      float scale = 1.f;
      int bias = -1, cur = mm.out[0];
      bool seen_other = false;
      for (size_t k = 1; k < gr.chain.size(); ++k) {
        const Op& op = G.ops[gr.chain[k]];
        const int o = op.in.size() > 1 ? (op.in[0] == cur ? op.in[1] : op.in[0]) : -1;
        if (op.kind == SOD2_OP_MUL) scale *= (float)G.tensors[o].fdata.at(0);
        else if (op.kind == SOD2_OP_ADD && G.tensors[o].role == SOD2_WEIGHT && bias < 0 && !seen_other) bias = o;
        else if (op.kind != SOD2_OP_TRANSPOSE) seen_other = true;
        cur = op.out[0];
      }
      auto wptr = [&](int t) -> const void* {
        if (t < 0) return nullptr;
        if (G.weight_pos[t] < 0) throw Error(SOD2_ERR_UNSUPPORTED, "folded LayerNorm parameter is not a weight: " + G.tensors[t].name);
        const void* q = weights[G.weight_pos[t]];
        if (!q) throw Error(SOD2_ERR_INVALID_ARG, "null weight pointer");
        return q;
      };
      if (G.weight_pos[ln.in[1]] < 0 || G.weight_pos[ln.in[2]] < 0) continue;   // such a pair never folds at run time
      if (bias >= 0 && G.weight_pos[bias] < 0) continue;
      const LS& sw = p.rdp->S[mm.in[1]];
      const int N = (int)sw.d[0].e.const_value(), K = (int)sw.d[1].e.const_value();
      char* base = (char*)constants + kv.second;
      hipError_t e = launch_fold_constants(wptr(mm.in[1]), wptr(ln.in[1]), wptr(ln.in[2]), wptr(bias), scale, N, K, base,
                                           base + 4ll * N, (hipStream_t)stream);
      if (e != hipSuccess) throw Error(SOD2_ERR_HIP, std::string("constants kernel: ") + hipGetErrorString(e));
    }
    return SOD2_OK;
  } catch (const Error& e) {
    set_error(e.what());
    return e.code;
  } catch (const std::exception& e) {
    set_error(e.what());
    return SOD2_ERR_INVALID_ARG;
  }
}

extern "C" sod2_status sod2_binding_set_constants(sod2_binding_t* h, const void* constants, size_t bytes) {
  if (!h) { set_error("null argument"); return SOD2_ERR_INVALID_ARG; }
  if (constants && ((uintptr_t)constants & 255)) { set_error("constants buffer must be 256-byte aligned"); return SOD2_ERR_INVALID_ARG; }
  h->constants = constants;
  h->constants_bytes = constants ? bytes : 0;
  h->launches_valid = false;
  return SOD2_OK;
}

extern "C" sod2_status sod2_run_static(sod2_binding_t* h, void* arena, size_t arena_bytes, const void* const* weights,
                                       int32_t n_weights, const void* const* inputs, int32_t n_inputs, void* const* outputs,
                                       int32_t n_outputs, void* stream) {
  return run_impl(h, arena, arena_bytes, weights, n_weights, inputs, n_inputs, outputs, n_outputs, stream, true);
}
