// Symbolic integer expressions (see internal.hpp).  Canonical text: terms ordered by
// (degree, atom names); "coeff", "a*b" or "coeff*a*b"; joined by " + "; zero prints "0".
#include <algorithm>
#include <mutex>
#include <sstream>

#include "internal.hpp"

namespace sod2 {
namespace {
// kind: 0 symbol, 1 floordiv(inner, c), 2 mod(inner, c), 3 bcast(inner, inner2): the extent two aligned dims broadcast to
struct AtomDef { int kind; std::string sym; std::shared_ptr<Expr> inner; int64_t c; std::shared_ptr<Expr> inner2; };
int64_t bcast_value(int64_t a, int64_t b, const std::string& what) {
  if (a == b || b == 1) return a;
  if (a == 1) return b;
  throw Error(SOD2_ERR_SHAPE_MISMATCH, "extents " + std::to_string(a) + " and " + std::to_string(b) + " do not broadcast (" + what + ")");
}
std::map<std::string, AtomDef>& atoms() { static std::map<std::string, AtomDef> a; return a; }
std::mutex& atoms_mu() { static std::mutex m; return m; }

// (entries are never erased and std::map nodes do not move: the reference stays valid)
const AtomDef& atom_of(const std::string& name) {
  std::lock_guard<std::mutex> lk(atoms_mu());
  auto it = atoms().find(name);
  if (it == atoms().end()) throw Error(SOD2_ERR_INVALID_ARG, "unknown atom " + name);
  return it->second;
}
void put_atom(const std::string& name, const AtomDef& d) {
  std::lock_guard<std::mutex> lk(atoms_mu());
  atoms().emplace(name, d);
}
int64_t floor_div(int64_t a, int64_t b) { int64_t q = a / b; return (a % b != 0 && ((a < 0) != (b < 0))) ? q - 1 : q; }
int64_t floor_mod(int64_t a, int64_t b) { return a - floor_div(a, b) * b; }
void prune(std::map<Expr::Mono, int64_t>& t) {
  for (auto it = t.begin(); it != t.end();) it = (it->second == 0) ? t.erase(it) : std::next(it);
}
}  // namespace

Expr Expr::constant(int64_t c) { Expr e; if (c) e.terms[Mono()] = c; return e; }
Expr Expr::symbol(const std::string& name) {
  put_atom(name, AtomDef{0, name, nullptr, 0, nullptr});
  Expr e; e.terms[Mono{name}] = 1; return e;
}
Expr Expr::parse(const std::string& text) {
  Expr e;
  std::stringstream ss(text);
  std::string part;
  while (std::getline(ss, part, '+')) {
    size_t a = part.find_first_not_of(" \t"), b = part.find_last_not_of(" \t");
    if (a == std::string::npos) throw Error(SOD2_ERR_INVALID_ARG, "empty dim term in '" + text + "'");
    part = part.substr(a, b - a + 1);
    bool num = true;
    for (size_t i = 0; i < part.size(); ++i)
      if (!(isdigit((unsigned char)part[i]) || (i == 0 && part[i] == '-' && part.size() > 1))) num = false;
    e = e + (num ? Expr::constant(std::stoll(part)) : Expr::symbol(part));
  }
  return e;
}
bool Expr::is_const() const { return terms.empty() || (terms.size() == 1 && terms.begin()->first.empty()); }
int64_t Expr::const_value() const { return terms.empty() ? 0 : terms.begin()->second; }
bool Expr::is_symbol() const {
  if (terms.size() != 1) return false;
  const auto& t = *terms.begin();
  return t.second == 1 && t.first.size() == 1 && atom_of(t.first[0]).kind == 0;
}
int Expr::cls() const { return is_const() ? 0 : (is_symbol() ? 1 : 2); }

std::string Expr::str() const {
  if (terms.empty()) return "0";
  std::vector<std::pair<Mono, int64_t>> v(terms.begin(), terms.end());
  std::stable_sort(v.begin(), v.end(), [](const std::pair<Mono, int64_t>& a, const std::pair<Mono, int64_t>& b) {
    if (a.first.size() != b.first.size()) return a.first.size() < b.first.size();
    return a.first < b.first;
  });
  std::string out;
  for (size_t i = 0; i < v.size(); ++i) {
    if (i) out += " + ";
    const Mono& m = v[i].first;
    if (m.empty()) { out += std::to_string(v[i].second); continue; }
    if (v[i].second != 1) out += std::to_string(v[i].second) + "*";
    for (size_t j = 0; j < m.size(); ++j) { if (j) out += "*"; out += m[j]; }
  }
  return out;
}

Expr Expr::operator+(const Expr& o) const {
  Expr r = *this;
  for (const auto& t : o.terms) r.terms[t.first] += t.second;
  prune(r.terms);
  return r;
}
Expr Expr::operator-(const Expr& o) const {
  Expr r = *this;
  for (const auto& t : o.terms) r.terms[t.first] -= t.second;
  prune(r.terms);
  return r;
}
Expr Expr::operator*(const Expr& o) const {
  Expr r;
  for (const auto& a : terms)
    for (const auto& b : o.terms) {
      Mono m = a.first;
      m.insert(m.end(), b.first.begin(), b.first.end());
      std::sort(m.begin(), m.end());
      r.terms[m] += a.second * b.second;
    }
  prune(r.terms);
  return r;
}
Expr Expr::floordiv(int64_t c) const {
  if (c <= 0) throw Error(SOD2_ERR_INVALID_ARG, "floordiv by a non-positive constant");
  if (c == 1) return *this;
  bool all = true;
  for (const auto& t : terms) if (floor_mod(t.second, c) != 0) all = false;
  if (all) { Expr r; for (const auto& t : terms) r.terms[t.first] = t.second / c; return r; }
  if (is_const()) return Expr::constant(floor_div(const_value(), c));
  if (terms.size() == 1 && terms.begin()->second == 1 && terms.begin()->first.size() == 1) {
    AtomDef d = atom_of(terms.begin()->first[0]);
    if (d.kind == 1) return d.inner->floordiv(d.c * c);        // floor(floor(e/a)/b) = floor(e/(a*b))
  }
  std::string name = "floordiv(" + str() + ", " + std::to_string(c) + ")";
  put_atom(name, AtomDef{1, "", std::make_shared<Expr>(*this), c, nullptr});
  Expr r; r.terms[Mono{name}] = 1; return r;
}
Expr Expr::bcast(const Expr& o) const {
  if (*this == o) return *this;
  if (is_const() && const_value() == 1) return o;
  if (o.is_const() && o.const_value() == 1) return *this;
  if (is_const() && o.is_const()) throw Error(SOD2_ERR_SHAPE_MISMATCH, "cannot broadcast " + str() + " with " + o.str());
  const bool first = str() <= o.str();
  const Expr &a = first ? *this : o, &b = first ? o : *this;
  std::string name = "bcast(" + a.str() + ", " + b.str() + ")";
  put_atom(name, AtomDef{3, "", std::make_shared<Expr>(a), 0, std::make_shared<Expr>(b)});
  Expr r; r.terms[Mono{name}] = 1; return r;
}
Expr Expr::mod(int64_t c) const {
  if (c <= 0) throw Error(SOD2_ERR_INVALID_ARG, "mod by a non-positive constant");
  bool all = true;
  for (const auto& t : terms) if (floor_mod(t.second, c) != 0) all = false;
  if (all) return Expr();
  if (is_const()) return Expr::constant(floor_mod(const_value(), c));
  std::string name = "mod(" + str() + ", " + std::to_string(c) + ")";
  put_atom(name, AtomDef{2, "", std::make_shared<Expr>(*this), c, nullptr});
  Expr r; r.terms[Mono{name}] = 1; return r;
}
bool Expr::exact_div(const Expr& o, Expr* q) const {
  if (o.terms.size() != 1) return false;
  const Mono& dm = o.terms.begin()->first;
  int64_t dc = o.terms.begin()->second;
  Expr r;
  for (const auto& t : terms) {
    if (t.second % dc != 0) return false;
    Mono rest = t.first;
    for (const auto& a : dm) {
      auto it = std::find(rest.begin(), rest.end(), a);
      if (it == rest.end()) return false;
      rest.erase(it);
    }
    r.terms[rest] += t.second / dc;
  }
  prune(r.terms);
  *q = r;
  return true;
}
int64_t Expr::eval(const std::map<std::string, int64_t>& env) const {
  int64_t total = 0;
  for (const auto& t : terms) {
    int64_t v = t.second;
    for (const auto& a : t.first) {
      const AtomDef& d = atom_of(a);
      if (d.kind == 0) {
        auto it = env.find(d.sym);
        if (it == env.end()) throw Error(SOD2_ERR_INVALID_ARG, "symbol without a value: " + d.sym);
        v *= it->second;
      } else {
        int64_t inner = d.inner->eval(env);
        v *= d.kind == 3 ? bcast_value(inner, d.inner2->eval(env), a) : ((d.kind == 1) ? floor_div(inner, d.c) : floor_mod(inner, d.c));
      }
    }
    total += v;
  }
  return total;
}

bool mentions_exec(const Expr& e) {
  for (const auto& t : e.terms)
    for (const auto& a : t.first) if (a.find("@nz") != std::string::npos) return true;
  return false;
}

// ---- flattened form ----------------------------------------------------------------------------
int ExprCompiler::intern(const std::string& name) {
  auto it = index.find(name);
  if (it != index.end()) return it->second;
  const AtomDef& d = atom_of(name);
  Atom a{d.kind, -1, d.c, CompiledExpr(), CompiledExpr(), name};
  if (d.kind == 0) {
    for (size_t i = 0; i < symbols.size(); ++i) if (symbols[i] == d.sym) a.sym = (int)i;
    if (a.sym < 0) throw Error(SOD2_ERR_INVALID_ARG, "symbol without a declaration: " + d.sym);
  } else {
    a.inner = compile(*d.inner);                   // its atoms get smaller indices than this one
    if (d.kind == 3) a.inner2 = compile(*d.inner2);
  }
  atoms.push_back(a);
  index[name] = (int)atoms.size() - 1;
  return (int)atoms.size() - 1;
}
CompiledExpr ExprCompiler::compile(const Expr& e) {
  CompiledExpr c;
  for (const auto& t : e.terms) {
    CompiledExpr::Term ct{t.second, {}};
    for (const auto& a : t.first) ct.atoms.push_back(intern(a));
    c.terms.push_back(ct);
  }
  return c;
}
void ExprCompiler::atom_values(const std::vector<int64_t>& sv, std::vector<int64_t>* out) const {
  out->assign(atoms.size(), 0);
  for (size_t i = 0; i < atoms.size(); ++i) {
    const Atom& a = atoms[i];
    if (a.kind == 0) { (*out)[i] = sv[a.sym]; continue; }
    int64_t inner = a.inner.eval(*out);
    (*out)[i] = a.kind == 3 ? bcast_value(inner, a.inner2.eval(*out), a.name) : (a.kind == 1 ? floor_div(inner, a.c) : floor_mod(inner, a.c));
  }
}

// ---- lattice ----------------------------------------------------------------------------------
LV meet(const LV& a, const LV& b) {
  if (a.k == LV::UNDEF) return b;
  if (b.k == LV::UNDEF) return a;
  if (a.k == LV::NAC || b.k == LV::NAC) return LV::nac();
  if (a.e == b.e) return a;
  if (a.e.is_const() && b.e.is_const())
    throw Error(SOD2_ERR_SHAPE_MISMATCH, "known constants disagree: " + a.e.str() + " vs " + b.e.str());
  return LV::nac();
}
LS meet(const LS& a, const LS& b) {
  if (a.k == LS::UNDEF) return b;
  if (b.k == LS::UNDEF) return a;
  if (a.k == LS::NAC || b.k == LS::NAC) return LS::nac();
  if (a.d.size() != b.d.size())
    throw Error(SOD2_ERR_SHAPE_MISMATCH, "ranks disagree: " + std::to_string(a.d.size()) + " vs " + std::to_string(b.d.size()));
  LS r = LS::list({});
  for (size_t i = 0; i < a.d.size(); ++i) r.d.push_back(meet(a.d[i], b.d[i]));
  return r;
}
bool LS::resolved() const {
  if (k != LIST) return false;
  for (const auto& x : d) if (!x.val()) return false;
  return true;
}
bool LS::same(const LS& o) const {
  if (k != o.k) return false;
  if (k != LIST) return true;
  if (d.size() != o.d.size()) return false;
  for (size_t i = 0; i < d.size(); ++i) if (!d[i].same(o.d[i])) return false;
  return true;
}
bool LS::has_undef() const {
  if (k == UNDEF) return true;
  if (k == LIST) for (const auto& x : d) if (x.k == LV::UNDEF) return true;
  return false;
}
static std::string lv_str(const LV& v) {
  if (v.k == LV::UNDEF) return "undef";
  if (v.k == LV::NAC) return "nac";
  static const char* tag[] = {"k", "s", "e"};
  return std::string(tag[v.e.cls()]) + ":" + v.e.str();
}
std::string LS::str() const {
  if (k == UNDEF) return "undef";
  if (k == NAC) return "nac";
  std::string s = "[";
  for (size_t i = 0; i < d.size(); ++i) { if (i) s += ", "; s += lv_str(d[i]); }
  return s + "]";
}
}  // namespace sod2
