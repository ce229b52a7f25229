// Access-pattern programs as text: reader, shape rules, evaluation on the GPU, rewrites.
//
// The paper writes tensor kernels as s-expressions over the transformers of Table 1 and the
// operators of Table 2 (Figs. 2a-2c, 5, 7) and transforms them with rewrite rules (Figs. 3, 4, 6).
// This file is the host side of that: it reads such text, infers every node's access-pattern
// shape with the rules of Table 1, and
//   * evaluates a program by dispatching its nodes to the library's kernels: the pattern the
//     paper maps to hardware, (compute dotProd (cartProd ?a0 ?a1)) (Fig. 3, Sec. 5.2), becomes one
//     MFMA contraction without the Cartesian product ever existing in memory; the whole listing
//     of Fig. 2a becomes the direct convolution; (compute reduceX (windows ...)) becomes the fused
//     pooling kernel; (compute reduceX (pair a b)) the element-wise kernel; every other
//     transformer is a descriptor change (access, squeeze, flatten, reshape, outermost slice) or
//     one of the data-moving kernels (transpose, slice, concat, pair, pad, windows).  Identical
//     sub-programs are evaluated once.
//   * applies the rewrites: the three rules of Fig. 4 that turn the convolution of Fig. 2a into
//     its im2col form (Fig. 5), the systolic-array rule of Fig. 3, and the blocking rules of
//     Fig. 6 that turn a matMul into a program of block products (Fig. 7).  The rules are applied
//     by a small directed strategy (no equality saturation, no e-graph): each strategy names the
//     rule sequence that derives one figure from another.
// Nothing here runs on the device; the kernels are reached through the C entry points.
#include "common.h"

#include <string.h>

#include <map>
#include <memory>
#include <string>
#include <vector>

extern "C" size_t glenside_conv2d_direct_workspace(const gs_ap*, const gs_ap*, const int64_t*, const int64_t*);

namespace {

using gs::round_up;

// ---------------------------------------------------------------------------------------------
// Text <-> tree
// ---------------------------------------------------------------------------------------------
struct Tree;
using TreeP = std::shared_ptr<const Tree>;
struct Tree {
  enum Kind { kList, kSymbol, kInt } kind;
  std::string sym;
  int64_t value = 0;
  std::vector<TreeP> items;
};

TreeP mk_int(int64_t v) {
  auto t = std::make_shared<Tree>();
  t->kind = Tree::kInt;
  t->value = v;
  return t;
}
TreeP mk_sym(const std::string& s) {
  auto t = std::make_shared<Tree>();
  t->kind = Tree::kSymbol;
  t->sym = s;
  return t;
}
TreeP mk_list(std::vector<TreeP> items) {
  auto t = std::make_shared<Tree>();
  t->kind = Tree::kList;
  t->items = std::move(items);
  return t;
}
TreeP call(const std::string& head, std::vector<TreeP> args) {
  std::vector<TreeP> items;
  items.push_back(mk_sym(head));
  for (auto& a : args) items.push_back(a);
  return mk_list(std::move(items));
}
TreeP int_tuple(const std::string& head, const std::vector<int64_t>& v) {
  std::vector<TreeP> items;
  for (int64_t x : v) items.push_back(mk_int(x));
  return call(head, items);
}

std::string to_text(const TreeP& t) {
  if (t->kind == Tree::kInt) return std::to_string(t->value);
  if (t->kind == Tree::kSymbol) return t->sym;
  std::string s = "(";
  for (size_t i = 0; i < t->items.size(); ++i) {
    if (i) s += " ";
    s += to_text(t->items[i]);
  }
  return s + ")";
}

struct Parser {
  const char* p;
  bool ok = true;
  void skip() {
    while (*p == ' ' || *p == '\n' || *p == '\t' || *p == '\r') ++p;
  }
  TreeP read(int depth) {
    skip();
    if (!*p || depth > 256) {
      ok = false;
      return nullptr;
    }
    if (*p == '(') {
      ++p;
      std::vector<TreeP> items;
      for (;;) {
        skip();
        if (!*p) {
          ok = false;
          return nullptr;
        }
        if (*p == ')') {
          ++p;
          break;
        }
        TreeP c = read(depth + 1);
        if (!ok) return nullptr;
        items.push_back(c);
      }
      return mk_list(std::move(items));
    }
    if (*p == ')') {
      ok = false;
      return nullptr;
    }
    const char* b = p;
    while (*p && *p != ' ' && *p != '\n' && *p != '\t' && *p != '\r' && *p != '(' && *p != ')') ++p;
    std::string tok(b, p);
    bool is_int = !tok.empty();
    for (size_t i = 0; i < tok.size(); ++i)
      if (!(tok[i] >= '0' && tok[i] <= '9') && !(i == 0 && tok[i] == '-' && tok.size() > 1)) is_int = false;
    if (is_int && tok.size() < 18) return mk_int(strtoll(tok.c_str(), nullptr, 10));
    return mk_sym(tok);
  }
};

TreeP parse(const char* text) {
  if (!text) return nullptr;
  Parser ps{text};
  TreeP t = ps.read(0);
  if (!ps.ok) return nullptr;
  ps.skip();
  return *ps.p ? nullptr : t;
}

bool is_call(const TreeP& t, const char* head, size_t nargs) {
  return t && t->kind == Tree::kList && t->items.size() == nargs + 1 && t->items[0]->kind == Tree::kSymbol &&
         t->items[0]->sym == head;
}
const TreeP& arg(const TreeP& t, size_t i) { return t->items[i + 1]; }

// ---------------------------------------------------------------------------------------------
// Environment, shapes (Table 1, Table 2)
// ---------------------------------------------------------------------------------------------
struct Env {
  const gs_named_ap* tensors;
  int n_tensors;
  const gs_named_int* ints;
  int n_ints;
  const gs_ap* tensor(const std::string& name) const {
    for (int i = 0; i < n_tensors; ++i)
      if (tensors[i].name && name == tensors[i].name) return &tensors[i].tensor;
    return nullptr;
  }
  bool integer(const TreeP& t, int64_t* v) const {
    if (!t) return false;
    if (t->kind == Tree::kInt) {
      *v = t->value;
      return true;
    }
    if (t->kind != Tree::kSymbol) return false;
    for (int i = 0; i < n_ints; ++i)
      if (ints[i].name && t->sym == ints[i].name) {
        *v = ints[i].value;
        return true;
      }
    return false;
  }
  bool tuple(const TreeP& t, const char* head, std::vector<int64_t>* v) const {
    if (!t || t->kind != Tree::kList || t->items.empty() || t->items[0]->kind != Tree::kSymbol ||
        t->items[0]->sym != head)
      return false;
    v->clear();
    for (size_t i = 1; i < t->items.size(); ++i) {
      int64_t x;
      if (!integer(t->items[i], &x)) return false;
      v->push_back(x);
    }
    return true;
  }
};

struct Shape {           // an access pattern's shape and element type
  std::vector<int64_t> d;
  int na = 0;
  int dtype = GS_F32;
  int nc() const { return int(d.size()) - na; }
  int64_t numel() const {
    int64_t n = 1;
    for (int64_t x : d) n *= x;
    return n;
  }
  int64_t access_numel() const {
    int64_t n = 1;
    for (int i = 0; i < na; ++i) n *= d[i];
    return n;
  }
  int64_t compute_numel() const { return numel() / (access_numel() ? access_numel() : 1); }
};

int dot_out_dtype(int in) { return in == GS_I8 ? GS_I32 : (in == GS_BF16 || in == GS_F8) ? GS_F32 : -1; }

// Shape of a node; GS_OK or the status that evaluation would return.
int infer(const TreeP& t, const Env& env, Shape* out);

int infer_compute(const TreeP& t, const Env& env, Shape* out) {
  const TreeP& op = arg(t, 0);
  if (op->kind != Tree::kSymbol) return GS_ERR_UNSUPPORTED;
  Shape in;
  if (op->sym == "dotProd") {
    int st = infer(arg(t, 1), env, &in);
    if (st) return st;
    if (in.nc() < 1 || in.d[in.na] != 2) return GS_ERR_SHAPE;     // (t, s_0 .. s_n) with t = 2 (Table 2)
    out->d.assign(in.d.begin(), in.d.begin() + in.na);
    out->na = in.na;
    out->dtype = dot_out_dtype(in.dtype);
    return out->dtype < 0 ? GS_ERR_DTYPE : GS_OK;
  }
  int st = infer(arg(t, 1), env, &in);
  if (st) return st;
  out->d.assign(in.d.begin(), in.d.begin() + in.na);
  out->na = in.na;
  if (op->sym == "reduceSum") {
    out->dtype = in.dtype == GS_I8 ? GS_I32 : in.dtype;
    return GS_OK;
  }
  if (op->sym == "reduceMax") {
    if (in.compute_numel() == 0 && in.access_numel() > 0) return GS_ERR_SHAPE;
    out->dtype = in.dtype;
    return GS_OK;
  }
  if (op->sym == "relu") {           // EXT
    if (in.nc() != 0) return GS_ERR_SHAPE;
    if (in.dtype == GS_I8) return GS_ERR_DTYPE;
    out->dtype = in.dtype;
    return GS_OK;
  }
  return GS_ERR_UNSUPPORTED;
}

int infer(const TreeP& t, const Env& env, Shape* out) {
  if (!t) return GS_ERR_NULL;
  if (t->kind == Tree::kSymbol) {
    const gs_ap* a = env.tensor(t->sym);
    if (!a) return GS_ERR_NULL;
    if (a->rank < 0 || a->rank > GS_MAX_RANK || a->dtype < GS_I8 || a->dtype > GS_F8) return GS_ERR_RANK;
    out->d.assign(a->shape, a->shape + a->rank);
    for (int64_t x : out->d)
      if (x < 0) return GS_ERR_SHAPE;
    out->na = 0;                      // a tensor is all compute dimensions until accessed
    out->dtype = a->dtype;
    return GS_OK;
  }
  if (t->kind != Tree::kList || t->items.empty() || t->items[0]->kind != Tree::kSymbol) return GS_ERR_UNSUPPORTED;
  const std::string& h = t->items[0]->sym;
  const size_t n = t->items.size() - 1;
  Shape a, b;
  int st;
  if (h == "access" && n == 2) {
    int64_t i;
    if ((st = infer(arg(t, 0), env, &a))) return st;
    if (!env.integer(arg(t, 1), &i)) return GS_ERR_UNSUPPORTED;
    if (i < 0 || i > int64_t(a.d.size())) return GS_ERR_RANK;
    *out = a;
    out->na = int(i);
    return GS_OK;
  }
  if (h == "transpose" && n == 2) {
    std::vector<int64_t> perm;
    if ((st = infer(arg(t, 0), env, &a))) return st;
    if (!env.tuple(arg(t, 1), "list", &perm)) return GS_ERR_UNSUPPORTED;
    if (perm.size() != a.d.size()) return GS_ERR_SHAPE;
    std::vector<bool> seen(perm.size(), false);
    *out = a;
    for (size_t k = 0; k < perm.size(); ++k) {
      if (perm[k] < 0 || perm[k] >= int64_t(perm.size()) || seen[perm[k]]) return GS_ERR_SHAPE;
      seen[perm[k]] = true;
      out->d[k] = a.d[perm[k]];
    }
    return GS_OK;
  }
  if (h == "cartProd" && n == 2) {
    if ((st = infer(arg(t, 0), env, &a))) return st;
    if ((st = infer(arg(t, 1), env, &b))) return st;
    if (a.nc() != b.nc() || a.dtype != b.dtype) return a.dtype != b.dtype ? GS_ERR_DTYPE : GS_ERR_SHAPE;
    for (int k = 0; k < a.nc(); ++k)
      if (a.d[a.na + k] != b.d[b.na + k]) return GS_ERR_SHAPE;
    out->d.assign(a.d.begin(), a.d.begin() + a.na);
    out->d.insert(out->d.end(), b.d.begin(), b.d.begin() + b.na);
    out->na = a.na + b.na;
    out->d.push_back(2);
    out->d.insert(out->d.end(), a.d.begin() + a.na, a.d.end());
    out->dtype = a.dtype;
    return out->d.size() > GS_MAX_RANK + 1 ? GS_ERR_RANK : GS_OK;
  }
  if (h == "windows" && n == 3) {
    std::vector<int64_t> w, s;
    if ((st = infer(arg(t, 0), env, &a))) return st;
    if (!env.tuple(arg(t, 1), "shape", &w) || !env.tuple(arg(t, 2), "shape", &s)) return GS_ERR_UNSUPPORTED;
    if (int(w.size()) != a.nc() || int(s.size()) != a.nc() || a.nc() < 1) return GS_ERR_RANK;
    out->d.assign(a.d.begin(), a.d.begin() + a.na);
    for (int k = 0; k < a.nc(); ++k) {
      const int64_t bdim = a.d[a.na + k];
      if (w[k] < 1 || s[k] < 1 || w[k] > bdim) return GS_ERR_SHAPE;
      out->d.push_back((bdim - (w[k] - 1) + s[k] - 1) / s[k]);
    }
    out->na = int(out->d.size());
    out->d.insert(out->d.end(), w.begin(), w.end());
    out->dtype = a.dtype;
    return out->d.size() > GS_MAX_RANK ? GS_ERR_RANK : GS_OK;
  }
  if (h == "slice" && n == 4) {
    int64_t dim, lo, hi;
    if ((st = infer(arg(t, 0), env, &a))) return st;
    if (!env.integer(arg(t, 1), &dim) || !env.integer(arg(t, 2), &lo) || !env.integer(arg(t, 3), &hi))
      return GS_ERR_UNSUPPORTED;
    if (dim < 0 || dim >= int64_t(a.d.size())) return GS_ERR_RANK;
    if (lo < 0 || lo > hi || hi > a.d[dim]) return GS_ERR_SHAPE;
    *out = a;
    out->d[dim] = hi - lo;
    return GS_OK;
  }
  if (h == "squeeze" && n == 2) {
    int64_t dim;
    if ((st = infer(arg(t, 0), env, &a))) return st;
    if (!env.integer(arg(t, 1), &dim)) return GS_ERR_UNSUPPORTED;
    if (dim < 0 || dim >= int64_t(a.d.size())) return GS_ERR_RANK;
    if (a.d[dim] != 1) return GS_ERR_SHAPE;
    *out = a;
    out->d.erase(out->d.begin() + dim);
    if (dim < a.na) out->na = a.na - 1;
    return GS_OK;
  }
  if (h == "flatten" && n == 1) {
    if ((st = infer(arg(t, 0), env, &a))) return st;
    out->d.clear();
    if (a.na > 0) out->d.push_back(a.access_numel());
    out->na = a.na > 0 ? 1 : 0;
    if (a.nc() > 0) out->d.push_back(a.compute_numel());
    out->dtype = a.dtype;
    return GS_OK;
  }
  if (h == "reshape" && n == 3) {
    std::vector<int64_t> sa, sc;
    if ((st = infer(arg(t, 0), env, &a))) return st;
    if (!env.tuple(arg(t, 1), "shape", &sa) || !env.tuple(arg(t, 2), "shape", &sc)) return GS_ERR_UNSUPPORTED;
    int64_t pa = 1, pc = 1;
    for (int64_t x : sa) pa *= x;
    for (int64_t x : sc) pc *= x;
    for (int64_t x : sa)
      if (x < 0) return GS_ERR_SHAPE;
    for (int64_t x : sc)
      if (x < 0) return GS_ERR_SHAPE;
    if (pa != a.access_numel() || pc * pa != a.numel()) return GS_ERR_SHAPE;
    out->d = sa;
    out->na = int(sa.size());
    out->d.insert(out->d.end(), sc.begin(), sc.end());
    out->dtype = a.dtype;
    return out->d.size() > GS_MAX_RANK ? GS_ERR_RANK : GS_OK;
  }
  if (h == "pair" && n == 2) {
    if ((st = infer(arg(t, 0), env, &a))) return st;
    if ((st = infer(arg(t, 1), env, &b))) return st;
    if (a.d != b.d || a.na != b.na) return GS_ERR_SHAPE;
    if (a.dtype != b.dtype) return GS_ERR_DTYPE;
    *out = a;
    out->d.insert(out->d.begin() + a.na, 2);
    return out->d.size() > GS_MAX_RANK ? GS_ERR_RANK : GS_OK;
  }
  if (h == "concat" && n == 3) {
    int64_t dim;
    if ((st = infer(arg(t, 0), env, &a))) return st;
    if ((st = infer(arg(t, 1), env, &b))) return st;
    if (!env.integer(arg(t, 2), &dim)) return GS_ERR_UNSUPPORTED;
    if (a.d.size() != b.d.size() || a.na != b.na) return GS_ERR_RANK;
    if (dim < 0 || dim >= int64_t(a.d.size())) return GS_ERR_RANK;
    if (a.dtype != b.dtype) return GS_ERR_DTYPE;
    for (size_t k = 0; k < a.d.size(); ++k)
      if (int64_t(k) != dim && a.d[k] != b.d[k]) return GS_ERR_SHAPE;
    *out = a;
    out->d[dim] = a.d[dim] + b.d[dim];
    return GS_OK;
  }
  if (h == "pad" && n == 4) {           // EXT: zero padding
    int64_t dim, lo, hi;
    if ((st = infer(arg(t, 0), env, &a))) return st;
    if (!env.integer(arg(t, 1), &dim) || !env.integer(arg(t, 2), &lo) || !env.integer(arg(t, 3), &hi))
      return GS_ERR_UNSUPPORTED;
    if (dim < 0 || dim >= int64_t(a.d.size())) return GS_ERR_RANK;
    if (lo < 0 || hi < 0) return GS_ERR_SHAPE;
    *out = a;
    out->d[dim] += lo + hi;
    return GS_OK;
  }
  if (h == "compute" && n == 2) return infer_compute(t, env, out);
  if (h == "systolicArray" && n == 4) {
    int64_t rows, cols;
    if (!env.integer(arg(t, 0), &rows) || !env.integer(arg(t, 1), &cols)) return GS_ERR_UNSUPPORTED;
    if ((st = infer(arg(t, 2), env, &a))) return st;
    if ((st = infer(arg(t, 3), env, &b))) return st;
    if (a.d.size() != 2 || a.na != 1 || b.d.size() != 2 || b.na != 0) return GS_ERR_RANK;
    if (a.d[1] != rows || b.d[0] != rows || b.d[1] != cols) return GS_ERR_SHAPE;
    if (a.dtype != b.dtype) return GS_ERR_DTYPE;
    out->d = {a.d[0], cols};
    out->na = 2;
    out->dtype = dot_out_dtype(a.dtype);
    return out->dtype < 0 ? GS_ERR_DTYPE : GS_OK;
  }
  return GS_ERR_UNSUPPORTED;
}

// ---------------------------------------------------------------------------------------------
// Evaluation
// ---------------------------------------------------------------------------------------------
gs_ap make_ap(void* data, const Shape& s) {
  gs_ap a;
  memset(&a, 0, sizeof(a));
  a.data = data;
  a.dtype = s.dtype;
  a.rank = int(s.d.size());
  a.n_access = s.na;
  for (size_t i = 0; i < s.d.size(); ++i) a.shape[i] = s.d[i];
  return a;
}

struct Value {
  Shape s;
  void* data = nullptr;
};

// The listing of Fig. 2a, with the sizes of its shape literals.
struct ConvMatch {
  TreeP act, weights;
  std::vector<int64_t> window, stride;
};
bool match_conv2d(const TreeP& t, const Env& env, ConvMatch* m) {
  std::vector<int64_t> perm;
  int64_t one;
  if (!is_call(t, "transpose", 2) || !env.tuple(arg(t, 1), "list", &perm)) return false;
  if (perm != std::vector<int64_t>({0, 3, 1, 2})) return false;
  const TreeP& sq = arg(t, 0);
  if (!is_call(sq, "squeeze", 2) || !env.integer(arg(sq, 1), &one) || one != 1) return false;
  const TreeP& cp = arg(sq, 0);
  if (!is_call(cp, "compute", 2) || arg(cp, 0)->kind != Tree::kSymbol || arg(cp, 0)->sym != "dotProd") return false;
  const TreeP& c = arg(cp, 1);
  if (!is_call(c, "cartProd", 2)) return false;
  const TreeP& w = arg(c, 0);
  const TreeP& f = arg(c, 1);
  int64_t i;
  if (!is_call(w, "windows", 3) || !is_call(arg(w, 0), "access", 2) || !env.integer(arg(arg(w, 0), 1), &i) || i != 1)
    return false;
  if (!is_call(f, "access", 2) || !env.integer(arg(f, 1), &i) || i != 1) return false;
  if (!env.tuple(arg(w, 1), "shape", &m->window) || !env.tuple(arg(w, 2), "shape", &m->stride)) return false;
  m->act = arg(arg(w, 0), 0);
  m->weights = arg(f, 0);
  Shape a, b;
  if (infer(m->act, env, &a) || infer(m->weights, env, &b)) return false;
  if (a.d.size() != 4 || b.d.size() != 4 || m->window.size() != 3 || m->stride.size() != 3) return false;
  // window = the weights' (C, Kh, Kw), covering every channel; stride 1 over the channels
  return m->window[0] == a.d[1] && m->window[0] == b.d[1] && m->window[1] == b.d[2] && m->window[2] == b.d[3] &&
         m->stride[0] == 1 && (a.dtype == GS_I8 || a.dtype == GS_BF16) && a.dtype == b.dtype;
}

struct Evaluator {
  const Env& env;
  bool dry;                // only add up the workspace
  uint8_t* ws;
  size_t ws_bytes, used = 0;
  void* stream;
  std::map<std::string, Value> memo;     // identical sub-programs are evaluated once

  void* alloc(int64_t bytes, int* st) {
    const size_t need = size_t(round_up(bytes > 0 ? bytes : 1, 256));
    void* p = nullptr;
    if (!dry) {
      if (used + need > ws_bytes) {
        *st = GS_ERR_WORKSPACE;
        return nullptr;
      }
      p = ws + used;
    }
    used += need;
    return p;
  }

  // Evaluates node t.  `dst` (may be null): where a data-producing node must put its result.
  // `want` (or -1): the element type asked of the result when it is not the node's own: only a
  // bfloat16 contraction may store narrower than it accumulates, and the transformers between it
  // and the root pass the request down (they keep the element type).
  int eval(const TreeP& t, void* dst, Value* out, int want = -1) {
    const std::string key = dst ? std::string() : to_text(t) + (want >= 0 ? "#" + std::to_string(want) : std::string());
    if (!dst) {
      auto it = memo.find(key);
      if (it != memo.end()) {
        *out = it->second;
        return GS_OK;
      }
    }
    int st = eval_node(t, dst, out, want);
    if (st == GS_OK && !dst) memo[key] = *out;
    return st;
  }

  int materialize(const Shape& s, void* dst, Value* out) {
    int st = GS_OK;
    out->s = s;
    out->data = dst ? dst : alloc(s.numel() * int64_t(gs::dtype_size(s.dtype)), &st);
    return st;
  }

  int eval_node(const TreeP& t, void* dst, Value* out, int want) {
    Shape s;
    int st = infer(t, env, &s);
    if (st) return st;
    int pass = -1;                     // request handed to the operand of a transformer
    if (want >= 0 && want != s.dtype) {
      if (s.dtype != GS_F32 || want != GS_BF16 || t->kind != Tree::kList) return GS_ERR_DTYPE;
      const std::string& hh = t->items[0]->sym;
      const bool dot = hh == "compute" && arg(t, 0)->sym == "dotProd";
      ConvMatch cm;
      if (dot || hh == "systolicArray" || match_conv2d(t, env, &cm)) {
        // the contraction stores bfloat16 itself
      } else if (hh == "access" || hh == "squeeze" || hh == "flatten" || hh == "reshape" || hh == "transpose" ||
                 hh == "slice") {
        pass = want;
      } else {
        return GS_ERR_DTYPE;
      }
      s.dtype = want;
    }
    if (t->kind == Tree::kSymbol) {
      const gs_ap* a = env.tensor(t->sym);
      out->s = s;
      out->data = a->data;
      if (!dry && s.numel() > 0 && (!a->data || reinterpret_cast<uintptr_t>(a->data) % 16)) return GS_ERR_NULL;
      return dst ? copy_to(*out, dst, out) : GS_OK;
    }
    const std::string& h = t->items[0]->sym;
    // --- descriptor-only transformers: the dense row-major data is unchanged -----------------
    if (h == "access" || h == "squeeze" || h == "flatten" || h == "reshape") {
      Value in;
      if ((st = eval(arg(t, 0), dst, &in, pass))) return st;
      out->s = s;
      out->data = in.data;
      return GS_OK;
    }
    if (h == "slice") {
      int64_t dim, lo, hi;
      env.integer(arg(t, 1), &dim);
      env.integer(arg(t, 2), &lo);
      env.integer(arg(t, 3), &hi);
      Shape in_s;
      if ((st = infer(arg(t, 0), env, &in_s))) return st;
      int64_t lead = 1;
      for (int64_t k = 0; k < dim; ++k) lead *= in_s.d[k];
      int64_t inner = 1;
      for (size_t k = dim + 1; k < in_s.d.size(); ++k) inner *= in_s.d[k];
      const int64_t off_bytes = lo * inner * int64_t(gs::dtype_size(s.dtype));
      if (!dst && lead == 1 && off_bytes % 16 == 0) {       // a contiguous range: a view
        Value in;
        if ((st = eval(arg(t, 0), nullptr, &in, pass))) return st;
        out->s = s;
        out->data = in.data ? static_cast<uint8_t*>(in.data) + off_bytes : nullptr;
        return GS_OK;
      }
      Value in;
      if ((st = eval(arg(t, 0), nullptr, &in, pass))) return st;
      if ((st = materialize(s, dst, out))) return st;
      if (dry) return GS_OK;
      gs_ap ia = make_ap(in.data, in.s), oa = make_ap(out->data, s);
      return glenside_slice(&ia, int(dim), lo, hi, &oa, stream);
    }
    // --- data-moving transformers ----------------------------------------------------------------
    if (h == "transpose") {
      ConvMatch cm;
      if (match_conv2d(t, env, &cm)) return eval_conv2d(cm, s, dst, out);
      std::vector<int64_t> perm;
      env.tuple(arg(t, 1), "list", &perm);
      Value in;
      if ((st = eval(arg(t, 0), nullptr, &in, pass))) return st;
      bool identity = true;
      for (size_t k = 0; k < perm.size(); ++k) identity = identity && perm[k] == int64_t(k);
      if (identity && !dst) {
        *out = in;
        out->s = s;
        return GS_OK;
      }
      if ((st = materialize(s, dst, out))) return st;
      if (dry) return GS_OK;
      gs_ap ia = make_ap(in.data, in.s), oa = make_ap(out->data, s);
      return glenside_transpose(&ia, perm.data(), &oa, stream);
    }
    if (h == "windows") {
      std::vector<int64_t> w, sd;
      env.tuple(arg(t, 1), "shape", &w);
      env.tuple(arg(t, 2), "shape", &sd);
      Value in;
      if ((st = eval(arg(t, 0), nullptr, &in))) return st;
      if ((st = materialize(s, dst, out))) return st;
      if (dry) return GS_OK;
      gs_ap ia = make_ap(in.data, in.s), oa = make_ap(out->data, s);
      return glenside_access_windows(&ia, w.data(), sd.data(), nullptr, nullptr, GS_PAD_ZERO, &oa, stream);
    }
    if (h == "pair" || h == "concat") {
      Value a, b;
      if ((st = eval(arg(t, 0), nullptr, &a))) return st;
      if ((st = eval(arg(t, 1), nullptr, &b))) return st;
      if ((st = materialize(s, dst, out))) return st;
      if (dry) return GS_OK;
      gs_ap aa = make_ap(a.data, a.s), ba = make_ap(b.data, b.s), oa = make_ap(out->data, s);
      if (h == "pair") return glenside_pair(&aa, &ba, &oa, stream);
      int64_t dim;
      env.integer(arg(t, 2), &dim);
      return glenside_concat(&aa, &ba, int(dim), &oa, stream);
    }
    if (h == "pad") {
      int64_t dim, lo, hi;
      env.integer(arg(t, 1), &dim);
      env.integer(arg(t, 2), &lo);
      env.integer(arg(t, 3), &hi);
      Value in;
      if ((st = eval(arg(t, 0), nullptr, &in))) return st;
      if ((st = materialize(s, dst, out))) return st;
      if (dry) return GS_OK;
      gs_ap ia = make_ap(in.data, in.s), oa = make_ap(out->data, s);
      return glenside_pad(&ia, int(dim), lo, hi, GS_PAD_ZERO, &oa, stream);
    }
    if (h == "cartProd") return GS_ERR_UNSUPPORTED;   // only as the operand of compute dotProd
    // --- compute ---------------------------------------------------------------------------------
    if (h == "systolicArray") {
      // out[b, c] = sum_r a0[b, r] w[r, c]: the contraction of a0 with w's transposition.  The
      // rewrite of Fig. 3 writes w as (access (transpose ?a1 (list 1 0)) 0): then ?a1 is used as is.
      Value a0, a1;
      if ((st = eval(arg(t, 2), nullptr, &a0))) return st;
      const TreeP& w = arg(t, 3);
      std::vector<int64_t> perm;
      int64_t zero;
      if (is_call(w, "access", 2) && env.integer(arg(w, 1), &zero) && zero == 0 && is_call(arg(w, 0), "transpose", 2) &&
          env.tuple(arg(arg(w, 0), 1), "list", &perm) && perm == std::vector<int64_t>({1, 0})) {
        if ((st = eval(arg(arg(w, 0), 0), nullptr, &a1))) return st;
      } else {
        TreeP tr = call("transpose", {w, int_tuple("list", {1, 0})});
        if ((st = eval(tr, nullptr, &a1))) return st;
      }
      a1.s.na = 1;
      if ((st = materialize(s, dst, out))) return st;
      if (dry) return GS_OK;
      gs_ap x = make_ap(a0.data, a0.s), y = make_ap(a1.data, a1.s), oa = make_ap(out->data, s);
      return glenside_cartesian_dot(&x, &y, &oa, GS_ACT_NONE, nullptr, 0, stream);
    }
    if (h == "compute") {
      const std::string& op = arg(t, 0)->sym;
      const TreeP& x = arg(t, 1);
      if (op == "dotProd") {                      // Fig. 3, left-hand side: one contraction
        if (!is_call(x, "cartProd", 2)) return GS_ERR_UNSUPPORTED;   // the tuple dimension is never materialised
        Value a, b;
        if ((st = eval(arg(x, 0), nullptr, &a))) return st;
        if ((st = eval(arg(x, 1), nullptr, &b))) return st;
        if ((st = materialize(s, dst, out))) return st;
        if (dry) return GS_OK;
        gs_ap aa = make_ap(a.data, a.s), ba = make_ap(b.data, b.s), oa = make_ap(out->data, s);
        return glenside_cartesian_dot(&aa, &ba, &oa, GS_ACT_NONE, nullptr, 0, stream);
      }
      const int rop = op == "reduceMax" ? GS_MAX : GS_SUM;
      if (op == "relu") {                         // EXT: max(x, x) with the fused ReLU
        Value in;
        if ((st = eval(x, nullptr, &in))) return st;
        if ((st = materialize(s, dst, out))) return st;
        if (dry) return GS_OK;
        gs_ap ia = make_ap(in.data, in.s), oa = make_ap(out->data, s);
        return glenside_pair_reduce(&ia, &ia, GS_MAX, GS_ACT_RELU, &oa, stream);
      }
      Shape xs;
      if ((st = infer(x, env, &xs))) return st;
      if (is_call(x, "windows", 3) && xs.nc() <= 3) {        // Fig. 2c: pooling without the windows in memory
        std::vector<int64_t> w, sd;
        env.tuple(arg(x, 1), "shape", &w);
        env.tuple(arg(x, 2), "shape", &sd);
        Value in;
        if ((st = eval(arg(x, 0), nullptr, &in))) return st;
        if ((st = materialize(s, dst, out))) return st;
        if (dry) return GS_OK;
        gs_ap ia = make_ap(in.data, in.s), oa = make_ap(out->data, s);
        return glenside_windows_reduce(&ia, w.data(), sd.data(), nullptr, nullptr, rop, 1.0f, &oa, stream);
      }
      if (is_call(x, "pair", 2) && xs.nc() == 1 && xs.dtype != GS_I8) {   // Sec. 5.4: element-wise sum / max
        Value a, b;
        if ((st = eval(arg(x, 0), nullptr, &a))) return st;
        if ((st = eval(arg(x, 1), nullptr, &b))) return st;
        if ((st = materialize(s, dst, out))) return st;
        if (dry) return GS_OK;
        gs_ap aa = make_ap(a.data, a.s), ba = make_ap(b.data, b.s), oa = make_ap(out->data, s);
        return glenside_pair_reduce(&aa, &ba, rop, GS_ACT_NONE, &oa, stream);
      }
      Value in;
      if ((st = eval(x, nullptr, &in))) return st;
      if ((st = materialize(s, dst, out))) return st;
      if (dry) return GS_OK;
      gs_ap ia = make_ap(in.data, in.s), oa = make_ap(out->data, s);
      return glenside_reduce(&ia, rop, 1.0f, &oa, stream);
    }
    return GS_ERR_UNSUPPORTED;
  }

  int eval_conv2d(const ConvMatch& m, const Shape& s, void* dst, Value* out) {
    Value a, w;
    int st;
    if ((st = eval(m.act, nullptr, &a))) return st;
    if ((st = eval(m.weights, nullptr, &w))) return st;
    a.s.na = 1;
    w.s.na = 1;
    gs_ap aa = make_ap(a.data, a.s), wa = make_ap(w.data, w.s);
    const int64_t stride[2] = {m.stride[1], m.stride[2]}, pad[2] = {0, 0};
    const size_t cws = glenside_conv2d_direct_workspace(&aa, &wa, stride, pad);
    if (cws == 0) return GS_ERR_UNSUPPORTED;
    void* scratch = alloc(int64_t(cws), &st);
    if (st) return st;
    if ((st = materialize(s, dst, out))) return st;
    if (dry) return GS_OK;
    gs_ap oa = make_ap(out->data, s);
    return glenside_conv2d_direct(&aa, &wa, stride, pad, nullptr, GS_ACT_NONE, &oa, scratch, cws, stream);
  }

  // The root names an input (or a view of one): copy it to the result.
  int copy_to(const Value& src, void* dst, Value* out) {
    const Value in = src;          // `out` may be the same object
    out->s = in.s;
    out->data = dst;
    if (dry || in.s.numel() == 0) return GS_OK;
    std::vector<int64_t> perm(in.s.d.size());
    for (size_t k = 0; k < perm.size(); ++k) perm[k] = int64_t(k);
    gs_ap ia = make_ap(in.data, in.s), oa = make_ap(dst, in.s);
    if (perm.empty()) {            // a scalar: a one-element slice
      Shape one = in.s;
      one.d = {1};
      one.na = 0;
      ia = make_ap(in.data, one);
      oa = make_ap(dst, one);
      return glenside_slice(&ia, 0, 0, 1, &oa, stream);
    }
    return glenside_transpose(&ia, perm.data(), &oa, stream);
  }
};

bool views_input(const TreeP& t) {       // the value of t is (a view of) a named tensor
  if (t->kind == Tree::kSymbol) return true;
  if (t->kind != Tree::kList || t->items.empty()) return false;
  const std::string& h = t->items[0]->sym;
  if (h == "access" || h == "squeeze" || h == "flatten" || h == "reshape") return views_input(arg(t, 0));
  return false;
}

int run(const char* text, const Env& env, gs_ap* out, void* ws, size_t ws_bytes, void* stream, bool dry,
        size_t* need) {
  TreeP t = parse(text);
  if (!t) return GS_ERR_UNSUPPORTED;
  Shape s;
  int st = infer(t, env, &s);
  if (st) return st;
  Evaluator ev{env, dry, static_cast<uint8_t*>(ws), ws_bytes};
  ev.stream = stream;
  void* dst = nullptr;
  if (!dry) {
    if (!out) return GS_ERR_NULL;
    if (out->rank != int(s.d.size()) || out->n_access != s.na) return GS_ERR_RANK;
    for (size_t k = 0; k < s.d.size(); ++k)
      if (out->shape[k] != s.d[k]) return GS_ERR_SHAPE;
    if (s.numel() > 0 && (!out->data || reinterpret_cast<uintptr_t>(out->data) % 16)) return GS_ERR_NULL;
    if (ws_bytes > 0 && (!ws || reinterpret_cast<uintptr_t>(ws) % 16)) return GS_ERR_WORKSPACE;
    dst = out->data;
  }
  Value v;
  // A root that only re-describes an input produces no data of its own: evaluate, then copy.
  const int want = (!dry && out->dtype != s.dtype) ? out->dtype : -1;
  if (views_input(t)) {
    if ((st = ev.eval(t, nullptr, &v, want))) return st;
    if (!dry) st = ev.copy_to(v, dst, &v);
  } else {
    st = ev.eval(t, dry ? nullptr : dst, &v, want);
  }
  if (need) *need = ev.used;
  return st;
}

// ---------------------------------------------------------------------------------------------
// Rewrites
// ---------------------------------------------------------------------------------------------
TreeP shape_lit(const std::vector<int64_t>& v) { return int_tuple("shape", v); }

// Fig. 4, rule 1:  ?a  =>  (reshape (flatten ?a) ?shape), ?shape = the shape of ?a.
TreeP rule_flatten_reshape(const TreeP& a, const Env& env) {
  Shape s;
  if (infer(a, env, &s)) return nullptr;
  std::vector<int64_t> sa(s.d.begin(), s.d.begin() + s.na), sc(s.d.begin() + s.na, s.d.end());
  return call("reshape", {call("flatten", {a}), shape_lit(sa), shape_lit(sc)});
}
// Fig. 4, rule 2:  (cartProd (reshape ?a0 ?s0) (reshape ?a1 ?s1)) => (reshape (cartProd ?a0 ?a1) ?new),
// ?new = (S_A(s0) ++ S_A(s1), (2) ++ S_C(s0)); needs S_C(s0) = S_C(s1).
TreeP rule_cartprod_reshape(const TreeP& t, const Env& env) {
  if (!is_call(t, "cartProd", 2) || !is_call(arg(t, 0), "reshape", 3) || !is_call(arg(t, 1), "reshape", 3)) return nullptr;
  std::vector<int64_t> a0, c0, a1, c1;
  if (!env.tuple(arg(arg(t, 0), 1), "shape", &a0) || !env.tuple(arg(arg(t, 0), 2), "shape", &c0) ||
      !env.tuple(arg(arg(t, 1), 1), "shape", &a1) || !env.tuple(arg(arg(t, 1), 2), "shape", &c1) || c0 != c1)
    return nullptr;
  TreeP inner = call("cartProd", {arg(arg(t, 0), 0), arg(arg(t, 1), 0)});
  Shape chk;
  if (infer(inner, env, &chk)) return nullptr;        // the flattened operands must still pair up
  std::vector<int64_t> na = a0, nc = {2};
  na.insert(na.end(), a1.begin(), a1.end());
  nc.insert(nc.end(), c0.begin(), c0.end());
  return call("reshape", {inner, shape_lit(na), shape_lit(nc)});
}
// Fig. 4, rule 3:  (compute dotProd (reshape ?a ?shape)) => (reshape (compute dotProd ?a) ?new),
// ?new = (S_A(?shape), ()).
TreeP rule_dot_reshape(const TreeP& t, const Env& env) {
  if (!is_call(t, "compute", 2) || arg(t, 0)->sym != "dotProd" || !is_call(arg(t, 1), "reshape", 3)) return nullptr;
  std::vector<int64_t> sa;
  if (!env.tuple(arg(arg(t, 1), 1), "shape", &sa)) return nullptr;
  return call("reshape", {call("compute", {mk_sym("dotProd"), arg(arg(t, 1), 0)}), shape_lit(sa), shape_lit({})});
}
// Fig. 3:  (compute dotProd (cartProd ?a0 ?a1)) => (systolicArray ?rows ?cols ?a0 (access (transpose ?a1 (list 1 0)) 0))
// where ?a0 : ((?batch),(?rows)) and ?a1 : ((?cols),(?rows)).
TreeP rule_systolic(const TreeP& t, const Env& env) {
  if (!is_call(t, "compute", 2) || arg(t, 0)->sym != "dotProd" || !is_call(arg(t, 1), "cartProd", 2)) return nullptr;
  Shape a0, a1;
  const TreeP& c = arg(t, 1);
  if (infer(arg(c, 0), env, &a0) || infer(arg(c, 1), env, &a1)) return nullptr;
  if (a0.d.size() != 2 || a0.na != 1 || a1.d.size() != 2 || a1.na != 1 || a0.d[1] != a1.d[1]) return nullptr;
  return call("systolicArray", {mk_int(a0.d[1]), mk_int(a1.d[0]), arg(c, 0),
                                call("access", {call("transpose", {arg(c, 1), int_tuple("list", {1, 0})}), mk_int(0)})});
}
// Applies `rule` to the first node (pre-order) where it fires.
template <typename F>
TreeP rewrite_first(const TreeP& t, F&& rule, bool* fired) {
  if (TreeP r = rule(t)) {
    *fired = true;
    return r;
  }
  if (t->kind != Tree::kList) return t;
  std::vector<TreeP> items;
  bool changed = false;
  for (const TreeP& c : t->items) {
    if (!*fired) {
      TreeP n = rewrite_first(c, rule, fired);
      changed = changed || n != c;
      items.push_back(n);
    } else {
      items.push_back(c);
    }
  }
  return changed ? mk_list(items) : t;
}

// Fig. 2a -> Fig. 5.
TreeP derive_im2col(const TreeP& t, const Env& env) {
  bool fired = false;
  // rule 1 on both operands of the cartProd that feeds the dotProd
  TreeP r = rewrite_first(t, [&](const TreeP& n) -> TreeP {
    if (!is_call(n, "compute", 2) || arg(n, 0)->sym != "dotProd" || !is_call(arg(n, 1), "cartProd", 2)) return nullptr;
    const TreeP& c = arg(n, 1);
    TreeP a = rule_flatten_reshape(arg(c, 0), env), b = rule_flatten_reshape(arg(c, 1), env);
    if (!a || !b) return nullptr;
    return call("compute", {mk_sym("dotProd"), call("cartProd", {a, b})});
  }, &fired);
  if (!fired) return nullptr;
  fired = false;
  r = rewrite_first(r, [&](const TreeP& n) { return rule_cartprod_reshape(n, env); }, &fired);
  if (!fired) return nullptr;
  fired = false;
  r = rewrite_first(r, [&](const TreeP& n) { return rule_dot_reshape(n, env); }, &fired);
  return fired ? r : nullptr;
}

// Fig. 6, rule 1, applied repeatedly:  ?a => (concat (slice ?a d 0 b) (slice ?a d b e) d), the second
// part split again; `leaf` is applied to every block that is not split further.
template <typename F>
TreeP split_dim(const TreeP& a, int dim, int64_t extent, int64_t block, F&& leaf) {
  if (block <= 0 || extent <= block) return leaf(a);
  TreeP head = call("slice", {a, mk_int(dim), mk_int(0), mk_int(block)});
  TreeP rest = call("slice", {a, mk_int(dim), mk_int(block), mk_int(extent)});
  return call("concat", {leaf(head), split_dim(rest, dim, extent - block, block, leaf), mk_int(dim)});
}
// Fig. 6, rules 2-5 (and the mirror image of rule 2 for the first operand), to a fixed point.
TreeP push_blocking(const TreeP& t, const Env& env) {
  if (t->kind != Tree::kList) return t;
  std::vector<TreeP> items;
  for (const TreeP& c : t->items) items.push_back(push_blocking(c, env));
  TreeP n = mk_list(items);
  if (is_call(n, "cartProd", 2)) {
    const TreeP &a = arg(n, 0), &b = arg(n, 1);
    Shape sa, sb;
    if (infer(a, env, &sa) || infer(b, env, &sb)) return n;
    int64_t da = -1, db = -1;
    const bool ca = is_call(a, "concat", 3) && env.integer(arg(a, 2), &da);
    const bool cb = is_call(b, "concat", 3) && env.integer(arg(b, 2), &db);
    // rule 3: both operands concatenated along the same compute dimension
    if (ca && cb && da >= sa.na && db >= sb.na && da - sa.na == db - sb.na) {
      const int64_t nd = sa.na + sb.na + 1 + (da - sa.na);
      return push_blocking(call("concat", {call("cartProd", {arg(a, 0), arg(b, 0)}),
                                           call("cartProd", {arg(a, 1), arg(b, 1)}), mk_int(nd)}), env);
    }
    // rule 2: second operand concatenated along an access dimension
    if (cb && db < sb.na)
      return push_blocking(call("concat", {call("cartProd", {a, arg(b, 0)}), call("cartProd", {a, arg(b, 1)}),
                                           mk_int(db + sa.na)}), env);
    // its mirror image: first operand concatenated along an access dimension
    if (ca && da < sa.na)
      return push_blocking(call("concat", {call("cartProd", {arg(a, 0), b}), call("cartProd", {arg(a, 1), b}),
                                           mk_int(da)}), env);
    return n;
  }
  if (is_call(n, "compute", 2) && arg(n, 0)->sym == "dotProd" && is_call(arg(n, 1), "concat", 3)) {
    const TreeP& c = arg(n, 1);
    Shape sc;
    int64_t d;
    if (infer(c, env, &sc) || !env.integer(arg(c, 2), &d)) return n;
    TreeP l = push_blocking(call("compute", {mk_sym("dotProd"), arg(c, 0)}), env);
    TreeP r = push_blocking(call("compute", {mk_sym("dotProd"), arg(c, 1)}), env);
    if (d < sc.na) return call("concat", {l, r, mk_int(d)});                     // rule 4
    return call("compute", {mk_sym("reduceSum"), call("pair", {l, r})});         // rule 5
  }
  return n;
}
// Fig. 2b -> the blocked program of Fig. 7 with blocks of (bm, bn, bk).
TreeP derive_blocked(const TreeP& t, const Env& env, int64_t bm, int64_t bn, int64_t bk) {
  bool fired = false;
  TreeP r = rewrite_first(t, [&](const TreeP& n) -> TreeP {
    if (!is_call(n, "compute", 2) || arg(n, 0)->sym != "dotProd" || !is_call(arg(n, 1), "cartProd", 2)) return nullptr;
    const TreeP& c = arg(n, 1);
    Shape a, b;
    if (infer(arg(c, 0), env, &a) || infer(arg(c, 1), env, &b)) return nullptr;
    if (a.d.size() != 2 || a.na != 1 || b.d.size() != 2 || b.na != 1) return nullptr;
    // rule 1 on every blocked dimension: each operand's access dimension, then the compute
    // dimension of every block of rows
    auto blocks = [&](const TreeP& x, const Shape& s, int64_t bacc) {
      return split_dim(x, 0, s.d[0], bacc, [&](const TreeP& rows) {
        return split_dim(rows, 1, s.d[1], bk, [](const TreeP& blk) { return blk; });
      });
    };
    return call("compute", {mk_sym("dotProd"), call("cartProd", {blocks(arg(c, 0), a, bm), blocks(arg(c, 1), b, bn)})});
  }, &fired);
  if (!fired) return nullptr;
  return push_blocking(r, env);
}

int copy_out(const TreeP& t, char* out, size_t cap, size_t* need) {
  const std::string s = to_text(t);
  if (need) *need = s.size() + 1;
  if (!out || cap < s.size() + 1) return GS_ERR_WORKSPACE;
  memcpy(out, s.c_str(), s.size() + 1);
  return GS_OK;
}

}  // namespace

extern "C" {

int glenside_program_shape(const char* text, const gs_named_ap* tensors, int n_tensors, const gs_named_int* ints,
                           int n_ints, gs_ap* out) {
  if (!text || !out || (n_tensors > 0 && !tensors) || (n_ints > 0 && !ints)) return GS_ERR_NULL;
  Env env{tensors, n_tensors, ints, n_ints};
  TreeP t = parse(text);
  if (!t) return GS_ERR_UNSUPPORTED;
  Shape s;
  int st = infer(t, env, &s);
  if (st) return st;
  if (s.d.size() > GS_MAX_RANK) return GS_ERR_RANK;
  void* keep = out->data;
  *out = make_ap(keep, s);
  return GS_OK;
}

size_t glenside_program_workspace(const char* text, const gs_named_ap* tensors, int n_tensors,
                                  const gs_named_int* ints, int n_ints) {
  if (!text || (n_tensors > 0 && !tensors) || (n_ints > 0 && !ints)) return 0;
  Env env{tensors, n_tensors, ints, n_ints};
  size_t need = 0;
  if (run(text, env, nullptr, nullptr, 0, nullptr, true, &need)) return 0;
  return need + 256;
}

int glenside_program_eval(const char* text, const gs_named_ap* tensors, int n_tensors, const gs_named_int* ints,
                          int n_ints, gs_ap* out, void* workspace, size_t workspace_bytes, void* stream) {
  if (!text || !out || (n_tensors > 0 && !tensors) || (n_ints > 0 && !ints)) return GS_ERR_NULL;
  Env env{tensors, n_tensors, ints, n_ints};
  return run(text, env, out, workspace, workspace_bytes, stream, false, nullptr);
}

int glenside_program_rewrite(const char* text, const char* strategy, const int64_t* params, int n_params,
                             const gs_named_ap* tensors, int n_tensors, const gs_named_int* ints, int n_ints,
                             char* out_text, size_t out_capacity, size_t* out_needed) {
  if (!text || !strategy || (n_tensors > 0 && !tensors) || (n_ints > 0 && !ints) || (n_params > 0 && !params))
    return GS_ERR_NULL;
  Env env{tensors, n_tensors, ints, n_ints};
  TreeP t = parse(text);
  if (!t) return GS_ERR_UNSUPPORTED;
  Shape before;
  int st = infer(t, env, &before);
  if (st) return st;
  TreeP r;
  const std::string s = strategy;
  if (s == "im2col") {
    r = derive_im2col(t, env);
  } else if (s == "systolic") {
    bool fired = false;
    r = rewrite_first(t, [&](const TreeP& n) { return rule_systolic(n, env); }, &fired);
    if (!fired) r = nullptr;
  } else if (s == "block") {
    if (n_params != 3 || params[0] < 1 || params[1] < 1 || params[2] < 1) return GS_ERR_SHAPE;
    r = derive_blocked(t, env, params[0], params[1], params[2]);
  } else {
    return GS_ERR_UNSUPPORTED;
  }
  if (!r) return GS_ERR_UNSUPPORTED;          // no rule of the strategy applies to this program
  // A rewrite preserves the access-pattern shape of the program: checked, not assumed.
  Shape after;
  if ((st = infer(r, env, &after))) return st;
  if (after.d != before.d || after.na != before.na || after.dtype != before.dtype) return GS_ERR_SHAPE;
  return copy_out(r, out_text, out_capacity, out_needed);
}

}  // extern "C"
