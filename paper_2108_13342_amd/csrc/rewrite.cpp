// Mathematical-property-based graph rewriting (paper Sec. 4.2, Table 4).
//
// Two stages:
//  1. Canonicalisation: exporter decompositions are recognised and replaced by one operator of the
//     same mapping type they would fuse to (decomposed softmax -> Softmax, decomposed LayerNorm
//     statistics -> Normalize), BatchNormalization becomes a per-channel multiply-add whose
//     coefficients are weight-only expressions, Pow/Div by constants are strength-reduced.
//  2. The rule engine: the graph is partitioned at operators that have none of the associative,
//     commutative or distributive properties; inside a partition every rule is matched everywhere,
//     the match with the largest #FLOPS reduction is applied, and this repeats until nothing
//     matches (the greedy scheme of Sec. 4.2).  The rules are the ten printed in Table 4, with the
//     operand orders commutativity allows.
#include <algorithm>
#include <cmath>
#include <functional>
#include <numeric>

#include "ir.hpp"

namespace dnnf {

namespace {

struct Rewriter {
  Graph& g;
  RewriteStats& st;
  explicit Rewriter(Graph& g_, RewriteStats& s_) : g(g_), st(s_) {}

  const Op* producer(int t) const {
    int p = g.tensors[t].producer;
    return p >= 0 && g.ops[p].alive ? &g.ops[p] : nullptr;
  }
  bool is_scalar_const(int t, double* v = nullptr) const {
    const Tensor& T = g.tensors[t];
    if (T.kind != DNNF_WEIGHT || !T.has_cval || T.n() != 1) return false;
    if (v) *v = T.cval[0];
    return true;
  }
  int n_uses(int t) const {
    return (int)g.tensors[t].consumers.size() + (g.tensors[t].kind == DNNF_OUTPUT ? 1 : 0);
  }
  int emit(const std::string& kind, const std::vector<int>& in, const Attrs& a = {}, int dtype = -1) {
    Op tmp;
    tmp.kind = kind;
    tmp.info = find_op_kind(kind);
    tmp.in = in;
    tmp.attrs = a;
    tmp.out = {0};
    Dims d = infer_shape(g, tmp, 0);
    int dt = dtype >= 0 ? dtype : g.tensors[in[0]].dtype;
    int o = g.new_tensor_like(kind, dt, d);
    g.add_op(kind, in, {o}, a);
    return o;
  }
  // every consumer of `from` reads `to` instead; a graph output keeps its identity by renaming
  void replace_uses(int from, int to) {
    if (g.tensors[to].origin.empty())
      g.tensors[to].origin = g.tensors[from].origin.empty() ? g.tensors[from].name : g.tensors[from].origin;
    for (auto& op : g.ops)
      if (op.alive)
        for (int& t : op.in) if (t == from) t = to;
    if (g.tensors[from].kind == DNNF_OUTPUT) {
      // the producer of `to` now writes the graph output tensor directly
      for (auto& op : g.ops)
        if (op.alive) {
          for (int& t : op.out) if (t == to) t = from;
          for (int& t : op.in) if (t == to) t = from;
        }
      int p = g.tensors[from].producer;
      if (p >= 0) g.ops[p].alive = false;
    }
  }
  void dce() {
    bool again = true;
    while (again) {
      again = false;
      g.relink();
      for (auto& op : g.ops) {
        if (!op.alive) continue;
        bool used = false;
        for (int o : op.out) used = used || n_uses(o) > 0;
        if (!used) { op.alive = false; again = true; }
      }
    }
    g.relink();
  }

  // ---------------------------------------------------------------- canonicalisation
  bool canon_batchnorm() {
    bool any = false;
    size_t n = g.ops.size();
    for (size_t i = 0; i < n; i++) {
      if (!g.ops[i].alive || g.ops[i].kind != "BatchNormalization") continue;
      Op op = g.ops[i];
      int x = op.in[0];
      bool wo = true;
      for (int k = 1; k < 5; k++) wo = wo && g.tensors[op.in[k]].weight_only;
      if (!wo) continue;
      const Dims xd = g.tensors[x].dims;   // copy: new tensors are appended below
      int dt = g.tensors[op.in[1]].dtype;
      int eps = g.new_const("bn_eps", DNNF_F32, {}, {op.f("epsilon", 1e-5)});
      int ve = emit("Add", {op.in[4], eps}, {}, DNNF_F32);
      int sd = emit("Sqrt", {ve}, {}, DNNF_F32);
      int scale = emit("Div", {op.in[1], sd}, {}, DNNF_F32);
      int ms = emit("Mul", {op.in[3], scale}, {}, DNNF_F32);
      int shift = emit("Sub", {op.in[2], ms}, {}, DNNF_F32);
      (void)dt;
      std::vector<double> shp = {(double)xd[1]};
      for (size_t d = 2; d < xd.size(); d++) shp.push_back(1.0);
      int scale_r = emit("Reshape", {scale}, {{"shape", shp}}, DNNF_F32);
      int shift_r = emit("Reshape", {shift}, {{"shape", shp}}, DNNF_F32);
      int y = emit("Mul", {x, scale_r});
      int z = emit("Add", {y, shift_r});
      replace_uses(op.out[0], z);
      g.ops[i].alive = false;
      st.log.push_back("canonicalise: BatchNormalization -> Mul, Add with folded coefficients");
      st.canonicalisations++;
      any = true;
      g.relink();
    }
    return any;
  }

  // Cast pairs around regions a 16-bit export keeps in fp32 (LayerNorm, softmax, Pow).  Every block of this executor
  // evaluates in fp32 and rounds once, when it stores a result in that result's own type, so: a widening Cast (or one
  // between equal types) changes no value and its readers take its operand; a narrowing Cast whose operand has no
  // other reader is merged into the operator that computes the operand, which then produces the narrow tensor directly.
  bool canon_casts() {
    bool any = false;
    for (size_t i = 0; i < g.ops.size(); i++) {
      if (!g.ops[i].alive || g.ops[i].kind != "Cast") continue;
      const int in = g.ops[i].in[0], out = g.ops[i].out[0];
      const Tensor& I = g.tensors[in];
      const Tensor& O = g.tensors[out];
      if (!is_float(I.dtype) || !is_float(O.dtype)) continue;
      const bool widening = I.dtype == O.dtype || (dtype_bytes(O.dtype) > dtype_bytes(I.dtype));
      if (widening && O.kind != DNNF_OUTPUT) {
        replace_uses(out, in);
        g.ops[i].alive = false;
      } else if (dtype_bytes(O.dtype) < dtype_bytes(I.dtype) && I.kind == DNNF_INTERMEDIATE && n_uses(in) == 1 && producer(in) &&
                 !g.tensors[in].weight_only) {
        Op& p = g.ops[I.producer];
        for (int& t : p.out) if (t == in) t = out;
        g.ops[i].alive = false;
      } else continue;
      st.log.push_back("canonicalise: Cast between float types merged away");
      st.canonicalisations++;
      any = true;
      g.relink();
    }
    return any;
  }

  // Index-only clean-up around Transpose (Shuffle operators, Sec. 3.1).
  //  (a) Transpose(Transpose(x, p1), p2) is one Transpose by the composed permutation (or x itself).
  //  (b) Data format for the dominant operator (Sec. 4.4.2): the MFMA GEMM reads its second operand fastest when the
  //      stored tensor is contiguous along K, i.e. stored as [.., N, K].  When a MatMul reads T = Transpose(R, pa) and a
  //      sibling Y = Transpose(R, pb) with pa = pb o (swap of the last two axes) is stored anyway (the key tensor an
  //      attention layer also returns), the MatMul reads Transpose(Y, swap) instead: the swap folds into the GEMM's
  //      operand addresses, T need not exist, and one stored tensor serves both readers.
  bool canon_transposes() {
    bool any = false;
    auto perm_of = [&](const Op& op) {
      auto p = op.ints("perm");
      if (p.empty()) for (int i = (int)g.tensors[op.in[0]].dims.size() - 1; i >= 0; i--) p.push_back(i);
      return p;
    };
    for (size_t i = 0; i < g.ops.size(); i++) {
      if (!g.ops[i].alive || g.ops[i].kind != "Transpose" || g.ops[i].has("materialize")) continue;
      const Op* in = producer(g.ops[i].in[0]);
      if (!in || in->kind != "Transpose" || in->has("materialize") || g.tensors[g.ops[i].out[0]].weight_only) continue;
      auto p1 = perm_of(*in), p2 = perm_of(g.ops[i]);
      std::vector<double> p;
      bool ident = true;
      for (size_t d = 0; d < p2.size(); d++) { p.push_back((double)p1[(size_t)p2[d]]); ident = ident && p1[(size_t)p2[d]] == (int64_t)d; }
      if (ident) {
        if (g.tensors[g.ops[i].out[0]].kind == DNNF_OUTPUT) continue;
        replace_uses(g.ops[i].out[0], in->in[0]);
        g.ops[i].alive = false;
      } else {
        g.ops[i].in[0] = in->in[0];
        g.ops[i].attrs["perm"] = p;
      }
      st.log.push_back("canonicalise: consecutive Transposes composed");
      st.canonicalisations++;
      any = true;
      g.relink();
    }
    size_t n = g.ops.size();
    for (size_t i = 0; i < n; i++) {
      if (!g.ops[i].alive || g.ops[i].kind != "MatMul") continue;
      const int t = g.ops[i].in[1];
      const Op* ta = producer(t);
      if (!ta || ta->kind != "Transpose" || g.tensors[t].weight_only || g.tensors[t].dims.size() < 2) continue;
      const auto pa = perm_of(*ta);
      const size_t r = pa.size();
      std::vector<int64_t> pb = pa;
      std::swap(pb[r - 1], pb[r - 2]);           // pb o swap = pa
      int sibling = -1;
      for (int cidx : g.tensors[ta->in[0]].consumers) {
        const Op& o2 = g.ops[cidx];
        if (!o2.alive || &o2 == ta || o2.kind != "Transpose" || o2.has("materialize")) continue;
        if (perm_of(o2) == pb && n_uses(o2.out[0]) >= 1) sibling = o2.out[0];
      }
      if (sibling < 0) continue;
      std::vector<double> sw;
      for (size_t d = 0; d < r; d++) sw.push_back((double)d);
      std::swap(sw[r - 1], sw[r - 2]);
      int nt = emit("Transpose", {sibling}, {{"perm", sw}});
      g.ops[i].in[1] = nt;
      st.log.push_back("layout: MatMul operand read through its K-contiguous sibling");
      st.canonicalisations++;
      any = true;
      g.relink();
    }
    if (any) dce();
    return any;
  }

  // Operators whose operands are all scalar constants are evaluated here (in double, as the constants are held):
  // the shape arithmetic exporters leave behind, e.g. Sqrt(Cast(head size)) in front of the attention scale.
  bool canon_fold_scalars() {
    bool any = false;
    for (bool again = true; again;) {
      again = false;
      for (size_t i = 0; i < g.ops.size(); i++) {
        if (!g.ops[i].alive || g.ops[i].out.size() != 1) continue;
        const Op op = g.ops[i];
        if (g.tensors[op.out[0]].kind == DNNF_OUTPUT || g.tensors[op.out[0]].n() != 1) continue;
        std::vector<double> v;
        bool ok = !op.in.empty();
        for (int t : op.in) { double x; ok = ok && is_scalar_const(t, &x); if (ok) v.push_back(x); }
        if (!ok) continue;
        double r;
        const std::string& k = op.kind;
        if (k == "Cast" || k == "Identity") r = v[0];
        else if (k == "Sqrt") r = std::sqrt(v[0]);
        else if (k == "Neg") r = -v[0];
        else if (k == "Reciprocal") r = 1.0 / v[0];
        else if (k == "Add" && v.size() == 2) r = v[0] + v[1];
        else if (k == "Sub" && v.size() == 2) r = v[0] - v[1];
        else if (k == "Mul" && v.size() == 2) r = v[0] * v[1];
        else if (k == "Div" && v.size() == 2) r = v[0] / v[1];
        else if (k == "Pow" && v.size() == 2) r = std::pow(v[0], v[1]);
        else continue;
        if (!std::isfinite(r)) continue;
        const Tensor& O = g.tensors[op.out[0]];
        int c = g.new_const("folded", O.dtype, O.dims, {r});
        replace_uses(op.out[0], c);
        g.ops[i].alive = false;
        st.log.push_back("canonicalise: " + k + " of scalar constants folded");
        st.canonicalisations++;
        any = again = true;
        g.relink();
      }
    }
    return any;
  }

  bool canon_strength() {
    bool any = false;
    size_t n = g.ops.size();
    for (size_t i = 0; i < n; i++) {
      if (!g.ops[i].alive) continue;
      Op op = g.ops[i];
      double c;
      if (op.kind == "Pow" && is_scalar_const(op.in[1], &c) && (c == 2.0 || c == 0.5 || c == 1.0)) {
        int y = c == 2.0 ? emit("Square", {op.in[0]}) : c == 0.5 ? emit("Sqrt", {op.in[0]}) : op.in[0];
        replace_uses(op.out[0], y);
        g.ops[i].alive = false;
        st.log.push_back("canonicalise: Pow by constant -> cheaper operator");
      } else if (op.kind == "Div" && is_scalar_const(op.in[1], &c) && c != 0.0 && !g.tensors[op.in[0]].weight_only) {
        int r = g.new_const("recip", g.tensors[op.in[1]].dtype == DNNF_F32 ? DNNF_F32 : DNNF_F32, {}, {1.0 / c});
        int y = emit("Mul", {op.in[0], r});
        replace_uses(op.out[0], y);
        g.ops[i].alive = false;
        st.log.push_back("canonicalise: Div by constant -> Mul by reciprocal");
      } else continue;
      st.canonicalisations++;
      any = true;
      g.relink();
    }
    return any;
  }

  static bool last_axis_reduce(const Graph& g, const Op& r) {
    auto ax = r.ints("axes");
    size_t rank = g.tensors[r.in[0]].dims.size();
    return ax.size() == 1 && (ax[0] == -1 || ax[0] == (int64_t)rank - 1) && r.i("keepdims", 1) == 1;
  }

  // p = Div(Exp(Sub(s, ReduceMax(s))), ReduceSum(Exp(...)))  ->  Softmax(s)
  bool canon_softmax() {
    bool any = false;
    size_t n = g.ops.size();
    for (size_t i = 0; i < n; i++) {
      if (!g.ops[i].alive || g.ops[i].kind != "Div") continue;
      Op dv = g.ops[i];
      const Op* ex = producer(dv.in[0]);
      const Op* sm = producer(dv.in[1]);
      if (!ex || !sm || ex->kind != "Exp" || sm->kind != "ReduceSum" || sm->in[0] != ex->out[0] || !last_axis_reduce(g, *sm)) continue;
      const Op* sb = producer(ex->in[0]);
      if (!sb || sb->kind != "Sub") continue;
      const Op* mx = producer(sb->in[1]);
      if (!mx || mx->kind != "ReduceMax" || mx->in[0] != sb->in[0] || !last_axis_reduce(g, *mx)) continue;
      if (n_uses(ex->out[0]) != 2 || n_uses(sm->out[0]) != 1 || n_uses(sb->out[0]) != 1 || n_uses(mx->out[0]) != 1) continue;
      int y = emit("Softmax", {sb->in[0]}, {{"axis", {-1.0}}});
      replace_uses(dv.out[0], y);
      g.ops[i].alive = false;
      st.log.push_back("canonicalise: ReduceMax/Sub/Exp/ReduceSum/Div -> Softmax");
      st.canonicalisations++;
      any = true;
      dce();
    }
    return any;
  }

  // n = Div(d, Sqrt(Add(ReduceMean(Square(d)), eps))), d = Sub(x, ReduceMean(x))  ->  Normalize(x)
  bool canon_normalize() {
    bool any = false;
    size_t n = g.ops.size();
    for (size_t i = 0; i < n; i++) {
      if (!g.ops[i].alive || g.ops[i].kind != "Div") continue;
      Op dv = g.ops[i];
      const Op* d = producer(dv.in[0]);
      const Op* sq = producer(dv.in[1]);
      if (!d || !sq || d->kind != "Sub" || sq->kind != "Sqrt") continue;
      const Op* ad = producer(sq->in[0]);
      if (!ad || ad->kind != "Add") continue;
      double eps;
      int var_t = -1;
      if (is_scalar_const(ad->in[1], &eps)) var_t = ad->in[0];
      else if (is_scalar_const(ad->in[0], &eps)) var_t = ad->in[1];
      else continue;
      const Op* var = producer(var_t);
      if (!var || var->kind != "ReduceMean" || !last_axis_reduce(g, *var)) continue;
      const Op* s2 = producer(var->in[0]);
      if (!s2) continue;
      double two;
      bool is_sq = (s2->kind == "Square" && s2->in[0] == d->out[0]) ||
                   (s2->kind == "Pow" && s2->in[0] == d->out[0] && is_scalar_const(s2->in[1], &two) && two == 2.0) ||
                   (s2->kind == "Mul" && s2->in[0] == d->out[0] && s2->in[1] == d->out[0]);
      if (!is_sq) continue;
      const Op* mu = producer(d->in[1]);
      if (!mu || mu->kind != "ReduceMean" || mu->in[0] != d->in[0] || !last_axis_reduce(g, *mu)) continue;
      int d_uses = s2->kind == "Mul" ? 3 : 2;
      if (n_uses(d->out[0]) != d_uses || n_uses(mu->out[0]) != 1 || n_uses(s2->out[0]) != 1 || n_uses(var->out[0]) != 1 ||
          n_uses(ad->out[0]) != 1 || n_uses(sq->out[0]) != 1)
        continue;
      int y = emit("Normalize", {d->in[0]}, {{"epsilon", {eps}}});
      replace_uses(dv.out[0], y);
      g.ops[i].alive = false;
      st.log.push_back("canonicalise: LayerNorm statistics -> Normalize");
      st.canonicalisations++;
      any = true;
      dce();
    }
    return any;
  }

  // Einsum (Many-to-Many in Table 2) as the batched matrix product it denotes.  Labels fall into four groups:
  // batch (both operands and the result), M (first operand and result), N (second operand and result) and K (both
  // operands, summed).  A is brought to [batch, M, K] and B to [batch, K, N] by a Transpose and a Reshape each, the
  // product is a MatMul, and a Reshape and a Transpose give the result its labels' order.  The index operators
  // fold into the GEMM block's operand and result addresses, so no copy is made.
  bool canon_einsum() {
    bool any = false;
    size_t n = g.ops.size();
    for (size_t i = 0; i < n; i++) {
      if (!g.ops[i].alive || g.ops[i].kind != "Einsum") continue;
      const Op op = g.ops[i];
      const EinsumSpec e = parse_einsum(op);
      const Dims da = g.tensors[op.in[0]].dims, db = g.tensors[op.in[1]].dims;
      auto has = [](const std::string& s, char c) { return s.find(c) != std::string::npos; };
      std::string batch, M, N, K;
      for (char l : e.out) {
        if (has(e.a, l) && has(e.b, l)) batch.push_back(l);
        else if (has(e.a, l)) M.push_back(l);
        else N.push_back(l);
      }
      for (char l : e.a) {
        if (has(e.out, l)) continue;
        DNNF_CHECK(has(e.b, l), DNNF_UNSUPPORTED_OP, std::string("Einsum: label ") + l + " is summed inside one operand");
        K.push_back(l);
      }
      for (char l : e.b) DNNF_CHECK(has(e.out, l) || has(e.a, l), DNNF_UNSUPPORTED_OP, std::string("Einsum: label ") + l + " is summed inside one operand");
      auto extent = [&](char l) { return has(e.a, l) ? da[e.a.find(l)] : db[e.b.find(l)]; };
      auto prod = [&](const std::string& ls) { int64_t p = 1; for (char l : ls) p *= extent(l); return p; };
      auto arrange = [&](int t, const std::string& have, const std::string& want, const std::vector<int64_t>& shape3) {
        std::vector<double> perm;
        bool ident = true;
        for (size_t d = 0; d < want.size(); d++) {
          perm.push_back((double)have.find(want[d]));
          ident = ident && have.find(want[d]) == d;
        }
        if (!ident) t = emit("Transpose", {t}, {{"perm", perm}});
        std::vector<double> shp(shape3.begin(), shape3.end());
        return emit("Reshape", {t}, {{"shape", shp}});
      };
      const int64_t Bt = prod(batch), Mt = prod(M), Nt = prod(N), Kt = prod(K);
      const int a3 = arrange(op.in[0], e.a, batch + M + K, {Bt, Mt, Kt});
      const int b3 = arrange(op.in[1], e.b, batch + K + N, {Bt, Kt, Nt});
      int y = emit("MatMul", {a3, b3});
      const std::string got = batch + M + N;
      std::vector<double> full;
      for (char l : got) full.push_back((double)extent(l));
      y = emit("Reshape", {y}, {{"shape", full}});
      if (got != e.out) {
        std::vector<double> perm;
        for (char l : e.out) perm.push_back((double)got.find(l));
        y = emit("Transpose", {y}, {{"perm", perm}});
      }
      replace_uses(op.out[0], y);
      g.ops[i].alive = false;
      st.log.push_back("canonicalise: Einsum -> Transpose / Reshape / MatMul");
      st.canonicalisations++;
      any = true;
      g.relink();
    }
    return any;
  }

  // Data layout for the dominant operator of a block (Sec. 4.4.2, inter-block optimisation): the
  // MFMA GEMM kernel wants both operands contiguous along K.  A constant [K, N] weight is therefore
  // re-laid out once, at prepare time, as [N, K]: W becomes Transpose(Transpose(W)) where the inner
  // Transpose is materialised (weight-only, runs once) and the outer one is folded into the GEMM's
  // operand index by the planner, so the kernel streams K-contiguous rows of the re-laid-out copy.
  bool canon_weight_layout() {
    bool any = false;
    size_t n = g.ops.size();
    for (size_t i = 0; i < n; i++) {
      if (!g.ops[i].alive || g.ops[i].kind != "MatMul") continue;
      int w = g.ops[i].in[1];
      const Tensor& W = g.tensors[w];
      if (!W.weight_only || W.dims.size() != 2 || !is_float(W.dtype)) continue;
      if (const Op* p = producer(w)) if (p->kind == "Transpose") continue;   // already K-contiguous through an index map
      int64_t K = W.dims[0], N = W.dims[1];
      int vec = dtype_bytes(W.dtype) == 2 ? 8 : 4;
      if (K % vec != 0 || N < 16 || K < 16) continue;
      int t1 = emit("Transpose", {w}, {{"perm", {1.0, 0.0}}, {"materialize", {1.0}}});
      int t2 = emit("Transpose", {t1}, {{"perm", {1.0, 0.0}}});
      g.ops[i].in[1] = t2;
      st.log.push_back("layout: constant MatMul operand re-laid out K-contiguous");
      st.canonicalisations++;
      any = true;
      g.relink();
    }
    return any;
  }

  // ---------------------------------------------------------------- Table 4 rule engine
  // A pattern is a small expression tree over operator kinds with named holes.
  struct Pat {
    std::string kind;            // operator kind, or "" for a hole
    std::string var;             // hole name
    std::vector<Pat> kids;
  };
  static Pat H(const std::string& v) { return Pat{"", v, {}}; }
  static Pat P(const std::string& k, std::vector<Pat> kids) { return Pat{k, "", std::move(kids)}; }

  using Bind = std::map<std::string, int>;

  // textual form of a sub-pattern; two occurrences of the same form inside one rule (the sqrt(B), rsum(B) and
  // A + B of Table 4) denote the same value
  static std::string pat_sig(const Pat& p) {
    if (p.kind.empty()) return "$" + p.var;
    std::string s = p.kind + "(";
    for (auto& k : p.kids) s += pat_sig(k) + ",";
    return s + ")";
  }

  bool match(const Pat& p, int t, Bind& b, std::vector<int>& ops) const {
    if (p.kind.empty()) {
      auto it = b.find(p.var);
      if (it != b.end()) return it->second == t;
      b[p.var] = t;
      return true;
    }
    const Op* op = producer(t);
    if (!op || op->kind != p.kind || op->out.size() != 1 || op->in.size() != p.kids.size()) return false;
    if (g.tensors[t].weight_only) return false;
    // A repeated sub-pattern must be the same value: matching operands is not enough when the operator has
    // attributes (two ReduceSum of one tensor over different axes are different values).
    const std::string sig = "@" + pat_sig(p);
    {
      auto it = b.find(sig);
      if (it != b.end() && it->second != t) {
        const Op* first = producer(it->second);
        if (!first || first->attrs != op->attrs) return false;
      }
    }
    auto attempt = [&](const std::vector<int>& order) {
      Bind b2 = b;
      std::vector<int> ops2 = ops;
      for (size_t k = 0; k < p.kids.size(); k++)
        if (!match(p.kids[k], op->in[order[k]], b2, ops2)) return false;
      b = b2;
      ops = ops2;
      return true;
    };
    bool ok = attempt({0, 1, 2, 3});
    if (!ok && p.kids.size() == 2 && op->info->commut) ok = attempt({1, 0});   // commutative row of Table 4
    if (ok) {
      ops.push_back(g.tensors[t].producer);
      if (!b.count(sig)) b[sig] = t;
    }
    return ok;
  }

  // true when every element of tensor t is known to be >= 0 from the operator that produces it
  bool provably_nonneg(int t, int depth = 0) const {
    const Tensor& T = g.tensors[t];
    if (T.has_cval) {
      for (double v : T.cval) if (!(v >= 0)) return false;
      return !T.cval.empty();
    }
    const Op* p = producer(t);
    if (!p || depth > 8) return false;
    const std::string& k = p->kind;
    if (k == "Square" || k == "Abs" || k == "Exp" || k == "Sigmoid" || k == "Relu" || k == "Softmax" || k == "Sqrt") return true;
    if (k == "Mul" && p->in[0] == p->in[1]) return true;
    if (k == "Add" || k == "Mul" || k == "Max") {
      if (k == "Max") return provably_nonneg(p->in[0], depth + 1) || provably_nonneg(p->in[1], depth + 1);
      return provably_nonneg(p->in[0], depth + 1) && provably_nonneg(p->in[1], depth + 1);
    }
    if (k == "Clip") return p->has("min") && p->f("min", -1) >= 0;
    if (k == "Reshape" || k == "Transpose" || k == "Identity" || k == "Expand" || k == "Slice" || k == "ReduceSum" || k == "ReduceMean" || k == "ReduceMax")
      return provably_nonneg(p->in[0], depth + 1);
    return false;
  }

  struct Rule {
    const char* name;
    const char* property;
    Pat lhs;
    std::function<int(Rewriter&, const Bind&)> build;   // returns the replacement tensor
    bool apply_on_tie;   // Table 4 rows marked with the load-count footnote: no #FLOPS gain, fewer loads
    std::function<bool(const Rewriter&, const Bind&)> guard;
    bool derived = false;   // not printed in Table 4: an instance of a printed row after an identity on one operand
  };

  std::vector<Rule> rules() {
    std::vector<Rule> R;
    auto mul = [](Pat a, Pat b) { return P("Mul", {std::move(a), std::move(b)}); };
    auto add = [](Pat a, Pat b) { return P("Add", {std::move(a), std::move(b)}); };
    auto un = [](const char* k, Pat a) { return P(k, {std::move(a)}); };
    auto same_shape = [](const char* x, const char* y) {
      return [x, y](const Rewriter& r, const Bind& b) { return r.g.tensors[b.at(x)].dims == r.g.tensors[b.at(y)].dims; };
    };
    // ---- Associative
    R.push_back({"recip(A)*recip(A*B) -> square(recip(A))*recip(B)", "associative",
                 mul(un("Reciprocal", H("A")), un("Reciprocal", mul(H("A"), H("B")))),
                 [](Rewriter& r, const Bind& b) {
                   int ra = r.emit("Reciprocal", {b.at("A")});
                   return r.emit("Mul", {r.emit("Square", {ra}), r.emit("Reciprocal", {b.at("B")})});
                 }, true, nullptr});
    R.push_back({"(A*sqrt(B))*(sqrt(B)*C) -> A*B*C", "associative",
                 mul(mul(H("A"), un("Sqrt", H("B"))), mul(un("Sqrt", H("B")), H("C"))),
                 [](Rewriter& r, const Bind& b) { return r.emit("Mul", {r.emit("Mul", {b.at("A"), b.at("B")}), b.at("C")}); },
                 // Table 4 prints no domain; for B < 0 the left side is NaN and the right side is not, so the rule
                 // fires only where B >= 0 follows from the operator that produces B
                 false, [](const Rewriter& r, const Bind& b) { return r.provably_nonneg(b.at("B")); }});
    R.push_back({"abs(A)*B*abs(C) -> abs(A*C)*B", "associative",
                 mul(mul(un("Abs", H("A")), H("B")), un("Abs", H("C"))),
                 [](Rewriter& r, const Bind& b) {
                   return r.emit("Mul", {r.emit("Abs", {r.emit("Mul", {b.at("A"), b.at("C")})}), b.at("B")});
                 }, false, same_shape("A", "C")});
    {
      Pat rs = P("ReduceSum", {H("B")});
      R.push_back({"(A*rsum(B))*(rsum(B)*C) -> A*square(rsum(B))*C", "associative", mul(mul(H("A"), rs), mul(rs, H("C"))),
                   [](Rewriter& r, const Bind& b) {
                     int s = b.at("#rs");
                     return r.emit("Mul", {r.emit("Mul", {b.at("A"), r.emit("Square", {s})}), b.at("C")});
                   }, false, nullptr});
    }
    // ---- Distributive
    R.push_back({"A*C + A*B -> A*(B+C)", "distributive", add(mul(H("A"), H("C")), mul(H("A"), H("B"))),
                 [](Rewriter& r, const Bind& b) { return r.emit("Mul", {b.at("A"), r.emit("Add", {b.at("B"), b.at("C")})}); },
                 false, nullptr});
    R.push_back({"A + A*B -> A*(B+1)", "distributive", add(H("A"), mul(H("A"), H("B"))),
                 [](Rewriter& r, const Bind& b) {
                   int one = r.g.new_const("one", DNNF_F32, {}, {1.0});
                   return r.emit("Mul", {b.at("A"), r.emit("Add", {b.at("B"), one})});
                 }, true, [](const Rewriter& r, const Bind& b) {
                   // the product must have A's shape, otherwise A + (A*B) broadcasts differently
                   return r.g.tensors[b.at("A")].n() >= r.g.tensors[b.at("B")].n();
                 }});
    {
      Pat ab = add(H("A"), H("B"));
      R.push_back({"square(A+B) - (A+B)*C -> (A+B)*(A+B-C)", "distributive",
                   P("Sub", {un("Square", ab), mul(ab, H("C"))}),
                   [](Rewriter& r, const Bind& b) {
                     int s = r.emit("Add", {b.at("A"), b.at("B")});
                     return r.emit("Mul", {s, r.emit("Sub", {s, b.at("C")})});
                   }, false, nullptr});
    }
    // Derived from the row above with A^3 = A * A^2 (the polynomial inside the tanh form of GELU, x + c x^3): the cube
    // becomes a square and A is read once.  A third power by a constant counts as its two multiplications, so the
    // #FLOPS tie of the printed row (and its load-count footnote) carries over.
    R.push_back({"A + K*pow(A,3) -> A*(K*square(A) + 1)", "distributive", add(H("A"), mul(H("K"), P("Pow", {H("A"), H("E")}))),
                 [](Rewriter& r, const Bind& b) {
                   int one = r.g.new_const("one", DNNF_F32, {}, {1.0});
                   int inner = r.emit("Add", {r.emit("Mul", {b.at("K"), r.emit("Square", {b.at("A")})}), one});
                   return r.emit("Mul", {b.at("A"), inner});
                 }, true, [](const Rewriter& r, const Bind& b) {
                   double e;
                   return r.is_scalar_const(b.at("E"), &e) && e == 3.0 && r.g.tensors[b.at("A")].n() >= r.g.tensors[b.at("K")].n();
                 }, true});
    // ---- Commutative (swapping an elementwise operator with a reduction)
    R.push_back({"rsum(bitshift(A)) -> bitshift(rsum(A))", "commutative", P("ReduceSum", {P("BitShift", {H("A"), H("S")})}),
                 [](Rewriter& r, const Bind& b) {
                   const Op* red = r.producer(b.at("#root"));
                   Attrs ra = red->attrs, sa = r.producer(red->in[0])->attrs;   // copies: emit() grows the op list
                   int sum = r.emit("ReduceSum", {b.at("A")}, ra);
                   return r.emit("BitShift", {sum, b.at("S")}, sa);
                 }, false, [](const Rewriter& r, const Bind& b) {
                   // wrap-around left shift distributes over addition; a right shift floors and does not.
                   const Op* red = r.producer(b.at("#root"));
                   const Op* sh = r.producer(red->in[0]);
                   double s;
                   return sh->f("direction_right", 0) == 0 && r.is_scalar_const(b.at("S"), &s);
                 }});
    R.push_back({"rprod(exp(A)) -> exp(rsum(A))", "commutative", P("ReduceProd", {un("Exp", H("A"))}),
                 [](Rewriter& r, const Bind& b) {
                   Attrs ra = r.producer(b.at("#root"))->attrs;
                   int sum = r.emit("ReduceSum", {b.at("A")}, ra);
                   return r.emit("Exp", {sum});
                 }, false, nullptr});
    return R;
  }

  struct Candidate {
    int rule = -1, root = -1;
    Bind bind;
    std::vector<int> ops;
    double gain = 0;
  };

  // #FLOPS of the matched operators that die when `root` is replaced
  double dead_flops(int root, const std::vector<int>& ops) const {
    std::set<int> dead;
    dead.insert(g.tensors[root].producer);
    bool again = true;
    std::set<int> cand(ops.begin(), ops.end());
    while (again) {
      again = false;
      for (int o : cand) {
        if (dead.count(o)) continue;
        bool all_dead = true;
        for (int t : g.ops[o].out) {
          if (g.tensors[t].kind == DNNF_OUTPUT) all_dead = false;
          for (int c : g.tensors[t].consumers) all_dead = all_dead && dead.count(c);
        }
        if (all_dead) { dead.insert(o); again = true; }
      }
    }
    double f = 0;
    for (int o : dead) f += g.ops[o].flops;
    return f;
  }

  std::vector<int> partitions() const {
    // union-find over operators that carry a mathematical property; others are partition points
    std::vector<int> parent(g.ops.size());
    std::iota(parent.begin(), parent.end(), 0);
    std::function<int(int)> find = [&](int x) { return parent[x] == x ? x : parent[x] = find(parent[x]); };
    auto has_prop = [&](const Op& o) { return o.alive && (o.info->assoc || o.info->commut || o.info->distrib); };
    for (size_t i = 0; i < g.ops.size(); i++) {
      if (!has_prop(g.ops[i])) continue;
      for (int t : g.ops[i].in) {
        int p = g.tensors[t].producer;
        if (p >= 0 && has_prop(g.ops[p])) parent[find((int)i)] = find(p);
      }
    }
    std::vector<int> r(g.ops.size());
    for (size_t i = 0; i < g.ops.size(); i++) r[i] = find((int)i);
    return r;
  }

  void run_rules() {
    std::vector<Rule> R = rules();
    for (int iter = 0; iter < 10000; iter++) {
      std::vector<int> part = partitions();
      std::map<int, Candidate> best;   // per partition
      for (size_t t = 0; t < g.tensors.size(); t++) {
        if (!producer((int)t)) continue;
        for (size_t ri = 0; ri < R.size(); ri++) {
          Bind b;
          std::vector<int> ops;
          if (!match(R[ri].lhs, (int)t, b, ops)) continue;
          b["#root"] = (int)t;
          // the shared ReduceSum of the fourth associative rule
          for (int o : ops) if (g.ops[o].kind == "ReduceSum") b["#rs"] = g.ops[o].out[0];
          if (R[ri].guard && !R[ri].guard(*this, b)) continue;
          // cost of the replacement: build it on a scratch copy
          Graph saved = g;
          int nt = R[ri].build(*this, b);
          (void)nt;
          double newf = 0;
          for (size_t o = saved.ops.size(); o < g.ops.size(); o++) newf += op_flops(g, g.ops[o]);
          g = saved;
          double gain = dead_flops((int)t, ops) - newf;
          if (gain < 0 || (gain == 0 && !R[ri].apply_on_tie)) continue;
          int pid = part[g.tensors[t].producer];
          auto it = best.find(pid);
          if (it == best.end() || gain > it->second.gain) best[pid] = Candidate{(int)ri, (int)t, b, ops, gain};
        }
      }
      if (best.empty()) break;
      for (auto& kv : best) {
        Candidate& c = kv.second;
        if (!producer(c.root)) continue;
        int nt = R[c.rule].build(*this, c.bind);
        replace_uses(c.root, nt);
        if (g.tensors[c.root].kind != DNNF_OUTPUT) g.ops[g.tensors[c.root].producer].alive = false;
        st.rules_fired++;
        if (R[c.rule].derived) st.derived_rules_fired++;
        st.log.push_back(std::string("rule (") + R[c.rule].property + (R[c.rule].derived ? ", derived): " : "): ") + R[c.rule].name);
        dce();
      }
    }
  }
};

}  // namespace

void rewrite_graph(Graph& g, RewriteStats& st) {
  st.ops_before = g.live_ops();
  st.flops_before = g.total_flops();
  Rewriter rw(g, st);
  rw.canon_einsum();
  rw.canon_batchnorm();
  rw.canon_casts();
  rw.canon_transposes();
  rw.canon_fold_scalars();
  rw.canon_strength();
  rw.dce();
  rw.canon_softmax();
  rw.canon_normalize();
  rw.dce();
  rw.canon_weight_layout();
  rw.run_rules();
  rw.dce();
  g.finalized = true;
  st.ops_after = g.live_ops();
  st.flops_after = g.total_flops();
}

}  // namespace dnnf
