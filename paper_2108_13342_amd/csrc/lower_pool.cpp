// Window pooling blocks: MaxPool / AveragePool (Many-to-Many in Table 2) as the block's anchor, the block's
// One-to-One operators applied to the elements as they are read (prologue) and to the pooled value before it
// is stored (epilogue).
//
// Direct kernel, no staging: a window is a handful of elements and neighbouring outputs share most of
// them, so the caches serve the overlap and HBM sees every input element once.  Lanes run along the
// fastest-varying output axis of the block's first result - the pixel row in the declared NCHW order, the
// channels for a channels-last tensor - so loads and stores coalesce in either data format; when that axis
// is the channel axis and operand and results are contiguous along it, a lane takes 8 (4) channels and
// moves them as 16-byte vectors.
#include <algorithm>

#include "lower_ctx.hpp"

namespace dnnf {

namespace {
int64_t stride_at(const Affine& a, int atom) {
  auto it = a.stride.find(atom);
  return it == a.stride.end() ? 0 : it->second;
}
}  // namespace

Lowered lower_pool(LowerCtx& c) {
  const Graph& g = c.g;
  const Op& A = g.ops[c.anchor_op];
  const Tensor& X = g.tensors[A.in[0]];
  const Tensor& Y = g.tensors[A.out[0]];
  DNNF_CHECK(is_float(X.dtype), DNNF_UNSUPPORTED_OP, "pooling over a non-float tensor");
  const bool is_max = A.kind == "MaxPool";
  auto ks = A.ints("kernel_shape");
  auto st = A.ints("strides");
  if (st.empty()) st = {1, 1};
  auto pd = A.ints("pads");
  if (pd.empty()) pd = {0, 0, 0, 0};
  const int64_t H = X.dims[2], Wd = X.dims[3], KH = ks[0], KW = ks[1], SH = st[0], SW = st[1], PT = pd[0], PL = pd[1];
  const bool include_pad = A.i("count_include_pad", 0) != 0;
  DNNF_CHECK(KH * KW <= 64, DNNF_UNSUPPORTED_OP, "pooling window larger than 64 elements");

  TIdx oi = c.fresh_index(Y.dims);
  c.tidx[c.anchor_out] = oi;
  std::vector<int> ein, eout, removed;
  block_io(g, c.blk, ein, eout, removed);
  c.forward_all();
  for (int t : eout)
    DNNF_CHECK(c.tidx.count(t), DNNF_UNSUPPORTED_OP, "block output " + g.tensors[t].name + " does not follow the pooling");
  c.collect_stores(eout);

  // the pooled tensor as a function of four index atoms whose values the kernel computes
  const int xn = c.new_atom(std::max<int64_t>(X.dims[0], 2)), xc = c.new_atom(std::max<int64_t>(X.dims[1], 2)),
            xh = c.new_atom(std::max<int64_t>(H, 2)), xw = c.new_atom(std::max<int64_t>(Wd, 2));
  TIdx xi(4);
  xi[0].atoms = {xn};
  xi[1].atoms = {xc};
  xi[2].atoms = {xh};
  xi[3].atoms = {xw};
  const int xnode = c.value(A.in[0], xi);

  std::vector<int> out_atoms[4];
  for (int d = 0; d < 4; d++) c.resolve(oi[d].atoms, out_atoms[d]);
  auto digit = [&](int d) {
    std::string e;
    int64_t mult = 1;
    for (int i = (int)out_atoms[d].size() - 1; i >= 0; i--) {
      e = "a" + std::to_string(out_atoms[d][i]) + (mult == 1 ? "" : " * " + std::to_string(mult)) + (e.empty() ? "" : " + " + e);
      mult *= c.atom_extent[out_atoms[d][i]];
    }
    return e.empty() ? std::string("0") : e;
  };

  // parameters: tensors the prologue / epilogue load, then the outputs
  std::vector<int> params;
  std::map<int, int> pslot;
  std::set<int> written, need;
  {
    std::vector<int> stack = {xnode};
    for (auto& s : c.stores) stack.push_back(s.value);
    while (!stack.empty()) {
      int n = stack.back();
      stack.pop_back();
      if (need.count(n)) continue;
      need.insert(n);
      for (int a : c.nodes[n].args) stack.push_back(a);
      if (c.nodes[n].kind == ENode::LOAD) for (auto& p : c.nodes[n].addr.indirect) stack.push_back(p.first);
    }
    for (int n : need)
      if (c.nodes[n].kind == ENode::LOAD && !pslot.count(c.nodes[n].tensor)) {
        pslot[c.nodes[n].tensor] = (int)params.size();
        params.push_back(c.nodes[n].tensor);
      }
  }
  const size_t n_in = params.size();
  for (auto& s : c.stores) {
    DNNF_CHECK(!pslot.count(s.tensor), DNNF_UNSUPPORTED_OP, "block reads and writes the same tensor");
    pslot[s.tensor] = (int)params.size();
    params.push_back(s.tensor);
    written.insert(s.tensor);
  }
  const bool wide = [&] {
    for (int t : params) if (g.tensors[t].n() >= (int64_t)1 << 31) return true;
    return false;
  }();

  // lanes follow the first result's storage order
  const Affine raddr = c.resolved(c.stores[0].addr);
  std::vector<int> order;
  for (int d = 0; d < 4; d++) order.insert(order.end(), out_atoms[d].begin(), out_atoms[d].end());
  std::sort(order.begin(), order.end(), [&](int x, int y) {
    int64_t sx = stride_at(raddr, x), sy = stride_at(raddr, y);
    return sx != sy ? sx > sy : x < y;
  });
  const int64_t total = numel(Y.dims);

  // channel vectors: the fastest axis is the (unsplit) channel axis and the operand is a stored tensor
  // contiguous along it
  int V = 1;
  const int ca = out_atoms[1].size() == 1 ? out_atoms[1][0] : -1;
  Affine xaddr;
  const std::vector<int> xatoms = {xn, xc, xh, xw};
  const bool x_cut = c.is_split(xn) || c.is_split(xc) || c.is_split(xh) || c.is_split(xw);   // by an index map in front
  if (!x_cut && ca >= 0 && !order.empty() && order.back() == ca && c.nodes[xnode].kind == ENode::LOAD && !c.nodes[xnode].is_int &&
      c.nodes[xnode].addr.indirect.empty() && c.opts.force_variant != 2) {
    xaddr = c.resolved(c.nodes[xnode].addr);
    const int v = 16 / dtype_bytes(g.tensors[c.nodes[xnode].tensor].dtype);
    bool ok = stride_at(xaddr, xc) == 1 && X.dims[1] % v == 0 && xaddr.offset % v == 0;
    for (auto& kv : xaddr.stride) if (kv.first != xc && kv.second % v) ok = false;
    for (auto& s : c.stores) {
      Affine sa = c.resolved(s.addr);
      ok = ok && stride_at(sa, ca) == 1 && sa.offset % v == 0 && sa.indirect.empty() && 16 / dtype_bytes(g.tensors[s.tensor].dtype) >= v;
      for (auto& kv : sa.stride) if (kv.first != ca && kv.second % v) ok = false;
      for (auto& pr : s.preds) {
        std::vector<int> r;
        c.resolve(pr.atoms, r);
        if (std::find(r.begin(), r.end(), ca) != r.end()) ok = false;
      }
    }
    if (ok) V = v;
  }

  std::ostringstream k;
  k << "typedef " << (wide ? "long long" : "int") << " idx_t;\n";
  k << "extern \"C\" __global__ __launch_bounds__(256) void KNAME(" << c.param_list(params, written) << ") {\n";
  k << "  const idx_t gid = (idx_t)blockIdx.x * 256 + threadIdx.x;\n  if (gid >= (idx_t)" << total / V << ") return;\n";
  {
    // mixed-radix digits of the lane's index, minor atom first (the channel atom counts vectors)
    std::string rem = "gid";
    k << "  idx_t rem = gid;\n";
    for (int i = (int)order.size() - 1; i >= 0; i--) {
      const int a = order[i];
      const int64_t e = (a == ca && V > 1) ? c.atom_extent[a] / V : c.atom_extent[a];
      k << "  const idx_t a" << a << (a == ca && V > 1 ? "_0" : "") << " = (rem % " << e << ")" << (a == ca && V > 1 ? " * " + std::to_string(V) : "")
        << "; rem /= " << e << ";\n";
    }
  }
  const char* ident = is_max ? "-__builtin_inff()" : "0.0f";
  if (V > 1) {
    const Tensor& XT = g.tensors[c.nodes[xnode].tensor];
    const std::string px = "p" + std::to_string(pslot.at(c.nodes[xnode].tensor));
    k << "  const idx_t a" << ca << " = a" << ca << "_0;\n";
    k << "  const idx_t a" << xn << " = " << digit(0) << ", a" << xc << " = a" << ca << "_0;\n";
    k << "  const idx_t oh = " << digit(2) << ", ow = " << digit(3) << ";\n";
    k << "  typedef " << c.ctype(XT.dtype) << " xvec_t __attribute__((ext_vector_type(" << V << ")));\n";
    k << "  float acc[" << V << "];\n#pragma unroll\n  for (int e = 0; e < " << V << "; ++e) acc[e] = " << ident << ";\n  int cnt = 0;\n";
    // window positions outside the map: the address is clamped into it and the element ignored afterwards, so no
    // load waits behind a branch
    k << "#pragma unroll\n  for (int i = 0; i < " << KH << "; ++i) {\n    const int h_ = (int)oh * " << SH << " + i - " << PT << ";\n";
    k << "    const idx_t a" << xh << " = min(max(h_, 0), " << H - 1 << ");\n";
    k << "#pragma unroll\n    for (int j = 0; j < " << KW << "; ++j) {\n      const int w_ = (int)ow * " << SW << " + j - " << PL << ";\n";
    k << "      const idx_t a" << xw << " = min(max(w_, 0), " << Wd - 1 << ");\n";
    k << "      const bool in_ = h_ >= 0 && h_ < " << H << " && w_ >= 0 && w_ < " << Wd << ";\n      {\n";
    k << "        const xvec_t xv = *(const xvec_t*)(" << px << " + (" << c.addr_expr(xaddr) << "));\n";
    k << "#pragma unroll\n        for (int e = 0; e < " << V << "; ++e) acc[e] = in_ ? " << (is_max ? "fmaxf(acc[e], cvt_in(xv[e]))" : "acc[e] + cvt_in(xv[e])") << " : acc[e];\n";
    k << "        cnt += in_ ? 1 : 0;\n      }\n    }\n  }\n";
    if (!is_max) k << "  const float inv = 1.0f / (float)" << (include_pad ? std::to_string(KH * KW) : std::string("cnt")) << ";\n";
    // epilogue per channel; contiguous operands and the results move as vectors
    std::map<int, std::string> ov;
    for (int n : need) {
      const ENode& e = c.nodes[n];
      if (e.kind != ENode::LOAD || e.is_int || n == xnode || !e.addr.indirect.empty()) continue;
      Affine la = c.resolved(e.addr);
      bool vec = stride_at(la, ca) == 1 && la.offset % V == 0 && 16 / dtype_bytes(g.tensors[e.tensor].dtype) >= V;
      for (auto& kv : la.stride) if (kv.first != ca && kv.second % V) vec = false;
      if (!vec) continue;
      k << "  typedef " << c.ctype(g.tensors[e.tensor].dtype) << " lv" << n << "_t __attribute__((ext_vector_type(" << V << ")));\n";
      k << "  const lv" << n << "_t lv" << n << " = *(const lv" << n << "_t*)(p" << pslot.at(e.tensor) << " + (" << c.addr_expr(e.addr) << "));\n";
      ov[n] = "cvt_in(lv" + std::to_string(n) + "[e])";
    }
    for (size_t i = 0; i < c.stores.size(); i++)
      k << "  typedef " << c.ctype(g.tensors[c.stores[i].tensor].dtype) << " sv" << i << "_t __attribute__((ext_vector_type(" << V << ")));\n  sv" << i
        << "_t sv" << i << ";\n";
    k << "  {\n#pragma unroll\n  for (int e = 0; e < " << V << "; ++e) {\n    const idx_t a" << ca << " = a" << ca << "_0 + e;\n";
    k << "    const float anchor_v = " << (is_max ? "acc[e]" : "acc[e] * inv") << ";\n";
    {
      std::set<int> done;
      std::vector<int> roots;
      for (auto& s : c.stores) roots.push_back(s.value);
      c.emit_values(k, roots, done, pslot, "    ", &ov);
      for (size_t i = 0; i < c.stores.size(); i++)
        k << "    { " << c.ctype(g.tensors[c.stores[i].tensor].dtype) << " tmp; cvt_out(&tmp, " << c.vname(c.stores[i].value) << "); sv" << i << "[e] = tmp; }\n";
    }
    k << "  }\n  }\n";
    for (size_t i = 0; i < c.stores.size(); i++) {
      const Store& s = c.stores[i];
      std::string stt = "*(sv" + std::to_string(i) + "_t*)(p" + std::to_string(pslot.at(s.tensor)) + " + (" + c.addr_expr(s.addr) + ")) = sv" + std::to_string(i) + ";";
      if (s.preds.empty()) k << "  " << stt << "\n";
      else k << "  if (" << c.pred_expr(s.preds) << ") { " << stt << " }\n";
    }
  } else {
    k << "  const idx_t a" << xn << " = " << digit(0) << ", a" << xc << " = " << digit(1) << ";\n";
    k << "  const idx_t oh = " << digit(2) << ", ow = " << digit(3) << ";\n";
    k << "  float acc = " << ident << ";\n  int cnt = 0;\n";
    k << "#pragma unroll\n  for (int i = 0; i < " << KH << "; ++i) {\n    const int h_ = (int)oh * " << SH << " + i - " << PT << ";\n";
    k << "    const idx_t a" << xh << " = min(max(h_, 0), " << H - 1 << ");\n";
    k << "#pragma unroll\n    for (int j = 0; j < " << KW << "; ++j) {\n      const int w_ = (int)ow * " << SW << " + j - " << PL << ";\n";
    k << "      const idx_t a" << xw << " = min(max(w_, 0), " << Wd - 1 << ");\n";
    k << "      const bool in_ = h_ >= 0 && h_ < " << H << " && w_ >= 0 && w_ < " << Wd << ";\n      {\n";
    k << c.decl_parts(xatoms, "        ");
    {
      std::set<int> done;
      c.emit_values(k, {xnode}, done, pslot, "        ");
    }
    k << "        acc = in_ ? " << (is_max ? "fmaxf(acc, " + c.vname(xnode) + ")" : "acc + " + c.vname(xnode)) << " : acc;\n        cnt += in_ ? 1 : 0;\n      }\n    }\n  }\n";
    if (is_max) k << "  const float anchor_v = acc;\n";
    else k << "  const float anchor_v = acc / (float)" << (include_pad ? std::to_string(KH * KW) : std::string("cnt")) << ";\n";
    std::set<int> done;
    std::vector<int> roots;
    for (auto& s : c.stores) roots.push_back(s.value);
    c.emit_values(k, roots, done, pslot, "  ");
    for (auto& s : c.stores) {
      std::string stt = c.store_stmt(s, pslot, c.addr_expr(s.addr));
      if (s.preds.empty()) k << "  " << stt << "\n";
      else k << "  if (" << c.pred_expr(s.preds) << ") { " << stt << " }\n";
    }
  }
  k << "}\n";

  Lowered Lw;
  Lw.family = FAM_DWCONV;     // a direct stencil, like the depthwise convolution
  Lw.ext_in.assign(params.begin(), params.begin() + n_in);
  Lw.ext_out.assign(params.begin() + n_in, params.end());
  Launch Kn;
  Kn.params = params;
  Kn.grid[0] = (unsigned)((total / V + 255) / 256);
  Kn.block[0] = 256;
  std::string src = std::string(device_preamble()) + k.str();
  Kn.name = fnv_name("dnnf_pool", src);
  size_t pos;
  while ((pos = src.find("KNAME")) != std::string::npos) src.replace(pos, 5, Kn.name);
  Kn.source = src;
  Lw.launches.push_back(Kn);
  Lw.variant = std::string(is_max ? "max" : "avg") + "pool" + (V > 1 ? "_chan" + std::to_string(V) : "_direct") + "_" + std::to_string(KH) + "x" + std::to_string(KW) +
               "s" + std::to_string(SH);
  return Lw;
}

}  // namespace dnnf
