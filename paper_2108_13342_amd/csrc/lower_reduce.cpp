// Row-reduction kernels: a block anchored on Softmax, Normalize (LayerNorm statistics),
// Reduce{Sum,Mean,Max,Prod} over trailing axes or GlobalAveragePool, with the block's One-to-One
// operators applied to the elements as they are loaded (prologue) and to the results before they
// are stored (epilogue).  One 64-lane wavefront owns one row: partial results are combined with
// cross-lane shuffles only, nothing goes through LDS, and a row is read from HBM exactly once
// (values stay in registers between the passes of softmax / normalisation).
#include <algorithm>

#include "lower_ctx.hpp"

namespace dnnf {

namespace {
void decl_digits(std::ostringstream& os, const LowerCtx& c, const std::vector<int>& atoms_major_minor,
                 const std::string& counter, const std::string& ind, const std::string& tag) {
  std::string rem = counter;
  for (int k = (int)atoms_major_minor.size() - 1; k >= 0; k--) {
    int a = atoms_major_minor[k];
    int64_t e = c.atom_extent[a];
    if (k == 0) os << ind << "const idx_t a" << a << " = " << rem << ";\n";
    else {
      os << ind << "const idx_t a" << a << " = " << rem << " % " << e << ";\n";
      os << ind << "const idx_t " << tag << a << " = " << rem << " / " << e << ";\n";
      rem = tag + std::to_string(a);
    }
  }
}
}  // namespace

Lowered lower_reduce(LowerCtx& c) {
  const Graph& g = c.g;
  const Op& A = g.ops[c.anchor_op];
  const Tensor& X = g.tensors[A.in[0]];
  const Tensor& Y = g.tensors[A.out[0]];
  size_t rank = X.dims.size();
  // which trailing axes are reduced
  size_t first_red = rank;
  bool per_element = false;   // output has the input's shape (softmax, normalize)
  std::string mode;
  switch (A.info->cls) {
    case OC_SOFTMAX: {
      int64_t ax = A.i("axis", -1);
      DNNF_CHECK(ax == -1 || ax == (int64_t)rank - 1, DNNF_UNSUPPORTED_OP, "Softmax over an axis other than the last");
      first_red = rank - 1;
      per_element = true;
      mode = "softmax";
      break;
    }
    case OC_NORMALIZE:
      first_red = rank - 1;
      per_element = true;
      mode = "normalize";
      break;
    case OC_GAP:
      first_red = 2;
      mode = "mean";
      break;
    default: {
      auto axes = A.ints("axes");
      std::set<int> ax;
      for (auto a : axes) ax.insert((int)(a < 0 ? a + (int64_t)rank : a));
      DNNF_CHECK(!ax.empty(), DNNF_UNSUPPORTED_OP, "reduction over all axes");
      first_red = (size_t)*ax.begin();
      for (size_t d = first_red; d < rank; d++)
        DNNF_CHECK(ax.count((int)d) || X.dims[d] == 1, DNNF_UNSUPPORTED_OP, "reduction axes must be the trailing axes");
      mode = A.kind == "ReduceSum" ? "sum" : A.kind == "ReduceMean" ? "mean" : A.kind == "ReduceMax" ? "max" : "prod";
    }
  }
  int64_t L = 1, rows = 1;
  for (size_t d = 0; d < rank; d++) (d < first_red ? rows : L) *= X.dims[d];
  DNNF_CHECK(L >= 1 && rows >= 1, DNNF_UNSUPPORTED_OP, "empty reduction");

  // iteration atoms = the anchor input's index space
  TIdx xi = c.fresh_index(X.dims);
  TIdx yi;
  if (per_element) yi = xi;
  else {
    bool keep = Y.dims.size() == rank;
    for (size_t d = 0; d < rank; d++) {
      if (d < first_red) yi.push_back(xi[d]);
      else if (keep) yi.push_back(DimIdx());
    }
    DNNF_CHECK(yi.size() == Y.dims.size(), DNNF_UNSUPPORTED_OP, "reduction output rank");
  }
  c.tidx[c.anchor_out] = yi;
  std::vector<int> ein, eout, removed;
  block_io(g, c.blk, ein, eout, removed);
  c.forward_all();
  // every block output must sit after the anchor
  for (int t : eout)
    DNNF_CHECK(c.tidx.count(t), DNNF_UNSUPPORTED_OP, "block output " + g.tensors[t].name + " does not follow the reduction");
  c.collect_stores(eout);
  int xin = c.value(A.in[0], xi);   // prologue

  std::vector<int> row_atoms, col_atoms;
  for (size_t d = 0; d < rank; d++) {
    std::vector<int> r;
    c.resolve(xi[d].atoms, r);
    auto& dst = d < first_red ? row_atoms : col_atoms;
    dst.insert(dst.end(), r.begin(), r.end());
  }

  // parameters
  std::vector<int> params;
  std::map<int, int> pslot;
  std::set<int> written;
  {
    std::set<int> need;
    std::vector<int> stack = {xin};
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
  size_t n_in = params.size();
  for (auto& s : c.stores) {
    DNNF_CHECK(!pslot.count(s.tensor), DNNF_UNSUPPORTED_OP, "block reads and writes the same tensor");
    pslot[s.tensor] = (int)params.size();
    params.push_back(s.tensor);
    written.insert(s.tensor);
  }

  const int W = 64;
  int64_t npl = (L + W - 1) / W;        // elements per lane
  bool cached = per_element && npl <= 32;
  bool unrolled = npl <= 32;
  const bool wide = [&] {
    for (int t : params) if (g.tensors[t].n() >= (int64_t)1 << 31) return true;
    return false;
  }();

  std::ostringstream k;
  k << "typedef " << (wide ? "long long" : "int") << " idx_t;\n";
  k << "extern \"C\" __global__ __launch_bounds__(256) void KNAME(" << c.param_list(params, written) << ") {\n";
  k << "  const int lane = threadIdx.x & 63;\n";
  k << "  const idx_t row = (idx_t)blockIdx.x * 4 + (threadIdx.x >> 6);\n";
  k << "  if (row >= (idx_t)" << rows << ") return;\n";
  decl_digits(k, c, row_atoms, "row", "  ", "qr");
  const char* ident = mode == "max" || mode == "softmax" ? "-__builtin_inff()" : mode == "prod" ? "1.0f" : "0.0f";
  auto combine = [&](const std::string& acc, const std::string& v) {
    if (mode == "max" || mode == "softmax") return acc + " = fmaxf(" + acc + ", " + v + ");";
    if (mode == "prod") return acc + " *= " + v + ";";
    return acc + " += " + v + ";";
  };
  // declares the column atoms for `col`, then evaluates the prologue into a fresh variable `dst`
  auto load_elem = [&](const std::string& ind, const std::string& dst) {
    decl_digits(k, c, col_atoms, "col", ind, "qc");
    k << ind << "float " << dst << ";\n" << ind << "{\n";
    std::set<int> done;
    c.emit_values(k, {xin}, done, pslot, ind + "  ");
    k << ind << "  " << dst << " = " << c.vname(xin) << ";\n" << ind << "}\n";
  };
  auto loop_open = [&](const std::string& jvar) {
    if (unrolled) k << "#pragma unroll\n  for (int " << jvar << " = 0; " << jvar << " < " << npl << "; ++" << jvar << ") {\n";
    else k << "  for (int " << jvar << " = 0; " << jvar << " < " << npl << "; ++" << jvar << ") {\n";
    k << "    const idx_t col = (idx_t)" << jvar << " * 64 + lane;\n";
  };
  if (cached) k << "  float xs[" << npl << "];\n";
  k << "  float acc = " << ident << ";\n";
  // ---- pass 1
  loop_open("j");
  k << "    if (col < " << L << ") {\n";
  load_elem("      ", "x0");
  if (cached) k << "      xs[j] = x0;\n";
  k << "      " << combine("acc", "x0") << "\n";
  k << "    }" << (cached ? std::string(" else xs[j] = ") + ident + ";" : "") << "\n  }\n";
  if (mode == "max" || mode == "softmax") k << "  acc = dn_wave_max(acc);\n";
  else if (mode == "prod") k << "#pragma unroll\n  for (int o = 32; o > 0; o >>= 1) acc *= __shfl_xor(acc, o, 64);\n";
  else k << "  acc = dn_wave_sum(acc);\n";

  auto elem_value = [&](const std::string& ind, const std::string& dst) {
    // value of the (prologue-transformed) input element in this pass
    if (cached) k << ind << "const float " << dst << " = xs[j];\n";
    else load_elem(ind, dst);
  };
  auto emit_stores = [&](const std::string& ind) {
    std::set<int> done;
    std::vector<int> roots;
    for (auto& s : c.stores) roots.push_back(s.value);
    c.emit_values(k, roots, done, pslot, ind);
    for (auto& s : c.stores) {
      std::string st = c.store_stmt(s, pslot, c.addr_expr(s.addr));
      if (s.preds.empty()) k << ind << st << "\n";
      else k << ind << "if (" << c.pred_expr(s.preds) << ") { " << st << " }\n";
    }
  };

  if (mode == "softmax") {
    k << "  const float row_max = acc;\n  float den = 0.0f;\n";
    loop_open("j");
    k << "    if (col < " << L << ") {\n";
    elem_value("      ", "xe");
    if (cached) k << "      xs[j] = expf(xe - row_max);\n      den += xs[j];\n";
    else k << "      den += expf(xe - row_max);\n";
    k << "    }\n  }\n  den = dn_wave_sum(den);\n  const float inv_den = dn_div(1.0f, den);\n";
    loop_open("j");
    k << "    if (col < " << L << ") {\n";
    if (cached) {
      decl_digits(k, c, col_atoms, "col", "      ", "qc");
      k << "      const float anchor_v = xs[j] * inv_den;\n";
    } else {
      elem_value("      ", "xe");
      k << "      const float anchor_v = expf(xe - row_max) * inv_den;\n";
    }
    emit_stores("      ");
    k << "    }\n  }\n";
  } else if (mode == "normalize") {
    k << "  const float mean = acc * " << "(1.0f / " << L << ".0f);\n  float sq = 0.0f;\n";
    loop_open("j");
    k << "    if (col < " << L << ") {\n";
    elem_value("      ", "xe");
    k << "      const float dlt = xe - mean;\n      sq += dlt * dlt;\n";
    k << "    }\n  }\n  sq = dn_wave_sum(sq);\n";
    k << "  const float rstd = dn_div(1.0f, sqrtf(sq * (1.0f / " << L << ".0f) + " << (float)A.f("epsilon", 1e-5) << "f));\n";
    loop_open("j");
    k << "    if (col < " << L << ") {\n";
    if (cached) decl_digits(k, c, col_atoms, "col", "      ", "qc");
    elem_value("      ", "xe");
    k << "      const float anchor_v = (xe - mean) * rstd;\n";
    emit_stores("      ");
    k << "    }\n  }\n";
  } else {
    if (mode == "mean") k << "  const float anchor_v = acc * (1.0f / " << L << ".0f);\n";
    else k << "  const float anchor_v = acc;\n";
    k << "  if (lane == 0) {\n";
    emit_stores("    ");
    k << "  }\n";
  }
  k << "}\n";

  Lowered Lw;
  Lw.family = FAM_REDUCE;
  Lw.ext_in.assign(params.begin(), params.begin() + n_in);
  Lw.ext_out.assign(params.begin() + n_in, params.end());
  Launch K;
  K.params = params;
  K.grid[0] = (unsigned)((rows + 3) / 4);
  K.block[0] = 256;
  std::string src = std::string(device_preamble()) + k.str();
  K.name = fnv_name("dnnf_red", src);
  size_t pos;
  while ((pos = src.find("KNAME")) != std::string::npos) src.replace(pos, 5, K.name);
  K.source = src;
  Lw.launches.push_back(K);
  Lw.variant = mode + (cached ? "_regs" : unrolled ? "_stream" : "_loop");
  return Lw;
}

}  // namespace dnnf
