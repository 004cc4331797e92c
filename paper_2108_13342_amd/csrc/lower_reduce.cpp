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
      // the LayerNorm statistics chain normalises the last axis; InstanceNormalization every axis behind the
      // channel axis, followed by its own per-channel scale and bias
      first_red = A.kind == "InstanceNormalization" ? 2 : rank - 1;
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
  int in_scale = -1, in_bias = -1;  // InstanceNormalization's per-channel operands
  if (A.kind == "InstanceNormalization") {
    DNNF_CHECK(rank >= 3, DNNF_UNSUPPORTED_OP, "InstanceNormalization needs rank >= 3");
    auto chan_value = [&](int t) {
      const Tensor& P = g.tensors[t];
      TIdx pi(P.dims.size());
      for (size_t d = 0; d < P.dims.size(); d++) if (P.dims[d] == X.dims[1]) { pi[d] = xi[1]; break; }
      return c.value(t, pi);
    };
    in_scale = chan_value(A.in[1]);
    in_bias = chan_value(A.in[2]);
  }

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
    if (in_scale >= 0) { stack.push_back(in_scale); stack.push_back(in_bias); }
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

  // Reductions over integer tensors (the ReduceSum of Table 4's BitShift rule): 64-bit accumulation, exact, wrapping
  // like the operator's integer arithmetic; every value of the block then travels as an integer.
  const bool ints = !is_float(X.dtype);
  DNNF_CHECK(!ints || mode == "sum" || mode == "max" || mode == "prod", DNNF_UNSUPPORTED_OP, "only sums, products and maxima of integer tensors are exact");
  const char* acc_t = ints ? "long long" : "float";
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
  unsigned grid0 = (unsigned)((rows + 3) / 4);
  std::string variant;

  // Channels-last operand (the fastest axis of the input is the last kept axis, e.g. GlobalAveragePool
  // over [n, h, w, c]): lanes run along the channels, V of them per lane as one 16-byte vector, and the
  // reduced positions are dealt to the remaining lanes of the workgroup; partial results meet through
  // cross-lane shuffles and one LDS exchange between the four wavefronts.
  int chanV = 0;
  Affine xaddr;
  if (!ints && !per_element && mode != "prod" && !row_atoms.empty() && c.nodes[xin].kind == ENode::LOAD && !c.nodes[xin].is_int &&
      c.nodes[xin].addr.indirect.empty() && c.opts.force_variant != 2) {
    xaddr = c.resolved(c.nodes[xin].addr);
    const int ch = row_atoms.back();
    const int v = 16 / dtype_bytes(g.tensors[c.nodes[xin].tensor].dtype);
    auto it = xaddr.stride.find(ch);
    bool ok = it != xaddr.stride.end() && it->second == 1 && c.atom_extent[ch] % v == 0 && xaddr.offset % v == 0 && L > 1;
    for (auto& kv : xaddr.stride) if (kv.first != ch && kv.second % v) ok = false;
    if (ok) chanV = v;
  }
  std::string stage2;          // source of a second kernel (two-stage variant)
  unsigned grid2 = 0;
  int64_t scratch_bytes = 0;
  if (chanV) {
    const int V = chanV, ch = row_atoms.back();
    const int64_t CH = c.atom_extent[ch], CV = CH / V, orows = rows / CH;
    int XW = 64;
    while (XW > 1 && (XW / 2 >= CV || orows * ((CV + XW - 1) / XW) < 512)) XW /= 2;
    // A large map over few channels leaves that choice with narrow channel lanes (short contiguous pieces) and a
    // long serial walk per lane.  Then the reduced positions are split between S workgroups as well, each adding
    // its part for all channel lanes of a pixel at full contiguity; the S partial sums go through the block's
    // scratch area and a second, tiny kernel adds them and runs the block's epilogue.
    int S = 1;
    {
      int xw_full = 64;
      while (xw_full / 2 >= CV) xw_full /= 2;
      const int64_t base = orows * ((CV + xw_full - 1) / xw_full);
      if (xw_full > XW && L >= 512 && c.opts.force_variant != 3) {
        XW = xw_full;
        S = (int)std::min<int64_t>((1024 + base - 1) / base, std::max<int64_t>(1, L / ((256 / XW) * 4)));
        if (S < 2) S = 1;
      }
    }
    const int YH = 256 / XW;
    const int64_t NCH = (CV + XW - 1) / XW;
    const int64_t LS = (L + S - 1) / S;
    std::vector<int> outer_rows(row_atoms.begin(), row_atoms.end() - 1);
    const Tensor& XT = g.tensors[c.nodes[xin].tensor];
    const std::string px = "p" + std::to_string(pslot.at(c.nodes[xin].tensor));
    const bool is_max = mode == "max";
    k << "extern \"C\" __global__ __launch_bounds__(256) void KNAME(" << c.param_list(params, written) << (S > 1 ? ", float* __restrict__ scratch" : "") << ") {\n";
    k << "  __shared__ float part[4][" << XW << "][" << V << "];\n";
    k << "  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, x = tid % " << XW << ", y = tid / " << XW << ";\n";
    if (S > 1) k << "  const idx_t part_s = (idx_t)blockIdx.x % " << S << ", bq = (idx_t)blockIdx.x / " << S << ";\n";
    else k << "  const idx_t bq = blockIdx.x;\n";
    k << "  const idx_t chunk = bq % " << NCH << ", orow = bq / " << NCH << ";\n";
    decl_digits(k, c, outer_rows, "orow", "  ", "qr");
    k << "  const idx_t cv = chunk * " << XW << " + x;\n";
    k << "  typedef " << c.ctype(XT.dtype) << " xvec_t __attribute__((ext_vector_type(" << V << ")));\n";
    k << "  float acc[" << V << "];\n#pragma unroll\n  for (int e = 0; e < " << V << "; ++e) acc[e] = " << (is_max ? "-__builtin_inff()" : "0.0f") << ";\n";
    k << "  if (cv < " << CV << ") {\n    const idx_t a" << ch << " = cv * " << V << ";\n";
    if (S > 1) k << "    const idx_t col_end = (part_s + 1) * " << LS << " < " << L << " ? (part_s + 1) * " << LS << " : " << L << ";\n";
    k << "#pragma unroll 4\n    for (idx_t col = " << (S > 1 ? "part_s * " + std::to_string(LS) + " + y" : std::string("y")) << "; col < "
      << (S > 1 ? std::string("col_end") : std::to_string(L)) << "; col += " << YH << ") {\n";
    decl_digits(k, c, col_atoms, "col", "      ", "qc");
    k << "      const xvec_t xv = *(const xvec_t*)(" << px << " + (" << c.addr_expr(xaddr) << "));\n";
    k << "#pragma unroll\n      for (int e = 0; e < " << V << "; ++e) acc[e] = "
      << (is_max ? "fmaxf(acc[e], cvt_in(xv[e]))" : "acc[e] + cvt_in(xv[e])") << ";\n    }\n  }\n";
    k << "#pragma unroll\n  for (int o = 32; o >= " << XW << "; o >>= 1)\n#pragma unroll\n    for (int e = 0; e < " << V << "; ++e) acc[e] = "
      << (is_max ? "fmaxf(acc[e], __shfl_xor(acc[e], o, 64))" : "acc[e] + __shfl_xor(acc[e], o, 64)") << ";\n";
    k << "  if (lane < " << XW << ") {\n#pragma unroll\n    for (int e = 0; e < " << V << "; ++e) part[wave][lane][e] = acc[e];\n  }\n";
    k << "  __syncthreads();\n";
    k << "  if (tid < " << XW * V << ") {\n    const int x2 = tid / " << V << ", e2 = tid % " << V << ";\n";
    k << "    const idx_t cv2 = chunk * " << XW << " + x2;\n    if (cv2 < " << CV << ") {\n";
    if (XW == 64) {
      k << "      float r = part[0][x2][e2];\n#pragma unroll\n      for (int w = 1; w < 4; ++w) r = " << (is_max ? "fmaxf(r, part[w][x2][e2])" : "r + part[w][x2][e2]") << ";\n";
    } else {
      // with fewer than 64 channel lanes every wavefront holds several of the y groups and all four hold partials
      k << "      float r = part[0][x2][e2];\n#pragma unroll\n      for (int w = 1; w < 4; ++w) r = " << (is_max ? "fmaxf(r, part[w][x2][e2])" : "r + part[w][x2][e2]") << ";\n";
    }
    if (S > 1) {
      // partial result of this slice: scratch[(orow * S + part_s) * CH + channel]
      k << "      scratch[(orow * " << S << " + part_s) * " << CH << " + cv2 * " << V << " + e2] = r;\n    }\n  }\n}\n";
      std::ostringstream k2;
      k2 << "extern \"C\" __global__ __launch_bounds__(256) void KNAME2(" << c.param_list(params, written) << ", float* __restrict__ scratch) {\n";
      k2 << "  const idx_t gid = (idx_t)blockIdx.x * 256 + threadIdx.x;\n  if (gid >= (idx_t)" << rows << ") return;\n";
      k2 << "  const idx_t orow = gid / " << CH << ";\n  const idx_t a" << ch << " = gid % " << CH << ";\n";
      decl_digits(k2, c, outer_rows, "orow", "  ", "qr");
      k2 << "  float r = scratch[orow * " << S * CH << " + a" << ch << "];\n";
      k2 << "#pragma unroll\n  for (int s = 1; s < " << S << "; ++s) r = "
         << (is_max ? "fmaxf(r, scratch[(orow * " + std::to_string(S) + " + s) * " + std::to_string(CH) + " + a" + std::to_string(ch) + "])"
                    : "r + scratch[(orow * " + std::to_string(S) + " + s) * " + std::to_string(CH) + " + a" + std::to_string(ch) + "]") << ";\n";
      if (mode == "mean") k2 << "  const float anchor_v = r * (1.0f / " << L << ".0f);\n";
      else k2 << "  const float anchor_v = r;\n";
      std::set<int> done;
      std::vector<int> roots;
      for (auto& s_ : c.stores) roots.push_back(s_.value);
      c.emit_values(k2, roots, done, pslot, "  ");
      for (auto& s_ : c.stores) {
        std::string st = c.store_stmt(s_, pslot, c.addr_expr(s_.addr));
        if (s_.preds.empty()) k2 << "  " << st << "\n";
        else k2 << "  if (" << c.pred_expr(s_.preds) << ") { " << st << " }\n";
      }
      k2 << "}\n";
      stage2 = k2.str();
      grid2 = (unsigned)((rows + 255) / 256);
      scratch_bytes = orows * S * CH * 4;
    } else {
    k << "      const idx_t a" << ch << " = cv2 * " << V << " + e2;\n";
    if (mode == "mean") k << "      const float anchor_v = r * (1.0f / " << L << ".0f);\n";
    else k << "      const float anchor_v = r;\n";
    {
      std::set<int> done;
      std::vector<int> roots;
      for (auto& s_ : c.stores) roots.push_back(s_.value);
      c.emit_values(k, roots, done, pslot, "      ");
      for (auto& s_ : c.stores) {
        std::string st = c.store_stmt(s_, pslot, c.addr_expr(s_.addr));
        if (s_.preds.empty()) k << "      " << st << "\n";
        else k << "      if (" << c.pred_expr(s_.preds) << ") { " << st << " }\n";
      }
    }
    k << "    }\n  }\n}\n";
    }
    grid0 = (unsigned)(orows * NCH * S);
    variant = mode + "_chan" + std::to_string(XW) + "x" + std::to_string(YH) + (S > 1 ? "_split" + std::to_string(S) : "");
  } else {
  k << "extern \"C\" __global__ __launch_bounds__(256) void KNAME(" << c.param_list(params, written) << ") {\n";
  k << "  const int lane = threadIdx.x & 63;\n";
  k << "  const idx_t row = (idx_t)blockIdx.x * 4 + (threadIdx.x >> 6);\n";
  k << "  if (row >= (idx_t)" << rows << ") return;\n";
  decl_digits(k, c, row_atoms, "row", "  ", "qr");
  const char* ident = ints ? (mode == "max" ? "(-9223372036854775807LL - 1)" : mode == "prod" ? "1LL" : "0LL")
                           : mode == "max" || mode == "softmax" ? "-__builtin_inff()" : mode == "prod" ? "1.0f" : "0.0f";
  auto combine = [&](const std::string& acc, const std::string& v) {
    if (ints && mode == "max") return acc + " = " + acc + " > " + v + " ? " + acc + " : " + v + ";";
    if (mode == "max" || mode == "softmax") return acc + " = fmaxf(" + acc + ", " + v + ");";
    if (mode == "prod") return acc + " *= " + v + ";";
    return acc + " += " + v + ";";
  };
  // declares the column atoms for `col`, then evaluates the prologue into a fresh variable `dst`
  auto load_elem = [&](const std::string& ind, const std::string& dst) {
    decl_digits(k, c, col_atoms, "col", ind, "qc");
    k << ind << acc_t << " " << dst << ";\n" << ind << "{\n";
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
  k << "  " << acc_t << " acc = " << ident << ";\n";
  // ---- pass 1
  loop_open("j");
  k << "    if (col < " << L << ") {\n";
  load_elem("      ", "x0");
  if (cached) k << "      xs[j] = x0;\n";
  k << "      " << combine("acc", "x0") << "\n";
  k << "    }" << (cached ? std::string(" else xs[j] = ") + ident + ";" : "") << "\n  }\n";
  if (ints) {
    k << "#pragma unroll\n  for (int o = 32; o > 0; o >>= 1) { const long long other = __shfl_xor(acc, o, 64); " << combine("acc", "other") << " }\n";
  } else if (mode == "max" || mode == "softmax") k << "  acc = dn_wave_max(acc);\n";
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
    if (in_scale >= 0) {
      k << "      float anchor_v;\n      {\n";
      std::set<int> done;
      c.emit_values(k, {in_scale, in_bias}, done, pslot, "        ");
      k << "        anchor_v = (xe - mean) * rstd * " << c.vname(in_scale) << " + " << c.vname(in_bias) << ";\n      }\n";
    } else
    k << "      const float anchor_v = (xe - mean) * rstd;\n";
    emit_stores("      ");
    k << "    }\n  }\n";
  } else {
    if (mode == "mean") k << "  const float anchor_v = acc * (1.0f / " << L << ".0f);\n";
    else k << "  const " << acc_t << " anchor_v = acc;\n";
    k << "  if (lane == 0) {\n";
    emit_stores("    ");
    k << "  }\n";
  }
  k << "}\n";
  variant = mode + (cached ? "_regs" : unrolled ? "_stream" : "_loop");
  }

  Lowered Lw;
  Lw.family = FAM_REDUCE;
  Lw.ext_in.assign(params.begin(), params.begin() + n_in);
  Lw.ext_out.assign(params.begin() + n_in, params.end());
  Launch K;
  K.params = params;
  K.grid[0] = grid0;
  K.block[0] = 256;
  std::string src = std::string(device_preamble()) + k.str();
  K.name = fnv_name("dnnf_red", src);
  size_t pos;
  while ((pos = src.find("KNAME")) != std::string::npos) src.replace(pos, 5, K.name);
  K.source = src;
  K.scratch = scratch_bytes > 0;
  Lw.launches.push_back(K);
  if (!stage2.empty()) {
    Launch K2;
    K2.params = params;
    K2.grid[0] = grid2;
    K2.block[0] = 256;
    K2.scratch = true;
    std::string src2 = std::string(device_preamble()) + "typedef " + (wide ? "long long" : "int") + " idx_t;\n" + stage2;
    K2.name = fnv_name("dnnf_red2", src2);
    while ((pos = src2.find("KNAME2")) != std::string::npos) src2.replace(pos, 6, K2.name);
    K2.source = src2;
    Lw.launches.push_back(K2);
    Lw.scratch_bytes = scratch_bytes;
  }
  Lw.variant = variant;
  return Lw;
}

}  // namespace dnnf
