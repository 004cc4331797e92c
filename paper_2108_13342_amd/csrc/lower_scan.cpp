// Prefix-sum blocks: CumSum (Many-to-Many in Table 2) as the block's anchor.  The block's One-to-One
// operators in front are applied to each element as the scan reads it, those behind to each prefix sum
// before it is stored, at the same index: the scan's input and result share their index atoms.
//
// Two kernels.  When lines are many and the scanned axis is not the one lanes should run along, a lane
// owns a whole line and walks it (neighbouring lanes hold neighbouring lines: coalesced in the storage
// order of the first result).  Otherwise a wavefront owns a line and takes it 64 elements at a time: a
// shuffle scan inside the wavefront, the running total carried from chunk to chunk.  fp32 accumulation.
#include <algorithm>

#include "lower_ctx.hpp"

namespace dnnf {

namespace {
}  // namespace

Lowered lower_scan(LowerCtx& c) {
  const Graph& g = c.g;
  const Op& A = g.ops[c.anchor_op];
  const Tensor& X = g.tensors[A.in[0]];
  const Tensor& Y = g.tensors[A.out[0]];
  DNNF_CHECK(is_float(X.dtype), DNNF_UNSUPPORTED_OP, "CumSum over a non-float tensor");
  const int rank = (int)X.dims.size();
  int ax = (int)A.i("axis", 0);
  if (ax < 0) ax += rank;
  const bool exclusive = A.i("exclusive", 0) != 0, reverse = A.i("reverse", 0) != 0;
  const int64_t L = X.dims[ax];

  TIdx oi = c.fresh_index(Y.dims);
  c.tidx[c.anchor_out] = oi;
  std::vector<int> ein, eout, removed;
  block_io(g, c.blk, ein, eout, removed);
  c.forward_all();
  for (int t : eout)
    DNNF_CHECK(c.tidx.count(t), DNNF_UNSUPPORTED_OP, "block output " + g.tensors[t].name + " does not follow the scan");
  c.collect_stores(eout);
  const int xnode = c.value(A.in[0], oi);

  // finest index atoms: those of the scanned axis are set per step, the others once per line
  std::vector<int> axis_atoms, line_atoms;
  for (int d = 0; d < rank; d++) {
    std::vector<int> r;
    c.resolve(oi[d].atoms, r);
    auto& dst = d == ax ? axis_atoms : line_atoms;
    dst.insert(dst.end(), r.begin(), r.end());
  }

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

  // lines in the storage order of the first result, fastest atom last
  const Affine raddr = c.resolved(c.stores[0].addr);
  std::sort(line_atoms.begin(), line_atoms.end(), [&](int x, int y) {
    int64_t sx = stride_of(raddr, x), sy = stride_of(raddr, y);
    return sx != sy ? sx > sy : x < y;
  });
  const int64_t lines = numel(Y.dims) / std::max<int64_t>(L, 1);
  int64_t min_axis_stride = INT64_MAX, min_line_stride = INT64_MAX;
  for (int a : axis_atoms) if (c.atom_extent[a] > 1) min_axis_stride = std::min(min_axis_stride, std::abs(stride_of(raddr, a)));
  for (int a : line_atoms) if (c.atom_extent[a] > 1) min_line_stride = std::min(min_line_stride, std::abs(stride_of(raddr, a)));
  // a lane per line when neighbouring lines are neighbours in memory (or there is nothing to scan in parallel)
  const bool lane_per_line = (lines >= 64 && min_line_stride < min_axis_stride) || L <= 4;

  std::ostringstream k;
  k << "typedef " << (wide ? "long long" : "int") << " idx_t;\n";
  k << "extern \"C\" __global__ __launch_bounds__(256) void KNAME(" << c.param_list(params, written) << ") {\n";
  k << "  const idx_t gid = (idx_t)blockIdx.x * 256 + threadIdx.x;\n";
  if (lane_per_line) k << "  const idx_t line = gid;\n  if (line >= (idx_t)" << lines << ") return;\n";
  else k << "  const idx_t line = gid >> 6;\n  const int lane = threadIdx.x & 63;\n  if (line >= (idx_t)" << lines << ") return;\n";   // whole wavefronts leave together
  k << "  idx_t rem = line;\n";
  for (int i = (int)line_atoms.size() - 1; i >= 0; i--)
    k << "  const idx_t a" << line_atoms[i] << " = rem % " << c.atom_extent[line_atoms[i]] << "; rem /= " << c.atom_extent[line_atoms[i]] << ";\n";
  // position along the axis -> its atoms (mixed radix, last atom fastest)
  auto axis_decl = [&](const std::string& pos, const std::string& ind) {
    std::string out = ind + "idx_t q_ = " + pos + ";\n";
    for (int i = (int)axis_atoms.size() - 1; i >= 0; i--)
      out += ind + "const idx_t a" + std::to_string(axis_atoms[i]) + " = q_ % " + std::to_string(c.atom_extent[axis_atoms[i]]) + "; q_ /= " +
             std::to_string(c.atom_extent[axis_atoms[i]]) + ";\n";
    return out;
  };
  std::set<int> done;      // values already declared in the loop body: the operators in front and behind share them
  auto body_tail = [&](const std::string& ind) {
    // the block's operators behind the scan, and its stores
    std::vector<int> roots;
    for (auto& s : c.stores) roots.push_back(s.value);
    c.emit_values(k, roots, done, pslot, ind);
    for (auto& s : c.stores) {
      std::string stt = c.store_stmt(s, pslot, c.addr_expr(s.addr));
      if (s.preds.empty()) k << ind << stt << "\n";
      else k << ind << "if (" << c.pred_expr(s.preds) << ") { " << stt << " }\n";
    }
  };
  const std::string pos_of_j = reverse ? "(idx_t)" + std::to_string(L - 1) + " - j" : "j";
  if (lane_per_line) {
    k << "  float run = 0.0f;\n";
    k << "  for (idx_t j = 0; j < (idx_t)" << L << "; ++j) {\n";
    k << axis_decl(pos_of_j, "    ");
    c.emit_values(k, {xnode}, done, pslot, "    ");
    k << "    const float x_ = " << c.vname(xnode) << ";\n";
    if (exclusive) k << "    const float anchor_v = run;\n    run += x_;\n";
    else k << "    run += x_;\n    const float anchor_v = run;\n";
    body_tail("    ");
    k << "  }\n";
  } else {
    k << "  float carry = 0.0f;\n";
    k << "  for (idx_t j0 = 0; j0 < (idx_t)" << L << "; j0 += 64) {\n";
    k << "    const bool in_ = j0 + lane < (idx_t)" << L << ";\n";
    k << "    const idx_t j = in_ ? j0 + lane : (idx_t)" << L - 1 << ";\n";      // lanes past the end re-read the last element and drop it
    k << axis_decl(pos_of_j, "    ");
    c.emit_values(k, {xnode}, done, pslot, "    ");
    k << "    const float x_ = in_ ? " << c.vname(xnode) << " : 0.0f;\n";
    k << "    float s_ = x_;\n";
    k << "#pragma unroll\n    for (int d = 1; d < 64; d <<= 1) {\n      const float up = __shfl_up(s_, d, 64);\n      s_ += lane >= d ? up : 0.0f;\n    }\n";
    k << "    const float anchor_v = carry + " << (exclusive ? "(s_ - x_)" : "s_") << ";\n";
    k << "    carry += __shfl(s_, 63, 64);\n";
    k << "    if (in_) {\n";
    body_tail("      ");
    k << "    }\n  }\n";
  }
  k << "}\n";

  Lowered Lw;
  Lw.family = FAM_REDUCE;
  Lw.ext_in.assign(params.begin(), params.begin() + n_in);
  Lw.ext_out.assign(params.begin() + n_in, params.end());
  Launch Kn;
  Kn.params = params;
  const int64_t threads = lane_per_line ? lines : lines * 64;
  Kn.grid[0] = (unsigned)((threads + 255) / 256);
  Kn.block[0] = 256;
  std::string src = std::string(device_preamble()) + k.str();
  Kn.name = fnv_name("dnnf_scan", src);
  size_t pos;
  while ((pos = src.find("KNAME")) != std::string::npos) src.replace(pos, 5, Kn.name);
  Kn.source = src;
  Lw.launches.push_back(Kn);
  Lw.variant = std::string("cumsum_") + (lane_per_line ? "lane_per_line" : "wave_per_line") + (exclusive ? "_excl" : "") + (reverse ? "_rev" : "");
  return Lw;
}

}  // namespace dnnf
