// Elementwise-chain kernels: a block of One-to-One / Reorganize / Shuffle / One-to-Many operators
// becomes a single pass over the output index space (paper Sec. 4.4: the rules for fusing
// One-to-One with Reorganize/Shuffle permute the loop instead of moving data).
//
// Two templates:
//   linear : the block's main input and its output share the fastest-varying atom; each lane
//            handles V consecutive elements with vector loads/stores.
//   tiled  : the fastest atoms differ (a transposition survives the index folding).  A 64x64 tile
//            is computed with lanes running along the input's fastest atoms, staged in LDS, and
//            written with lanes running along the output's fastest atoms, so both the global
//            read and the global write are coalesced.
#include <algorithm>

#include "lower_ctx.hpp"

namespace dnnf {

namespace {

struct Access {
  int tensor;
  Affine addr;   // resolved
  bool is_store;
  int node;      // LOAD node id, or index into stores
};

struct Loop {
  std::vector<int> atoms;  // major -> minor, all merged into one counter
  int64_t extent;
};


// Atoms that follow each other contiguously in `a` starting from element stride 1.
std::vector<int> contiguous_group(const LowerCtx& c, const Affine& a, const std::vector<int>& atoms) {
  std::vector<int> grp;
  int64_t want = 1;
  for (;;) {
    int found = -1;
    for (int at : atoms)
      if (stride_of(a, at) == want && std::find(grp.begin(), grp.end(), at) == grp.end()) { found = at; break; }
    if (found < 0) break;
    grp.push_back(found);            // minor -> major
    want *= c.atom_extent[found];
  }
  return grp;
}

void collect_accesses(LowerCtx& c, std::vector<Access>& acc, std::set<int>& pinned) {
  std::set<int> need;
  std::vector<int> stack;
  for (auto& s : c.stores) stack.push_back(s.value);
  while (!stack.empty()) {
    int n = stack.back();
    stack.pop_back();
    if (need.count(n)) continue;
    need.insert(n);
    for (int a : c.nodes[n].args) stack.push_back(a);
    if (c.nodes[n].kind == ENode::LOAD)
      for (auto& p : c.nodes[n].addr.indirect) stack.push_back(p.first);
  }
  for (int n : need)
    if (c.nodes[n].kind == ENode::LOAD) acc.push_back({c.nodes[n].tensor, c.resolved(c.nodes[n].addr), false, n});
  for (size_t i = 0; i < c.stores.size(); i++) {
    acc.push_back({c.stores[i].tensor, c.resolved(c.stores[i].addr), true, (int)i});
    for (auto& p : c.stores[i].preds) {
      std::vector<int> r;
      c.resolve(p.atoms, r);
      pinned.insert(r.begin(), r.end());
    }
  }
}

void decl_atoms_from_counter(std::ostringstream& os, const LowerCtx& c, const std::vector<int>& atoms_major_minor,
                             const std::string& counter, const std::string& ind) {
  // mixed-radix digits of `counter`, least significant atom last in the list
  std::string rem = counter;
  for (int k = (int)atoms_major_minor.size() - 1; k >= 0; k--) {
    int a = atoms_major_minor[k];
    int64_t e = c.atom_extent[a];
    if (k == 0) os << ind << "const idx_t a" << a << " = " << rem << ";\n";
    else {
      os << ind << "const idx_t a" << a << " = " << rem << " % " << e << ";\n";
      os << ind << "const idx_t q" << a << " = " << rem << " / " << e << ";\n";
      rem = "q" + std::to_string(a);
    }
  }
}

}  // namespace

Lowered lower_elementwise(LowerCtx& c) {
  const Graph& g = c.g;
  Lowered L;
  L.family = FAM_EW;
  std::vector<int> ein, eout, removed;
  block_io(g, c.blk, ein, eout, removed);
  if (!c.only_outputs.empty()) eout = c.only_outputs;   // one kernel per output (see lower_block)
  DNNF_CHECK(!eout.empty(), DNNF_INVALID_ARG, "block without outputs");
  // pivot = the last block output in topological order, unless the caller names another; everything else hangs
  // off its index space
  if (c.pivot_out >= 0) {
    auto it = std::find(eout.begin(), eout.end(), c.pivot_out);
    DNNF_CHECK(it != eout.end(), DNNF_INVALID_ARG, "pivot is not a block output");
    eout.erase(it);
    eout.push_back(c.pivot_out);
  }
  int root = eout.back();
  if (c.concat_part >= 0) {
    // the pivot space is the operand's: its atoms index the result at the operand's offset
    const Op& co = g.ops[c.concat_op];
    int a = (int)co.i("axis", 0);
    if (a < 0) a += (int)g.tensors[root].dims.size();
    TIdx ix = c.fresh_index(g.tensors[co.in[c.concat_part]].dims);
    for (int k = 0; k < c.concat_part; k++) ix[a].offset += g.tensors[co.in[k]].dims[a];
    c.tidx[root] = ix;
  } else
  c.tidx[root] = c.fresh_index(g.tensors[root].dims);
  // the root's own value first (gives indices to everything upstream), then siblings
  {
    TIdx ix = c.tidx[root];
    c.value(root, ix);
  }
  c.forward_all();
  c.collect_stores(eout);

  std::vector<Access> acc;
  std::set<int> pinned;
  collect_accesses(c, acc, pinned);
  std::vector<int> atoms = c.final_atoms();

  // kernel parameters: external inputs actually loaded, then outputs
  std::vector<int> params;
  std::map<int, int> pslot;
  std::set<int> written;
  for (auto& a : acc)
    if (!a.is_store && !pslot.count(a.tensor)) { pslot[a.tensor] = (int)params.size(); params.push_back(a.tensor); }
  for (auto& s : c.stores) {
    DNNF_CHECK(!pslot.count(s.tensor), DNNF_UNSUPPORTED_OP, "block reads and writes the same tensor");
    pslot[s.tensor] = (int)params.size();
    params.push_back(s.tensor);
    written.insert(s.tensor);
  }
  L.ext_in.assign(params.begin(), params.begin() + (params.size() - c.stores.size()));
  L.ext_out.assign(params.begin() + L.ext_in.size(), params.end());

  // root store and dominant load decide the template
  const Store& rs = c.stores.back();
  Affine raddr = c.resolved(rs.addr);
  int dom = -1;
  int64_t dom_n = 0;
  for (size_t i = 0; i < acc.size(); i++)
    if (!acc[i].is_store && acc[i].addr.indirect.empty() && g.tensors[acc[i].tensor].n() > dom_n) {
      dom = (int)i;
      dom_n = g.tensors[acc[i].tensor].n();
    }
  std::vector<int> ogrp = contiguous_group(c, raddr, atoms);
  std::vector<int> igrp;
  if (dom >= 0 && dom_n * 4 >= g.tensors[rs.tensor].n()) igrp = contiguous_group(c, acc[dom].addr, atoms);
  bool tiled = !ogrp.empty() && !igrp.empty() && ogrp[0] != igrp[0] && c.stores.size() == 1 && rs.preds.empty() &&
               c.opts.force_variant != 1;
  if (tiled) {
    // make the groups disjoint: cut each at the first atom owned by the other
    // each group takes just enough of its fastest atoms to fill a 64-wide tile edge and never an
    // atom the other group needs
    std::vector<int> o2, i2;
    int64_t e = 1;
    for (int a : ogrp) {
      if (e >= 64 || a == igrp[0]) break;
      o2.push_back(a);
      e *= c.atom_extent[a];
    }
    e = 1;
    for (int a : igrp) {
      if (e >= 64 || std::find(o2.begin(), o2.end(), a) != o2.end()) break;
      i2.push_back(a);
      e *= c.atom_extent[a];
    }
    ogrp = o2;
    igrp = i2;
    tiled = !ogrp.empty() && !igrp.empty() && c.extent_of(ogrp) >= 8 && c.extent_of(igrp) >= 8;
  }

  std::ostringstream body;
  const bool wide = [&] {
    for (int t : params) if (g.tensors[t].n() >= (int64_t)1 << 31) return true;
    return false;
  }();
  body << "typedef " << (wide ? "long long" : "int") << " idx_t;\n";
  Launch K;
  K.params = params;

  if (!tiled) {
    // ---- linear template: loops = atoms ordered by root-output stride (major first), merged
    //      where every access agrees they are contiguous.
    std::vector<int> order = atoms;
    std::sort(order.begin(), order.end(), [&](int x, int y) {
      int64_t sx = stride_of(raddr, x), sy = stride_of(raddr, y);
      return sx != sy ? sx > sy : x < y;
    });
    int inner = order.empty() ? -1 : order.back();
    int V = 1;
    if (inner >= 0 && stride_of(raddr, inner) == 1 && !pinned.count(inner)) {
      int eb = 4;
      for (int t : params) eb = std::min(eb, dtype_bytes(g.tensors[t].dtype));
      for (int cand : {16 / std::max(eb, 2), 4, 2}) {
        bool ok = c.atom_extent[inner] % cand == 0;
        for (auto& a : acc) {
          int64_t s = stride_of(a.addr, inner);
          ok = ok && (s == 0 || s == 1) && a.addr.indirect.empty() == true;
          if (s == 1) {
            ok = ok && a.addr.offset % cand == 0;
            for (auto& kv : a.addr.stride) if (kv.first != inner) ok = ok && kv.second % cand == 0;
          }
          if (!is_float(g.tensors[a.tensor].dtype)) ok = false;
        }
        if (ok) { V = cand; break; }
      }
    }
    int64_t total = 1;
    for (int a : atoms) total *= c.atom_extent[a];
    int64_t nthreads = total / V;
    std::ostringstream k;
    k << "extern \"C\" __global__ __launch_bounds__(256) void KNAME(" << c.param_list(params, written) << ") {\n";
    k << "  const idx_t gid = (idx_t)blockIdx.x * 256 + threadIdx.x;\n";
    k << "  if (gid >= (idx_t)" << nthreads << ") return;\n";
    if (V == 1) {
      decl_atoms_from_counter(k, c, order, "gid", "  ");
      std::set<int> done;
      std::vector<int> roots;
      for (auto& s : c.stores) roots.push_back(s.value);
      c.emit_values(k, roots, done, pslot, "  ");
      for (auto& s : c.stores) {
        std::string st = c.store_stmt(s, pslot, c.addr_expr(s.addr));
        if (s.preds.empty()) k << "  " << st << "\n";
        else k << "  if (" << c.pred_expr(s.preds) << ") { " << st << " }\n";
      }
    } else {
      // inner atom advances by V per thread; vector loads for stride-1 accesses
      std::vector<int> outer(order.begin(), order.end() - 1);
      int64_t ev = c.atom_extent[inner] / V;
      if (outer.empty()) k << "  const idx_t a" << inner << "_0 = gid * " << V << ";\n";
      else {
        k << "  const idx_t a" << inner << "_0 = (gid % " << ev << ") * " << V << ";\n";
        k << "  const idx_t gq = gid / " << ev << ";\n";
        decl_atoms_from_counter(k, c, outer, "gq", "  ");
      }
      k << "  { const idx_t a" << inner << " = a" << inner << "_0;\n";
      std::map<int, std::string> ov;
      for (auto& a : acc) {
        if (a.is_store) continue;
        int64_t s = stride_of(a.addr, inner);
        std::string ct = c.ctype(g.tensors[a.tensor].dtype);
        int slot = pslot[a.tensor];
        if (s == 1) {
          k << "  typedef " << ct << " lv" << a.node << "_t __attribute__((ext_vector_type(" << V << ")));\n";
          k << "  const lv" << a.node << "_t lv" << a.node << " = *(const lv" << a.node << "_t*)(p" << slot << " + ("
            << c.addr_expr(a.addr) << "));\n";
          ov[a.node] = "cvt_in(lv" + std::to_string(a.node) + "[u])";
        } else {
          k << "  const float ls" << a.node << " = cvt_in(p" << slot << "[" << c.addr_expr(a.addr) << "]);\n";
          ov[a.node] = "ls" + std::to_string(a.node);
        }
      }
      for (size_t i = 0; i < c.stores.size(); i++) {
        std::string ct = c.ctype(g.tensors[c.stores[i].tensor].dtype);
        k << "  typedef " << ct << " sv" << i << "_t __attribute__((ext_vector_type(" << V << ")));\n";
        k << "  sv" << i << "_t sv" << i << ";\n";
      }
      k << "#pragma unroll\n  for (int u = 0; u < " << V << "; ++u) {\n";
      std::set<int> done;
      std::vector<int> roots;
      for (auto& s : c.stores) roots.push_back(s.value);
      c.emit_values(k, roots, done, pslot, "    ", &ov);
      for (size_t i = 0; i < c.stores.size(); i++) {
        std::string ct = c.ctype(g.tensors[c.stores[i].tensor].dtype);
        k << "    { " << ct << " tmp; cvt_out(&tmp, " << c.vname(c.stores[i].value) << "); sv" << i << "[u] = tmp; }\n";
      }
      k << "  }\n";
      for (size_t i = 0; i < c.stores.size(); i++) {
        const Store& s = c.stores[i];
        std::string st = "*(sv" + std::to_string(i) + "_t*)(p" + std::to_string(pslot[s.tensor]) + " + (" + c.addr_expr(s.addr) + ")) = sv" + std::to_string(i) + ";";
        // a result that does not move along the vector atom (it sits in front of a Resize / Expand inside the block):
        // the V lanes hold the same element, stored once
        if (stride_of(c.resolved(s.addr), inner) == 0)
          st = "p" + std::to_string(pslot[s.tensor]) + "[" + c.addr_expr(s.addr) + "] = sv" + std::to_string(i) + "[0];";
        if (s.preds.empty()) k << "  " << st << "\n";
        else k << "  if (" << c.pred_expr(s.preds) << ") { " << st << " }\n";
      }
      k << "  }\n";
    }
    k << "}\n";
    body << k.str();
    K.grid[0] = (unsigned)((nthreads + 255) / 256);
    K.block[0] = 256;
    L.variant = "linear_v" + std::to_string(V);
  } else {
    // ---- tiled template
    int64_t EI = c.extent_of(igrp), EO = c.extent_of(ogrp);
    const int T = 64;
    int64_t ti = (EI + T - 1) / T, to = (EO + T - 1) / T;
    std::vector<int> rest;
    for (int a : atoms)
      if (std::find(igrp.begin(), igrp.end(), a) == igrp.end() && std::find(ogrp.begin(), ogrp.end(), a) == ogrp.end())
        rest.push_back(a);
    std::sort(rest.begin(), rest.end(), [&](int x, int y) {
      int64_t sx = stride_of(raddr, x), sy = stride_of(raddr, y);
      return sx != sy ? sx > sy : x < y;
    });
    int64_t nrest = 1;
    for (int a : rest) nrest *= c.atom_extent[a];
    std::vector<int> imaj(igrp.rbegin(), igrp.rend()), omaj(ogrp.rbegin(), ogrp.rend());
    std::string ot = c.ctype(g.tensors[rs.tensor].dtype);
    std::ostringstream k;
    k << "extern \"C\" __global__ __launch_bounds__(256) void KNAME(" << c.param_list(params, written) << ") {\n";
    k << "  __shared__ " << ot << " tile[" << T << "][" << T + (dtype_bytes(g.tensors[rs.tensor].dtype) == 4 ? 1 : 2) << "];\n";
    // ty is the same for the 64 lanes of a wavefront: held in a scalar register, so that indices built from
    // it alone (per-channel operands in the first phase) are computed once per wavefront and read with scalar loads
    k << "  const int tx = threadIdx.x & 63, ty = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);\n";
    k << "  idx_t bid = blockIdx.x;\n";
    k << "  const idx_t tile_i = bid % " << ti << "; bid /= " << ti << ";\n";
    k << "  const idx_t tile_o = bid % " << to << "; bid /= " << to << ";\n";
    decl_atoms_from_counter(k, c, rest, "bid", "  ");
    k << "  {\n    const idx_t gi = tile_i * " << T << " + tx;\n";
    decl_atoms_from_counter(k, c, imaj, "gi", "    ");
    k << "#pragma unroll 4\n    for (int r = 0; r < " << T / 4 << "; ++r) {\n";
    k << "      const int ol = ty + 4 * r;\n      const idx_t go = tile_o * " << T << " + ol;\n";
    k << "      if (gi < " << EI << " && go < " << EO << ") {\n";
    decl_atoms_from_counter(k, c, omaj, "go", "        ");
    {
      std::set<int> done;
      c.emit_values(k, {rs.value}, done, pslot, "        ");
    }
    k << "        cvt_out(&tile[ol][tx], " << c.vname(rs.value) << ");\n";
    k << "      }\n    }\n  }\n  __syncthreads();\n";
    k << "  {\n    const idx_t go = tile_o * " << T << " + tx;\n";
    decl_atoms_from_counter(k, c, omaj, "go", "    ");
    k << "#pragma unroll 4\n    for (int r = 0; r < " << T / 4 << "; ++r) {\n";
    k << "      const int il = ty + 4 * r;\n      const idx_t gi = tile_i * " << T << " + il;\n";
    k << "      if (gi < " << EI << " && go < " << EO << ") {\n";
    decl_atoms_from_counter(k, c, imaj, "gi", "        ");
    k << "        p" << pslot[rs.tensor] << "[" << c.addr_expr(rs.addr) << "] = tile[tx][il];\n";
    k << "      }\n    }\n  }\n}\n";
    body << k.str();
    K.grid[0] = (unsigned)(ti * to * nrest);
    K.block[0] = 256;
    L.variant = "tiled_64x64";
  }

  std::string src = std::string(device_preamble()) + body.str();
  K.name = fnv_name("dnnf_ew", src);
  size_t pos;
  while ((pos = src.find("KNAME")) != std::string::npos) src.replace(pos, 5, K.name);
  K.source = src;
  L.launches.push_back(K);
  return L;
}

}  // namespace dnnf
