// Convolution blocks (NCHW / OIHW).
//   dense (group 1): implicit GEMM on the MFMA template shared with MatMul - rows are output
//     channels (the weight matrix is K-contiguous), columns are output pixels (n, p, q), which are
//     contiguous in NCHW so accumulator columns store coalesced.  A 1x1 stride-1 unpadded
//     convolution over an external tensor has an affine operand and uses the vector loaders; any
//     other window gathers the operand element by element (im2col on the fly, zero padding by
//     predicate), applying the block's prologue operators to each gathered element.
//   depthwise (group = channels): direct stencil, one output element per lane, fp32 accumulate.
// The block's successors (folded-BN affine, activation, residual add, ...) run as the epilogue.
#include <algorithm>
#include <cstdlib>

#include "lower_ctx.hpp"

namespace dnnf {

namespace {

void collect_params(const LowerCtx& c, const std::vector<int>& roots, std::vector<int>& params, std::map<int, int>& pslot) {
  std::set<int> need;
  std::vector<int> stack = roots;
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
}  // namespace

Lowered lower_conv(LowerCtx& c) {
  const Graph& g = c.g;
  const Op& A = g.ops[c.anchor_op];
  const Tensor& X = g.tensors[A.in[0]];
  const Tensor& Wt = g.tensors[A.in[1]];
  const Tensor& Y = g.tensors[A.out[0]];
  const int bias_t = A.in.size() > 2 ? A.in[2] : -1;
  DNNF_CHECK(c.is_external(A.in[1]) && (bias_t < 0 || c.is_external(bias_t)), DNNF_UNSUPPORTED_OP,
             "convolution weights computed inside the block");
  DNNF_CHECK(is_float(X.dtype) && Wt.dtype == X.dtype, DNNF_UNSUPPORTED_OP, "Conv operands must share a float type");
  const int64_t N = X.dims[0], C = X.dims[1], H = X.dims[2], Wd = X.dims[3];
  const int64_t CO = Wt.dims[0], CG = Wt.dims[1], KH = Wt.dims[2], KW = Wt.dims[3];
  const int64_t HO = Y.dims[2], WO = Y.dims[3];
  const int64_t grp = A.i("group", 1);
  auto st = A.ints("strides");
  if (st.empty()) st = {1, 1};
  auto pd = A.ints("pads");
  if (pd.empty()) pd = {0, 0, 0, 0};
  const int64_t SH = st[0], SW = st[1], PT = pd[0], PL = pd[1];
  const bool depthwise = grp == C && CG == 1 && CO == C && grp > 1;
  DNNF_CHECK(grp == 1 || depthwise, DNNF_UNSUPPORTED_OP, "grouped convolution other than depthwise has no kernel template");

  TIdx oi = c.fresh_index(Y.dims);
  c.tidx[c.anchor_out] = oi;
  std::vector<int> ein, eout, removed;
  block_io(g, c.blk, ein, eout, removed);
  c.allow_replication = grp == 1;          // the implicit-GEMM epilogue can store a result at several destinations
  c.forward_all();
  for (int t : eout)
    DNNF_CHECK(c.tidx.count(t), DNNF_UNSUPPORTED_OP, "block output " + g.tensors[t].name + " does not follow the convolution");
  c.collect_stores(eout);

  // the conv input as a function of four index atoms whose values the kernel computes
  const int xn = c.new_atom(std::max<int64_t>(N, 2)), xc = c.new_atom(std::max<int64_t>(C, 2)),
            xh = c.new_atom(std::max<int64_t>(H, 2)), xw = c.new_atom(std::max<int64_t>(Wd, 2));
  TIdx xi(4);
  xi[0].atoms = {xn};
  xi[1].atoms = {xc};
  xi[2].atoms = {xh};
  xi[3].atoms = {xw};
  const int xnode = c.value(A.in[0], xi);
  // an index map in front of the convolution (Reshape, DepthToSpace, ...) may have cut one of the four operand
  // atoms into parts: the affine operand loaders, which work on the atoms as wholes, are then not used, and the
  // element-wise paths declare the parts from the whole
  const std::vector<int> xatoms = {xn, xc, xh, xw};
  const bool x_cut = c.is_split(xn) || c.is_split(xc) || c.is_split(xh) || c.is_split(xw);

  std::vector<int> out_atoms[4];
  for (int d = 0; d < 4; d++) c.resolve(oi[d].atoms, out_atoms[d]);

  std::vector<int> params;
  std::map<int, int> pslot;
  std::set<int> written;
  {
    std::vector<int> roots = {xnode};
    for (auto& s : c.stores) roots.push_back(s.value);
    collect_params(c, roots, params, pslot);
  }
  auto add_param = [&](int t) {
    if (!pslot.count(t)) { pslot[t] = (int)params.size(); params.push_back(t); }
    return pslot[t];
  };
  const int wslot = add_param(A.in[1]);
  // depthwise filter [c, 1, kh, kw]: element (channel, tap) in the declared order, or in the re-laid [kh, kw, 1, c] order
  const Tensor& Wdecl = g.tensors[A.in[1]];
  const bool w_relaid = Wdecl.perm == std::vector<int>{2, 3, 1, 0};
  const bool w_taps_major = Wdecl.perm == std::vector<int>{0, 2, 3, 1};
  DNNF_CHECK(Wdecl.perm.empty() || w_relaid || w_taps_major, DNNF_UNSUPPORTED_OP, "filter in an unknown storage order");
  const int64_t w_chan_stride = w_relaid ? 1 : (Wdecl.dims.size() == 4 ? Wdecl.dims[2] * Wdecl.dims[3] : 1);
  const int64_t w_tap_stride = w_relaid ? Wdecl.dims[0] : 1;
  const int bslot = bias_t >= 0 ? add_param(bias_t) : -1;
  size_t n_in = params.size();
  for (auto& s : c.stores) {
    DNNF_CHECK(!pslot.count(s.tensor), DNNF_UNSUPPORTED_OP, "block reads and writes the same tensor");
    pslot[s.tensor] = (int)params.size();
    params.push_back(s.tensor);
    written.insert(s.tensor);
  }
  // a global average pool taken inside this kernel (a depthwise convolution whose workgroup covers a whole image plane)
  int pool_src = -1, pool_dst = -1;
  if (c.opts.pool_op >= 0) {
    const Op& PO = g.ops[c.opts.pool_op];
    pool_src = PO.in[0];
    pool_dst = PO.out[0];
    DNNF_CHECK(written.count(pool_src) && !pslot.count(pool_dst), DNNF_UNSUPPORTED_OP, "the pooled tensor is not a stored result of the convolution's block");
    DNNF_CHECK(g.tensors[pool_src].dims == Y.dims && g.tensors[pool_dst].dtype == g.tensors[pool_src].dtype, DNNF_UNSUPPORTED_OP,
               "the pooled tensor does not have the convolution's index space");
    pslot[pool_dst] = (int)params.size();
    params.push_back(pool_dst);
    written.insert(pool_dst);
  }
  const bool wide = [&] {
    for (int t : params) if (g.tensors[t].n() >= (int64_t)1 << 31) return true;
    return false;
  }();
  std::string kparams = c.param_list(params, written), kargs;
  for (size_t i = 0; i < params.size(); i++) kargs += (i ? ", p" : "p") + std::to_string(i);

  auto emit_epilogue_body = [&](std::ostringstream& k, const std::string& ind) {
    std::set<int> done;
    std::vector<int> roots;
    for (auto& s : c.stores) roots.push_back(s.value);
    c.emit_values(k, roots, done, pslot, ind);
    for (auto& s : c.stores) {
      std::string stt = c.store_stmt(s, pslot, c.addr_expr(s.addr));
      if (s.preds.empty()) k << ind << stt << "\n";
      else k << ind << "if (" << c.pred_expr(s.preds) << ") { " << stt << " }\n";
    }
  };

  Lowered Lw;
  Launch Kn;
  std::ostringstream k;
  k << "typedef " << (wide ? "long long" : "int") << " idx_t;\n";

  if (depthwise) {
    // 100: the direct channels-last kernel; 101-104: the staged one with its largest patch, with a patch of fewer rows
    // (more, smaller workgroups), with 32 instead of 64 channels per workgroup, and with both
    DNNF_CHECK(c.opts.force_variant < 105, DNNF_UNSUPPORTED_OP, "no such depthwise variant");
    // Each lane produces TP vertically adjacent outputs of one (n, c, q): the (TP-1)*SH + KH input
    // rows they cover are loaded once and shared between them; lanes run along q, so every load and
    // store instruction of a wavefront touches consecutive addresses.
    const bool p_single = out_atoms[2].size() == 1;
    const int TP = (p_single && HO >= 4) ? 4 : 1;
    const int64_t ptiles = (HO + TP - 1) / TP;
    const int R = (TP - 1) * (int)SH + (int)KH;
    const int64_t total = N * C * ptiles * WO;
    auto digit = [&](int d) {   // value of output dimension d as a C expression
      std::string e;
      int64_t mult = 1;
      for (int i = (int)out_atoms[d].size() - 1; i >= 0; i--) {
        e = "a" + std::to_string(out_atoms[d][i]) + (mult == 1 ? "" : " * " + std::to_string(mult)) + (e.empty() ? "" : " + " + e);
        mult *= c.atom_extent[out_atoms[d][i]];
      }
      return e.empty() ? std::string("0") : e;
    };
    auto peel = [&](const std::vector<int>& atoms) {   // minor -> major digits off the running counter
      for (int i = (int)atoms.size() - 1; i >= 0; i--)
        k << "  const idx_t a" << atoms[i] << " = rem % " << c.atom_extent[atoms[i]] << "; rem /= " << c.atom_extent[atoms[i]] << ";\n";
    };
    // Vector variant: a lane owns VW horizontally adjacent outputs as well, so each input row costs it
    // one aligned vector load plus the halo elements instead of KW scalar loads per output column.
    int VW = 0;
    Affine xaddr;
    if (!x_cut && p_single && out_atoms[3].size() == 1 && c.nodes[xnode].kind == ENode::LOAD && !c.nodes[xnode].is_int &&
        c.nodes[xnode].addr.indirect.empty() && Wd == WO * SW && TP > 1) {
      xaddr = c.resolved(c.nodes[xnode].addr);
      const int ebx = dtype_bytes(g.tensors[c.nodes[xnode].tensor].dtype);
      auto itw = xaddr.stride.find(xw);
      if (itw != xaddr.stride.end() && itw->second == 1) {
        for (int vw = (int)(16 / (ebx * SW)); vw >= 2 && !VW; vw /= 2) {
          const int64_t span = vw * SW;
          bool ok = WO % vw == 0 && xaddr.offset % span == 0;
          for (auto& kv : xaddr.stride) if (kv.first != xw && kv.second % span) ok = false;
          if (ok) VW = vw;
        }
      }
    }
    // Channels-last variant: the operand, the (re-laid) filter and the result are all contiguous along
    // the channels.  A lane owns V channels (one 16-byte vector) of a TPc x TQc patch of output pixels:
    // every tap is one vector load of the input and one of the filter, neighbouring lanes take the next
    // channels of the same pixel, so a wavefront's loads and stores run over whole pixels' worth of
    // contiguous bytes.  Input columns are shared between the TQc outputs of a row, input rows between
    // the TPc output rows; filter rows are fetched as the window reaches them, never all at once.
    int VC = 0;
    Affine xaddr_c, waddr;
    int wkh = -1, wkw = -1;
    {
      bool single = true;
      for (int d = 0; d < 4; d++) single = single && out_atoms[d].size() <= 1;
      const ENode& xe = c.nodes[xnode];
      if (!x_cut && single && xe.kind == ENode::LOAD && !xe.is_int && xe.addr.indirect.empty() && c.opts.force_variant != 2) {
        xaddr_c = c.resolved(xe.addr);
        const int v = 16 / dtype_bytes(g.tensors[xe.tensor].dtype);
        auto itc = xaddr_c.stride.find(xc);
        bool ok = itc != xaddr_c.stride.end() && itc->second == 1 && C % v == 0 && xaddr_c.offset % v == 0 &&
                  g.tensors[xe.tensor].dtype == Wt.dtype;
        for (auto& kv : xaddr_c.stride) if (kv.first != xc && kv.second % v) ok = false;
        if (ok) {
          wkh = c.new_atom(std::max<int64_t>(KH, 2));
          wkw = c.new_atom(std::max<int64_t>(KW, 2));
          TIdx wi(4);
          wi[0].atoms = {xc};
          wi[2].atoms = {wkh};
          wi[3].atoms = {wkw};
          waddr = c.resolved(c.affine(Wt, wi));
          auto itw = waddr.stride.find(xc);
          ok = itw != waddr.stride.end() && itw->second == 1 && waddr.offset % v == 0;
          for (auto& kv : waddr.stride) if (kv.first != xc && kv.second % v) ok = false;
        }
        if (ok) VC = v;
      }
    }
    DNNF_CHECK(c.opts.force_variant < 100 || VC, DNNF_UNSUPPORTED_OP, "depthwise variants exist for channels-last operands only");
    // Second channels-last kernel, through LDS: a workgroup stages the input window of a TH x TW patch of output
    // pixels for CB channels (all its loads in flight at once, each input element fetched once per workgroup
    // instead of once per tap), keeps the filter taps of its channel vector in registers and then reads the taps'
    // inputs from LDS.  The default for 5x5 filters, where the direct kernel is bound by cache bandwidth and by the
    // latency of its dependent rows of loads; a tuning build times both.
    int ldsTH = 0, ldsTW = 0, ldsXC = 0;
    if (VC) {
      const int64_t CV = C / VC;
      const int lds_mode = c.opts.force_variant >= 101 ? c.opts.force_variant - 101 : 0;       // bit 0: fewer rows, bit 1: 32 channels
      ldsXC = (CV % 8 == 0 && !(lds_mode & 2)) ? 8 : 4;
      // (a pool that rides along needs the whole plane in one patch: four channel vectors per workgroup when eight do not leave room)
      if (c.opts.pool_op >= 0 && ldsXC == 8 && ((HO - 1) * SH + KH) * ((WO - 1) * SW + KW) * 8 * 16 > 40 * 1024) ldsXC = 4;
      const int PS = 256 / ldsXC;
      auto largest_divisor = [](int64_t n, int64_t cap) { int64_t best = 0; for (int64_t d = 1; d <= n && d <= cap; d++) if (n % d == 0) best = d; return (int)best; };
      ldsTW = largest_divisor(WO, 16);
      if (CV >= 4 && ldsTW >= 7) {
        const int IW = (ldsTW - 1) * (int)SW + (int)KW;
        for (int th = (int)std::min<int64_t>(HO, 16); th >= 1 && !ldsTH; th--) {
          if (HO % th) continue;
          const int IH = (th - 1) * (int)SH + (int)KH;
          if ((int64_t)IH * IW * ldsXC * 16 <= 40 * 1024 && th * ldsTW <= 8 * PS) ldsTH = th;
        }
        if ((lds_mode & 1) && ldsTH > 1 && c.opts.pool_op < 0)
          for (int th = ldsTH / 2; th >= 1; th--)
            if (HO % th == 0) { ldsTH = th; break; }
      }
    }
    bool use_lds = ldsTH > 0 && (c.opts.force_variant >= 101 || (c.opts.force_variant < 100 && KH * KW > 9));
    if (pool_dst >= 0) {
      // one workgroup must see every pixel of an image for its channels: the staged kernel with the whole plane as its patch
      DNNF_CHECK(VC && ldsTH == HO && ldsTW == WO && c.opts.force_variant != 100, DNNF_UNSUPPORTED_OP,
                 "the pool joins a depthwise convolution only when one workgroup's patch is the whole image plane");
      use_lds = true;
    }
    if (const char* e = getenv("DNNF_DW_VARIANT"))       // developer override for tuning runs and tests: "chan" or "lds"
      if (c.opts.force_variant < 100) use_lds = ldsTH > 0 && std::string(e) == "lds";
    DNNF_CHECK(c.opts.force_variant < 101 || use_lds, DNNF_UNSUPPORTED_OP, "no LDS variant for this depthwise shape");
    if (VC) {
      const int V = VC;
      const int64_t CV = C / V;
      // patch size: as much reuse as still leaves every SIMD four wavefronts to hide the load latency with
      // (a lane's taps are a chain of dependent round trips; with fewer wavefronts nothing covers them)
      std::vector<std::pair<int, int>> tiles;
      {
        std::vector<int> tq = WO % 4 == 0 ? std::vector<int>{4, 2, 1} : WO % 2 == 0 ? std::vector<int>{2, 1} : std::vector<int>{1};
        for (int q : tq) {
          if (HO % 2 == 0) tiles.push_back({2, q});
          tiles.push_back({1, q});
        }
        std::sort(tiles.begin(), tiles.end(), [](const std::pair<int, int>& a, const std::pair<int, int>& b) { return a.first * a.second > b.first * b.second; });
      }
      int TPc = 1, TQc = 1;
      int64_t want_threads = 256 * 4 * 4 * 64;
      if (const char* e = getenv("DNNF_DW_THREADS")) want_threads = atoll(e);     // developer override for tuning runs
      for (auto& t : tiles)
        if (N * CV * (HO / t.first) * (WO / t.second) >= want_threads) { TPc = t.first; TQc = t.second; break; }
      const int64_t PTn = HO / TPc, QTn = WO / TQc, ctotal = N * CV * PTn * QTn;
      const int Rc = (TPc - 1) * (int)SH + (int)KH, WINQ = (TQc - 1) * (int)SW + (int)KW;
      const Tensor& XT = g.tensors[c.nodes[xnode].tensor];
      const std::string px = "p" + std::to_string(pslot.at(c.nodes[xnode].tensor)), pw = "p" + std::to_string(wslot);
      auto atom_or_zero = [&](int d) { return out_atoms[d].empty() ? -1 : out_atoms[d][0]; };
      const int na = atom_or_zero(0), ca = atom_or_zero(1), pa = atom_or_zero(2), qa = atom_or_zero(3);
      // epilogue: per output pixel, V channels; operands and results contiguous along the channels move as vectors
      std::set<int> need;
      {
        std::vector<int> stack;
        for (auto& st_ : c.stores) stack.push_back(st_.value);
        while (!stack.empty()) {
          int n = stack.back();
          stack.pop_back();
          if (need.count(n)) continue;
          need.insert(n);
          for (int a : c.nodes[n].args) stack.push_back(a);
        }
      }
      auto chan_contig = [&](const Affine& a0, int elems) {
        Affine a = c.resolved(a0);
        auto it = a.stride.find(ca);
        if (ca < 0 || it == a.stride.end() || it->second != 1 || a.offset % elems || !a.indirect.empty()) return false;
        for (auto& kv : a.stride) if (kv.first != ca && kv.second % elems) return false;
        return true;
      };
      // emits the epilogue of one output pixel: its V channels run through the block's successors; operands and
      // results that are contiguous along the channels move as vectors
      bool pool_vec_ok = false;      // the pooled result leaves as a vector store (whose rounded values the pool sums)
      auto chan_epilogue = [&](const std::string& n_expr, const std::string& p_expr, const std::string& q_expr, const std::string& acc_expr) {
      k << "      {\n";
      if (na >= 0) k << "      const idx_t a" << na << " = " << n_expr << ";\n";
      if (pa >= 0) k << "      const idx_t a" << pa << " = " << p_expr << ";\n";
      if (qa >= 0) k << "      const idx_t a" << qa << " = " << q_expr << ";\n";
      k << "      const idx_t c0_ = oc0;\n";
      std::map<int, std::string> ov;
      k << "      {\n";
      if (ca >= 0) k << "      const idx_t a" << ca << " = c0_;\n";
      for (int n : need) {
        const ENode& e = c.nodes[n];
        if (e.kind != ENode::LOAD || e.is_int) continue;
        const Tensor& T = g.tensors[e.tensor];
        if (16 / dtype_bytes(T.dtype) < V || !chan_contig(e.addr, V)) continue;
        k << "      typedef " << c.ctype(T.dtype) << " lv" << n << "_t __attribute__((ext_vector_type(" << V << ")));\n";
        k << "      const lv" << n << "_t lv" << n << " = *(const lv" << n << "_t*)(p" << pslot.at(e.tensor) << " + (" << c.addr_expr(e.addr) << "));\n";
        ov[n] = "cvt_in(lv" + std::to_string(n) + "[e])";
      }
      std::vector<bool> vstore;
      for (size_t i = 0; i < c.stores.size(); i++) {
        const Store& st_ = c.stores[i];
        bool v = 16 / dtype_bytes(g.tensors[st_.tensor].dtype) >= V && chan_contig(st_.addr, V);
        for (auto& pr : st_.preds) {
          std::vector<int> r;
          c.resolve(pr.atoms, r);
          if (std::find(r.begin(), r.end(), ca) != r.end()) v = false;
        }
        vstore.push_back(v);
        if (v && st_.tensor == pool_src && st_.preds.empty()) pool_vec_ok = true;
        if (v)
          k << "      typedef " << c.ctype(g.tensors[st_.tensor].dtype) << " sv" << i << "_t __attribute__((ext_vector_type(" << V
            << ")));\n      sv" << i << "_t sv" << i << ";\n";
      }
      k << "      {\n#pragma unroll\n      for (int e = 0; e < " << V << "; ++e) {\n";
      if (ca >= 0) k << "        const idx_t a" << ca << " = c0_ + e;\n";
      k << "        const float anchor_v = " << acc_expr << ";\n";
      {
        std::set<int> done;
        std::vector<int> roots;
        for (auto& st_ : c.stores) roots.push_back(st_.value);
        c.emit_values(k, roots, done, pslot, "        ", &ov);
        for (size_t i = 0; i < c.stores.size(); i++) {
          const Store& st_ = c.stores[i];
          if (vstore[i]) {
            k << "        { " << c.ctype(g.tensors[st_.tensor].dtype) << " tmp; cvt_out(&tmp, " << c.vname(st_.value) << "); sv" << i << "[e] = tmp;"
              << (st_.tensor == pool_src ? " pool_acc[e] += cvt_in(tmp);" : "") << " }\n";
          } else {
            std::string stt = c.store_stmt(st_, pslot, c.addr_expr(st_.addr));
            if (st_.preds.empty()) k << "        " << stt << "\n";
            else k << "        if (" << c.pred_expr(st_.preds) << ") { " << stt << " }\n";
          }
        }
      }
      k << "      }\n      }\n";
      for (size_t i = 0; i < c.stores.size(); i++) {
        if (!vstore[i]) continue;
        const Store& st_ = c.stores[i];
        std::string stt = "*(sv" + std::to_string(i) + "_t*)(p" + std::to_string(pslot.at(st_.tensor)) + " + (" + c.addr_expr(st_.addr) + ")) = sv" + std::to_string(i) + ";";
        if (st_.preds.empty()) k << "      " << stt << "\n";
        else k << "      if (" << c.pred_expr(st_.preds) << ") { " << stt << " }\n";
      }
      k << "      }\n      }\n";
      };
      // One tap for V channels: acc[e] += x[e] * w[e] in fp32.  For fp16 data that is two v_fma_mix_f32 per packed
      // pair (the instruction reads either half of a register as fp16 and accumulates in fp32), a third of the
      // convert-convert-multiply-add sequence the compiler otherwise builds from the element-wise expression -
      // and these kernels are bound by vector instruction issue, not by memory.
      k << "typedef " << c.ctype(XT.dtype) << " xvec_t __attribute__((ext_vector_type(" << V << ")));\n";
      if (XT.dtype == DNNF_F16) {
        k << "typedef unsigned int dwu4_t __attribute__((ext_vector_type(4)));\n";
        k << "DEV void mac_vec(float* acc, const xvec_t x, const xvec_t w) {\n";
        k << "  const dwu4_t xu = __builtin_bit_cast(dwu4_t, x), wu = __builtin_bit_cast(dwu4_t, w);\n";
        k << "#pragma unroll\n  for (int q = 0; q < 4; ++q) {\n";
        k << "    asm(\"v_fma_mix_f32 %0, %1, %2, %0 op_sel_hi:[1,1,0]\" : \"+v\"(acc[2 * q]) : \"v\"(xu[q]), \"v\"(wu[q]));\n";
        k << "    asm(\"v_fma_mix_f32 %0, %1, %2, %0 op_sel:[1,1,0] op_sel_hi:[1,1,0]\" : \"+v\"(acc[2 * q + 1]) : \"v\"(xu[q]), \"v\"(wu[q]));\n";
        k << "  }\n}\n";
      } else {
        k << "DEV void mac_vec(float* acc, const xvec_t x, const xvec_t w) {\n#pragma unroll\n  for (int e = 0; e < " << V
          << "; ++e) acc[e] += cvt_in(x[e]) * cvt_in(w[e]);\n}\n";
      }
      if (use_lds) {
        const int XC = ldsXC, TH = ldsTH, TW = ldsTW, PS = 256 / XC, CB = XC * V;
        const int IH = (TH - 1) * (int)SH + (int)KH, IW = (TW - 1) * (int)SW + (int)KW;
        const int NLD = (IH * IW + PS - 1) / PS, NIT = (TH * TW + PS - 1) / PS, KK = (int)(KH * KW);
        const int64_t NCHK = (CV + XC - 1) / XC, NTH = HO / TH, NTW = WO / TW;
        const std::string xt = c.ctype(XT.dtype);
        k << "extern \"C\" __global__ __launch_bounds__(256) void KNAME(" << kparams << ") {\n";
        k << "  typedef " << xt << " xvec_t __attribute__((ext_vector_type(" << V << ")));\n";
        k << "  __shared__ __attribute__((aligned(16))) " << xt << " in_s[" << IH * IW * CB << "];\n";
        k << "  const int tid = threadIdx.x, cvl = tid % " << XC << ", slot = tid / " << XC << ";\n";
        k << "  idx_t bid = blockIdx.x;\n";
        k << "  const idx_t tw = bid % " << NTW << "; bid /= " << NTW << ";\n";
        k << "  const idx_t th = bid % " << NTH << "; bid /= " << NTH << ";\n";
        k << "  const idx_t chunk = bid % " << NCHK << ";\n  const idx_t on = bid / " << NCHK << ";\n";
        k << "  const idx_t cv = chunk * " << XC << " + cvl;\n";
        k << "  const bool cok = " << (CV % XC == 0 ? std::string("true") : "cv < " + std::to_string(CV)) << ";\n";
        k << "  const idx_t oc0 = (cok ? cv : 0) * " << V << ";     // lanes past the last channel vector read in bounds and store nothing\n";
        k << "  const idx_t a" << xn << " = on, a" << xc << " = oc0;\n";
        k << "  const int h0 = (int)th * " << TH * SH << " - " << PT << ", w0 = (int)tw * " << TW * SW << " - " << PL << ";\n";
        k << "  xvec_t stage[" << NLD << "];\n";
        k << "#pragma unroll\n  for (int i = 0; i < " << NLD << "; ++i) {\n";
        k << "    const int pix = slot + " << PS << " * i;\n";
        k << "    const int h_ = h0 + pix / " << IW << ", w_ = w0 + pix % " << IW << ";\n";
        k << "    const idx_t a" << xh << " = min(max(h_, 0), " << H - 1 << "), a" << xw << " = min(max(w_, 0), " << Wd - 1 << ");\n";
        k << "    stage[i] = *(const xvec_t*)(" << px << " + (" << c.addr_expr(xaddr_c) << "));      // clamped address: no branch in front of the load\n";
        k << "    if (!(h_ >= 0 && h_ < " << H << " && w_ >= 0 && w_ < " << Wd << ")) {\n#pragma unroll\n      for (int e = 0; e < " << V << "; ++e) stage[i][e] = 0;\n    }\n  }\n";
        k << "  xvec_t wv[" << KK << "];\n";
        k << "#pragma unroll\n  for (int t = 0; t < " << KK << "; ++t) {\n";
        k << "    const idx_t a" << wkh << " = t / " << KW << ", a" << wkw << " = t % " << KW << ";\n";
        k << "    wv[t] = *(const xvec_t*)(" << pw << " + (" << c.addr_expr(waddr) << "));\n  }\n";
        k << "#pragma unroll\n  for (int i = 0; i < " << NLD << "; ++i) {\n";
        k << "    const int pix = slot + " << PS << " * i;\n";
        k << "    if (pix < " << IH * IW << ") *(xvec_t*)&in_s[(pix * " << XC << " + cvl) * " << V << "] = stage[i];\n  }\n";
        k << "  __syncthreads();\n";
        if (pool_dst >= 0) k << "  float pool_acc[" << V << "];\n#pragma unroll\n  for (int e = 0; e < " << V << "; ++e) pool_acc[e] = 0.0f;\n";
        k << "#pragma unroll 1\n  for (int it = 0; it < " << NIT << "; ++it) {\n";
        k << "    const int p = slot + " << PS << " * it;\n    if (p < " << TH * TW << " && cok) {\n";
        k << "      const int oh = p / " << TW << ", ow = p % " << TW << ";\n";
        k << "      float acc[" << V << "];\n#pragma unroll\n      for (int e = 0; e < " << V << "; ++e) acc[e] = "
          << (bslot >= 0 ? "cvt_in(p" + std::to_string(bslot) + "[oc0 + e])" : std::string("0.0f")) << ";\n";
        k << "#pragma unroll\n      for (int i = 0; i < " << KH << "; ++i)\n#pragma unroll\n        for (int j = 0; j < " << KW << "; ++j) {\n";
        k << "          const xvec_t xv = *(const xvec_t*)&in_s[(((oh * " << SH << " + i) * " << IW << " + ow * " << SW << " + j) * " << XC << " + cvl) * " << V << "];\n";
        k << "          mac_vec(acc, xv, wv[i * " << KW << " + j]);\n        }\n";
        chan_epilogue("on", "th * " + std::to_string(TH) + " + oh", "tw * " + std::to_string(TW) + " + ow", "acc[e]");
        k << "    }\n  }\n";
        if (pool_dst >= 0) {
          // The workgroup has seen every pixel of its image for its CB channels: a lane's sums (of the values as stored)
          // meet the other pixel slots' in LDS, and one lane per channel writes the mean.
          DNNF_CHECK(NTH == 1 && NTW == 1 && pool_vec_ok, DNNF_UNSUPPORTED_OP, "the pool joins a depthwise convolution only when one workgroup's patch is the whole image plane");
          const std::string pt = c.ctype(g.tensors[pool_dst].dtype);
          k << "  __shared__ float pool_red[" << PS * CB << "];\n";
          k << "#pragma unroll\n  for (int e = 0; e < " << V << "; ++e) pool_red[slot * " << CB << " + cvl * " << V << " + e] = pool_acc[e];\n";
          k << "  __syncthreads();\n";
          k << "  if (tid < " << CB << ") {\n    float s_ = 0.0f;\n    for (int sl = 0; sl < " << PS << "; ++sl) s_ += pool_red[sl * " << CB << " + tid];\n";
          k << "    const idx_t ch = chunk * " << CB << " + tid;\n";
          k << "    if (ch < " << C << ") { " << pt << " o_; cvt_out(&o_, s_ * " << std::scientific << 1.0 / (double)(HO * WO) << std::defaultfloat << "f); p" << pslot.at(pool_dst)
            << "[on * " << C << " + ch] = o_; }\n  }\n";
        }
        k << "}\n";
        Lw.family = FAM_DWCONV;
        Kn.grid[0] = (unsigned)(N * NCHK * NTH * NTW);
        Lw.variant = "dw_lds" + std::to_string(TH) + "x" + std::to_string(TW) + "c" + std::to_string(CB) + "_" + std::to_string(KH) + "x" + std::to_string(KW) + "s" + std::to_string(SH) +
                     (pool_dst >= 0 ? "_pool" : "");
      } else {
      k << "extern \"C\" __global__ __launch_bounds__(256) void KNAME(" << kparams << ") {\n";
      k << "  const idx_t gid = (idx_t)blockIdx.x * 256 + threadIdx.x;\n  if (gid >= (idx_t)" << ctotal << ") return;\n";
      k << "  idx_t rem = gid;\n";
      k << "  const idx_t oc0 = (rem % " << CV << ") * " << V << "; rem /= " << CV << ";\n";
      k << "  const idx_t qt = rem % " << QTn << "; rem /= " << QTn << ";\n";
      k << "  const idx_t pt = rem % " << PTn << "; rem /= " << PTn << ";\n";
      k << "  const idx_t on = rem;\n";
      k << "  typedef " << c.ctype(XT.dtype) << " xvec_t __attribute__((ext_vector_type(" << V << ")));\n";
      k << "  float acc[" << TPc << "][" << TQc << "][" << V << "];\n";
      k << "#pragma unroll\n  for (int t = 0; t < " << TPc << "; ++t)\n#pragma unroll\n    for (int u = 0; u < " << TQc << "; ++u)\n#pragma unroll\n"
        << "      for (int e = 0; e < " << V << "; ++e) acc[t][u][e] = "
        << (bslot >= 0 ? "cvt_in(p" + std::to_string(bslot) + "[oc0 + e])" : std::string("0.0f")) << ";\n";
      k << "  const idx_t a" << xn << " = on, a" << xc << " = oc0;\n";
      k << "#pragma unroll\n  for (int rr = 0; rr < " << Rc << "; ++rr) {\n";
      k << "    const int a" << xh << "_ = (int)pt * " << TPc * SH << " + rr - " << PT << ";\n";
      k << "    const idx_t a" << xh << " = min(max(a" << xh << "_, 0), " << H - 1 << ");\n";
      k << "    xvec_t wr[" << TPc << "][" << KW << "];\n";
      k << "#pragma unroll\n    for (int t = 0; t < " << TPc << "; ++t) {\n      const int i = rr - t * " << SH << ";\n";
      k << "      if (i >= 0 && i < " << KH << ") {\n#pragma unroll\n        for (int j = 0; j < " << KW << "; ++j) {\n";
      k << "          const idx_t a" << wkh << " = i, a" << wkw << " = j;\n";
      k << "          wr[t][j] = *(const xvec_t*)(" << pw << " + (" << c.addr_expr(waddr) << "));\n        }\n      }\n    }\n";
      // padding without branches (clamped address, zeroed value): all taps' loads are in flight together
      k << "    const bool hin = a" << xh << "_ >= 0 && a" << xh << "_ < " << H << ";\n";
      k << "    {\n";
      k << "#pragma unroll\n      for (int jj = 0; jj < " << WINQ << "; ++jj) {\n";
      k << "        const int w_ = (int)qt * " << TQc * SW << " + jj - " << PL << ";\n";
      k << "        const idx_t a" << xw << " = min(max(w_, 0), " << Wd - 1 << ");\n";
      k << "        {\n";
      k << "          xvec_t xv = *(const xvec_t*)(" << px << " + (" << c.addr_expr(xaddr_c) << "));\n";
      k << "          if (!(hin && w_ >= 0 && w_ < " << Wd << ")) {\n#pragma unroll\n            for (int e = 0; e < " << V << "; ++e) xv[e] = 0;\n          }\n";
      k << "#pragma unroll\n          for (int t = 0; t < " << TPc << "; ++t) {\n            const int i = rr - t * " << SH << ";\n";
      k << "            if (i >= 0 && i < " << KH << ") {\n#pragma unroll\n              for (int u = 0; u < " << TQc << "; ++u) {\n";
      k << "                const int j = jj - u * " << SW << ";\n                if (j >= 0 && j < " << KW << ") {\n";
      k << "                  mac_vec(acc[t][u], xv, wr[t][j]);\n";
      k << "                }\n              }\n            }\n          }\n        }\n      }\n    }\n  }\n";
      k << "#pragma unroll\n  for (int t = 0; t < " << TPc << "; ++t)\n#pragma unroll\n    for (int u = 0; u < " << TQc << "; ++u) {\n";
      chan_epilogue("on", "pt * " + std::to_string(TPc) + " + t", "qt * " + std::to_string(TQc) + " + u", "acc[t][u][e]");
      k << "    }\n}\n";
      Lw.family = FAM_DWCONV;
      Kn.grid[0] = (unsigned)((ctotal + 255) / 256);
      Lw.variant = "dw_chan" + std::to_string(TPc) + "x" + std::to_string(TQc) + "_" + std::to_string(KH) + "x" + std::to_string(KW) + "s" + std::to_string(SH);
      }
    } else if (VW) {
      const int64_t qv = WO / VW, vtotal = N * C * ptiles * qv;
      const int RH = (int)std::max<int64_t>(0, KW - SW - PL), SPAN = VW * (int)SW, WIN = (int)PL + SPAN + RH;
      const Tensor& XT = g.tensors[c.nodes[xnode].tensor];
      const std::string px = "p" + std::to_string(pslot.at(c.nodes[xnode].tensor));
      const int qa = out_atoms[3][0], pa = out_atoms[2][0];
      k << "extern \"C\" __global__ __launch_bounds__(256) void KNAME(" << kparams << ") {\n";
      k << "  const idx_t gid = (idx_t)blockIdx.x * 256 + threadIdx.x;\n  if (gid >= (idx_t)" << vtotal << ") return;\n";
      k << "  idx_t rem = gid;\n";
      k << "  const idx_t oq0 = (rem % " << qv << ") * " << VW << "; rem /= " << qv << ";\n";
      k << "  const idx_t pt = rem % " << ptiles << "; rem /= " << ptiles << ";\n";
      peel(out_atoms[1]);
      peel(out_atoms[0]);
      k << "  const idx_t on = " << digit(0) << ", oc = " << digit(1) << ";\n";
      k << "  float w[" << KH * KW << "];\n#pragma unroll\n  for (int t = 0; t < " << KH * KW << "; ++t) w[t] = cvt_in(p" << wslot
        << "[oc * " << w_chan_stride << " + t * " << w_tap_stride << "]);\n";
      k << "  float acc[" << TP << "][" << VW << "];\n#pragma unroll\n  for (int t = 0; t < " << TP << "; ++t)\n#pragma unroll\n"
        << "    for (int u = 0; u < " << VW << "; ++u) acc[t][u] = "
        << (bslot >= 0 ? "cvt_in(p" + std::to_string(bslot) + "[oc])" : std::string("0.0f")) << ";\n";
      k << "  const idx_t a" << xn << " = on, a" << xc << " = oc;\n";
      k << "  typedef " << c.ctype(XT.dtype) << " xvec_t __attribute__((ext_vector_type(" << SPAN << ")));\n";
      k << "#pragma unroll\n  for (int rr = 0; rr < " << R << "; ++rr) {\n";
      // rows and halo columns outside the map: clamped address, value zeroed afterwards (no load behind a branch)
      k << "    const int h_ = (int)pt * " << TP * SH << " + rr - " << PT << ";\n";
      k << "    const bool hin = h_ >= 0 && h_ < " << H << ";\n";
      k << "    const idx_t a" << xh << " = min(max(h_, 0), " << H - 1 << ");\n";
      k << "    float win[" << WIN << "];\n";
      k << "    {\n";
      k << "      {\n        const idx_t a" << xw << " = oq0 * " << SW << ";\n";
      k << "        const xvec_t xv = *(const xvec_t*)(" << px << " + (" << c.addr_expr(xaddr) << "));\n";
      k << "#pragma unroll\n        for (int u = 0; u < " << SPAN << "; ++u) win[" << PL << " + u] = hin ? cvt_in(xv[u]) : 0.0f;\n      }\n";
      if (PL > 0) {
        k << "#pragma unroll\n      for (int l = 0; l < " << PL << "; ++l) {\n";
        k << "        const int w_ = (int)oq0 * " << SW << " - " << PL << " + l;\n        const idx_t a" << xw << " = max(w_, 0);\n";
        k << "        const float hv = cvt_in(" << px << "[" << c.addr_expr(xaddr) << "]);\n        win[l] = (hin && w_ >= 0) ? hv : 0.0f;\n      }\n";
      }
      if (RH > 0) {
        k << "#pragma unroll\n      for (int l = 0; l < " << RH << "; ++l) {\n";
        k << "        const int w_ = (int)oq0 * " << SW << " + " << SPAN << " + l;\n        const idx_t a" << xw << " = min(w_, " << Wd - 1 << ");\n";
        k << "        const float hv = cvt_in(" << px << "[" << c.addr_expr(xaddr) << "]);\n        win[" << PL + SPAN << " + l] = (hin && w_ < " << Wd << ") ? hv : 0.0f;\n      }\n";
      }
      k << "    }\n";
      k << "#pragma unroll\n    for (int t = 0; t < " << TP << "; ++t) {\n";
      k << "      const int i = rr - t * " << SH << ";\n";
      k << "      if (i >= 0 && i < " << KH << ") {\n#pragma unroll\n        for (int j = 0; j < " << KW << "; ++j)\n#pragma unroll\n"
        << "          for (int u = 0; u < " << VW << "; ++u) acc[t][u] += win[u * " << SW << " + j] * w[i * " << KW << " + j];\n      }\n    }\n  }\n";
      // epilogue: VW results per row; stores that run along q leave as one vector
      std::vector<bool> vstore;
      for (auto& st_ : c.stores) {
        Affine sa = c.resolved(st_.addr);
        auto it = sa.stride.find(qa);
        bool v = it != sa.stride.end() && it->second == 1 && sa.offset % VW == 0 && sa.indirect.empty();
        for (auto& kv : sa.stride) if (kv.first != qa && kv.second % VW) v = false;
        for (auto& pr : st_.preds) {
          std::vector<int> r;
          c.resolve(pr.atoms, r);
          if (std::find(r.begin(), r.end(), qa) != r.end()) v = false;
        }
        vstore.push_back(v);
      }
      k << "#pragma unroll\n  for (int t = 0; t < " << TP << "; ++t) {\n";
      k << "    const idx_t a" << pa << " = pt * " << TP << " + t;\n";
      k << "    if (a" << pa << " < " << HO << ") {\n";
      for (size_t i = 0; i < c.stores.size(); i++)
        if (vstore[i])
          k << "      typedef " << c.ctype(g.tensors[c.stores[i].tensor].dtype) << " sv" << i << "_t __attribute__((ext_vector_type(" << VW
            << ")));\n      sv" << i << "_t sv" << i << ";\n";
      k << "#pragma unroll\n      for (int u = 0; u < " << VW << "; ++u) {\n";
      k << "        const idx_t a" << qa << " = oq0 + u;\n        const float anchor_v = acc[t][u];\n";
      {
        std::set<int> done;
        std::vector<int> roots;
        for (auto& st_ : c.stores) roots.push_back(st_.value);
        c.emit_values(k, roots, done, pslot, "        ");
        for (size_t i = 0; i < c.stores.size(); i++) {
          const Store& st_ = c.stores[i];
          if (vstore[i]) {
            k << "        { " << c.ctype(g.tensors[st_.tensor].dtype) << " tmp; cvt_out(&tmp, " << c.vname(st_.value) << "); sv" << i << "[u] = tmp; }\n";
          } else {
            std::string stt = c.store_stmt(st_, pslot, c.addr_expr(st_.addr));
            if (st_.preds.empty()) k << "        " << stt << "\n";
            else k << "        if (" << c.pred_expr(st_.preds) << ") { " << stt << " }\n";
          }
        }
      }
      k << "      }\n";
      k << "      {\n        const idx_t a" << qa << " = oq0;\n";
      for (size_t i = 0; i < c.stores.size(); i++) {
        if (!vstore[i]) continue;
        const Store& st_ = c.stores[i];
        std::string stt = "*(sv" + std::to_string(i) + "_t*)(p" + std::to_string(pslot.at(st_.tensor)) + " + (" + c.addr_expr(st_.addr) + ")) = sv" + std::to_string(i) + ";";
        if (st_.preds.empty()) k << "        " << stt << "\n";
        else k << "        if (" << c.pred_expr(st_.preds) << ") { " << stt << " }\n";
      }
      k << "      }\n    }\n  }\n}\n";
      Lw.family = FAM_DWCONV;
      Kn.grid[0] = (unsigned)((vtotal + 255) / 256);
      Lw.variant = "dw_tile" + std::to_string(TP) + "x" + std::to_string(VW) + "_" + std::to_string(KH) + "x" + std::to_string(KW) + "s" + std::to_string(SH);
    } else {
    k << "extern \"C\" __global__ __launch_bounds__(256) void KNAME(" << kparams << ") {\n";
    k << "  const idx_t gid = (idx_t)blockIdx.x * 256 + threadIdx.x;\n  if (gid >= (idx_t)" << total << ") return;\n";
    k << "  idx_t rem = gid;\n";
    peel(out_atoms[3]);
    k << "  const idx_t pt = rem % " << ptiles << "; rem /= " << ptiles << ";\n";
    peel(out_atoms[1]);
    peel(out_atoms[0]);
    if (TP == 1) decl_digits(k, c, out_atoms[2], "pt", "  ", "qp");
    k << "  const idx_t on = " << digit(0) << ", oc = " << digit(1) << ", oq = " << digit(3) << ";\n";
    k << "  float w[" << KH * KW << "];\n#pragma unroll\n  for (int t = 0; t < " << KH * KW << "; ++t) w[t] = cvt_in(p" << wslot
      << "[oc * " << w_chan_stride << " + t * " << w_tap_stride << "]);\n";
    k << "  float acc[" << TP << "];\n#pragma unroll\n  for (int t = 0; t < " << TP << "; ++t) acc[t] = "
      << (bslot >= 0 ? "cvt_in(p" + std::to_string(bslot) + "[oc])" : std::string("0.0f")) << ";\n";
    k << "  const idx_t a" << xn << " = on, a" << xc << " = oc;\n";
    k << "#pragma unroll\n  for (int rr = 0; rr < " << R << "; ++rr) {\n";
    k << "    const int h_ = (int)pt * " << TP * SH << " + rr - " << PT << ";\n";
    k << "    const idx_t a" << xh << " = min(max(h_, 0), " << H - 1 << ");\n";
    k << "#pragma unroll\n    for (int j = 0; j < " << KW << "; ++j) {\n";
    k << "      const int w_ = (int)oq * " << SW << " + j - " << PL << ";\n";
    k << "      const idx_t a" << xw << " = min(max(w_, 0), " << Wd - 1 << ");\n";
    k << "      float xv;\n";
    k << "      {\n";
    k << c.decl_parts(xatoms, "        ");
    {
      std::set<int> done;
      c.emit_values(k, {xnode}, done, pslot, "        ");
    }
    k << "        xv = (h_ >= 0 && h_ < " << H << " && w_ >= 0 && w_ < " << Wd << ") ? " << c.vname(xnode) << " : 0.0f;\n      }\n";
    k << "#pragma unroll\n      for (int t = 0; t < " << TP << "; ++t) {\n";
    k << "        const int i = rr - t * " << SH << ";\n";
    k << "        if (i >= 0 && i < " << KH << ") acc[t] += xv * w[i * " << KW << " + j];\n      }\n    }\n  }\n";
    if (TP == 1) {
      k << "  const float anchor_v = acc[0];\n";
      emit_epilogue_body(k, "  ");
    } else {
      k << "#pragma unroll\n  for (int t = 0; t < " << TP << "; ++t) {\n";
      k << "    const idx_t a" << out_atoms[2][0] << " = pt * " << TP << " + t;\n";
      k << "    if (a" << out_atoms[2][0] << " < " << HO << ") {\n      const float anchor_v = acc[t];\n";
      emit_epilogue_body(k, "      ");
      k << "    }\n  }\n";
    }
    k << "}\n";
    Lw.family = FAM_DWCONV;
    Kn.grid[0] = (unsigned)((total + 255) / 256);
    Lw.variant = "dw_rows" + std::to_string(TP) + "_" + std::to_string(KH) + "x" + std::to_string(KW) + "s" + std::to_string(SH);
    }
  } else {
    // ---- implicit GEMM: rows = output channels, columns = (n, p, q), K = (ci, kh, kw)
    const int64_t K = C * KH * KW, GM = CO, GN = N * HO * WO;
    const int eb = dtype_bytes(X.dtype), VEC = eb == 2 ? 8 : 4;
    std::vector<int> rows = out_atoms[1], cols;
    for (int d : {0, 2, 3}) cols.insert(cols.end(), out_atoms[d].begin(), out_atoms[d].end());
    DNNF_CHECK(rows.size() <= 1, DNNF_UNSUPPORTED_OP, "output channel axis was split by a reshape in the block");
    const int katom = c.new_atom(std::max<int64_t>(K, 2));
    Affine aa;   // weight matrix [CO, K]
    if (!rows.empty()) aa.stride[rows[0]] = K;
    aa.stride[katom] = 1;
    // The operand of a pointwise convolution is an affine function of (column, k) when it is a stored tensor,
    // or One-to-One operators over one stored tensor that has the operand's index space (the main load) and
    // over tensors that are constant across the image plane (a squeeze-excite scale, per-channel constants):
    // those operators then run on the loaded vectors on their way into LDS (operand prologue).
    int main_load = -1;
    bool prologue = false;
    if (c.nodes[xnode].kind == ENode::LOAD) main_load = xnode;
    else if (c.nodes[xnode].kind == ENode::OP) {
      std::set<int> seen;
      std::vector<int> stack = {xnode};
      bool ok = true;
      while (!stack.empty() && ok) {
        int n = stack.back();
        stack.pop_back();
        if (seen.count(n)) continue;
        seen.insert(n);
        const ENode& e = c.nodes[n];
        if (e.kind == ENode::ANCHOR) ok = false;
        if (e.kind == ENode::LOAD) {
          Affine la = c.resolved(e.addr);
          const bool plane = (la.stride.count(xh) && la.stride.at(xh) != 0) || (la.stride.count(xw) && la.stride.at(xw) != 0);
          if (!e.addr.indirect.empty() || e.is_int) ok = false;
          else if (plane) { if (main_load >= 0) ok = false; main_load = n; }
        }
        for (int a : e.args) stack.push_back(a);
      }
      if (!ok || main_load < 0 || g.tensors[c.nodes[main_load].tensor].dtype != X.dtype) main_load = -1;
      prologue = main_load >= 0;
    }
    bool pointwise = !x_cut && KH == 1 && KW == 1 && SH == 1 && SW == 1 && PT == 0 && PL == 0 && pd[2] == 0 && pd[3] == 0 &&
                           main_load >= 0 && c.nodes[main_load].addr.indirect.empty();
    int amode = (K % VEC == 0) ? 0 : 2, bmode = 3;
    // A convolution with few outputs (the squeeze-and-excitation layers: 1x1 spatial, batch x channels
    // results) is a handful of dot products: one wavefront per output element, lanes striding over K,
    // finishes in one memory round trip where a tiled GEMM would walk K tile by tile in one workgroup.
    const bool dot = GM * GN <= 65536 && GM * GN * K <= ((int64_t)8 << 20) && c.rep_atoms.empty();
    int bcvec = 0;
    if (dot) pointwise = false;
    Affine ab;
    if (pointwise) {
      // x[n, ci, p, q] with ci = k: substitute the conv-input atoms by output / k atoms
      Affine xa = c.resolved(c.nodes[main_load].addr);
      ab.offset = xa.offset;
      auto put = [&](const std::vector<int>& outs, int xatom) {
        int64_t s = 0;
        auto it = xa.stride.find(xatom);
        if (it != xa.stride.end()) s = it->second;
        int64_t mult = 1;
        for (int i = (int)outs.size() - 1; i >= 0; i--) { ab.stride[outs[i]] += s * mult; mult *= c.atom_extent[outs[i]]; }
      };
      put(out_atoms[0], xn);
      put(out_atoms[2], xh);
      put(out_atoms[3], xw);
      auto it = xa.stride.find(xc);
      ab.stride[katom] = it == xa.stride.end() ? 0 : it->second;
      // channels-last operand: K-contiguous like the weights, 16-byte vectors straight into the operand tile
      bool kdirect = ab.stride[katom] == 1 && K % VEC == 0 && ab.offset % VEC == 0;
      for (auto& kv : ab.stride) if (kv.first != katom && kv.second % VEC) kdirect = false;
      // a vector of VEC pixels may run over several trailing column atoms as long as they are contiguous
      int64_t run = 1;
      std::set<int> in_run;            // trailing column atoms that form one contiguous index
      for (int i = (int)cols.size() - 1; i >= 0 && ab.stride[cols[i]] == run; i--) { run *= c.atom_extent[cols[i]]; in_run.insert(cols[i]); }
      // widest pixel vector (16 or 8 bytes) that never straddles a plane and is always aligned
      for (int cv = VEC; cv >= VEC / 2 && !bcvec; cv /= 2) {
        bool col_contig = !cols.empty() && ab.stride[cols.back()] == 1 && run % cv == 0 && GN % cv == 0;
        bool al = ab.offset % cv == 0;
        for (auto& kv : ab.stride) if (!in_run.count(kv.first) && kv.second % cv) al = false;
        if (col_contig && al) bcvec = cv;
      }
      // without vectors along the pixels the gathering loader (lanes along pixels) coalesces better
      // than the generic scalar one (lanes along K)
      if (kdirect) { bmode = 0; bcvec = 0; }
      else if (bcvec && !prologue) bmode = 1;
      else { bmode = 3; pointwise = false; }        // (a prologue is generated for K-contiguous vectors only)
    }
    if (!pointwise) prologue = false;
    // Filters re-laid [co, kh, kw, ci] by data-format selection: K runs tap by tap.  With a stored channels-last
    // operand every K vector is VEC channels of one tap (tap loader, B_MODE 4); any other operand is gathered
    // element by element in the same K order.
    const bool k_taps_major = Wt.perm == std::vector<int>{0, 2, 3, 1} && KH * KW > 1;
    Affine xaddr_t;
    if (k_taps_major && !x_cut && !pointwise && !dot && c.nodes[xnode].kind == ENode::LOAD && !c.nodes[xnode].is_int && c.nodes[xnode].addr.indirect.empty() &&
        g.tensors[c.nodes[xnode].tensor].dtype == X.dtype && C % VEC == 0) {
      xaddr_t = c.resolved(c.nodes[xnode].addr);
      auto itc = xaddr_t.stride.find(xc);
      bool ok = itc != xaddr_t.stride.end() && itc->second == 1 && xaddr_t.offset % VEC == 0;
      for (auto& kv : xaddr_t.stride) if (kv.first != xc && kv.second % VEC) ok = false;
      if (ok) bmode = 4;
    }
    // Tile configurations, largest first.  These products are short (K of 16 to 1152) and bound by memory
    // and by the latency of a tile's load - multiply - store chain rather than by the matrix cores, so the
    // default is the largest tile that still gives every compute unit about three workgroups to overlap;
    // a tuning build times all of them on the device instead (force_variant = 100 + index).
    auto nblocks = [&](int bm, int bn) { return ((GM + bm - 1) / bm) * ((GN + bn - 1) / bn); };
    int BK = eb == 2 ? (K <= 32 ? 32 : 64) : 16;
    struct Tile { int BM, BN, WM, WN, WK, BK; bool direct = false; };
    std::vector<Tile> tiles;
    // few output channels: a tile as tall as the channel count (four wavefronts side by side), so that a pixel's
    // channels are written by one workgroup as one contiguous run and no accumulator rows are staged for nothing
    if (GM <= 32) tiles.push_back({32, 128, 1, 4, 1, BK});
    else if (GM > 64 && GM <= 96) tiles.push_back({96, 128, 1, 4, 1, BK});
    if (GM > 64) { tiles.push_back({128, 128, 2, 2, 1, BK}); tiles.push_back({128, 64, 2, 2, 1, BK}); }
    tiles.push_back({64, 128, 2, 2, 1, BK});
    tiles.push_back({64, 64, 2, 2, 1, BK});
    if (K >= 8 * BK) tiles.push_back({32, 32, 1, 1, 4, BK});
    size_t pick = tiles.size() - 1;
    // the K-split tile without LDS staging (fp32, gathered operand): a lane keeps its share of both operands in
    // registers, two values per channel pair and tap
    const int cd_j = (int)((C + 7) / 8);
    const bool direct_ok = eb == 4 && !pointwise && !dot && bmode == 3 && !k_taps_major && K >= 64 && (int64_t)cd_j * KH * KW * 2 <= 176;
    if (direct_ok) tiles.push_back({32, 32, 1, 1, 4, BK, true});
    const size_t direct_idx = tiles.size() - 1;
    const size_t n_default = tiles.size();

    if (c.opts.force_variant >= 100) {
      DNNF_CHECK(!dot && c.opts.force_variant - 100 < (int)tiles.size(), DNNF_UNSUPPORTED_OP, "no such convolution tile variant");
      pick = (size_t)(c.opts.force_variant - 100);
    } else {
      for (size_t i = 0; i < n_default; i++)
        if (tiles[i].WK == 1 && nblocks(tiles[i].BM, tiles[i].BN) >= 768) { pick = i; break; }
      if (tiles[pick].WK == 4 && nblocks(64, 64) >= 192) pick--;     // K-split tiles only for problems that cannot fill the chip otherwise
      if (tiles[pick].WK == 4 && direct_ok) pick = direct_idx;
    }
    const bool direct = tiles[pick].direct;
    int BM = tiles[pick].BM, BN = tiles[pick].BN, WAVES_M = tiles[pick].WM, WAVES_N = tiles[pick].WN, WAVES_K = tiles[pick].WK;
    BK = tiles[pick].BK;
    // a K-split kernel is a chain of dependent K steps: fewer, longer steps keep more loads in flight
    if (WAVES_K == 4 && eb == 4 && K >= 256) BK = 64;
    // the pointer the template calls PB is only dereferenced by the affine loaders
    k << "typedef " << c.ctype(X.dtype) << " elem_t;\n";
    k << "#define ELEM_BYTES " << eb << "\n#define BM " << BM << "\n#define BN " << BN << "\n#define BK " << BK << "\n";
    k << "#define GM " << GM << "\n#define GN " << GN << "\n#define GK " << K << "\n";
    k << "#define WAVES_M " << WAVES_M << "\n#define WAVES_N " << WAVES_N << "\n#define WAVES_K " << WAVES_K
      << (K <= BK ? "\n#define NBUF 1\n#define PF 1\n" : "\n#define NBUF 2\n#define PF 2\n");   // a single K tile needs no second buffer
    k << "#define A_MODE " << amode << "\n#define B_MODE " << bmode << "\n#define PA p" << wslot << "\n";
    {
      // the filter matrix was last read an inference ago: every XCD touches all of it up front (see the MatMul template)
      const int64_t wbytes = Wt.n() * dtype_bytes(Wt.dtype);
      const char* e = getenv("DNNF_CONV_PREFETCH_KB");       // (developer switch for A/B runs: smallest filter, 0 = never)
      const int64_t min_kb = e ? atoll(e) : 64;
      if (!dot && !direct && min_kb > 0 && wbytes >= (min_kb << 10) && wbytes <= ((int64_t)16 << 20) && wbytes % 128 == 0)
        k << "#define W_PREFETCH_LINES " << wbytes / 128 << "\n#define W_PREFETCH_PTR p" << wslot << "\n";
    }
    if (bcvec) k << "#define B_CVEC " << bcvec << "\n";
    if (direct) {
      k << "#define CONV_DIRECT 1\n#define CD_TAPS " << KH * KW << "\n#define CD_J " << cd_j << "\n#define CD_C " << C << "\n";
    }
    k << "#define PB p" << (pointwise ? pslot[c.nodes[main_load].tensor] : wslot) << "\n";
    if (X.dtype == DNNF_F16) k << "typedef f16x8 frag_t;\n#define MFMA __builtin_amdgcn_mfma_f32_32x32x16_f16\n";
    else if (X.dtype == DNNF_BF16) k << "typedef bf16x8 frag_t;\n#define MFMA __builtin_amdgcn_mfma_f32_32x32x16_bf16\n";
    k << gemm_offset_fn(c, "offA_row", rows, aa) << gemm_offset_fn(c, "offA_k", {katom}, aa) << gemm_offset_fn(c, "offA_batch", {}, aa);
    if (pointwise) {
      k << gemm_offset_fn(c, "offB_col", cols, ab) << gemm_offset_fn(c, "offB_k", {katom}, ab) << gemm_offset_fn(c, "offB_batch", {}, ab);
    } else {
      k << "DEV idx_t offB_col(idx_t x) { return 0; }\nDEV idx_t offB_k(idx_t x) { return 0; }\nDEV idx_t offB_batch(idx_t x) { return 0; }\n";
      k << "#define KARGS_G " << kargs << "\n";
      // the column (n, p, q) is decoded once per thread, the K index (ci, kh, kw) once per element
      k << "struct gcol_t { idx_t n; int h0, w0; };\n";
      k << "DEV gcol_t gather_col(idx_t cc) {\n";
      decl_digits(k, c, cols, "cc", "  ", "qc");
      auto digit = [&](int d) {
        std::string e;
        int64_t mult = 1;
        for (int i = (int)out_atoms[d].size() - 1; i >= 0; i--) {
          e = "a" + std::to_string(out_atoms[d][i]) + (mult == 1 ? "" : " * " + std::to_string(mult)) + (e.empty() ? "" : " + " + e);
          mult *= c.atom_extent[out_atoms[d][i]];
        }
        return e.empty() ? std::string("0") : e;
      };
      k << "  gcol_t g;\n  g.n = " << digit(0) << ";\n  g.h0 = (int)(" << digit(2) << ") * " << SH << " - " << PT << ";\n";
      k << "  g.w0 = (int)(" << digit(3) << ") * " << SW << " - " << PL << ";\n  return g;\n}\n";
      k << "DEV elem_t loadB_gather_impl(idx_t kk, const gcol_t g, " << kparams << ") {\n";
      if (k_taps_major) {
        k << "  const int kw_ = (int)((kk / " << C << ") % " << KW << "), kh_ = (int)(kk / " << C * KW << ");\n";
        k << "  const idx_t a" << xc << " = kk % " << C << ", a" << xn << " = g.n;\n";
      } else {
      k << "  const int kw_ = (int)(kk % " << KW << "), kh_ = (int)((kk / " << KW << ") % " << KH << ");\n";
      k << "  const idx_t a" << xc << " = kk / " << KH * KW << ", a" << xn << " = g.n;\n";
      }
      // (a branch-free form - clamped address, value zeroed afterwards - was measured and is a few percent slower
      // here: the compiler already keeps a tile's gathers in flight together, and the clamps are extra work)
      k << "  const idx_t a" << xh << " = g.h0 + kh_;\n";
      k << "  const idx_t a" << xw << " = g.w0 + kw_;\n";
      k << "  if (a" << xh << " < 0 || a" << xh << " >= " << H << " || a" << xw << " < 0 || a" << xw << " >= " << Wd << ") return (elem_t)0;\n";
      k << c.decl_parts(xatoms, "  ");
      {
        std::set<int> done;
        c.emit_values(k, {xnode}, done, pslot, "  ");
      }
      k << "  elem_t o; cvt_out(&o, " << c.vname(xnode) << "); return o;\n}\n";
      k << "#define loadB_gather(Bb, kk, g) loadB_gather_impl(kk, g, KARGS_G)\n";
      if (direct) {
        // the operand value of (channel, tap) at a column, zero in the padding; tap is a constant after unrolling
        k << "DEV float conv_direct_b(const int ch, const int t, const gcol_t g, " << kparams << ") {\n";
        k << "  const int h_ = g.h0 + t / " << KW << ", w_ = g.w0 + t % " << KW << ";\n";
        k << "  const bool in_ = h_ >= 0 && h_ < " << H << " && w_ >= 0 && w_ < " << Wd << ";\n";
        k << "  const idx_t a" << xc << " = ch, a" << xn << " = g.n;\n";
        k << "  const idx_t a" << xh << " = min(max(h_, 0), " << H - 1 << ");\n  const idx_t a" << xw << " = min(max(w_, 0), " << Wd - 1 << ");\n";
        k << c.decl_parts(xatoms, "  ");
        {
          std::set<int> done;
          c.emit_values(k, {xnode}, done, pslot, "  ");
        }
        k << "  elem_t o; cvt_out(&o, " << c.vname(xnode) << ");\n  return in_ ? (float)o : 0.0f;\n}\n";
      }
      if (bmode == 4) {
        k << "DEV " << (eb == 2 ? "u16x8" : "f32x4") << " loadB_tap_impl(idx_t kk, const gcol_t g, " << kparams << ") {\n";
        k << "  const int tap = (int)(kk / " << C << "), kh_ = tap / " << KW << ", kw_ = tap % " << KW << ";\n";
        k << "  const idx_t a" << xc << " = kk % " << C << ", a" << xn << " = g.n;\n";
        k << "  const int h_ = g.h0 + kh_, w_ = g.w0 + kw_;\n";
        k << "  const bool in_ = h_ >= 0 && h_ < " << H << " && w_ >= 0 && w_ < " << Wd << ";\n";
        k << "  const idx_t a" << xh << " = min(max(h_, 0), " << H - 1 << ");\n  const idx_t a" << xw << " = min(max(w_, 0), " << Wd - 1 << ");\n";
        k << "  " << (eb == 2 ? "u16x8" : "f32x4") << " v = *(const " << (eb == 2 ? "u16x8" : "f32x4") << "*)(p" << pslot.at(c.nodes[xnode].tensor) << " + ("
          << c.addr_expr(xaddr_t) << "));\n";
        k << "#pragma unroll\n  for (int e = 0; e < " << VEC << "; ++e) v[e] = in_ ? v[e] : 0;\n  return v;\n}\n";
        k << "#define loadB_tap(kk, g) loadB_tap_impl(kk, g, KARGS_G)\n";
      }
    }
    k << gemm_epilogue_source(c, {}, rows, cols, pslot, kparams, GN, bslot, dot ? 0 : GM);
    k << "#define KPARAMS " << kparams << "\n#define KARGS " << kargs << "\n";
    if (prologue) {
      // vec_t b_prologue(raw vector of VEC consecutive k of one column, column, first k): the block's operators in
      // front of the convolution, element by element in fp32, rounded back to the storage type - the values the
      // separate kernel would have stored
      auto digit = [&](int d) {
        std::string e;
        int64_t mult = 1;
        for (int i = (int)out_atoms[d].size() - 1; i >= 0; i--) {
          e = "a" + std::to_string(out_atoms[d][i]) + (mult == 1 ? "" : " * " + std::to_string(mult)) + (e.empty() ? "" : " + " + e);
          mult *= c.atom_extent[out_atoms[d][i]];
        }
        return e.empty() ? std::string("0") : e;
      };
      k << "#define B_PROLOGUE 1\n";
      k << "typedef elem_t evec_t __attribute__((ext_vector_type(" << VEC << ")));\n";
      k << "DEV " << (eb == 2 ? "u16x8" : "f32x4") << " b_prologue(const " << (eb == 2 ? "u16x8" : "f32x4") << " raw, idx_t cc, idx_t kk, " << kparams << ") {\n";
      decl_digits(k, c, cols, "cc", "  ", "qc");
      k << "  const idx_t a" << xn << " = " << digit(0) << ", a" << xh << " = " << digit(2) << ", a" << xw << " = " << digit(3) << ";\n";
      k << "  const evec_t ev = __builtin_bit_cast(evec_t, raw);\n  evec_t ov;\n";
      std::map<int, std::string> ovr;
      ovr[main_load] = "cvt_in(ev[e])";
      {
        std::set<int> seen;
        std::vector<int> stack = {xnode};
        k << "  {\n  const idx_t a" << xc << " = kk;\n";
        while (!stack.empty()) {
          int n = stack.back();
          stack.pop_back();
          if (seen.count(n)) continue;
          seen.insert(n);
          const ENode& e = c.nodes[n];
          for (int a : e.args) stack.push_back(a);
          if (e.kind != ENode::LOAD || n == main_load) continue;
          Affine la = c.resolved(e.addr);
          auto it = la.stride.find(xc);
          bool vec = it != la.stride.end() && it->second == 1 && la.offset % VEC == 0 && dtype_bytes(g.tensors[e.tensor].dtype) * VEC <= 16;
          for (auto& kv : la.stride) if (kv.first != xc && kv.second % VEC) vec = false;
          if (!vec) continue;
          k << "  typedef " << c.ctype(g.tensors[e.tensor].dtype) << " pv" << n << "_t __attribute__((ext_vector_type(" << VEC << ")));\n";
          k << "  const pv" << n << "_t pv" << n << " = *(const pv" << n << "_t*)(p" << pslot.at(e.tensor) << " + (" << c.addr_expr(e.addr) << "));\n";
          ovr[n] = "cvt_in(pv" + std::to_string(n) + "[e])";
        }
      }
      k << "#pragma unroll\n  for (int e = 0; e < " << VEC << "; ++e) {\n    const idx_t a" << xc << " = kk + e;\n";
      {
        std::set<int> done;
        c.emit_values(k, {xnode}, done, pslot, "    ", &ovr);
      }
      k << "    elem_t t_; cvt_out(&t_, " << c.vname(xnode) << "); ov[e] = t_;\n  }\n  }\n";
      k << "  return __builtin_bit_cast(" << (eb == 2 ? "u16x8" : "f32x4") << ", ov);\n}\n";
    }
    Lw.family = FAM_CONV;
    if (dot) {
      k << R"KRN(
extern "C" __global__ __launch_bounds__(256) void KNAME(KPARAMS) {
  const int lane = threadIdx.x & 63;
  const idx_t o = (idx_t)blockIdx.x * 4 + (threadIdx.x >> 6);     // one wavefront per output element
  if (o >= (idx_t)GM * GN) return;
  const idx_t r = o / GN, cc = o % GN;
  const idx_t ar = offA_row(r);
  float acc = 0.0f;
  const gcol_t gc = gather_col(cc);
  for (idx_t kk = lane; kk < GK; kk += 64) acc += cvt_in(PA[ar + offA_k(kk)]) * cvt_in(loadB_gather(0, kk, gc));
  acc = dn_wave_sum(acc);
  if (lane == 0) {
    float colv[NCOLV > 0 ? NCOLV : 1];
    col_loads(cc, colv, KARGS);
    epilogue(0, r, cc, acc, colv, KARGS);
  }
}
)KRN";
      Kn.grid[0] = (unsigned)((GM * GN + 3) / 4);
      Lw.variant = "dot_wave_k" + std::to_string(K);
      if (K <= 64) {
        // A short K leaves most of a wavefront's lanes idle and the reduction across them costs more than the products:
        // one lane per output instead, walking K itself; neighbouring lanes take neighbouring output channels, so the
        // stores of a channels-last result coalesce and the column's operand values are the same address in every lane.
        const size_t at = k.str().rfind("extern \"C\" __global__");
        std::string head = k.str().substr(0, at);
        k.str("");
        k << head << R"KRN(
extern "C" __global__ __launch_bounds__(256) void KNAME(KPARAMS) {
  const idx_t o = (idx_t)blockIdx.x * 256 + threadIdx.x;          // one lane per output element
  if (o >= (idx_t)GM * GN) return;
  const idx_t r = o % GM, cc = o / GM;
  const idx_t ar = offA_row(r);
  const gcol_t gc = gather_col(cc);
  float acc = 0.0f;
#pragma unroll 8
  for (idx_t kk = 0; kk < GK; ++kk) acc += cvt_in(PA[ar + offA_k(kk)]) * cvt_in(loadB_gather(0, kk, gc));
  float colv[NCOLV > 0 ? NCOLV : 1];
  col_loads(cc, colv, KARGS);
  epilogue(0, r, cc, acc, colv, KARGS);
}
)KRN";
        Kn.grid[0] = (unsigned)((GM * GN + 255) / 256);
        Lw.variant = "dot_lane_k" + std::to_string(K);
      }
    } else {
      k << gemm_kernel_body();
      Kn.grid[0] = (unsigned)nblocks(BM, BN);
      Kn.block[0] = (unsigned)(64 * WAVES_M * WAVES_N * WAVES_K);
      Lw.variant = direct ? "direct_32x32_taps" + std::to_string(KH * KW) + "_k4"
                          : "igemm_" + std::to_string(BM) + "x" + std::to_string(BN) + "x" + std::to_string(BK) + "_a" + std::to_string(amode) + "b" + std::to_string(bmode) +
                                (prologue ? "_pro" : "");
    }
  }
  Lw.ext_in.assign(params.begin(), params.begin() + n_in);
  Lw.ext_out.assign(params.begin() + n_in, params.end());
  Kn.params = params;
  if (Kn.block[0] == 1) Kn.block[0] = 256;      // (the implicit-GEMM tiles set their own size above)
  std::string src = std::string(device_preamble()) + k.str();
  Kn.name = fnv_name(depthwise ? "dnnf_dwconv" : "dnnf_conv", src);
  size_t pos;
  while ((pos = src.find("KNAME")) != std::string::npos) src.replace(pos, 5, Kn.name);
  Kn.source = src;
  Lw.launches.push_back(Kn);
  return Lw;
}

}  // namespace dnnf
