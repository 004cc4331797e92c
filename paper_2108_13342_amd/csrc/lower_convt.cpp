// Transposed convolution blocks (ConvTranspose; NCHW input, [C, CO, KH, KW] filter, group 1), in gather form:
//   out[n, co, p, q] = bias[co] + sum over (c, i, j) with (p + pad_top - i) and (q + pad_left - j) divisible by the
//                      stride of x[n, c, (p + pad_top - i) / stride_h, (q + pad_left - j) / stride_w] * w[c, co, i, j]
// i.e. an implicit GEMM whose rows are output channels, columns output pixels and K = (c, i, j), on the MFMA
// template shared with MatMul and Conv.  The operand is gathered element by element (positions that fall between
// input pixels or outside the map read as zero, with the block's prologue operators applied to the gathered
// element); the filter's channel axis comes first in the declared order, so the filter matrix is strided along K
// and the A operand uses the scalar loader.  The block's successors run as the epilogue.  Few outputs: one
// wavefront per output element.
#include <algorithm>

#include "lower_ctx.hpp"

namespace dnnf {

namespace {
}  // namespace

Lowered lower_conv_transpose(LowerCtx& c) {
  const Graph& g = c.g;
  const Op& A = g.ops[c.anchor_op];
  const Tensor& X = g.tensors[A.in[0]];
  const Tensor& Wt = g.tensors[A.in[1]];
  const Tensor& Y = g.tensors[A.out[0]];
  const int bias_t = A.in.size() > 2 ? A.in[2] : -1;
  DNNF_CHECK(c.is_external(A.in[1]) && (bias_t < 0 || c.is_external(bias_t)), DNNF_UNSUPPORTED_OP,
             "convolution weights computed inside the block");
  DNNF_CHECK(is_float(X.dtype) && Wt.dtype == X.dtype, DNNF_UNSUPPORTED_OP, "ConvTranspose operands must share a float type");
  DNNF_CHECK(A.i("group", 1) == 1 && Wt.perm.empty(), DNNF_UNSUPPORTED_OP, "grouped ConvTranspose has no kernel template");
  const int64_t N = X.dims[0], C = X.dims[1], H = X.dims[2], Wd = X.dims[3];
  const int64_t CO = Wt.dims[1], KH = Wt.dims[2], KW = Wt.dims[3];
  const int64_t HO = Y.dims[2], WO = Y.dims[3];
  auto st = A.ints("strides");
  if (st.empty()) st = {1, 1};
  auto pd = A.ints("pads");
  if (pd.empty()) pd = {0, 0, 0, 0};
  const int64_t SH = st[0], SW = st[1], PT = pd[0], PL = pd[1];

  TIdx oi = c.fresh_index(Y.dims);
  c.tidx[c.anchor_out] = oi;
  std::vector<int> ein, eout, removed;
  block_io(g, c.blk, ein, eout, removed);
  c.forward_all();
  for (int t : eout)
    DNNF_CHECK(c.tidx.count(t), DNNF_UNSUPPORTED_OP, "block output " + g.tensors[t].name + " does not follow the convolution");
  c.collect_stores(eout);

  const int xn = c.new_atom(std::max<int64_t>(N, 2)), xc = c.new_atom(std::max<int64_t>(C, 2)),
            xh = c.new_atom(std::max<int64_t>(H, 2)), xw = c.new_atom(std::max<int64_t>(Wd, 2));
  TIdx xi(4);
  xi[0].atoms = {xn};
  xi[1].atoms = {xc};
  xi[2].atoms = {xh};
  xi[3].atoms = {xw};
  const int xnode = c.value(A.in[0], xi);
  const std::vector<int> xatoms = {xn, xc, xh, xw};

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

  std::vector<int> params;
  std::map<int, int> pslot;
  std::set<int> written;
  {
    std::set<int> need;
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
  auto add_param = [&](int t) {
    if (!pslot.count(t)) { pslot[t] = (int)params.size(); params.push_back(t); }
    return pslot[t];
  };
  const int wslot = add_param(A.in[1]);
  const int bslot = bias_t >= 0 ? add_param(bias_t) : -1;
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
  std::string kparams = c.param_list(params, written), kargs;
  for (size_t i = 0; i < params.size(); i++) kargs += (i ? ", p" : "p") + std::to_string(i);

  const int64_t KK = KH * KW, K = C * KK, GM = CO, GN = N * HO * WO;
  const int eb = dtype_bytes(X.dtype);
  std::vector<int> rows = out_atoms[1], cols;
  for (int d : {0, 2, 3}) cols.insert(cols.end(), out_atoms[d].begin(), out_atoms[d].end());
  DNNF_CHECK(rows.size() <= 1, DNNF_UNSUPPORTED_OP, "output channel axis was split by a reshape in the block");
  // filter matrix A[co][k], k = c * KK + tap, stored as w[c][co][tap]: two K atoms (channel, tap)
  const int kc = c.new_atom(std::max<int64_t>(C, 2)), ktap = c.new_atom(std::max<int64_t>(KK, 2));
  Affine aa;
  if (!rows.empty()) aa.stride[rows[0]] = KK;
  aa.stride[kc] = CO * KK;
  aa.stride[ktap] = 1;
  std::vector<int> katoms;
  if (C > 1) katoms.push_back(kc);
  if (KK > 1) katoms.push_back(ktap);
  const int amode = 2, bmode = 3;
  const bool dot = GM * GN <= 65536 && GM * GN * K <= ((int64_t)8 << 20);

  auto nblocks = [&](int bm, int bn) { return ((GM + bm - 1) / bm) * ((GN + bn - 1) / bn); };
  int BK = eb == 2 ? (K <= 32 ? 32 : 64) : 16;
  struct Tile { int BM, BN, WM, WN, WK; };
  std::vector<Tile> tiles;
  if (GM > 64) { tiles.push_back({128, 128, 2, 2, 1}); tiles.push_back({128, 64, 2, 2, 1}); }
  tiles.push_back({64, 128, 2, 2, 1});
  tiles.push_back({64, 64, 2, 2, 1});
  if (K >= 8 * BK) tiles.push_back({32, 32, 1, 1, 4});
  size_t pick = tiles.size() - 1;
  if (c.opts.force_variant >= 100) {
    DNNF_CHECK(!dot && c.opts.force_variant - 100 < (int)tiles.size(), DNNF_UNSUPPORTED_OP, "no such convolution tile variant");
    pick = (size_t)(c.opts.force_variant - 100);
  } else {
    for (size_t i = 0; i < tiles.size(); i++)
      if (tiles[i].WK == 1 && nblocks(tiles[i].BM, tiles[i].BN) >= 768) { pick = i; break; }
    if (tiles[pick].WK == 4 && nblocks(64, 64) >= 192) pick--;
  }
  const int BM = tiles[pick].BM, BN = tiles[pick].BN, WAVES_M = tiles[pick].WM, WAVES_N = tiles[pick].WN, WAVES_K = tiles[pick].WK;
  if (WAVES_K == 4 && eb == 4 && K >= 256) BK = 64;

  std::ostringstream k;
  k << "typedef " << (wide ? "long long" : "int") << " idx_t;\n";
  k << "typedef " << c.ctype(X.dtype) << " elem_t;\n";
  k << "#define ELEM_BYTES " << eb << "\n#define BM " << BM << "\n#define BN " << BN << "\n#define BK " << BK << "\n";
  k << "#define GM " << GM << "\n#define GN " << GN << "\n#define GK " << K << "\n";
  k << "#define WAVES_M " << WAVES_M << "\n#define WAVES_N " << WAVES_N << "\n#define WAVES_K " << WAVES_K
    << (K <= BK ? "\n#define NBUF 1\n#define PF 1\n" : "\n#define NBUF 2\n#define PF 2\n");
  k << "#define A_MODE " << amode << "\n#define B_MODE " << bmode << "\n#define PA p" << wslot << "\n#define PB p" << wslot << "\n";
  if (X.dtype == DNNF_F16) k << "typedef f16x8 frag_t;\n#define MFMA __builtin_amdgcn_mfma_f32_32x32x16_f16\n";
  else if (X.dtype == DNNF_BF16) k << "typedef bf16x8 frag_t;\n#define MFMA __builtin_amdgcn_mfma_f32_32x32x16_bf16\n";
  k << gemm_offset_fn(c, "offA_row", rows, aa) << gemm_offset_fn(c, "offA_k", katoms, aa) << gemm_offset_fn(c, "offA_batch", {}, aa);
  k << "DEV idx_t offB_col(idx_t x) { return 0; }\nDEV idx_t offB_k(idx_t x) { return 0; }\nDEV idx_t offB_batch(idx_t x) { return 0; }\n";
  k << "#define KARGS_G " << kargs << "\n";
  // the column (n, p, q) is decoded once per thread, the K index (c, i, j) once per element
  k << "struct gcol_t { idx_t n; int h0, w0; };\n";
  k << "DEV gcol_t gather_col(idx_t cc) {\n";
  decl_digits(k, c, cols, "cc", "  ", "qc");
  k << "  gcol_t g;\n  g.n = " << digit(0) << ";\n  g.h0 = (int)(" << digit(2) << ") + " << PT << ";\n";
  k << "  g.w0 = (int)(" << digit(3) << ") + " << PL << ";\n  return g;\n}\n";
  k << "DEV elem_t loadB_gather_impl(idx_t kk, const gcol_t g, " << kparams << ") {\n";
  k << "  const int kw_ = (int)(kk % " << KW << "), kh_ = (int)((kk / " << KW << ") % " << KH << ");\n";
  k << "  const idx_t a" << xc << " = kk / " << KK << ", a" << xn << " = g.n;\n";
  k << "  const int th = g.h0 - kh_, tw = g.w0 - kw_;\n";
  k << "  if (th < 0 || tw < 0 || th % " << SH << " != 0 || tw % " << SW << " != 0) return (elem_t)0;\n";
  k << "  const idx_t a" << xh << " = th / " << SH << ", a" << xw << " = tw / " << SW << ";\n";
  k << "  if (a" << xh << " >= " << H << " || a" << xw << " >= " << Wd << ") return (elem_t)0;\n";
  k << c.decl_parts(xatoms, "  ");
  {
    std::set<int> done;
    c.emit_values(k, {xnode}, done, pslot, "  ");
  }
  k << "  elem_t o; cvt_out(&o, " << c.vname(xnode) << "); return o;\n}\n";
  k << "#define loadB_gather(Bb, kk, g) loadB_gather_impl(kk, g, KARGS_G)\n";
  k << gemm_epilogue_source(c, {}, rows, cols, pslot, kparams, GN, bslot, dot ? 0 : GM);
  k << "#define KPARAMS " << kparams << "\n#define KARGS " << kargs << "\n";

  Lowered Lw;
  Launch Kn;
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
    Lw.variant = "dotT_wave_k" + std::to_string(K);
  } else {
    k << gemm_kernel_body();
    Kn.grid[0] = (unsigned)nblocks(BM, BN);
    Lw.variant = "igemmT_" + std::to_string(BM) + "x" + std::to_string(BN) + "x" + std::to_string(BK) + "_a" + std::to_string(amode) + "b" + std::to_string(bmode);
  }
  Lw.ext_in.assign(params.begin(), params.begin() + n_in);
  Lw.ext_out.assign(params.begin() + n_in, params.end());
  Kn.params = params;
  Kn.block[0] = 256;
  std::string src = std::string(device_preamble()) + k.str();
  Kn.name = fnv_name("dnnf_convt", src);
  size_t pos;
  while ((pos = src.find("KNAME")) != std::string::npos) src.replace(pos, 5, Kn.name);
  Kn.source = src;
  Lw.launches.push_back(Kn);
  return Lw;
}

}  // namespace dnnf
