// Squeeze-and-excitation tail as one kernel: [GlobalAveragePool ->] 1x1 Conv on the pooled vector -> One-to-One
// operators -> 1x1 Conv -> One-to-One operators.  The mapping-type table keeps every one of these apart
// (Many-to-Many behind Many-to-Many, Sec. 3.2); on this chip each of them is a launch of a few microseconds that
// moves kilobytes, so the plan option `squeeze_excite` offers the three as one block, like the attention block.
// One workgroup per image: the pooled vector and the hidden vector live in LDS, nothing between the pool's input and
// the second layer's result touches memory.
#include <algorithm>
#include <map>
#include <set>
#include <sstream>

#include "lower_ctx.hpp"

namespace dnnf {

namespace {

const char* kSeBody = R"KRN(
#define SE_NT 512
#define SE_EPW (4 / ELEM_BYTES)                 // elements per 32-bit word of the second layer's weights
#define SE_WR (SE_CR / SE_EPW)                  // words per weight row
#define SE_PW (SE_WR | 1)                       // row pitch of a wavefront's weight slice in LDS: odd, every row its own bank
#define SE_JPW ((SE_CR + SE_NT / 64 - 1) / (SE_NT / 64))                 // hidden units per wavefront
#define SE_CPW (((SE_CO + 63) / 64 + SE_NT / 64 - 1) / (SE_NT / 64))     // groups of 64 output rows per wavefront
extern "C" __global__ __launch_bounds__(SE_NT) void KNAME(KPARAMS) {
  __shared__ float pooled[SE_C];
  __shared__ float hid[SE_CR];
#if SE_HW > 1 && defined(SE_VEC)
  __shared__ float part[SE_G * SE_C];
#endif
  __shared__ unsigned int wt[SE_NT / 64][64 * SE_PW];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const idx_t n = blockIdx.x;

  // ---- the pooled vector
#if SE_HW == 1
  for (int c = tid; c < SE_C; c += SE_NT) pooled[c] = se_in(n, c, 0, KARGS);
#elif defined(SE_VEC)
  // lanes along the channels, SE_VEC of them per 16-byte load; the positions are dealt to SE_G groups of lanes
  for (int item = tid; item < (SE_C / SE_VEC) * SE_G; item += SE_NT) {
    const int cv = item % (SE_C / SE_VEC), grp = item / (SE_C / SE_VEC);
    float acc[SE_VEC];
#pragma unroll
    for (int u = 0; u < SE_VEC; ++u) acc[u] = 0.0f;
#pragma unroll 8
    for (int hw = grp; hw < SE_HW; hw += SE_G) {
      float v[SE_VEC];
      se_in_vec(n, cv * SE_VEC, hw, v, KARGS);
#pragma unroll
      for (int u = 0; u < SE_VEC; ++u) acc[u] += v[u];
    }
#pragma unroll
    for (int u = 0; u < SE_VEC; ++u) part[grp * SE_C + cv * SE_VEC + u] = acc[u];
  }
  __syncthreads();
  for (int c = tid; c < SE_C; c += SE_NT) {
    float s = 0.0f;
    for (int q = 0; q < SE_G; ++q) s += part[q * SE_C + c];
    pooled[c] = s * (1.0f / SE_HW);
  }
#else
  for (int c = tid; c < SE_C; c += SE_NT) {
    float s = 0.0f;
    for (int hw = 0; hw < SE_HW; ++hw) s += se_in(n, c, hw, KARGS);
    pooled[c] = s * (1.0f / SE_HW);
  }
#endif
  __syncthreads();

  // ---- first layer: one wavefront per hidden unit, lanes along the channels.  A wavefront's units are walked with
  // compile-time bounds and separate sums, so that every weight load of the layer is issued before the first reduction
  // (the layer is a handful of memory round trips otherwise, one per unit).
  {
    float s[SE_JPW];
#pragma unroll
    for (int q = 0; q < SE_JPW; ++q) {
      s[q] = 0.0f;
      const int j = wave + q * (SE_NT / 64);
      if (j < SE_CR) {
#ifdef SE_W1VEC
        typedef elem_t w1vec_t __attribute__((ext_vector_type(SE_W1VEC)));
#pragma unroll
        for (int it = 0; it < (SE_C / SE_W1VEC + 63) / 64; ++it) {
          const int cv = lane + it * 64;
          if (cv < SE_C / SE_W1VEC) {
            const w1vec_t w = *(const w1vec_t*)(PW1 + (idx_t)j * SE_C + cv * SE_W1VEC);
#pragma unroll
            for (int u = 0; u < SE_W1VEC; ++u) s[q] += pooled[cv * SE_W1VEC + u] * cvt_in(w[u]);
          }
        }
#else
#pragma unroll 4
        for (int c = lane; c < SE_C; c += 64) s[q] += pooled[c] * cvt_in(PW1[(idx_t)j * SE_C + c]);
#endif
      }
    }
#pragma unroll
    for (int q = 0; q < SE_JPW; ++q) {
      const int j = wave + q * (SE_NT / 64);
      const float t = dn_wave_sum(s[q]);
      if (j < SE_CR && lane == 0) hid[j] = se_mid(n, j, t, KARGS);
    }
  }
  __syncthreads();

  // ---- second layer.  A wavefront takes 64 output rows at a time: their weights (64 x SE_CR, contiguous in memory)
  // are fetched with lanes along the words - all of the wavefront's groups before anything else, for the same reason -
  // and copied into its own LDS slice, then lane = row walks its row; the slice belongs to the wavefront alone,
  // whose LDS operations complete in order, so no barrier is involved.
  {
    unsigned int wreg[SE_CPW][SE_WR];
#pragma unroll
    for (int q = 0; q < SE_CPW; ++q) {
      const int r0 = (wave + q * (SE_NT / 64)) * 64;
      const int nrows = r0 >= SE_CO ? 0 : (SE_CO - r0 < 64 ? SE_CO - r0 : 64);
      const unsigned int* __restrict__ src = (const unsigned int*)(PW2 + (idx_t)(r0 < SE_CO ? r0 : 0) * SE_CR);
#pragma unroll
      for (int t = 0; t < SE_WR; ++t) {
        const int i = lane + t * 64;
        wreg[q][t] = i < nrows * SE_WR ? src[i] : 0u;
      }
    }
#pragma unroll
    for (int q = 0; q < SE_CPW; ++q) {
      const int r0 = (wave + q * (SE_NT / 64)) * 64;
      const int nrows = r0 >= SE_CO ? 0 : (SE_CO - r0 < 64 ? SE_CO - r0 : 64);
#pragma unroll
      for (int t = 0; t < SE_WR; ++t) {
        const int i = lane + t * 64;
        wt[wave][(i / SE_WR) * SE_PW + i % SE_WR] = wreg[q][t];
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
      if (lane < nrows) {
        float s = 0.0f;
#pragma unroll 4
        for (int w = 0; w < SE_WR; ++w) {
          const unsigned int word = wt[wave][lane * SE_PW + w];
#if ELEM_BYTES == 2
          typedef elem_t epair_t __attribute__((ext_vector_type(2)));
          const epair_t pr = __builtin_bit_cast(epair_t, word);
          s += hid[2 * w] * cvt_in(pr[0]) + hid[2 * w + 1] * cvt_in(pr[1]);
#else
          s += hid[w] * __builtin_bit_cast(float, word);
#endif
        }
        se_out(n, r0 + lane, s, KARGS);
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
  }
}
)KRN";

struct FcFrame {
  int64_t N = 0, C = 0, CO = 0;
  int wt = -1, bias = -1;
  std::vector<int> n_atoms, c_atoms;      // output index digits: image, channel
};

// A 1x1 convolution over a [N, C, 1, 1] tensor as the fully connected layer it is; sets up the context's index space
// over the layer's result and walks the block's operators behind it.
FcFrame analyse_fc(LowerCtx& c, const std::vector<int>& eout) {
  const Graph& g = c.g;
  const Op& A = g.ops[c.anchor_op];
  const Tensor& X = g.tensors[A.in[0]];
  const Tensor& W = g.tensors[A.in[1]];
  const Tensor& Y = g.tensors[A.out[0]];
  DNNF_CHECK(X.dims.size() == 4 && W.dims.size() == 4 && Y.dims.size() == 4, DNNF_UNSUPPORTED_OP, "squeeze-excite layers are 2-d convolutions");
  DNNF_CHECK(X.dims[2] == 1 && X.dims[3] == 1 && W.dims[2] == 1 && W.dims[3] == 1 && Y.dims[2] == 1 && Y.dims[3] == 1, DNNF_UNSUPPORTED_OP,
             "squeeze-excite layers work on 1x1 maps with 1x1 filters");
  DNNF_CHECK(A.i("group", 1) == 1 && W.dims[1] == X.dims[1], DNNF_UNSUPPORTED_OP, "grouped squeeze-excite layer");
  DNNF_CHECK(is_float(X.dtype) && W.dtype == X.dtype, DNNF_UNSUPPORTED_OP, "Conv operands must share a float type");
  DNNF_CHECK(c.is_external(A.in[1]) && (A.in.size() < 3 || c.is_external(A.in[2])), DNNF_UNSUPPORTED_OP, "convolution weights computed inside the block");
  const bool known_order = W.perm.empty() || W.perm == std::vector<int>{0, 2, 3, 1};      // (the same bytes for a 1x1 filter)
  DNNF_CHECK(known_order, DNNF_UNSUPPORTED_OP, "filter in an unknown storage order");
  FcFrame f;
  f.N = X.dims[0];
  f.C = X.dims[1];
  f.CO = W.dims[0];
  f.wt = A.in[1];
  f.bias = A.in.size() > 2 ? A.in[2] : -1;
  TIdx oi = c.fresh_index(Y.dims);
  c.tidx[c.anchor_out] = oi;
  c.forward_all();
  for (int t : eout)
    DNNF_CHECK(c.tidx.count(t), DNNF_UNSUPPORTED_OP, "block output " + g.tensors[t].name + " does not follow the convolution");
  c.collect_stores(eout);
  DNNF_CHECK(c.rep_atoms.empty(), DNNF_UNSUPPORTED_OP, "replicated results behind a squeeze-excite layer");
  c.resolve(oi[0].atoms, f.n_atoms);
  c.resolve(oi[1].atoms, f.c_atoms);
  return f;
}

void collect_loads(const LowerCtx& c, std::vector<int> stack, std::vector<int>& params, std::map<int, int>& pslot) {
  std::set<int> need;
  while (!stack.empty()) {
    int n = stack.back();
    stack.pop_back();
    if (need.count(n)) continue;
    need.insert(n);
    for (int a : c.nodes[n].args) stack.push_back(a);
    if (c.nodes[n].kind == ENode::LOAD) {
      DNNF_CHECK(c.nodes[n].addr.indirect.empty(), DNNF_UNSUPPORTED_OP, "gathered operand in a squeeze-excite block");
      if (!pslot.count(c.nodes[n].tensor)) { pslot[c.nodes[n].tensor] = (int)params.size(); params.push_back(c.nodes[n].tensor); }
    }
  }
}

}  // namespace

Lowered lower_squeeze_excite(const Graph& g, const Block& b, const LowerOpts& o) {
  int gap = -1;
  std::vector<int> convs;
  for (int oi : b.ops) {
    const OpClass cl = g.ops[oi].info->cls;
    if (cl == OC_GAP) { DNNF_CHECK(gap < 0, DNNF_UNSUPPORTED_OP, "two pooling operators in one block"); gap = oi; }
    else if (cl == OC_CONV) convs.push_back(oi);
    else DNNF_CHECK(cl == OC_UNARY || cl == OC_BINARY, DNNF_UNSUPPORTED_OP, "operator " + g.ops[oi].kind + " in a squeeze-excite block");
  }
  DNNF_CHECK(convs.size() == 2, DNNF_UNSUPPORTED_OP, "not a squeeze-excite tail (two 1x1 convolutions)");
  // the first layer is the one the second layer's operand depends on
  std::set<int> in_block(b.ops.begin(), b.ops.end()), front;
  auto upstream = [&](int t0, std::set<int>& acc) {
    std::vector<int> stack = {t0};
    while (!stack.empty()) {
      int t = stack.back();
      stack.pop_back();
      int p = g.tensors[t].producer;
      if (p < 0 || !in_block.count(p) || acc.count(p)) continue;
      acc.insert(p);
      for (int i : g.ops[p].in) stack.push_back(i);
    }
  };
  int c1 = -1, c2 = -1;
  for (int cand : convs) {
    std::set<int> up;
    upstream(g.ops[cand].in[0], up);
    const int other = cand == convs[0] ? convs[1] : convs[0];
    if (up.count(other)) { c2 = cand; c1 = other; front = up; }
  }
  DNNF_CHECK(c1 >= 0, DNNF_UNSUPPORTED_OP, "the two convolutions of a squeeze-excite tail must follow one another");
  if (gap >= 0)
    DNNF_CHECK(g.ops[c1].in[0] == g.ops[gap].out[0] && g.tensors[g.ops[gap].out[0]].consumers.size() == 1 &&
                   g.tensors[g.ops[gap].out[0]].kind == DNNF_INTERMEDIATE,
               DNNF_UNSUPPORTED_OP, "the pooled vector must feed the first layer and nothing else");
  Block b1, b2, bp;
  for (int oi : b.ops) {
    if (oi == gap) bp.ops.push_back(oi);
    else if (front.count(oi)) b1.ops.push_back(oi);
    else b2.ops.push_back(oi);
  }
  b1.fused_type = b2.fused_type = bp.fused_type = DNNF_MANY_TO_MANY;
  const int X2 = g.ops[c2].in[0];
  DNNF_CHECK(g.tensors[X2].consumers.size() == 1 && g.tensors[X2].kind == DNNF_INTERMEDIATE, DNNF_UNSUPPORTED_OP,
             "the hidden vector must feed the second layer and nothing else");

  LowerCtx k1(g, b1, o), k2(g, b2, o), kp(g, bp.ops.empty() ? b1 : bp, o);
  k1.anchor_op = c1;
  k1.anchor_out = g.ops[c1].out[0];
  k2.anchor_op = c2;
  k2.anchor_out = g.ops[c2].out[0];
  std::vector<int> ein, eout, removed, eout2;
  block_io(g, b, ein, eout, removed);
  {
    std::vector<int> e2, r2;
    block_io(g, b2, e2, eout2, r2);
  }
  FcFrame f1 = analyse_fc(k1, {X2});
  FcFrame f2 = analyse_fc(k2, eout2);
  DNNF_CHECK(std::set<int>(eout.begin(), eout.end()) == std::set<int>(eout2.begin(), eout2.end()), DNNF_UNSUPPORTED_OP,
             "an intermediate of the squeeze-excite tail is read outside the block");
  DNNF_CHECK(f2.C == f1.CO && f2.N == f1.N, DNNF_UNSUPPORTED_OP, "the two layers do not fit one another");
  DNNF_CHECK(k1.stores.size() == 1 && k1.stores[0].tensor == X2 && k1.stores[0].preds.empty(), DNNF_UNSUPPORTED_OP, "hidden vector only partly written");
  {
    // the hidden vector in the first layer's own (image, channel) order
    const TIdx& xi = k1.tidx.at(X2);
    std::vector<int> d0, d1;
    DNNF_CHECK(xi.size() == 4 && xi[0].offset == 0 && xi[1].offset == 0 && xi[0].indirect < 0 && xi[1].indirect < 0, DNNF_UNSUPPORTED_OP, "sliced hidden vector");
    k1.resolve(xi[0].atoms, d0);
    k1.resolve(xi[1].atoms, d1);
    DNNF_CHECK(d0 == f1.n_atoms && d1 == f1.c_atoms, DNNF_UNSUPPORTED_OP, "operators between the two layers permute the hidden vector");
  }
  const int dtype = g.tensors[g.ops[c1].in[0]].dtype;
  DNNF_CHECK(g.tensors[X2].dtype == dtype, DNNF_UNSUPPORTED_OP, "the hidden vector changes type between the layers");
  const int eb = dtype_bytes(dtype);
  const int64_t C = f1.C, CR = f1.CO, CO = f2.CO, N = f1.N;
  DNNF_CHECK((CR * eb) % 4 == 0, DNNF_UNSUPPORTED_OP, "hidden width not a whole number of 32-bit words");
  DNNF_CHECK(C <= 4096 && CR <= (eb == 2 ? 94 : 47), DNNF_UNSUPPORTED_OP, "squeeze-excite vectors too long for one workgroup's LDS");
  // (a lane holds its share of the second layer's weights in registers: groups of 64 rows per wavefront x words per row)
  DNNF_CHECK(((CO + 63) / 64 + 7) / 8 * (CR * eb / 4) <= 160, DNNF_UNSUPPORTED_OP, "second squeeze-excite layer too large for one workgroup per image");

  // ---- the pooled vector's source
  int64_t HW = 1, Wd = 1;
  const int src_t = gap >= 0 ? g.ops[gap].in[0] : g.ops[c1].in[0];
  {
    const Tensor& T = g.tensors[src_t];
    DNNF_CHECK(T.dims.size() == 4 && T.dims[0] == N && T.dims[1] == C && T.dtype == dtype, DNNF_UNSUPPORTED_OP, "pooled tensor does not match the first layer");
    HW = T.dims[2] * T.dims[3];
    Wd = T.dims[3];
    DNNF_CHECK(gap >= 0 || HW == 1, DNNF_UNSUPPORTED_OP, "first layer on a map larger than 1x1");
    DNNF_CHECK(HW <= 1024, DNNF_UNSUPPORTED_OP, "map too large to pool in one workgroup per image");
  }
  const int xn = kp.new_atom(std::max<int64_t>(N, 2)), xc = kp.new_atom(std::max<int64_t>(C, 2)),
            xh = kp.new_atom(std::max<int64_t>(g.tensors[src_t].dims[2], 2)), xw = kp.new_atom(std::max<int64_t>(Wd, 2));
  TIdx xi(4);
  xi[0].atoms = {xn};
  xi[1].atoms = {xc};
  xi[2].atoms = {xh};
  xi[3].atoms = {xw};
  const int xnode = kp.value(src_t, xi);
  const std::vector<int> xatoms = {xn, xc, xh, xw};

  // ---- parameters: pooled source, both layers' weights and biases, what the operators read, the results
  std::vector<int> params;
  std::map<int, int> pslot;
  std::set<int> written;
  collect_loads(kp, {xnode}, params, pslot);
  auto add_param = [&](int t) {
    if (!pslot.count(t)) { pslot[t] = (int)params.size(); params.push_back(t); }
    return pslot[t];
  };
  const int w1 = add_param(f1.wt), w2 = add_param(f2.wt);
  const int bs1 = f1.bias >= 0 ? add_param(f1.bias) : -1, bs2 = f2.bias >= 0 ? add_param(f2.bias) : -1;
  collect_loads(k1, {k1.stores[0].value}, params, pslot);
  {
    std::vector<int> roots;
    for (auto& s : k2.stores) roots.push_back(s.value);
    collect_loads(k2, roots, params, pslot);
  }
  DNNF_CHECK(!pslot.count(X2) && (gap < 0 || !pslot.count(g.ops[gap].out[0])), DNNF_UNSUPPORTED_OP, "an on-chip vector of the block is read from memory");
  const size_t n_in = params.size();
  for (auto& s : k2.stores) {
    DNNF_CHECK(!pslot.count(s.tensor), DNNF_UNSUPPORTED_OP, "block reads and writes the same tensor");
    pslot[s.tensor] = (int)params.size();
    params.push_back(s.tensor);
    written.insert(s.tensor);
  }
  DNNF_CHECK(params.size() <= 24, DNNF_UNSUPPORTED_OP, "too many operands for one kernel");
  bool wide = false;
  for (int t : params) wide = wide || g.tensors[t].n() >= (int64_t)1 << 31;
  std::string kparams = k1.param_list(params, written), kargs;
  for (size_t i = 0; i < params.size(); i++) kargs += (i ? ", p" : "p") + std::to_string(i);

  // 16-byte loads of the pooled tensor along the channels (channels-last maps)
  int V = 0;
  if (HW > 1 && kp.nodes[xnode].kind == ENode::LOAD && !kp.nodes[xnode].is_int && kp.nodes[xnode].addr.indirect.empty() &&
      g.tensors[kp.nodes[xnode].tensor].dtype == dtype) {
    const int v = 16 / eb;
    Affine a = kp.resolved(kp.nodes[xnode].addr);
    bool ok = stride_of(a, xc) == 1 && C % v == 0 && a.offset % v == 0;
    for (auto& kv : a.stride) if (kv.first != xc && kv.second % v) ok = false;
    if (ok) V = v;
  }
  int64_t G = 1;
  if (V) G = std::max<int64_t>(1, std::min<int64_t>(512 / std::max<int64_t>(C / V, 1), HW));

  std::ostringstream k;
  k << "typedef " << (wide ? "long long" : "int") << " idx_t;\n";
  k << "typedef " << k1.ctype(dtype) << " elem_t;\n";
  k << "#define ELEM_BYTES " << eb << "\n#define SE_C " << C << "\n#define SE_CR " << CR << "\n#define SE_CO " << CO << "\n#define SE_HW " << HW << "\n";
  if (V) k << "#define SE_VEC " << V << "\n#define SE_G " << G << "\n";
  if (C % (16 / eb) == 0) k << "#define SE_W1VEC " << 16 / eb << "\n";
  k << "#define PW1 p" << w1 << "\n#define PW2 p" << w2 << "\n";
  auto decl_src_atoms = [&](const std::string& cexpr) {
    k << "  const idx_t a" << xn << " = n, a" << xc << " = " << cexpr << ", a" << xh << " = hw / " << Wd << ", a" << xw << " = hw % " << Wd << ";\n";
    k << kp.decl_parts(xatoms, "  ");
  };
  k << "DEV float se_in(idx_t n, idx_t c, idx_t hw, " << kparams << ") {\n";
  decl_src_atoms("c");
  {
    std::set<int> done;
    kp.emit_values(k, {xnode}, done, pslot, "  ");
  }
  k << "  return " << kp.vname(xnode) << ";\n}\n";
  if (V) {
    k << "DEV void se_in_vec(idx_t n, idx_t c, idx_t hw, float* v, " << kparams << ") {\n";
    decl_src_atoms("c");
    k << "  typedef elem_t xvec_t __attribute__((ext_vector_type(" << V << ")));\n";
    k << "  const xvec_t xv = *(const xvec_t*)(p" << pslot.at(kp.nodes[xnode].tensor) << " + (" << kp.addr_expr(kp.nodes[xnode].addr) << "));\n";
    k << "#pragma unroll\n  for (int u = 0; u < " << V << "; ++u) v[u] = cvt_in(xv[u]);\n}\n";
  }
  // first layer's result -> the second layer's operand, as the separate kernel would have stored it
  k << "DEV float se_mid(idx_t n, idx_t j, float anchor_v, " << kparams << ") {\n";
  decl_digits(k, k1, f1.n_atoms, "n", "  ", "qn");
  decl_digits(k, k1, f1.c_atoms, "j", "  ", "qj");
  if (bs1 >= 0) k << "  anchor_v += cvt_in(p" << bs1 << "[j]);\n";
  {
    std::set<int> done;
    k1.emit_values(k, {k1.stores[0].value}, done, pslot, "  ");
  }
  k << "  elem_t t_; cvt_out(&t_, " << k1.vname(k1.stores[0].value) << ");\n  return cvt_in(t_);\n}\n";
  // second layer's result -> the block's outputs
  k << "DEV void se_out(idx_t n, idx_t c, float anchor_v, " << kparams << ") {\n";
  decl_digits(k, k2, f2.n_atoms, "n", "  ", "qn");
  decl_digits(k, k2, f2.c_atoms, "c", "  ", "qc");
  if (bs2 >= 0) k << "  anchor_v += cvt_in(p" << bs2 << "[c]);\n";
  {
    std::set<int> done;
    std::vector<int> roots;
    for (auto& s : k2.stores) roots.push_back(s.value);
    k2.emit_values(k, roots, done, pslot, "  ");
    for (auto& s : k2.stores) {
      std::string st = k2.store_stmt(s, pslot, k2.addr_expr(s.addr));
      if (s.preds.empty()) k << "  " << st << "\n";
      else k << "  if (" << k2.pred_expr(s.preds) << ") { " << st << " }\n";
    }
  }
  k << "}\n";
  k << "#define KPARAMS " << kparams << "\n#define KARGS " << kargs << "\n";
  k << kSeBody;

  Lowered Lw;
  Lw.family = FAM_SE;
  Lw.ext_in.assign(params.begin(), params.begin() + n_in);
  Lw.ext_out.assign(params.begin() + n_in, params.end());
  Launch Kn;
  Kn.params = params;
  Kn.grid[0] = (unsigned)N;
  Kn.block[0] = 512;
  std::string src = std::string(device_preamble()) + k.str();
  Kn.name = fnv_name("dnnf_se", src);
  size_t pos;
  while ((pos = src.find("KNAME")) != std::string::npos) src.replace(pos, 5, Kn.name);
  Kn.source = src;
  Lw.launches.push_back(Kn);
  Lw.variant = std::string(gap >= 0 ? "pool" + std::to_string(HW) + "_" : "") + "fc" + std::to_string(C) + "x" + std::to_string(CR) + "x" + std::to_string(CO) +
               (V ? "_v" + std::to_string(V) : "");
  return Lw;
}

}  // namespace dnnf
