// Block lowering: data-flow walk (paper Sec. 4.4.1), index folding for Reorganize/Shuffle
// (Sec. 4.4.2), expression emission.
#include "lower_ctx.hpp"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <limits>

namespace dnnf {

// Device-side helpers prepended to every generated translation unit.
const char* device_preamble() {
  return R"PRE(
typedef unsigned short u16;
typedef unsigned int u32;
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef u16 u16x2 __attribute__((ext_vector_type(2)));
typedef u16 u16x4 __attribute__((ext_vector_type(4)));
typedef u16 u16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
#define DEV static __device__ __forceinline__
DEV float bf2f(u16 h) { return __builtin_bit_cast(float, ((u32)h) << 16); }
// (the compiler turns the conversion into gfx950's own instruction, two values at a time: round to nearest even, NaN
// stays NaN - two to three vector instructions per value less than rounding by integer arithmetic)
DEV u16 f2bf(float f) { return __builtin_bit_cast(u16, (__bf16)f); }
DEV float cvt_in(float v) { return v; }
DEV float cvt_in(_Float16 v) { return (float)v; }
DEV float cvt_in(u16 v) { return bf2f(v); }
DEV float cvt_in(int v) { return (float)v; }
DEV float cvt_in(long long v) { return (float)v; }
DEV void cvt_out(float* p, float v) { *p = v; }
DEV void cvt_out(_Float16* p, float v) { *p = (_Float16)v; }
DEV void cvt_out(u16* p, float v) { *p = f2bf(v); }
DEV void cvt_out(long long* p, long long v) { *p = v; }
DEV void cvt_out(int* p, long long v) { *p = (int)v; }
DEV void cvt_out(unsigned char* p, long long v) { *p = (unsigned char)(v != 0); }      // truth values are stored as 0 / 1
DEV void cvt_out(unsigned char* p, float v) { *p = (unsigned char)(v != 0.0f); }
// A vector store of a result too large to stay in the L2 caches until somebody reads it: the non-temporal form keeps the
// stream of results from displacing the operand tiles that neighbouring workgroups are about to read again.  (The
// compiler's builtin, not inline assembly: a store of more than 8 bytes needs wait states before its data registers are
// written again, which the compiler only inserts behind stores it has emitted itself - an assembly store followed by
// the next address computation in those registers stored the wrong values for some lanes.)
template <typename V> DEV void dn_store_stream(V* p, const V v) { __builtin_nontemporal_store(v, p); }
// fp32 math.  v_rcp_f32 / v_exp_f32 / v_sqrt_f32 are accurate to 1 ulp; the wrappers below add
// at most a few ulps.  The *_r variants are for arguments whose range the generator has proven
// (see node_range): they drop the work that only the excluded region needs.
DEV float dn_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
DEV float dn_div(float a, float b) { return a * __builtin_amdgcn_rcpf(b); }
DEV float dn_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
DEV float dn_sqrt_r(float x) { return __builtin_amdgcn_sqrtf(x); }           // x positive and normal
DEV float dn_exp_r(float x) { return dn_exp2(x * 1.44269504f); }             // |x| <= 16: error <= |x| * 2^-24 relative
DEV float dn_exp(float x) {
  // e^x = 2^(hi + lo) with x * log2(e) carried in two floats, so the error stays ~1 ulp for any x
  const float hi = x * 1.44269504f;
  const float lo = __builtin_fmaf(x, 1.44269504f, -hi) + x * 1.92596299e-8f;
  const float r = dn_exp2(hi);
  const float y = __builtin_fmaf(r, lo * 0.693147181f, r);
  return __builtin_fabsf(hi) < 160.0f ? y : r;                                // r is already 0 or inf out there
}
DEV float dn_sigmoid_r(float x) { return dn_rcp(1.0f + dn_exp2(x * -1.44269504f)); }   // x >= -16
DEV float dn_sigmoid(float x) { return dn_rcp(1.0f + dn_exp(-x)); }
// |x| >= 0.3, or any x where the result is stored in a 16-bit type: below 0.3 the closed form cancels, its absolute
// error stays <= 1.2e-7 (a fraction of a 16-bit ulp of any value above 1e-3; the polynomial costs nine more instructions)
DEV float dn_tanh_r(float x) {
  const float t = dn_exp2(__builtin_fabsf(x) * 2.88539008f);                 // e^(2|x|)
  return __builtin_copysignf(__builtin_fmaf(-2.0f, dn_rcp(1.0f + t), 1.0f), x);
}
DEV float dn_tanh_p(float x) {                                               // x >= 0.3: no sign to restore
  return __builtin_fmaf(-2.0f, dn_rcp(1.0f + dn_exp2(x * 2.88539008f)), 1.0f);
}
DEV float dn_tanh(float x) {
  // below 0.3 the closed form cancels; the odd Taylor polynomial through x^9 is exact to < 6e-8 there
  const float x2 = x * x;
  const float p = x * __builtin_fmaf(x2, __builtin_fmaf(x2, __builtin_fmaf(x2, __builtin_fmaf(x2, 0.0218694885f, -0.0539682540f),
                                                                             0.133333333f), -0.333333333f), 1.0f);
  return __builtin_fabsf(x) < 0.3f ? p : dn_tanh_r(x);
}
DEV float dn_erf_r(float x) {
  // rational approximation 7.1.26 of Abramowitz & Stegun, absolute error <= 1.5e-7; used where |x| >= 0.1
  // (relative error <= 2e-6) or where the result is stored in a 16-bit type
  const float ax = __builtin_fabsf(x);
  const float t = dn_rcp(__builtin_fmaf(0.3275911f, ax, 1.0f));
  const float p = t * __builtin_fmaf(t, __builtin_fmaf(t, __builtin_fmaf(t, __builtin_fmaf(t, 1.061405429f, -1.453152027f), 1.421413741f),
                                                       -0.284496736f), 0.254829592f);
  return __builtin_copysignf(__builtin_fmaf(-p, dn_exp2(ax * ax * -1.44269504f), 1.0f), x);
}
DEV float dn_erf_p(float x) {                                                // dn_erf_r for x >= 0
  const float t = dn_rcp(__builtin_fmaf(0.3275911f, x, 1.0f));
  const float p = t * __builtin_fmaf(t, __builtin_fmaf(t, __builtin_fmaf(t, __builtin_fmaf(t, 1.061405429f, -1.453152027f), 1.421413741f),
                                                       -0.284496736f), 0.254829592f);
  return __builtin_fmaf(-p, dn_exp2(x * x * -1.44269504f), 1.0f);
}
// index of a gathered axis of length n: negative values count from the end, the result always lies inside [0, n)
DEV long long dn_gidx(long long i, long long n) { i += i < 0 ? n : 0; return i < 0 ? 0 : (i < n ? i : n - 1); }
DEV long long dn_gidx(float v, long long n) { return v >= 9.0e18f ? n - 1 : (v > -9.0e18f ? dn_gidx((long long)v, n) : 0); }   // NaN -> 0
DEV float dn_wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
DEV float dn_wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
)PRE";
}

std::string fnv_name(const std::string& prefix, const std::string& body) {
  unsigned long long h = 1469598103934665603ull;
  for (unsigned char ch : body) { h ^= ch; h *= 1099511628211ull; }
  char buf[40];
  snprintf(buf, sizeof buf, "_%016llx", h);
  return prefix + buf;
}

void block_io(const Graph& g, const Block& b, std::vector<int>& ext_in, std::vector<int>& ext_out,
              std::vector<int>& removed) {
  std::set<int> inb(b.ops.begin(), b.ops.end());
  std::set<int> seen_in, seen_out;
  for (int oi : b.ops) {
    const Op& op = g.ops[oi];
    for (int t : op.in) {
      const Tensor& T = g.tensors[t];
      bool internal = T.producer >= 0 && inb.count(T.producer);
      if (!internal && !seen_in.count(t)) { seen_in.insert(t); ext_in.push_back(t); }
    }
    for (int t : op.out) {
      const Tensor& T = g.tensors[t];
      bool outside = T.kind == DNNF_OUTPUT;
      for (int c : T.consumers) outside = outside || !inb.count(c);
      if (outside) { if (!seen_out.count(t)) { seen_out.insert(t); ext_out.push_back(t); } }
      else removed.push_back(t);
    }
  }
}

LowerCtx::LowerCtx(const Graph& g_, const Block& b_, const LowerOpts& o_) : g(g_), blk(b_), opts(o_) {
  inblock.insert(b_.ops.begin(), b_.ops.end());
  std::vector<int> ein, eout, rem;
  block_io(g_, b_, ein, eout, rem);
  lowp = !eout.empty();
  for (int t : eout) lowp = lowp && dtype_bytes(g_.tensors[t].dtype) == 2;
}

int LowerCtx::new_atom(int64_t extent) {
  atom_extent.push_back(extent);
  atom_split.push_back({-1, -1});
  return (int)atom_extent.size() - 1;
}

void LowerCtx::resolve(const std::vector<int>& in, std::vector<int>& out) const {
  for (int a : in) {
    if (atom_split[a].first >= 0) resolve({atom_split[a].first, atom_split[a].second}, out);
    else if (atom_extent[a] > 1) out.push_back(a);
  }
}

std::string LowerCtx::decl_parts(const std::vector<int>& atoms, const std::string& ind) const {
  std::string s;
  for (int a : atoms) {
    if (atom_split[a].first < 0) continue;
    const int hi = atom_split[a].first, lo = atom_split[a].second;
    s += ind + "const idx_t a" + std::to_string(hi) + " = a" + std::to_string(a) + " / " + std::to_string(atom_extent[lo]) + ", a" + std::to_string(lo) +
         " = a" + std::to_string(a) + " % " + std::to_string(atom_extent[lo]) + ";\n";
    s += decl_parts({hi, lo}, ind);
  }
  return s;
}

int64_t LowerCtx::extent_of(const std::vector<int>& atoms) const {
  int64_t e = 1;
  for (int a : atoms) e *= atom_extent[a];
  return e;
}

TIdx LowerCtx::fresh_index(const Dims& dims) {
  TIdx t(dims.size());
  for (size_t d = 0; d < dims.size(); d++)
    if (dims[d] > 1) t[d].atoms.push_back(new_atom(dims[d]));
  return t;
}

// Re-express an index given for extents src_dims as an index for dst_dims of the same
// row-major element order (Reshape and friends).  Atoms are split where the new extents cut
// through them; an extent pair with no common factorisation has no index-only form.
TIdx LowerCtx::regroup(const TIdx& src, const Dims& src_dims, const Dims& dst_dims) {
  TIdx out(dst_dims.size());
  // The two shapes are cut into segments of equal element count (positions where the running products of the
  // extents coincide).  A segment that is one dimension on either side is an axis the Reshape leaves alone: its
  // index passes through whatever it is (a sliced, partial or gathered index included).  Any other segment has its
  // atoms re-dealt to the new extents.
  size_t i = 0, j = 0;
  while (i < src_dims.size() || j < dst_dims.size()) {
    size_t i1 = i, j1 = j;
    int64_t ps = 1, pd = 1;
    // extent-1 dimensions carry no index: skip them on either side
    if (i < src_dims.size() && src_dims[i] == 1 && !(j < dst_dims.size() && dst_dims[j] == 1)) { i++; continue; }
    if (j < dst_dims.size() && dst_dims[j] == 1 && !(i < src_dims.size() && src_dims[i] == 1)) { j++; continue; }
    DNNF_CHECK(i < src_dims.size() && j < dst_dims.size(), DNNF_UNSUPPORTED_OP, "Reshape: extents do not match");
    ps = src_dims[i1++];
    pd = dst_dims[j1++];
    while (ps != pd) {
      if (ps < pd) { DNNF_CHECK(i1 < src_dims.size(), DNNF_UNSUPPORTED_OP, "Reshape: extents do not match"); ps *= src_dims[i1++]; }
      else { DNNF_CHECK(j1 < dst_dims.size(), DNNF_UNSUPPORTED_OP, "Reshape: extents do not match"); pd *= dst_dims[j1++]; }
    }
    if (i1 - i == 1 && j1 - j == 1) {
      out[j] = src[i];
    } else {
      std::vector<int> flat;
      for (size_t d = i; d < i1; d++) {
        DNNF_CHECK(src[d].offset == 0 && src[d].indirect < 0, DNNF_UNSUPPORTED_OP,
                   "Reshape of a sliced or gathered axis has no index-only form");
        std::vector<int> r;
        resolve(src[d].atoms, r);
        DNNF_CHECK(extent_of(r) == src_dims[d] || (r.empty() && src_dims[d] >= 1), DNNF_UNSUPPORTED_OP,
                   "Reshape of a broadcast axis");
        if (r.empty() && src_dims[d] > 1) throw Error(DNNF_UNSUPPORTED_OP, "Reshape of a broadcast axis");
        flat.insert(flat.end(), r.begin(), r.end());
      }
      size_t pos = 0;
      for (size_t d = j; d < j1; d++) {
        int64_t need = dst_dims[d];
        while (need > 1) {
          DNNF_CHECK(pos < flat.size(), DNNF_UNSUPPORTED_OP, "Reshape: ran out of index atoms");
          int a = flat[pos];
          int64_t e = atom_extent[a];
          if (e <= need) {
            DNNF_CHECK(need % e == 0, DNNF_UNSUPPORTED_OP, "Reshape extents have no common factorisation");
            out[d].atoms.push_back(a);
            need /= e;
            pos++;
          } else {
            DNNF_CHECK(e % need == 0, DNNF_UNSUPPORTED_OP, "Reshape extents have no common factorisation");
            int hi = new_atom(need), lo = new_atom(e / need);
            atom_split[a] = {hi, lo};
            out[d].atoms.push_back(hi);
            flat[pos] = lo;
            need = 1;
          }
        }
      }
      DNNF_CHECK(pos == flat.size(), DNNF_UNSUPPORTED_OP, "Reshape: unused index atoms");
    }
    i = i1;
    j = j1;
  }
  return out;
}

// DepthToSpace / SpaceToDepth as Reshape(mid_in) - Transpose(perm) - Reshape(out); mid_out = mid_in permuted.
static void d2s_chain(const Op& op, const Dims& x, Dims& mid_in, std::vector<int>& perm, Dims& mid_out) {
  const int64_t b = op.i("blocksize", 1);
  if (op.kind == "DepthToSpace") {
    const int64_t cp = x[1] / (b * b);
    if (op.i("mode_crd", 0)) { mid_in = {x[0], cp, b, b, x[2], x[3]}; perm = {0, 1, 4, 2, 5, 3}; }     // column-row-depth
    else { mid_in = {x[0], b, b, cp, x[2], x[3]}; perm = {0, 3, 4, 1, 5, 2}; }                          // depth-column-row (default)
  } else {
    mid_in = {x[0], x[1], x[2] / b, b, x[3] / b, b};
    perm = {0, 3, 5, 1, 2, 4};
  }
  mid_out.clear();
  for (int p : perm) mid_out.push_back(mid_in[p]);
}

Affine LowerCtx::affine(const Tensor& T, const TIdx& idx) {
  const Dims& dims = T.dims;
  Affine a;
  int64_t stride = 1;
  for (int k = (int)dims.size() - 1; k >= 0; k--) {
    const int d = T.perm.empty() ? k : T.perm[k];
    const DimIdx& di = idx[d];
    if (di.indirect >= 0) a.indirect.push_back({di.indirect, stride, dims[d]});
    std::vector<int> r;
    resolve(di.atoms, r);
    int64_t mult = 1;
    for (int j = (int)r.size() - 1; j >= 0; j--) {
      a.stride[r[j]] += stride * mult;
      mult *= atom_extent[r[j]];
    }
    a.offset += di.offset * stride;
    stride *= dims[d];
  }
  return a;
}

Affine LowerCtx::resolved(const Affine& in) const {
  Affine out;
  out.offset = in.offset;
  out.indirect = in.indirect;
  for (auto& kv : in.stride) {
    std::vector<int> r;
    resolve({kv.first}, r);
    int64_t mult = 1;
    for (int k = (int)r.size() - 1; k >= 0; k--) {
      out.stride[r[k]] += kv.second * mult;
      mult *= atom_extent[r[k]];
    }
  }
  return out;
}

std::vector<int> LowerCtx::final_atoms() const {
  std::vector<int> r;
  for (size_t a = 0; a < atom_extent.size(); a++)
    if (atom_split[a].first < 0 && atom_extent[a] > 1) r.push_back((int)a);
  return r;
}

bool LowerCtx::is_external(int t) const {
  const Tensor& T = g.tensors[t];
  return T.producer < 0 || !inblock.count(T.producer);
}

static std::string affine_sig(const Affine& a) {
  std::ostringstream s;
  for (auto& kv : a.stride) if (kv.second) s << kv.first << "*" << kv.second << "+";
  s << a.offset;
  for (auto& p : a.indirect) s << "+n" << p.first << "*" << p.second << "%" << p.extent;
  return s.str();
}

int LowerCtx::add_node(const ENode& n) {
  std::ostringstream key;
  key << (int)n.kind << "|" << n.tensor << "|" << affine_sig(n.addr) << "|" << n.op << "|" << (const void*)n.src << "|";
  for (int a : n.args) key << a << ",";
  char cvb[40];
  snprintf(cvb, sizeof cvb, "%.17g", n.cv);
  key << "|" << cvb;
  auto it = cse.find(key.str());
  if (it != cse.end()) return it->second;   // common sub-tree: emitted once
  nodes.push_back(n);
  cse[key.str()] = (int)nodes.size() - 1;
  return (int)nodes.size() - 1;
}

static TIdx broadcast_index(const TIdx& out_idx, const Dims& out_dims, const Dims& in_dims) {
  TIdx r(in_dims.size());
  size_t shift = out_dims.size() - in_dims.size();
  for (size_t d = 0; d < in_dims.size(); d++)
    if (in_dims[d] != 1 || out_dims[d + shift] == 1) r[d] = out_idx[d + shift];
  return r;
}

int LowerCtx::value(int t, const TIdx& idx) {
  const Tensor& T = g.tensors[t];
  DNNF_CHECK(idx.size() == T.dims.size(), DNNF_UNSUPPORTED_OP, "index rank mismatch at " + T.name);
  if (!tidx.count(t)) tidx[t] = idx;
  if (t == anchor_out) {
    // The anchor's result exists only at the index its kernel computes it for.  A block that needs it at a second
    // index as well (the result and a channel-shuffled copy of it added together, say) has no single-pass kernel.
    const TIdx& own = tidx[t];
    for (size_t d = 0; d < idx.size(); d++) {
      if (T.dims[d] == 1) continue;
      bool same = idx[d].indirect < 0 && own[d].indirect < 0;
      // both indices as linear functions of the finest atoms
      std::map<int, int64_t> diff;
      for (int side = 0; side < 2 && same; side++) {
        std::vector<int> r;
        resolve(side ? own[d].atoms : idx[d].atoms, r);
        int64_t mult = 1;
        for (int k = (int)r.size() - 1; k >= 0; k--) {
          diff[r[k]] += side ? -mult : mult;
          mult *= atom_extent[r[k]];
        }
      }
      const int64_t dconst = idx[d].offset - own[d].offset;
      std::vector<int> moving;
      for (auto& kv : diff) if (kv.second != 0) moving.push_back(kv.first);
      if (same && (!moving.empty() || dconst != 0)) {
        // the two may still agree where a store's predicate holds: the parts of a Split behind the anchor are read
        // back at (offset of part k) + position, which is the anchor's own column when the part digit equals k
        // (only the predicate of the store being built counts: a value that combines two parts of the Split
        // would need the anchor at two columns at once)
        same = false;
        if (moving.size() == 1)
          for (auto& pr : cur_preds) {
            std::vector<int> pa;
            resolve(pr.atoms, pa);
            if (pr.hi <= pr.lo && pa.size() == 1 && pa[0] == moving[0] && diff[moving[0]] * pr.equals + dconst == 0) same = true;
          }
      }
      DNNF_CHECK(same, DNNF_UNSUPPORTED_OP, "the block reads " + T.name + " at an index other than the one its kernel produces it at");
    }
    ENode n;
    n.kind = ENode::ANCHOR;
    n.tensor = t;
    n.is_int = !is_float(T.dtype);      // the result of an integer reduction stays an integer
    return add_node(n);
  }
  if (T.has_cval && T.n() == 1 && is_external(t)) {
    ENode n;
    n.kind = ENode::CONSTV;
    n.cv = T.cval[0];
    return add_node(n);
  }
  if (is_external(t)) {
    ENode n;
    n.kind = ENode::LOAD;
    n.tensor = t;
    n.addr = affine(T, idx);
    n.is_int = !is_float(T.dtype);
    return add_node(n);
  }
  const Op& op = g.ops[T.producer];
  auto in_dims = [&](int k) -> const Dims& { return g.tensors[op.in[k]].dims; };
  ENode n;
  n.kind = ENode::OP;
  n.op = op.kind;
  n.src = &op;
  switch (op.info->cls) {
    case OC_UNARY:
      n.args = {value(op.in[0], idx)};
      if (op.kind == "Identity" || op.kind == "Cast") return n.args[0];
      return add_node(n);
    case OC_BINARY:
    case OC_WHERE:
      for (size_t k = 0; k < op.in.size(); k++)
        n.args.push_back(value(op.in[k], broadcast_index(idx, T.dims, in_dims((int)k))));
      if (op.kind == "BitShift") {
        // the one integer operator: 64-bit shift of an integer tensor, the result integer-typed as well
        DNNF_CHECK(!is_float(T.dtype) && !is_float(g.tensors[op.in[0]].dtype), DNNF_UNSUPPORTED_OP, "BitShift of a floating-point tensor");
        n.is_int = true;
      }
      return add_node(n);
    case OC_BATCHNORM: {
      DNNF_CHECK(op.in.size() == 5 && T.dims.size() >= 2, DNNF_INVALID_ARG, "BatchNormalization operands");
      n.args.push_back(value(op.in[0], idx));
      TIdx ch(1);
      ch[0] = idx[1];
      for (int k = 1; k < 5; k++) n.args.push_back(value(op.in[k], ch));
      return add_node(n);
    }
    case OC_RESHAPE:
      return value(op.in[0], regroup(idx, T.dims, in_dims(0)));
    case OC_TRANSPOSE: {
      auto perm = op.ints("perm");
      if (perm.empty()) for (int i = (int)T.dims.size() - 1; i >= 0; i--) perm.push_back(i);
      TIdx in(idx.size());
      for (size_t k = 0; k < idx.size(); k++) in[perm[k]] = idx[k];
      return value(op.in[0], in);
    }
    case OC_D2S: {
      // Reshape - Transpose - Reshape (the operator's definition), walked backwards: no code, only an index map
      Dims mid_in, mid_out;
      std::vector<int> perm;
      d2s_chain(op, in_dims(0), mid_in, perm, mid_out);
      TIdx t6 = regroup(idx, T.dims, mid_out), s6(t6.size());
      for (size_t k = 0; k < t6.size(); k++) s6[perm[k]] = t6[k];
      return value(op.in[0], regroup(s6, mid_in, in_dims(0)));
    }
    case OC_SLICE: {
      TIdx in = idx;
      auto st = op.ints("starts"), ax = op.ints("axes"), sp = op.ints("steps");
      for (size_t i = 0; i < st.size(); i++) {
        int a = (int)(ax.empty() ? (int64_t)i : ax[i]);
        if (a < 0) a += (int)idx.size();
        DNNF_CHECK(sp.empty() || sp[i] == 1, DNNF_UNSUPPORTED_OP, "Slice with step != 1");
        int64_t d = in_dims(0)[a], s = st[i] < 0 ? st[i] + d : st[i];
        in[a].offset += std::min(std::max<int64_t>(s, 0), d);
      }
      return value(op.in[0], in);
    }
    case OC_SPLIT: {
      TIdx in = idx;
      int a = (int)op.i("axis", 0);
      if (a < 0) a += (int)idx.size();
      int64_t start = 0;
      for (size_t k = 0; k < op.out.size() && op.out[k] != t; k++) start += g.tensors[op.out[k]].dims[a];
      in[a].offset += start;
      return value(op.in[0], in);
    }
    case OC_EXPAND:
      return value(op.in[0], broadcast_index(idx, T.dims, in_dims(0)));
    case OC_RESIZE: {
      // nearest neighbour by an integer factor s: output index i reads input index i / s, i.e. the
      // major digit when the axis index is regrouped as (extent / s, s)
      auto sc = op.ints("scales");
      TIdx in = idx;
      for (size_t d = 0; d < idx.size(); d++) {
        if (sc[d] == 1) continue;
        DNNF_CHECK(idx[d].offset == 0 && idx[d].indirect < 0, DNNF_UNSUPPORTED_OP, "Resize of a sliced axis");
        TIdx one(1);
        one[0] = idx[d];
        TIdx two = regroup(one, {T.dims[d]}, {in_dims(0)[d], sc[d]});
        in[d] = two[0];
      }
      return value(op.in[0], in);
    }
    case OC_CONCAT: {
      // only as the last operator of a block that is lowered part by part (see lower_block): this
      // context covers the index range of one operand
      DNNF_CHECK(concat_part >= 0 && &op == &g.ops[concat_op], DNNF_UNSUPPORTED_OP, "Concat inside a fused expression");
      int a = (int)op.i("axis", 0);
      if (a < 0) a += (int)idx.size();
      int64_t start = 0;
      for (int k = 0; k < concat_part; k++) start += g.tensors[op.in[k]].dims[a];
      TIdx in = idx;
      in[a].offset -= start;
      return value(op.in[concat_part], in);
    }
    case OC_GATHER: {
      // out[.., j.., ..] = data[.., indices[j..], ..]: the index tensor's axes stand where the gathered axis stood
      int64_t ax = op.i("axis", 0);
      if (ax < 0) ax += (int64_t)in_dims(0).size();
      const size_t a = (size_t)ax, ri = in_dims(1).size();
      TIdx ii(idx.begin() + a, idx.begin() + a + ri);
      int iv = value(op.in[1], ii);
      TIdx di(in_dims(0).size());
      for (size_t d = 0; d < a; d++) di[d] = idx[d];
      di[a].indirect = iv;
      for (size_t d = a + 1; d < di.size(); d++) di[d] = idx[ri + d - 1];
      return value(op.in[0], di);
    }
    default:
      throw Error(DNNF_UNSUPPORTED_OP, "operator " + op.kind + " cannot be evaluated inside a fused expression");
  }
}

// Forward direction: an element of an input known at pivot index I lands at which index of the
// operator's output?  Only operators whose index map is invertible are handled.
bool LowerCtx::forward_step(const Op& op) {
  bool progress = false;
  for (size_t oi = 0; oi < op.out.size(); oi++) {
    int o = op.out[oi];
    if (tidx.count(o)) continue;
    const Tensor& O = g.tensors[o];
    for (size_t k = 0; k < op.in.size() && !tidx.count(o); k++) {
      int i = op.in[k];
      if (!tidx.count(i)) continue;
      const Tensor& I = g.tensors[i];
      const TIdx& ti = tidx[i];
      std::vector<Pred> preds = tpred.count(i) ? tpred[i] : std::vector<Pred>();
      try {
      switch (op.info->cls) {
        case OC_UNARY: case OC_BINARY: case OC_WHERE: case OC_BATCHNORM: {
          if (I.n() != O.n()) break;
          if (op.info->cls == OC_BATCHNORM && k != 0) break;
          TIdx to(O.dims.size());
          size_t shift = O.dims.size() - I.dims.size();
          for (size_t d = 0; d < I.dims.size(); d++) to[d + shift] = ti[d];
          tidx[o] = to;
          break;
        }
        case OC_RESHAPE:
          tidx[o] = regroup(ti, I.dims, O.dims);
          break;
        case OC_TRANSPOSE: {
          auto perm = op.ints("perm");
          if (perm.empty()) for (int d = (int)I.dims.size() - 1; d >= 0; d--) perm.push_back(d);
          TIdx to(perm.size());
          for (size_t d = 0; d < perm.size(); d++) to[d] = ti[perm[d]];
          tidx[o] = to;
          break;
        }
        case OC_D2S: {
          Dims mid_in, mid_out;
          std::vector<int> perm;
          d2s_chain(op, I.dims, mid_in, perm, mid_out);
          TIdx s6 = regroup(ti, I.dims, mid_in), t6(s6.size());
          for (size_t d = 0; d < perm.size(); d++) t6[d] = s6[perm[d]];
          tidx[o] = regroup(t6, mid_out, O.dims);
          break;
        }
        case OC_SLICE: {
          // the element at input index i lands at i - start, if start <= i < end: a range predicate on the axis
          TIdx to = ti;
          auto st = op.ints("starts"), en = op.ints("ends"), ax = op.ints("axes"), sp = op.ints("steps");
          for (size_t q = 0; q < st.size(); q++) {
            int a = (int)(ax.empty() ? (int64_t)q : ax[q]);
            if (a < 0) a += (int)I.dims.size();
            DNNF_CHECK(sp.empty() || sp[q] == 1, DNNF_UNSUPPORTED_OP, "Slice with step != 1");
            DNNF_CHECK(ti[a].indirect < 0, DNNF_UNSUPPORTED_OP, "Slice of a gathered axis");
            const int64_t d = I.dims[a];
            const int64_t lo = std::min(std::max<int64_t>(st[q] < 0 ? st[q] + d : st[q], 0), d);
            const int64_t hi = std::min(std::max<int64_t>(en[q] < 0 ? en[q] + d : en[q], lo), d);
            DNNF_CHECK(hi - lo == O.dims[a], DNNF_SHAPE_MISMATCH, "Slice extent");
            if (lo == 0 && hi == d) continue;
            Pred p;                                   // on the digits alone: the index is digits + offset
            p.atoms = ti[a].atoms;
            p.lo = lo - ti[a].offset;
            p.hi = hi - ti[a].offset;
            preds.push_back(p);
            to[a].offset -= lo;
          }
          tidx[o] = to;
          break;
        }
        case OC_CONCAT: {
          // the block-closing Concat, seen from the one operand this context lowers: its elements land at the
          // operand's offset along the axis (the other operands are written by kernels of their own)
          if (concat_part < 0 || &op != &g.ops[concat_op] || (int)k != concat_part) break;
          int a = (int)op.i("axis", 0);
          if (a < 0) a += (int)I.dims.size();
          int64_t start = 0;
          for (int q = 0; q < concat_part; q++) start += g.tensors[op.in[q]].dims[a];
          TIdx to = ti;
          to[a].offset += start;
          tidx[o] = to;
          break;
        }
        case OC_RESIZE: {
          // nearest neighbour by integer factors: the element at input index i lands at i * s + r for every r < s
          if (!allow_replication || k != 0) break;
          auto sc = op.ints("scales");
          TIdx to = ti;
          for (size_t d = 0; d < ti.size(); d++) {
            if (sc[d] == 1) continue;
            DNNF_CHECK(ti[d].offset == 0 && ti[d].indirect < 0, DNNF_UNSUPPORTED_OP, "Resize of a sliced axis");
            const int r = new_atom(sc[d]);
            rep_atoms.push_back(r);
            to[d].atoms.push_back(r);
          }
          tidx[o] = to;
          break;
        }
        case OC_SPLIT: {
          int a = (int)op.i("axis", 0);
          if (a < 0) a += (int)I.dims.size();
          int64_t parts = (int64_t)op.out.size(), len = O.dims[a];
          DNNF_CHECK(len * parts == I.dims[a], DNNF_UNSUPPORTED_OP, "Split into unequal parts after the block's anchor");
          DNNF_CHECK(ti[a].offset == 0 && ti[a].indirect < 0, DNNF_UNSUPPORTED_OP, "Split of a sliced axis");
          TIdx one(1);
          one[0] = ti[a];
          TIdx two = regroup(one, {I.dims[a]}, {parts, len});
          // parts of length 1 pass through the regrouping as they are: an index that stays inside one part (the
          // block's pivot is another part of this Split) would leave a predicate that never holds
          std::vector<int> digit;
          resolve(two[0].atoms, digit);
          DNNF_CHECK(parts == 1 || extent_of(digit) == parts, DNNF_UNSUPPORTED_OP, "Split of an axis that the block's index space covers in part");
          TIdx to = ti;
          to[a] = two[1];
          Pred p;
          p.atoms = two[0].atoms;
          p.equals = (int64_t)oi;
          if (parts > 1) preds.push_back(p);
          tidx[o] = to;
          break;
        }
        default:
          break;
      }
      } catch (const Error&) {
        tidx.erase(o);   // no invertible index map along this edge
      }
      if (tidx.count(o)) {
        if (!preds.empty()) tpred[o] = preds;
        progress = true;
      }
    }
  }
  return progress;
}

void LowerCtx::forward_all() {
  bool again = true;
  while (again) {
    again = false;
    for (int oi : blk.ops) {
      if (oi == anchor_op) continue;
      again = forward_step(g.ops[oi]) || again;
    }
  }
}

void LowerCtx::collect_stores(const std::vector<int>& outs) {
  for (int t : outs) {
    if (t == anchor_out && !tidx.count(t)) throw Error(DNNF_UNSUPPORTED_OP, "anchor output has no index");
    DNNF_CHECK(tidx.count(t), DNNF_UNSUPPORTED_OP,
               "block output " + g.tensors[t].name + " is not reachable from the block's pivot by invertible index maps");
    Store s;
    s.tensor = t;
    TIdx ix = tidx[t];
    // The kernel's index space must reach every element of a result.  An index derived backwards through a Slice
    // (or a Gather) covers only the part its consumer reads: such a tensor cannot be stored from this pivot.
    if (concat_part < 0)
      for (size_t d = 0; d < ix.size(); d++) {
        std::vector<int> fine;
        resolve(ix[d].atoms, fine);
        int64_t span = 1;
        for (int a : fine) span *= atom_extent[a];
        // (an index space reaching beyond the tensor comes from a forward walk through a Slice, which also left
        // the range predicate that guards the store)
        const bool guarded = tpred.count(t) && !tpred[t].empty();
        const bool reaches = ix[d].offset <= 0 && ix[d].offset + span >= g.tensors[t].dims[d];
        const bool exact = ix[d].offset == 0 && span == g.tensors[t].dims[d];
        DNNF_CHECK(ix[d].indirect < 0 && (exact || (guarded && reaches)), DNNF_UNSUPPORTED_OP,
                   "block output " + g.tensors[t].name + " is only partly covered by the block's index space");
      }
    cur_preds = tpred.count(t) ? tpred[t] : std::vector<Pred>();
    s.value = value(t, ix);
    cur_preds.clear();
    s.addr = affine(g.tensors[t], ix);
    if (tpred.count(t)) s.preds = tpred[t];
    stores.push_back(s);
  }
}

// ------------------------------------------------------------------ emission
std::string LowerCtx::ctype(int dt) const {
  switch (dt) {
    case DNNF_F32: return "float";
    case DNNF_F16: return "_Float16";
    case DNNF_BF16: return "u16";
    case DNNF_I32: return "int";
    case DNNF_I64: return "long long";
    default: return "unsigned char";
  }
}

std::string LowerCtx::param_list(const std::vector<int>& params, const std::set<int>& written) const {
  std::ostringstream s;
  for (size_t k = 0; k < params.size(); k++) {
    if (k) s << ", ";
    const Tensor& T = g.tensors[params[k]];
    if (!written.count(params[k])) s << "const ";
    s << ctype(T.dtype) << "* __restrict__ p" << k;
  }
  return s.str();
}

std::string LowerCtx::addr_expr(const Affine& a0) const {
  Affine a = resolved(a0);
  std::ostringstream s;
  bool first = true;
  for (auto& kv : a.stride) {
    if (kv.second == 0) continue;
    if (!first) s << " + ";
    first = false;
    if (kv.second == 1) s << "a" << kv.first;
    else s << "a" << kv.first << " * " << kv.second;
  }
  for (auto& p : a.indirect) {
    if (!first) s << " + ";
    first = false;
    // an index outside the axis must never reach the address: negative values count from the end (as the
    // operator is defined), whatever is still outside is clamped to the nearest valid position
    s << "(idx_t)dn_gidx(" << vname(p.first) << ", " << p.extent << ") * " << p.second;
  }
  if (a.offset != 0 || first) {
    if (!first) s << " + ";
    s << a.offset;
  }
  return s.str();
}

std::string LowerCtx::pred_expr(const std::vector<Pred>& ps) const {
  std::ostringstream s;
  for (size_t i = 0; i < ps.size(); i++) {
    if (i) s << " && ";
    std::vector<int> r;
    resolve(ps[i].atoms, r);
    s << (ps[i].hi > ps[i].lo ? "(unsigned)((" : "(");
    if (r.empty()) s << "0";
    int64_t mult = 1;
    std::vector<std::string> terms;
    for (int k = (int)r.size() - 1; k >= 0; k--) {
      terms.push_back("a" + std::to_string(r[k]) + (mult == 1 ? "" : " * " + std::to_string(mult)));
      mult *= atom_extent[r[k]];
    }
    for (size_t k = 0; k < terms.size(); k++) s << (k ? " + " : "") << terms[k];
    if (ps[i].hi > ps[i].lo) s << ") - (" << ps[i].lo << ")) < (unsigned)" << ps[i].hi - ps[i].lo;      // one unsigned compare for the range
    else s << ") == " << ps[i].equals;
  }
  return s.str();
}

static std::string flit(double v) {
  char b[48];
  if (std::isinf(v)) return v > 0 ? "__builtin_inff()" : "(-__builtin_inff())";
  snprintf(b, sizeof b, "%.9g", (double)(float)v);
  std::string s = b;
  if (s.find('.') == std::string::npos && s.find('e') == std::string::npos && s.find("inf") == std::string::npos) s += ".0";
  return s + "f";
}

// Interval of values a node can take, propagated through the block's expression DAG.  It lets the
// generator pick a cheaper, equally accurate formulation of a transcendental when its argument is
// known to stay away from the region that needs the general one (e.g. exp of a clipped value,
// erf/tanh of a value bounded away from zero, sqrt of a value >= 1).
using Range = std::pair<double, double>;
static const double kInf = std::numeric_limits<double>::infinity();

static Range node_range(const LowerCtx& c, int n) {
  auto it = c.range_memo.find(n);
  if (it != c.range_memo.end()) return it->second;
  const ENode& e = c.nodes[n];
  Range r(-kInf, kInf);
  auto R = [&](int k) { return node_range(c, e.args[k]); };
  auto mono = [&](double (*f)(double), const Range& a) { return Range(f(a.first), f(a.second)); };
  if (e.kind == ENode::CONSTV) r = Range(e.cv, e.cv);
  else if (e.kind == ENode::OP) {
    const std::string& k = e.op;
    if (k == "Add") r = Range(R(0).first + R(1).first, R(0).second + R(1).second);
    else if (k == "Sub") r = Range(R(0).first - R(1).second, R(0).second - R(1).first);
    else if (k == "Neg") r = Range(-R(0).second, -R(0).first);
    else if (k == "Mul") {
      Range a = R(0), b = R(1);
      if (std::isfinite(a.first) && std::isfinite(a.second) && std::isfinite(b.first) && std::isfinite(b.second)) {
        double p[4] = {a.first * b.first, a.first * b.second, a.second * b.first, a.second * b.second};
        r = Range(*std::min_element(p, p + 4), *std::max_element(p, p + 4));
      } else if (e.args[0] == e.args[1]) r = Range(0, kInf);
    } else if (k == "Square" || (k == "Pow" && c.nodes[e.args[1]].kind == ENode::CONSTV && c.nodes[e.args[1]].cv == 2.0)) {
      Range a = R(0);
      double lo = (a.first <= 0 && a.second >= 0) ? 0.0 : std::min(a.first * a.first, a.second * a.second);
      r = Range(lo, std::max(a.first * a.first, a.second * a.second));
    } else if (k == "Abs") {
      Range a = R(0);
      double lo = (a.first <= 0 && a.second >= 0) ? 0.0 : std::min(std::fabs(a.first), std::fabs(a.second));
      r = Range(lo, std::max(std::fabs(a.first), std::fabs(a.second)));
    } else if (k == "Relu") r = Range(std::max(R(0).first, 0.0), std::max(R(0).second, 0.0));
    else if (k == "Clip") {
      Range a = R(0);
      double lo = e.src->has("min") ? e.src->f("min", 0) : -kInf, hi = e.src->has("max") ? e.src->f("max", 0) : kInf;
      r = Range(std::min(std::max(a.first, lo), hi), std::max(std::min(a.second, hi), lo));
    } else if (k == "Exp") r = mono([](double x) { return std::exp(x); }, R(0));
    else if (k == "Sigmoid") r = mono([](double x) { return 1.0 / (1.0 + std::exp(-x)); }, R(0));
    else if (k == "Tanh") r = mono([](double x) { return std::tanh(x); }, R(0));
    else if (k == "Erf") r = mono([](double x) { return std::erf(x); }, R(0));
    else if (k == "Sqrt") r = Range(std::sqrt(std::max(R(0).first, 0.0)), std::sqrt(std::max(R(0).second, 0.0)));
    else if (k == "Max") r = Range(std::max(R(0).first, R(1).first), std::max(R(0).second, R(1).second));
    else if (k == "Min") r = Range(std::min(R(0).first, R(1).first), std::min(R(0).second, R(1).second));
    if (std::isnan(r.first) || std::isnan(r.second)) r = Range(-kInf, kInf);
    // keep a safety margin for the rounding of the fp32 evaluation
    if (std::isfinite(r.first)) r.first -= 1e-5 * std::fabs(r.first) + 1e-30;
    if (std::isfinite(r.second)) r.second += 1e-5 * std::fabs(r.second) + 1e-30;
  }
  c.range_memo[n] = r;
  return r;
}

static std::string op_expr(const LowerCtx& c, const ENode& n) {
  auto A = [&](int k) { return c.vname(n.args[k]); };
  const std::string& k = n.op;
  const Op& op = *n.src;
  auto arg_range = [&](int i) { return node_range(c, n.args[i]); };
  auto within = [&](int i, double lo, double hi) { Range r = arg_range(i); return r.first >= lo && r.second <= hi; };
  if (k == "Add") return A(0) + " + " + A(1);
  if (k == "Sub") return A(0) + " - " + A(1);
  if (k == "Mul") return A(0) + " * " + A(1);
  if (k == "Div") {
    const ENode& d = c.nodes[n.args[1]];
    if (d.kind == ENode::CONSTV) {
      // division by a power of two is an exact multiplication
      int e;
      if (std::frexp(d.cv, &e) == 0.5) return A(0) + " * " + flit(1.0 / d.cv);
    }
    return "dn_div(" + A(0) + ", " + A(1) + ")";
  }
  if (k == "Pow") {
    const ENode& e = c.nodes[n.args[1]];
    if (e.kind == ENode::CONSTV) {
      if (e.cv == 2.0) return A(0) + " * " + A(0);
      if (e.cv == 3.0) return A(0) + " * " + A(0) + " * " + A(0);
      if (e.cv == 1.0) return A(0);
      if (e.cv == 0.5) return "sqrtf(" + A(0) + ")";
    }
    return "powf(" + A(0) + ", " + A(1) + ")";
  }
  if (k == "Max") return "fmaxf(" + A(0) + ", " + A(1) + ")";
  if (k == "Min") return "fminf(" + A(0) + ", " + A(1) + ")";
  if (k == "Greater") return "(" + A(0) + " > " + A(1) + " ? 1.0f : 0.0f)";
  if (k == "Where") return "(" + A(0) + " != 0.0f ? " + A(1) + " : " + A(2) + ")";
  if (k == "Relu") return "fmaxf(" + A(0) + ", 0.0f)";
  if (k == "Sigmoid") return (within(0, -16.0, kInf) || c.lowp ? "dn_sigmoid_r(" : "dn_sigmoid(") + A(0) + ")";
  if (k == "Tanh") {
    Range r = arg_range(0);
    return (r.first >= 0.3 ? "dn_tanh_p(" : (r.second <= -0.3 || c.lowp) ? "dn_tanh_r(" : "dn_tanh(") + A(0) + ")";
  }
  if (k == "Exp") return (within(0, -16.0, 16.0) || c.lowp ? "dn_exp_r(" : "dn_exp(") + A(0) + ")";
  if (k == "Log") return "logf(" + A(0) + ")";
  if (k == "Sqrt") return (within(0, 1e-30, 1e30) || c.lowp ? "dn_sqrt_r(" : "sqrtf(") + A(0) + ")";
  if (k == "Abs") return arg_range(0).first >= 0 ? A(0) : "fabsf(" + A(0) + ")";
  if (k == "Neg") return "-" + A(0);
  if (k == "Reciprocal") return "dn_div(1.0f, " + A(0) + ")";
  if (k == "Erf") {
    Range r = arg_range(0);
    return (r.first >= 0.1 ? "dn_erf_p(" : (r.second <= -0.1 || c.lowp) ? "dn_erf_r(" : "erff(") + A(0) + ")";
  }
  if (k == "Square") return A(0) + " * " + A(0);
  if (k == "Floor") return "floorf(" + A(0) + ")";
  if (k == "Round") return "rintf(" + A(0) + ")";          // halves to even, as the operator is defined
  if (k == "BitShift") return "((long long)" + A(0) + (op.i("direction_right", 0) ? " >> " : " << ") + "(long long)" + A(1) + ")";
  if (k == "Not") return "(" + A(0) + " != 0.0f ? 0.0f : 1.0f)";     // truth values travel as 0 / 1, like Greater's
  if (k == "Sin") return "sinf(" + A(0) + ")";
  if (k == "Cos") return "cosf(" + A(0) + ")";
  if (k == "Asin") return "asinf(" + A(0) + ")";
  if (k == "PRelu") return "(" + A(0) + " >= 0.0f ? " + A(0) + " : " + A(0) + " * " + A(1) + ")";
  if (k == "Ceil") return "ceilf(" + A(0) + ")";
  if (k == "Clip") {
    std::string e = A(0);
    if (op.has("min")) e = "fmaxf(" + e + ", " + flit(op.f("min", 0)) + ")";
    if (op.has("max")) e = "fminf(" + e + ", " + flit(op.f("max", 0)) + ")";
    return e;
  }
  if (k == "LeakyRelu") return "(" + A(0) + " >= 0.0f ? " + A(0) + " : " + A(0) + " * " + flit(op.f("alpha", 0.01)) + ")";
  if (k == "BatchNormalization")
    return "(" + A(0) + " - " + A(3) + ") * (" + A(1) + " * dn_div(1.0f, sqrtf(" + A(4) + " + " + flit(op.f("epsilon", 1e-5)) + "))) + " + A(2);
  throw Error(DNNF_UNSUPPORTED_OP, "no device expression for operator " + k);
}

void LowerCtx::emit_values(std::ostringstream& os, const std::vector<int>& roots, std::set<int>& done,
                           const std::map<int, int>& pslot, const std::string& ind,
                           const std::map<int, std::string>* load_override) const {
  // nodes are created children-first, so ascending id order is a valid schedule
  std::set<int> need;
  std::vector<int> stack(roots.begin(), roots.end());
  while (!stack.empty()) {
    int n = stack.back();
    stack.pop_back();
    if (need.count(n) || done.count(n)) continue;
    need.insert(n);
    for (int a : nodes[n].args) stack.push_back(a);
    if (nodes[n].kind == ENode::LOAD)
      for (auto& p : nodes[n].addr.indirect) stack.push_back(p.first);
  }
  for (int n : need) {
    const ENode& e = nodes[n];
    switch (e.kind) {
      case ENode::CONSTV:
        os << ind << "const float " << vname(n) << " = " << flit(e.cv) << ";\n";
        break;
      case ENode::ANCHOR:
        os << ind << (e.is_int ? "const long long " : "const float ") << vname(n) << " = anchor_v;\n";
        break;
      case ENode::LOAD: {
        if (load_override && load_override->count(n)) {
          os << ind << "const float " << vname(n) << " = " << load_override->at(n) << ";\n";
          break;
        }
        int slot = pslot.at(e.tensor);
        if (e.is_int)
          os << ind << "const long long " << vname(n) << " = (long long)p" << slot << "[" << addr_expr(e.addr) << "];\n";
        else
          os << ind << "const float " << vname(n) << " = cvt_in(p" << slot << "[" << addr_expr(e.addr) << "]);\n";
        break;
      }
      case ENode::OP:
        os << ind << (e.is_int ? "const long long " : "const float ") << vname(n) << " = " << op_expr(*this, e) << ";\n";
        break;
    }
    done.insert(n);
  }
}

std::string LowerCtx::store_stmt(const Store& s, const std::map<int, int>& pslot, const std::string& off) const {
  std::ostringstream o;
  int slot = pslot.at(s.tensor);
  o << "cvt_out(p" << slot << " + (" << off << "), " << vname(s.value) << ");";
  return o.str();
}

// ------------------------------------------------------------------ dispatcher
Lowered lower_block(const Graph& g, const Block& b, const LowerOpts& o) {
  DNNF_CHECK(!b.ops.empty(), DNNF_INVALID_ARG, "empty block");
  {
    std::vector<int> in0, out0, rem0;
    block_io(g, b, in0, out0, rem0);
    DNNF_CHECK(!out0.empty(), DNNF_INVALID_ARG, "block without outputs");     // every template stores at least one result
  }
  LowerCtx c(g, b, o);
  int anchors = 0, n_matmul = 0, n_softmax = 0, concat = -1;
  for (int oi : b.ops) {
    n_matmul += g.ops[oi].info->cls == OC_MATMUL;
    n_softmax += g.ops[oi].info->cls == OC_SOFTMAX;
  }
  const bool attention = n_matmul == 2 && n_softmax == 1;      // the one block shape with three anchors
  int n_norm = 0;
  for (int oi : b.ops) n_norm += g.ops[oi].info->cls == OC_NORMALIZE;
  const bool gemm_norm = n_matmul == 1 && n_norm == 1 && n_softmax == 0;   // and the one with a normalisation behind a MatMul
  int n_conv = 0, n_gap = 0;
  for (int oi : b.ops) { n_conv += g.ops[oi].info->cls == OC_CONV; n_gap += g.ops[oi].info->cls == OC_GAP; }
  const bool se_tail = n_conv == 2 && n_gap <= 1 && n_matmul == 0;          // and the squeeze-excite tail: [pool,] two 1x1 convolutions
  for (int oi : b.ops) {
    const Op& op = g.ops[oi];
    switch (op.info->cls) {
      case OC_CONV: case OC_CONVT: case OC_MATMUL: case OC_GEMM: case OC_REDUCE: case OC_SOFTMAX: case OC_NORMALIZE: case OC_GAP: case OC_POOL: case OC_SCAN:
        anchors++;
        c.anchor_op = oi;
        c.anchor_out = op.out[0];
        break;
      case OC_OTHER:
        throw Error(DNNF_UNSUPPORTED_OP, "operator " + op.kind + " has no kernel template");
      case OC_EINSUM:
        throw Error(DNNF_UNSUPPORTED_OP, "Einsum runs as the MatMul the rewriting pass expands it into: rewrite the graph first");
      case OC_CONCAT:
        DNNF_CHECK(concat < 0, DNNF_UNSUPPORTED_OP, "two Concat operators in one block");
        concat = oi;
        break;
      default:
        break;
    }
  }
  // and a depthwise convolution with the global average pool over its (activated) result: the pool is taken in the
  // convolution's kernel, which is lowered from the block without the pool operator
  if (n_conv == 1 && n_gap == 1 && anchors == 2 && n_matmul == 0 && o.pool_op < 0) {
    Block b2 = b;
    int gap = -1;
    for (int oi : b.ops) if (g.ops[oi].info->cls == OC_GAP) gap = oi;
    b2.ops.erase(std::remove(b2.ops.begin(), b2.ops.end(), gap), b2.ops.end());
    for (int oi : b2.ops)
      for (int t : g.ops[oi].in) DNNF_CHECK(t != g.ops[gap].out[0], DNNF_UNSUPPORTED_OP, "the pooled vector is read inside its own block");
    LowerOpts o2 = o;
    o2.pool_op = gap;
    Lowered Lp = lower_block(g, b2, o2);
    DNNF_CHECK(Lp.family == FAM_DWCONV && Lp.launches.size() == 1 && Lp.variant.find("_pool") != std::string::npos, DNNF_UNSUPPORTED_OP,
               "no kernel takes this pool inside the convolution in front of it");
    return Lp;
  }
  DNNF_CHECK(anchors <= 1 || (attention && anchors == 3) || (gemm_norm && anchors == 2) || (se_tail && anchors == n_conv + n_gap), DNNF_UNSUPPORTED_OP,
             "a block may hold one Many-to-Many operator");
  Lowered L;
  // a lone contiguous Reorganize operator moves nothing: its output shares the input's storage
  if (b.ops.size() == 1 && g.ops[b.ops[0]].info->cls == OC_RESHAPE &&
      g.tensors[g.ops[b.ops[0]].out[0]].kind == DNNF_INTERMEDIATE && g.tensors[g.ops[b.ops[0]].in[0]].perm.empty() &&
      g.tensors[g.ops[b.ops[0]].out[0]].perm.empty()) {
    L.family = FAM_ALIAS;
    L.alias_src = g.ops[b.ops[0]].in[0];
    L.alias_dst = g.ops[b.ops[0]].out[0];
    L.ext_in = {L.alias_src};
    L.ext_out = {L.alias_dst};
    L.variant = "alias";
    return L;
  }
  if (attention && anchors == 3) L = lower_attention(g, b, o);
  else if (se_tail && anchors == n_conv + n_gap) {
    DNNF_CHECK(concat < 0, DNNF_UNSUPPORTED_OP, "Concat in a squeeze-excite block");
    L = lower_squeeze_excite(g, b, o);
  } else if (gemm_norm && anchors == 2) {
    DNNF_CHECK(concat < 0, DNNF_UNSUPPORTED_OP, "Concat in a MatMul - normalisation block");
    L = lower_gemm_norm(g, b, o);
  } else if (concat >= 0) {
    // Concat closes its block: one kernel per operand computes that operand's chain over the operand's
    // own index range and writes it at its offset of the result (no copy of the finished operands).  The chain of
    // one operand may hold the block's Many-to-Many anchor: that operand is then written by the anchor's own kernel,
    // whose epilogue stores into the operand's range of the result.
    std::vector<int> ein0, eout0, rem0;
    block_io(g, b, ein0, eout0, rem0);
    DNNF_CHECK(anchors <= 1 && eout0.size() == 1 && eout0[0] == g.ops[concat].out[0], DNNF_UNSUPPORTED_OP,
               "Concat must be the last operator of its block");
    std::set<int> inb(b.ops.begin(), b.ops.end());
    auto chain_has_anchor = [&](int t) {
      if (anchors == 0) return false;
      std::set<int> seen;
      std::vector<int> stack = {t};
      while (!stack.empty()) {
        int x = stack.back();
        stack.pop_back();
        int p = g.tensors[x].producer;
        if (p < 0 || !inb.count(p) || seen.count(p)) continue;
        if (p == c.anchor_op) return true;
        seen.insert(p);
        for (int i : g.ops[p].in) stack.push_back(i);
      }
      return false;
    };
    // A Concat that stacks whole stored tensors along the outermost axis (with nothing but Reshape-class operators
    // in between: the Unsqueeze pair of a returned key / value stack) moves no data if its operands are simply kept
    // inside the result: the producers write there, the other readers read from there.
    if (anchors == 0 && o.alias_concat) {
      const Op& cc = g.ops[concat];
      const Tensor& R = g.tensors[cc.out[0]];
      int a = (int)cc.i("axis", 0);
      if (a < 0) a += (int)R.dims.size();
      bool ok = R.perm.empty();
      for (int d = 0; d < a; d++) ok = ok && R.dims[d] == 1;
      for (int oi : b.ops) ok = ok && (oi == concat || g.ops[oi].info->cls == OC_RESHAPE);
      std::vector<std::pair<int, int64_t>> parts;
      int64_t start = 0;
      for (size_t k = 0; k < cc.in.size() && ok; k++) {
        int t = cc.in[k];
        const int64_t part_bytes = g.tensors[t].bytes();
        while (g.tensors[t].producer >= 0 && inb.count(g.tensors[t].producer)) t = g.ops[g.tensors[t].producer].in[0];
        const Tensor& X = g.tensors[t];
        ok = ok && X.kind == DNNF_INTERMEDIATE && X.producer >= 0 && !X.weight_only && X.perm.empty() && X.dtype == R.dtype && X.bytes() == part_bytes &&
             g.ops[X.producer].info->cls != OC_RESHAPE && g.ops[X.producer].info->cls != OC_CONCAT;
        for (auto& pr : parts) ok = ok && pr.first != t;
        parts.push_back({t, start});
        start += part_bytes;
      }
      if (ok) {
        L.family = FAM_ALIAS;
        L.variant = "alias_concat";
        L.alias_dst = cc.out[0];
        L.alias_parts = parts;
        for (auto& pr : parts) L.ext_in.push_back(pr.first);
        L.ext_out = eout0;
        L.bytes = L.flops = 0;
        L.irs_removed = 0;
        return L;
      }
    }
    L.family = FAM_EW;
    L.variant = "concat_parts";
    L.ext_out = eout0;
    int anchored = 0;
    for (size_t k = 0; k < g.ops[concat].in.size(); k++) {
      LowerCtx ck(g, b, o);
      ck.concat_op = concat;
      ck.concat_part = (int)k;
      Lowered Lk;
      if (chain_has_anchor(g.ops[concat].in[k])) {
        anchored++;
        ck.anchor_op = c.anchor_op;
        ck.anchor_out = c.anchor_out;
        switch (g.ops[c.anchor_op].info->cls) {
          case OC_CONV:
            DNNF_CHECK(g.tensors[g.ops[c.anchor_op].in[0]].dims.size() == 4, DNNF_UNSUPPORTED_OP, "only 2-d convolutions write into a Concat");
            Lk = lower_conv(ck);
            break;
          case OC_MATMUL: case OC_GEMM: Lk = lower_gemm(ck); break;
          default: throw Error(DNNF_UNSUPPORTED_OP, "this Many-to-Many operator cannot write into a Concat");
        }
        L.family = Lk.family;
        L.variant = "concat_parts+" + Lk.variant;
        L.scratch_bytes = std::max(L.scratch_bytes, Lk.scratch_bytes);
      } else Lk = lower_elementwise(ck);
      for (int x : Lk.ext_in) if (std::find(L.ext_in.begin(), L.ext_in.end(), x) == L.ext_in.end()) L.ext_in.push_back(x);
      L.launches.insert(L.launches.end(), Lk.launches.begin(), Lk.launches.end());
    }
    DNNF_CHECK(anchored == anchors, DNNF_UNSUPPORTED_OP, "the block's Many-to-Many operator does not feed its Concat");
  }
  else if (anchors == 0) {
    try {
      L = lower_elementwise(c);
    } catch (const Error& e) {
      // outputs that share no index space (e.g. the parts of a lone Split): one kernel per output
      std::vector<int> ein0, eout0, rem0;
      block_io(g, b, ein0, eout0, rem0);
      if (e.code != DNNF_UNSUPPORTED_OP || eout0.size() < 2) throw;
      // another output may span an index space that reaches all of them (the last one may be a Slice of it)
      bool done = false;
      for (int k = (int)eout0.size() - 2; k >= 0 && !done; k--) {
        LowerCtx ck(g, b, o);
        ck.pivot_out = eout0[k];
        try {
          L = lower_elementwise(ck);
          done = true;
        } catch (const Error& e2) {
          if (e2.code != DNNF_UNSUPPORTED_OP) throw;
        }
      }
      if (!done) {
      L = Lowered();
      L.family = FAM_EW;
      L.variant = "per_output";
      for (int t : eout0) {
        LowerCtx c1(g, b, o);
        c1.only_outputs = {t};
        Lowered Li = lower_elementwise(c1);
        for (int x : Li.ext_in) if (std::find(L.ext_in.begin(), L.ext_in.end(), x) == L.ext_in.end()) L.ext_in.push_back(x);
        L.ext_out.push_back(t);
        L.launches.insert(L.launches.end(), Li.launches.begin(), Li.launches.end());
      }
      }
    }
  }
  else {
    switch (g.ops[c.anchor_op].info->cls) {
      case OC_CONV: L = g.tensors[g.ops[c.anchor_op].in[0]].dims.size() == 5 ? lower_conv3d(c) : lower_conv(c); break;
      case OC_POOL: L = lower_pool(c); break;
      case OC_SCAN: L = lower_scan(c); break;
      case OC_CONVT: L = lower_conv_transpose(c); break;
      case OC_MATMUL: case OC_GEMM: L = lower_gemm(c); break;
      default: L = lower_reduce(c); break;
    }
  }
  std::vector<int> ein, eout, removed;
  block_io(g, b, ein, eout, removed);
  L.bytes = 0;
  for (int t : ein) L.bytes += (double)g.tensors[t].bytes();
  for (int t : eout) L.bytes += (double)g.tensors[t].bytes();
  L.flops = 0;
  for (int oi : b.ops) L.flops += g.ops[oi].flops;
  L.irs_removed = 0;
  for (int t : removed) L.irs_removed += (double)g.tensors[t].bytes();
  return L;
}

}  // namespace dnnf
