// Graph construction, shape inference, mapping-type classification (paper Sec. 3.1, Table 2),
// the mapping-type analysis table (Sec. 3.2) and the #FLOPS cost model of Sec. 4.2.
#include <cctype>
#include <algorithm>
#include <functional>
#include <sstream>

#include "ir.hpp"

namespace dnnf {

// name, class, Table-2 mapping type, printed in Table 2?, associative, commutative, distributive, flops/output
static const std::vector<OpKindInfo> kOpKinds = {
    // ---- One-to-One row of Table 2
    {"Add", OC_BINARY, DNNF_ONE_TO_ONE, true, true, true, true, 1},
    {"Asin", OC_UNARY, DNNF_ONE_TO_ONE, true, false, false, false, 1},
    {"BatchNormalization", OC_BATCHNORM, DNNF_ONE_TO_ONE, true, false, false, false, 4},
    {"Cast", OC_UNARY, DNNF_ONE_TO_ONE, true, false, false, false, 0},
    {"Ceil", OC_UNARY, DNNF_ONE_TO_ONE, true, false, false, false, 1},
    {"Clip", OC_UNARY, DNNF_ONE_TO_ONE, true, false, false, false, 2},
    {"Concat", OC_CONCAT, DNNF_ONE_TO_ONE, true, false, false, false, 0},
    {"Cos", OC_UNARY, DNNF_ONE_TO_ONE, true, false, false, false, 1},
    {"Erf", OC_UNARY, DNNF_ONE_TO_ONE, true, false, false, false, 1},
    {"Exp", OC_UNARY, DNNF_ONE_TO_ONE, true, false, true, false, 1},
    {"Greater", OC_BINARY, DNNF_ONE_TO_ONE, true, false, false, false, 1},
    {"LeakyRelu", OC_UNARY, DNNF_ONE_TO_ONE, true, false, false, false, 1},
    {"Log", OC_UNARY, DNNF_ONE_TO_ONE, true, false, false, false, 1},
    {"Not", OC_UNARY, DNNF_ONE_TO_ONE, true, false, false, false, 1},
    {"PRelu", OC_BINARY, DNNF_ONE_TO_ONE, true, false, false, false, 1},
    {"Reciprocal", OC_UNARY, DNNF_ONE_TO_ONE, true, true, false, false, 1},
    {"Relu", OC_UNARY, DNNF_ONE_TO_ONE, true, false, false, false, 1},
    {"Round", OC_UNARY, DNNF_ONE_TO_ONE, true, false, false, false, 1},
    {"Sigmoid", OC_UNARY, DNNF_ONE_TO_ONE, true, false, false, false, 1},
    {"Sin", OC_UNARY, DNNF_ONE_TO_ONE, true, false, false, false, 1},
    {"Slice", OC_SLICE, DNNF_ONE_TO_ONE, true, false, false, false, 0},
    {"Split", OC_SPLIT, DNNF_ONE_TO_ONE, true, false, false, false, 0},
    {"Sqrt", OC_UNARY, DNNF_ONE_TO_ONE, true, true, false, false, 1},
    {"Tanh", OC_UNARY, DNNF_ONE_TO_ONE, true, false, false, false, 1},
    {"Where", OC_WHERE, DNNF_ONE_TO_ONE, true, false, false, false, 1},
    // ---- One-to-Many row ("Elementwise w/ broadcast" is a condition, handled in classify_op)
    {"Expand", OC_EXPAND, DNNF_ONE_TO_MANY, true, false, false, false, 0},
    {"Gather", OC_GATHER, DNNF_ONE_TO_MANY, true, false, false, false, 0},
    {"Resize", OC_RESIZE, DNNF_ONE_TO_MANY, true, false, false, false, 0},
    {"Upsample", OC_RESIZE, DNNF_ONE_TO_MANY, true, false, false, false, 0},
    // ---- Many-to-Many row
    {"AveragePool", OC_POOL, DNNF_MANY_TO_MANY, true, false, false, false, 1},
    {"Conv", OC_CONV, DNNF_MANY_TO_MANY, true, false, false, false, 0},
    {"ConvTranspose", OC_CONVT, DNNF_MANY_TO_MANY, true, false, false, false, 0},
    {"CumSum", OC_SCAN, DNNF_MANY_TO_MANY, true, false, false, false, 1},
    {"Einsum", OC_EINSUM, DNNF_MANY_TO_MANY, true, false, false, false, 0},
    {"Gemm", OC_GEMM, DNNF_MANY_TO_MANY, true, false, false, false, 0},
    {"InstanceNormalization", OC_NORMALIZE, DNNF_MANY_TO_MANY, true, false, false, false, 0},
    {"MaxPool", OC_POOL, DNNF_MANY_TO_MANY, true, false, false, false, 1},
    {"ReduceProd", OC_REDUCE, DNNF_MANY_TO_MANY, true, false, true, false, 0},
    {"ReduceMean", OC_REDUCE, DNNF_MANY_TO_MANY, true, false, false, false, 0},
    {"ReduceSum", OC_REDUCE, DNNF_MANY_TO_MANY, true, false, true, false, 0},
    {"ReduceMax", OC_REDUCE, DNNF_MANY_TO_MANY, true, false, false, false, 0},
    {"Softmax", OC_SOFTMAX, DNNF_MANY_TO_MANY, true, false, false, false, 0},
    // ---- Reorganize row
    {"Flatten", OC_RESHAPE, DNNF_REORGANIZE, true, false, false, false, 0},
    {"Reshape", OC_RESHAPE, DNNF_REORGANIZE, true, false, false, false, 0},
    {"Squeeze", OC_RESHAPE, DNNF_REORGANIZE, true, false, false, false, 0},
    {"Unsqueeze", OC_RESHAPE, DNNF_REORGANIZE, true, false, false, false, 0},
    // ---- Shuffle row
    {"DepthToSpace", OC_D2S, DNNF_SHUFFLE, true, false, false, false, 0},
    {"SpaceToDepth", OC_D2S, DNNF_SHUFFLE, true, false, false, false, 0},
    {"Transpose", OC_TRANSPOSE, DNNF_SHUFFLE, true, false, false, false, 0},
    // ---- not printed in Table 2; typed from the index-function definitions of Sec. 3.1.
    //      Elementwise operators of Table 4 (Mul, Sub, Abs, Square, ...) are One-to-One.
    {"Sub", OC_BINARY, DNNF_ONE_TO_ONE, false, false, false, true, 1},
    {"Mul", OC_BINARY, DNNF_ONE_TO_ONE, false, true, true, true, 1},
    {"Div", OC_BINARY, DNNF_ONE_TO_ONE, false, false, false, true, 1},
    {"Pow", OC_BINARY, DNNF_ONE_TO_ONE, false, false, false, false, 1},
    {"Max", OC_BINARY, DNNF_ONE_TO_ONE, false, true, true, false, 1},
    {"Min", OC_BINARY, DNNF_ONE_TO_ONE, false, true, true, false, 1},
    {"BitShift", OC_BINARY, DNNF_ONE_TO_ONE, false, false, true, false, 1},
    {"Neg", OC_UNARY, DNNF_ONE_TO_ONE, false, false, false, false, 1},
    {"Abs", OC_UNARY, DNNF_ONE_TO_ONE, false, true, false, false, 1},
    {"Square", OC_UNARY, DNNF_ONE_TO_ONE, false, true, false, true, 1},
    {"Floor", OC_UNARY, DNNF_ONE_TO_ONE, false, false, false, false, 1},
    {"Identity", OC_UNARY, DNNF_ONE_TO_ONE, false, false, false, false, 0},
    {"MatMul", OC_MATMUL, DNNF_MANY_TO_MANY, false, false, false, false, 0},
    {"GlobalAveragePool", OC_GAP, DNNF_MANY_TO_MANY, false, false, false, false, 0},
    {"Normalize", OC_NORMALIZE, DNNF_MANY_TO_MANY, false, false, false, false, 0},
};

const std::vector<OpKindInfo>& all_op_kinds() { return kOpKinds; }
const OpKindInfo* find_op_kind(const std::string& name) {
  for (auto& k : kOpKinds)
    if (name == k.name) return &k;
  return nullptr;
}

// ------------------------------------------------------------------ mapping-type analysis table
// The table itself is a figure in the paper; it is rebuilt from the section's prose:
//  - fused type: the operand with the higher transformation impedance decides, i.e. the more
//    complex of the two types in the order of the Sec. 3.1 footnote;
//  - red: second is Many-to-Many and first is One-to-Many or Many-to-Many;
//  - green: either operand is One-to-One, or both are Reorganize/Shuffle;
//  - yellow: the rest.  13 green + 10 yellow = the 23 code-generation rules of Sec. 4.4.1.
void fuse_relation(int first, int second, int* fused, int* colour) {
  *fused = std::max(first, second);
  bool heavy1 = first == DNNF_ONE_TO_MANY || first == DNNF_MANY_TO_MANY;
  bool mid1 = first == DNNF_REORGANIZE || first == DNNF_SHUFFLE;
  bool mid2 = second == DNNF_REORGANIZE || second == DNNF_SHUFFLE;
  if (second == DNNF_MANY_TO_MANY && heavy1) *colour = DNNF_RED;
  else if (first == DNNF_ONE_TO_ONE || second == DNNF_ONE_TO_ONE || (mid1 && mid2)) *colour = DNNF_GREEN;
  else *colour = DNNF_YELLOW;
}

// ------------------------------------------------------------------ construction
int Graph::add_tensor(const std::string& name, int dtype, const Dims& dims, int kind) {
  for (auto d : dims) DNNF_CHECK(d >= 0, DNNF_INVALID_ARG, "negative extent in tensor " + name);
  Tensor t;
  t.name = name;
  t.dtype = dtype;
  t.dims = dims;
  t.kind = kind;
  tensors.push_back(t);
  int id = (int)tensors.size() - 1;
  if (kind == DNNF_INPUT) { tensors[id].ext_index = (int)inputs.size(); inputs.push_back(id); }
  if (kind == DNNF_WEIGHT) { tensors[id].ext_index = (int)weights.size(); weights.push_back(id); }
  if (kind == DNNF_OUTPUT) { tensors[id].ext_index = (int)outputs.size(); outputs.push_back(id); }
  finalized = false;
  return id;
}

int Graph::add_op(const std::string& kind, const std::vector<int>& in, const std::vector<int>& out, const Attrs& a) {
  const OpKindInfo* info = find_op_kind(kind);
  DNNF_CHECK(info != nullptr, DNNF_UNSUPPORTED_OP, "unknown operator kind " + kind);
  for (int t : in) DNNF_CHECK(t >= 0 && t < (int)tensors.size(), DNNF_INVALID_ARG, kind + ": bad input tensor id");
  for (int t : out) DNNF_CHECK(t >= 0 && t < (int)tensors.size(), DNNF_INVALID_ARG, kind + ": bad output tensor id");
  Op op;
  op.kind = kind;
  op.info = info;
  op.in = in;
  op.out = out;
  op.attrs = a;
  ops.push_back(op);
  finalized = false;
  return (int)ops.size() - 1;
}

int Graph::new_tensor_like(const std::string& stem, int dtype, const Dims& dims) {
  Tensor t;
  t.name = stem + "#" + std::to_string(tensors.size());
  t.dtype = dtype;
  t.dims = dims;
  t.kind = DNNF_INTERMEDIATE;
  tensors.push_back(t);
  return (int)tensors.size() - 1;
}

// A compiler-made constant: a weight with host values and no device buffer of the caller's.
int Graph::new_const(const std::string& stem, int dtype, const Dims& dims, const std::vector<double>& v) {
  int id = new_tensor_like(stem, dtype, dims);
  tensors[id].kind = DNNF_WEIGHT;
  tensors[id].has_cval = true;
  tensors[id].cval = v;
  tensors[id].ext_index = -1;
  return id;
}

Dims broadcast_dims(const Dims& a, const Dims& b) {
  size_t r = std::max(a.size(), b.size());
  Dims out(r);
  for (size_t i = 0; i < r; i++) {
    int64_t x = i + a.size() >= r ? a[i + a.size() - r] : 1;
    int64_t y = i + b.size() >= r ? b[i + b.size() - r] : 1;
    DNNF_CHECK(x == y || x == 1 || y == 1, DNNF_SHAPE_MISMATCH, "operands do not broadcast");
    out[i] = std::max(x, y);
  }
  return out;
}

static int norm_axis(int64_t a, size_t rank) { return (int)(a < 0 ? a + (int64_t)rank : a); }

EinsumSpec parse_einsum(const Op& op) {
  std::string eq;
  auto it = op.attrs.find("equation");
  DNNF_CHECK(it != op.attrs.end(), DNNF_INVALID_ARG, "Einsum without an equation");
  for (double v : it->second) if ((char)v != ' ') eq.push_back((char)v);
  const size_t arrow = eq.find("->"), comma = eq.find(',');
  DNNF_CHECK(arrow != std::string::npos, DNNF_UNSUPPORTED_OP, "Einsum: the result term must be written out");
  DNNF_CHECK(comma != std::string::npos && comma < arrow && eq.find(',', comma + 1) == std::string::npos, DNNF_UNSUPPORTED_OP,
             "Einsum: exactly two operands are supported");
  EinsumSpec e{eq.substr(0, comma), eq.substr(comma + 1, arrow - comma - 1), eq.substr(arrow + 2)};
  for (const std::string* t : {&e.a, &e.b, &e.out})
    for (size_t i = 0; i < t->size(); i++) {
      DNNF_CHECK(std::isalpha((unsigned char)(*t)[i]), DNNF_UNSUPPORTED_OP, "Einsum: only letter labels are supported (no ellipsis)");
      DNNF_CHECK(t->find((*t)[i], i + 1) == std::string::npos, DNNF_UNSUPPORTED_OP, "Einsum: a label repeated inside one term");
    }
  return e;
}

Dims infer_shape(const Graph& g, const Op& op, int oi) {
  auto in = [&](int k) -> const Dims& { return g.tensors[op.in[k]].dims; };
  auto need = [&](size_t n) { DNNF_CHECK(op.in.size() >= n, DNNF_INVALID_ARG, op.kind + ": too few inputs"); };
  switch (op.info->cls) {
    case OC_UNARY: case OC_BATCHNORM: case OC_SOFTMAX: case OC_NORMALIZE:
      need(1);
      if (op.kind == "InstanceNormalization") {
        need(3);
        DNNF_CHECK(in(0).size() >= 3 && numel(in(1)) == in(0)[1] && numel(in(2)) == in(0)[1], DNNF_SHAPE_MISMATCH,
                   "InstanceNormalization: scale / bias need one value per channel");
      }
      return in(0);
    case OC_BINARY:
      need(2);
      return broadcast_dims(in(0), in(1));
    case OC_WHERE:
      need(3);
      return broadcast_dims(broadcast_dims(in(0), in(1)), in(2));
    case OC_CONV: {
      need(2);
      const Dims &x = in(0), &w = in(1);
      if (x.size() == 5 && w.size() == 5) {      // 3-d convolution, NCDHW / OIDHW
        DNNF_CHECK(op.i("group", 1) == 1 && w[1] == x[1], DNNF_SHAPE_MISMATCH, "3-d Conv: channel mismatch (group must be 1)");
        auto st = op.ints("strides"); if (st.empty()) st = {1, 1, 1};
        auto pd = op.ints("pads"); if (pd.empty()) pd = {0, 0, 0, 0, 0, 0};
        DNNF_CHECK(st.size() == 3 && pd.size() == 6 && st[0] >= 1 && st[1] >= 1 && st[2] >= 1, DNNF_INVALID_ARG, "3-d Conv strides/pads");
        if (op.in.size() > 2) DNNF_CHECK(numel(in(2)) == w[0], DNNF_SHAPE_MISMATCH, "Conv bias size");
        Dims out = {x[0], w[0]};
        for (int d = 0; d < 3; d++) {
          int64_t o = (x[2 + d] + pd[d] + pd[3 + d] - w[2 + d]) / st[d] + 1;
          DNNF_CHECK(o >= 1, DNNF_SHAPE_MISMATCH, "Conv output is empty");
          out.push_back(o);
        }
        return out;
      }
      DNNF_CHECK(x.size() == 4 && w.size() == 4, DNNF_SHAPE_MISMATCH, "Conv expects NCHW input and OIHW weight (or NCDHW / OIDHW)");
      int64_t grp = op.i("group", 1);
      DNNF_CHECK(grp >= 1 && w[1] * grp == x[1] && w[0] % grp == 0, DNNF_SHAPE_MISMATCH, "Conv channel/group mismatch");
      auto st = op.ints("strides"); if (st.empty()) st = {1, 1};
      auto pd = op.ints("pads"); if (pd.empty()) pd = {0, 0, 0, 0};
      DNNF_CHECK(st.size() == 2 && pd.size() == 4 && st[0] >= 1 && st[1] >= 1, DNNF_INVALID_ARG, "Conv strides/pads");
      if (op.in.size() > 2) DNNF_CHECK(numel(in(2)) == w[0], DNNF_SHAPE_MISMATCH, "Conv bias size");
      int64_t ho = (x[2] + pd[0] + pd[2] - w[2]) / st[0] + 1, wo = (x[3] + pd[1] + pd[3] - w[3]) / st[1] + 1;
      DNNF_CHECK(ho >= 1 && wo >= 1, DNNF_SHAPE_MISMATCH, "Conv output is empty");
      return {x[0], w[0], ho, wo};
    }
    case OC_CONVT: {
      need(2);
      const Dims &x = in(0), &w = in(1);
      DNNF_CHECK(x.size() == 4 && w.size() == 4 && op.i("group", 1) == 1 && w[0] == x[1], DNNF_SHAPE_MISMATCH,
                 "ConvTranspose expects NCHW input and a [C, CO, KH, KW] filter (group 1)");
      auto st = op.ints("strides"); if (st.empty()) st = {1, 1};
      auto pd = op.ints("pads"); if (pd.empty()) pd = {0, 0, 0, 0};
      auto op_ = op.ints("output_padding"); if (op_.empty()) op_ = {0, 0};
      DNNF_CHECK(st.size() == 2 && pd.size() == 4 && op_.size() == 2 && st[0] >= 1 && st[1] >= 1, DNNF_INVALID_ARG, "ConvTranspose strides/pads");
      if (op.in.size() > 2) DNNF_CHECK(numel(in(2)) == w[1], DNNF_SHAPE_MISMATCH, "ConvTranspose bias size");
      int64_t ho = (x[2] - 1) * st[0] - pd[0] - pd[2] + w[2] + op_[0], wo = (x[3] - 1) * st[1] - pd[1] - pd[3] + w[3] + op_[1];
      DNNF_CHECK(ho >= 1 && wo >= 1, DNNF_SHAPE_MISMATCH, "ConvTranspose output is empty");
      return {x[0], w[1], ho, wo};
    }
    case OC_MATMUL: {
      need(2);
      const Dims &a = in(0), &b = in(1);
      DNNF_CHECK(a.size() >= 2 && b.size() >= 2, DNNF_SHAPE_MISMATCH, "MatMul operands need rank >= 2");
      DNNF_CHECK(a[a.size() - 1] == b[b.size() - 2], DNNF_SHAPE_MISMATCH, "MatMul inner dimensions differ");
      Dims ba(a.begin(), a.end() - 2), bb(b.begin(), b.end() - 2);
      Dims out = broadcast_dims(ba, bb);
      out.push_back(a[a.size() - 2]);
      out.push_back(b[b.size() - 1]);
      return out;
    }
    case OC_GEMM: {
      need(2);
      const Dims &a = in(0), &b = in(1);
      DNNF_CHECK(a.size() == 2 && b.size() == 2, DNNF_SHAPE_MISMATCH, "Gemm operands need rank 2");
      bool ta = op.i("transA", 0), tb = op.i("transB", 0);
      int64_t m = ta ? a[1] : a[0], k = ta ? a[0] : a[1], k2 = tb ? b[1] : b[0], n = tb ? b[0] : b[1];
      DNNF_CHECK(k == k2, DNNF_SHAPE_MISMATCH, "Gemm inner dimensions differ");
      return {m, n};
    }
    case OC_REDUCE: {
      need(1);
      const Dims& x = in(0);
      auto axes = op.ints("axes");
      std::set<int> ax;
      for (auto a : axes) ax.insert(norm_axis(a, x.size()));
      if (ax.empty()) for (size_t i = 0; i < x.size(); i++) ax.insert((int)i);
      bool keep = op.i("keepdims", 1);
      Dims out;
      for (size_t i = 0; i < x.size(); i++) {
        if (ax.count((int)i)) { if (keep) out.push_back(1); }
        else out.push_back(x[i]);
      }
      return out;
    }
    case OC_GAP: {
      need(1);
      Dims out = in(0);
      DNNF_CHECK(out.size() >= 3, DNNF_SHAPE_MISMATCH, "GlobalAveragePool needs rank >= 3");
      for (size_t i = 2; i < out.size(); i++) out[i] = 1;
      return out;
    }
    case OC_EINSUM: {
      need(2);
      const EinsumSpec e = parse_einsum(op);
      DNNF_CHECK(e.a.size() == in(0).size() && e.b.size() == in(1).size(), DNNF_SHAPE_MISMATCH, "Einsum: a term's length differs from its operand's rank");
      std::map<char, int64_t> ext;
      for (size_t i = 0; i < e.a.size(); i++) ext[e.a[i]] = in(0)[i];
      for (size_t i = 0; i < e.b.size(); i++) {
        auto it = ext.find(e.b[i]);
        DNNF_CHECK(it == ext.end() || it->second == in(1)[i], DNNF_SHAPE_MISMATCH, std::string("Einsum: label ") + e.b[i] + " has two extents");
        ext[e.b[i]] = in(1)[i];
      }
      Dims out;
      for (char l : e.out) {
        DNNF_CHECK(ext.count(l), DNNF_INVALID_ARG, std::string("Einsum: result label ") + l + " is in no operand");
        out.push_back(ext[l]);
      }
      return out;
    }
    case OC_SCAN: {
      need(1);
      const Dims& x = in(0);
      const int64_t ax = op.i("axis", 0);
      DNNF_CHECK(ax >= -(int64_t)x.size() && ax < (int64_t)x.size(), DNNF_INVALID_ARG, op.kind + ": axis out of range");
      return x;
    }
    case OC_POOL: {
      need(1);
      const Dims& x = in(0);
      DNNF_CHECK(x.size() == 4, DNNF_SHAPE_MISMATCH, op.kind + " needs a rank-4 (NCHW) operand");
      auto ks = op.ints("kernel_shape");
      auto st = op.ints("strides"); if (st.empty()) st = {1, 1};
      auto pd = op.ints("pads"); if (pd.empty()) pd = {0, 0, 0, 0};
      DNNF_CHECK(ks.size() == 2 && st.size() == 2 && pd.size() == 4 && ks[0] >= 1 && ks[1] >= 1 && st[0] >= 1 && st[1] >= 1,
                 DNNF_INVALID_ARG, op.kind + " kernel_shape/strides/pads");
      DNNF_CHECK(pd[0] < ks[0] && pd[2] < ks[0] && pd[1] < ks[1] && pd[3] < ks[1], DNNF_INVALID_ARG, op.kind + ": padding as large as the window");
      DNNF_CHECK(op.i("ceil_mode", 0) == 0, DNNF_UNSUPPORTED_OP, op.kind + " with ceil_mode");
      int64_t ho = (x[2] + pd[0] + pd[2] - ks[0]) / st[0] + 1, wo = (x[3] + pd[1] + pd[3] - ks[1]) / st[1] + 1;
      DNNF_CHECK(ho >= 1 && wo >= 1, DNNF_SHAPE_MISMATCH, op.kind + " output is empty");
      return {x[0], x[1], ho, wo};
    }
    case OC_GATHER: {
      need(2);
      const Dims &d = in(0), &idx = in(1);
      int ax = norm_axis(op.i("axis", 0), d.size());
      Dims out(d.begin(), d.begin() + ax);
      out.insert(out.end(), idx.begin(), idx.end());
      out.insert(out.end(), d.begin() + ax + 1, d.end());
      return out;
    }
    case OC_RESHAPE: {
      need(1);
      const Dims& x = in(0);
      Dims out;
      if (op.kind == "Reshape") {
        out = op.ints("shape");
        int64_t known = 1; int neg = -1;
        for (size_t i = 0; i < out.size(); i++) {
          if (out[i] == 0 && i < x.size()) out[i] = x[i];
          if (out[i] == -1) neg = (int)i; else known *= out[i];
        }
        if (neg >= 0) { DNNF_CHECK(known > 0, DNNF_SHAPE_MISMATCH, "Reshape -1 with zero extent"); out[neg] = numel(x) / known; }
      } else if (op.kind == "Flatten") {
        int ax = norm_axis(op.i("axis", 1), x.size() + 1);
        int64_t a = 1, b = 1;
        for (int i = 0; i < (int)x.size(); i++) (i < ax ? a : b) *= x[i];
        out = {a, b};
      } else if (op.kind == "Squeeze") {
        auto axes = op.ints("axes");
        std::set<int> ax;
        for (auto a : axes) ax.insert(norm_axis(a, x.size()));
        for (size_t i = 0; i < x.size(); i++) {
          bool drop = axes.empty() ? x[i] == 1 : ax.count((int)i) != 0;
          if (drop) DNNF_CHECK(x[i] == 1, DNNF_SHAPE_MISMATCH, "Squeeze of an axis with extent != 1");
          else out.push_back(x[i]);
        }
      } else {  // Unsqueeze
        auto axes = op.ints("axes");
        size_t r = x.size() + axes.size();
        std::set<int> ax;
        for (auto a : axes) ax.insert(norm_axis(a, r));
        size_t k = 0;
        for (size_t i = 0; i < r; i++) out.push_back(ax.count((int)i) ? 1 : x[k++]);
      }
      DNNF_CHECK(numel(out) == numel(x), DNNF_SHAPE_MISMATCH, op.kind + " changes the element count");
      return out;
    }
    case OC_D2S: {
      need(1);
      const Dims& x = in(0);
      const int64_t b = op.i("blocksize", 0);
      DNNF_CHECK(x.size() == 4 && b >= 1, DNNF_INVALID_ARG, op.kind + " needs a rank-4 operand and a blocksize");
      if (op.kind == "DepthToSpace") {
        DNNF_CHECK(x[1] % (b * b) == 0, DNNF_SHAPE_MISMATCH, "DepthToSpace: channels not divisible by blocksize^2");
        return {x[0], x[1] / (b * b), x[2] * b, x[3] * b};
      }
      DNNF_CHECK(x[2] % b == 0 && x[3] % b == 0, DNNF_SHAPE_MISMATCH, "SpaceToDepth: map not divisible by blocksize");
      return {x[0], x[1] * b * b, x[2] / b, x[3] / b};
    }
    case OC_TRANSPOSE: {
      need(1);
      const Dims& x = in(0);
      auto perm = op.ints("perm");
      if (perm.empty()) for (int i = (int)x.size() - 1; i >= 0; i--) perm.push_back(i);
      DNNF_CHECK(perm.size() == x.size(), DNNF_SHAPE_MISMATCH, "Transpose perm rank");
      std::vector<int> seen(x.size(), 0);
      Dims out;
      for (auto p : perm) {
        DNNF_CHECK(p >= 0 && p < (int64_t)x.size() && !seen[p], DNNF_INVALID_ARG, "Transpose perm is not a permutation");
        seen[p] = 1;
        out.push_back(x[p]);
      }
      return out;
    }
    case OC_SLICE: {
      need(1);
      Dims out = in(0);
      auto st = op.ints("starts"), en = op.ints("ends"), ax = op.ints("axes"), sp = op.ints("steps");
      DNNF_CHECK(st.size() == en.size(), DNNF_INVALID_ARG, "Slice starts/ends");
      for (size_t i = 0; i < st.size(); i++) {
        int a = norm_axis(ax.empty() ? (int64_t)i : ax[i], out.size());
        int64_t step = sp.empty() ? 1 : sp[i];
        DNNF_CHECK(step >= 1, DNNF_UNSUPPORTED_OP, "Slice with non-positive step");
        int64_t d = in(0)[a], s = st[i] < 0 ? st[i] + d : st[i], e = en[i] < 0 ? en[i] + d : en[i];
        s = std::min(std::max<int64_t>(s, 0), d);
        e = std::min(std::max<int64_t>(e, 0), d);
        out[a] = e > s ? (e - s + step - 1) / step : 0;
      }
      return out;
    }
    case OC_SPLIT: {
      need(1);
      Dims out = in(0);
      int a = norm_axis(op.i("axis", 0), out.size());
      auto sp = op.ints("split");
      if (sp.empty()) {
        DNNF_CHECK(out[a] % (int64_t)op.out.size() == 0, DNNF_SHAPE_MISMATCH, "Split into unequal parts needs 'split'");
        sp.assign(op.out.size(), out[a] / (int64_t)op.out.size());
      }
      DNNF_CHECK(sp.size() == op.out.size(), DNNF_INVALID_ARG, "Split sizes");
      int64_t tot = 0;
      for (auto s : sp) tot += s;
      DNNF_CHECK(tot == out[a], DNNF_SHAPE_MISMATCH, "Split sizes do not add up");
      out[a] = sp[oi];
      return out;
    }
    case OC_CONCAT: {
      need(1);
      Dims out = in(0);
      int a = norm_axis(op.i("axis", 0), out.size());
      for (size_t k = 1; k < op.in.size(); k++) {
        const Dims& d = in((int)k);
        DNNF_CHECK(d.size() == out.size(), DNNF_SHAPE_MISMATCH, "Concat rank");
        for (size_t i = 0; i < d.size(); i++)
          if ((int)i != a) DNNF_CHECK(d[i] == out[i], DNNF_SHAPE_MISMATCH, "Concat extents");
        out[a] += d[a];
      }
      return out;
    }
    case OC_EXPAND:
      need(1);
      return broadcast_dims(in(0), op.ints("shape"));
    case OC_RESIZE: {
      need(1);
      Dims out = in(0);
      auto sc = op.ints("scales");
      DNNF_CHECK(sc.size() == out.size(), DNNF_INVALID_ARG, op.kind + " needs one integer scale per axis");
      for (size_t d = 0; d < out.size(); d++) {
        DNNF_CHECK(sc[d] >= 1, DNNF_UNSUPPORTED_OP, op.kind + ": only nearest-neighbour enlargement by integer factors is executable");
        out[d] *= sc[d];
      }
      return out;
    }
    default:
      throw Error(DNNF_UNSUPPORTED_OP, "operator " + op.kind + " is classified but cannot be executed");
  }
}

// ------------------------------------------------------------------ classification (Sec. 3.1)
// The operator's type is that of its most complex input/output pair.  Pairs are taken over
// activation operands: a broadcast weight or constant (bias, BatchNormalization vectors) does not
// raise the type - Table 2 lists Add and BatchNormalization as One-to-One - while a broadcast
// activation makes an elementwise operator "Elementwise w/ broadcast", i.e. One-to-Many.
int classify_op(const Graph& g, const Op& op) {
  int t = op.info->mapping;
  if (op.info->cls == OC_BINARY || op.info->cls == OC_WHERE) {
    int64_t on = g.tensors[op.out[0]].n();
    for (int i : op.in) {
      const Tensor& x = g.tensors[i];
      if (!x.weight_only && x.n() < on) t = std::max(t, (int)DNNF_ONE_TO_MANY);
    }
  }
  return t;
}

// ------------------------------------------------------------------ #FLOPS (Sec. 4.2 cost model)
// Elementwise operator: one per output element.  Reduction: one per input element.
// Contractions: 2 per multiply-accumulate.
double op_flops(const Graph& g, const Op& op) {
  double on = (double)g.tensors[op.out[0]].n();
  switch (op.info->cls) {
    case OC_REDUCE: case OC_GAP: return (double)g.tensors[op.in[0]].n();
    case OC_POOL: {
      auto ks = op.ints("kernel_shape");
      return on * (double)(ks.size() == 2 ? ks[0] * ks[1] : 1);
    }
    case OC_SOFTMAX: return 5.0 * on;
    case OC_NORMALIZE: return 6.0 * on;
    case OC_CONV: {
      const Dims& w = g.tensors[op.in[1]].dims;
      return 2.0 * on * (double)(w[1] * w[2] * w[3] * (w.size() == 5 ? w[4] : 1));
    }
    case OC_CONVT: {
      const Dims& w = g.tensors[op.in[1]].dims;
      return 2.0 * (double)g.tensors[op.in[0]].n() * (double)(w[1] * w[2] * w[3]);      // every input element meets every tap of every output channel
    }
    case OC_MATMUL: {
      const Dims& a = g.tensors[op.in[0]].dims;
      return 2.0 * on * (double)a.back();
    }
    case OC_GEMM: {
      const Dims& a = g.tensors[op.in[0]].dims;
      return 2.0 * on * (double)(op.i("transA", 0) ? a[0] : a[1]);
    }
    default: {
      double tot = 0;
      for (int o : op.out) tot += (double)g.tensors[o].n();
      // a third power by a constant is executed (and counted) as its two multiplications
      if (op.kind == "Pow" && op.in.size() == 2 && g.tensors[op.in[1]].has_cval && g.tensors[op.in[1]].cval.size() == 1 &&
          g.tensors[op.in[1]].cval[0] == 3.0)
        return 2.0 * tot;
      return op.info->flops_per_out * tot;
    }
  }
}

void Graph::relink() {
  for (auto& t : tensors) { t.producer = -1; t.consumers.clear(); }
  for (size_t i = 0; i < ops.size(); i++) {
    if (!ops[i].alive) continue;
    for (int o : ops[i].out) {
      DNNF_CHECK(tensors[o].producer < 0, DNNF_INVALID_ARG, "tensor " + tensors[o].name + " has two producers");
      DNNF_CHECK(tensors[o].kind == DNNF_INTERMEDIATE || tensors[o].kind == DNNF_OUTPUT, DNNF_INVALID_ARG,
                 "operator writes input/weight tensor " + tensors[o].name);
      tensors[o].producer = (int)i;
    }
    for (int t : ops[i].in) tensors[t].consumers.push_back((int)i);
  }
  // Kahn's algorithm; ties broken by op id so the order is deterministic.
  std::vector<int> indeg(ops.size(), 0);
  for (size_t i = 0; i < ops.size(); i++) {
    if (!ops[i].alive) continue;
    std::set<int> preds;
    for (int t : ops[i].in) {
      const Tensor& x = tensors[t];
      if (x.producer >= 0) preds.insert(x.producer);
      else DNNF_CHECK(x.kind == DNNF_INPUT || x.kind == DNNF_WEIGHT, DNNF_INVALID_ARG,
                      "tensor " + x.name + " is read but never produced");
    }
    indeg[i] = (int)preds.size();
  }
  std::set<int> ready;
  for (size_t i = 0; i < ops.size(); i++)
    if (ops[i].alive && indeg[i] == 0) ready.insert((int)i);
  topo.clear();
  while (!ready.empty()) {
    int i = *ready.begin();
    ready.erase(ready.begin());
    topo.push_back(i);
    std::set<int> succ;
    for (int o : ops[i].out) for (int c : tensors[o].consumers) succ.insert(c);
    for (int c : succ) if (--indeg[c] == 0) ready.insert(c);
  }
  DNNF_CHECK((int)topo.size() == live_ops(), DNNF_CYCLE, "the operator graph has a cycle");
  for (auto& t : tensors) t.weight_only = (t.kind == DNNF_WEIGHT);
  for (int i : topo) {
    bool wo = true;
    for (int t : ops[i].in) wo = wo && tensors[t].weight_only;
    for (int o : ops[i].out) tensors[o].weight_only = wo && tensors[o].kind != DNNF_OUTPUT;
  }
  for (int i : topo) {
    ops[i].mapping = classify_op(*this, ops[i]);
    ops[i].flops = op_flops(*this, ops[i]);
  }
}

void Graph::finalize() {
  for (auto& op : ops) {
    if (!op.alive) continue;
    DNNF_CHECK(!op.out.empty(), DNNF_INVALID_ARG, op.kind + ": no outputs");
    for (size_t k = 0; k < op.out.size(); k++) {
      Dims want = infer_shape(*this, op, (int)k);
      const Tensor& t = tensors[op.out[k]];
      if (want != t.dims) {
        std::ostringstream s;
        s << op.kind << ": output " << t.name << " declared [";
        for (auto d : t.dims) s << d << ",";
        s << "] but inferred [";
        for (auto d : want) s << d << ",";
        s << "]";
        throw Error(DNNF_SHAPE_MISMATCH, s.str());
      }
    }
    if (op.info->cls == OC_GATHER) {
      int dt = tensors[op.in[1]].dtype;
      DNNF_CHECK(dt == DNNF_I32 || dt == DNNF_I64, DNNF_INVALID_ARG, "Gather indices must be integer");
      // indices the compiler can read are checked here; indices that arrive at run time are wrapped and clamped by
      // the generated code, so neither kind can address outside the gathered axis
      const Tensor& I = tensors[op.in[1]];
      const Dims& dd = tensors[op.in[0]].dims;
      int64_t ax = op.i("axis", 0);
      if (ax < 0) ax += (int64_t)dd.size();
      DNNF_CHECK(ax >= 0 && ax < (int64_t)dd.size(), DNNF_INVALID_ARG, "Gather axis out of range");
      if (I.has_cval)
        for (double v : I.cval)
          DNNF_CHECK(v >= -(double)dd[ax] && v < (double)dd[ax], DNNF_INVALID_ARG,
                     "Gather: constant index " + std::to_string((long long)v) + " lies outside the axis of length " + std::to_string((long long)dd[ax]));
    }
  }
  relink();
  finalized = true;
}

}  // namespace dnnf
