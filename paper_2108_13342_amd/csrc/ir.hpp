// Extended Computational Graph (paper Sec. 3.2): operators annotated with mapping type,
// mathematical properties, and whether their result can be removed by fusion.
#pragma once
#include <cstdint>
#include <map>
#include <set>
#include <stdexcept>
#include <string>
#include <vector>

#include "../../include/dnnf.h"

namespace dnnf {

struct Error : std::runtime_error {
  dnnf_status code;
  Error(dnnf_status c, const std::string& m) : std::runtime_error(m), code(c) {}
};
#define DNNF_CHECK(cond, code, msg)                     \
  do {                                                  \
    if (!(cond)) throw ::dnnf::Error((code), (msg));    \
  } while (0)

using Dims = std::vector<int64_t>;
inline int64_t numel(const Dims& d) {
  int64_t n = 1;
  for (auto x : d) n *= x;
  return n;
}
inline int dtype_bytes(int dt) {
  switch (dt) {
    case DNNF_F32: case DNNF_I32: return 4;
    case DNNF_F16: case DNNF_BF16: return 2;
    case DNNF_I64: return 8;
    default: return 1;
  }
}
inline bool is_float(int dt) { return dt == DNNF_F32 || dt == DNNF_F16 || dt == DNNF_BF16; }

// Operator classes used by shape inference and lowering.
enum OpClass {
  OC_UNARY,      // y = f(x)
  OC_BINARY,     // y = f(a, b) with numpy broadcasting
  OC_WHERE,      // y = c ? a : b
  OC_BATCHNORM,  // inference BatchNormalization
  OC_CONV,
  OC_CONVT,      // ConvTranspose (2-d, group 1)
  OC_MATMUL,
  OC_GEMM,
  OC_REDUCE,     // ReduceSum/Mean/Max/Prod
  OC_SOFTMAX,
  OC_NORMALIZE,  // (x - mean) / sqrt(var + eps) over the last axis (internal, from the LayerNorm decomposition)
  OC_GAP,        // GlobalAveragePool
  OC_POOL,       // MaxPool / AveragePool over a 2-d window ("kernel_shape", "strides", "pads", "count_include_pad")
  OC_EINSUM,     // two-operand Einsum with an explicit result ("equation": the character codes of e.g. "bhid,bhjd->bhij");
                 // the rewriting pass expands it into Transpose / Reshape / MatMul, it has no kernel of its own
  OC_SCAN,       // CumSum along "axis" ("exclusive", "reverse" as in ONNX; the axis is an attribute here)
  OC_GATHER,
  OC_RESHAPE,    // Reshape / Flatten / Squeeze / Unsqueeze
  OC_TRANSPOSE,
  OC_SLICE,
  OC_SPLIT,
  OC_CONCAT,
  OC_EXPAND,
  OC_RESIZE,     // Resize / Upsample, nearest neighbour by integer factors ("scales", one per axis)
  OC_D2S,        // DepthToSpace / SpaceToDepth (classified only)
  OC_OTHER       // classified by Table 2, not executable here
};

struct OpKindInfo {
  const char* name;
  OpClass cls;
  int mapping;       // Table 2 mapping type
  bool in_table2;    // printed in Table 2 (others are classified from the Sec. 3.1 definitions)
  bool assoc, commut, distrib;  // mathematical properties recorded in the ECG
  double flops_per_out;         // elementwise cost used by the rewriting cost model (Sec. 4.2)
};
const OpKindInfo* find_op_kind(const std::string& name);
const std::vector<OpKindInfo>& all_op_kinds();

struct Tensor {
  std::string name;
  int dtype = DNNF_F32;
  Dims dims;
  int kind = DNNF_INTERMEDIATE;
  int producer = -1;            // op id, -1 for graph inputs / weights
  std::vector<int> consumers;   // op ids (live ops only after finalize)
  bool has_cval = false;
  std::vector<double> cval;     // host-readable values (small constants)
  bool weight_only = false;     // computed from weights alone (known at compile time)
  int ext_index = -1;           // position among tensors of its kind (INPUT / WEIGHT / OUTPUT)
  std::string origin;           // name of the tensor of the original graph whose value this one equals (set by rewrites)
  // Storage order of the dimensions, major to minor (empty = as declared, row-major).  Only tensors the
  // plan owns (intermediates, relaid-out weights) ever get one; the caller's buffers keep the declared order.
  std::vector<int> perm;
  int64_t n() const { return numel(dims); }
  int64_t bytes() const { return n() * dtype_bytes(dtype); }
};

using Attrs = std::map<std::string, std::vector<double>>;

struct Op {
  std::string kind;
  const OpKindInfo* info = nullptr;
  std::vector<int> in, out;
  Attrs attrs;
  int mapping = DNNF_ONE_TO_ONE;
  bool alive = true;
  double flops = 0;
  // attribute helpers
  bool has(const std::string& k) const { return attrs.count(k) != 0; }
  double f(const std::string& k, double dflt) const {
    auto it = attrs.find(k);
    return it == attrs.end() || it->second.empty() ? dflt : it->second[0];
  }
  int64_t i(const std::string& k, int64_t dflt) const { return (int64_t)f(k, (double)dflt); }
  std::vector<int64_t> ints(const std::string& k) const {
    std::vector<int64_t> r;
    auto it = attrs.find(k);
    if (it != attrs.end()) for (double v : it->second) r.push_back((int64_t)v);
    return r;
  }
};

// Einsum equation of an operator, parsed: one label string per operand and the result's.  Throws on forms that
// are not supported (ellipsis, implicit result, a label repeated inside one term, other than two operands).
struct EinsumSpec { std::string a, b, out; };
EinsumSpec parse_einsum(const Op& op);

struct Graph {
  std::vector<Tensor> tensors;
  std::vector<Op> ops;
  std::vector<int> topo;       // live op ids in topological order
  std::vector<int> inputs, weights, outputs;  // tensor ids by kind, declaration order
  bool finalized = false;

  int add_tensor(const std::string& name, int dtype, const Dims& dims, int kind);
  int add_op(const std::string& kind, const std::vector<int>& in, const std::vector<int>& out, const Attrs& a);
  void finalize();             // validate + infer + topo + classify
  void relink();               // rebuild producer/consumer lists, topo order, weight_only flags, classes
  int new_tensor_like(const std::string& stem, int dtype, const Dims& dims);
  int new_const(const std::string& stem, int dtype, const Dims& dims, const std::vector<double>& v);
  int live_ops() const {
    int n = 0;
    for (auto& o : ops) n += o.alive;
    return n;
  }
  double total_flops() const {
    double f = 0;
    for (auto& o : ops) if (o.alive) f += o.flops;
    return f;
  }
};

Dims infer_shape(const Graph& g, const Op& op, int out_index);
Dims broadcast_dims(const Dims& a, const Dims& b);
int classify_op(const Graph& g, const Op& op);      // Table 2 + most-complex-pair rule
double op_flops(const Graph& g, const Op& op);      // cost model of Sec. 4.2
void fuse_relation(int first, int second, int* fused, int* colour);  // mapping-type analysis table

struct RewriteStats {
  int rules_fired = 0, derived_rules_fired = 0, canonicalisations = 0, ops_before = 0, ops_after = 0;
  double flops_before = 0, flops_after = 0;
  std::vector<std::string> log;
};
void rewrite_graph(Graph& g, RewriteStats& st);
// Storage orders for the tensors between blocks (Sec. 4.4.2); returns how many tensors were given one.
int select_layouts(Graph& g);

}  // namespace dnnf
