// Shared machinery of the kernel generator: iteration atoms, per-tensor index descriptions,
// the expression DAG of a block (the data-flow tree of paper Sec. 4.4.1 with common sub-trees
// merged), and C source emission for it.
#pragma once
#include <map>
#include <set>
#include <sstream>
#include <string>
#include <vector>

#include "lower.hpp"

namespace dnnf {

// The index of one tensor dimension: a mixed-radix number over iteration atoms (major to minor)
// plus a constant, or a value read from an index tensor (Gather).
struct DimIdx {
  std::vector<int> atoms;
  int64_t offset = 0;
  int indirect = -1;  // expression node holding the (integer) index value
};
using TIdx = std::vector<DimIdx>;

// A gathered axis of an address: the index is the value of expression node `first`, `second` is the axis's
// element stride and `extent` its length (the generated code wraps negative indices and clamps to the axis).
struct IndirectTerm {
  int first;
  int64_t second;
  int64_t extent;
};

struct Affine {
  std::map<int, int64_t> stride;                     // atom -> element stride
  int64_t offset = 0;
  std::vector<IndirectTerm> indirect;
};

struct Pred {       // mixedradix(atoms) == equals, or lo <= mixedradix(atoms) < hi when hi > lo
  std::vector<int> atoms;
  int64_t equals = 0;
  int64_t lo = 0, hi = 0;
};

struct ENode {
  enum Kind { LOAD, CONSTV, OP, ANCHOR } kind = OP;
  int tensor = -1;       // LOAD
  Affine addr;           // LOAD
  std::string op;        // OP: operator kind
  const Op* src = nullptr;
  std::vector<int> args;
  double cv = 0;         // CONSTV
  bool is_int = false;   // integer-valued (Gather indices)
};

struct Store {
  int tensor;
  Affine addr;
  int value;
  std::vector<Pred> preds;
};

struct LowerCtx {
  const Graph& g;
  const Block& blk;
  LowerOpts opts;
  std::set<int> inblock;
  std::vector<int64_t> atom_extent;
  std::vector<std::pair<int, int>> atom_split;  // (-1,-1) or (hi, lo)
  std::vector<ENode> nodes;
  std::map<std::string, int> cse;
  std::map<int, TIdx> tidx;                     // first pivot-space index seen for a tensor
  std::map<int, std::vector<Pred>> tpred;       // predicates attached by forward walks
  int anchor_op = -1, anchor_out = -1;
  std::vector<Store> stores;
  std::vector<int> only_outputs;                // restrict the kernel to these block outputs
  std::vector<Pred> cur_preds;                  // predicates of the store whose value tree is being built
  int pivot_out = -1;                           // elementwise blocks: the output whose index space the kernel walks (-1: the last)
  mutable std::map<int, std::pair<double, double>> range_memo;   // value interval per expression node
  bool lowp = false;                            // every block output is stored in a 16-bit type
  int concat_op = -1, concat_part = -1;         // lowering one operand's range of a block-closing Concat
  // A Resize behind the block's anchor (Conv -> Resize, a yellow cell of the mapping-type table): every result of
  // the anchor is stored at s x s positions.  The forward walk gives the enlarged axes one more index digit each
  // (a replication atom); templates that set allow_replication run their epilogue once per value of those digits.
  bool allow_replication = false;
  std::vector<int> rep_atoms;

  LowerCtx(const Graph& g_, const Block& b_, const LowerOpts& o_);

  int new_atom(int64_t extent);
  void resolve(const std::vector<int>& in, std::vector<int>& out) const;  // expand split atoms
  int64_t extent_of(const std::vector<int>& atoms) const;
  TIdx fresh_index(const Dims& dims);
  TIdx regroup(const TIdx& src, const Dims& src_dims, const Dims& dst_dims);
  Affine affine(const Tensor& T, const TIdx& idx);   // element address under the tensor's storage order
  Affine resolved(const Affine& a) const;
  std::vector<int> final_atoms() const;         // unsplit atoms with extent > 1
  bool is_split(int atom) const { return atom_split[atom].first >= 0; }
  // declarations of the (recursively) split-off parts of atoms whose own values `a<id>` are in scope: an index
  // map further up the block (a Reshape, DepthToSpace, ...) may have cut an atom the kernel computes as a whole
  std::string decl_parts(const std::vector<int>& atoms, const std::string& ind) const;

  int add_node(const ENode& n);
  int value(int tensor, const TIdx& idx);       // backward data-flow walk
  bool forward_step(const Op& op);              // give pivot-space indices to op's outputs
  void forward_all();
  void collect_stores(const std::vector<int>& outs);
  bool is_external(int tensor) const;

  // ---- emission
  std::string ctype(int dtype) const;
  std::string param_list(const std::vector<int>& params, const std::set<int>& written) const;
  // Emits statements computing every node needed by `roots` (in order); atom variables are
  // expected to be in scope as `a<id>`.  `done` carries nodes already emitted in this scope.
  void emit_values(std::ostringstream& os, const std::vector<int>& roots, std::set<int>& done,
                   const std::map<int, int>& pslot, const std::string& indent,
                   const std::map<int, std::string>* load_override = nullptr) const;
  std::string addr_expr(const Affine& a) const;
  std::string store_stmt(const Store& s, const std::map<int, int>& pslot, const std::string& off) const;
  std::string pred_expr(const std::vector<Pred>& p) const;
  std::string vname(int node) const { return "v" + std::to_string(node); }
};

const char* device_preamble();
std::string fnv_name(const std::string& prefix, const std::string& body);

// A MatMul anchor analysed: operand tensors and addresses, and its iteration atoms sorted into contraction,
// row (M), column (N) and batch atoms (major to minor by output stride); loader modes 0 direct
// (K-contiguous, 16-byte vectors), 1 transpose (contiguous along M/N), 2 scalar.
struct MatmulFrame {
  int dtype = 0, ta = -1, tb = -1, amode = 2, bmode = 2;
  Affine aa, ab;
  std::vector<int> katoms, rows, cols, batch;
  int64_t K = 1, GM = 1, GN = 1, GZ = 1;
};
MatmulFrame analyse_matmul(LowerCtx& c);    // also runs the forward walk and collects the block's stores

// element stride of `atom` in an address (0 when the address does not move with it)
int64_t stride_of(const Affine& a, int atom);
// `const idx_t a<k> = ...;` for every atom of a mixed-radix counter (atoms major to minor), as generated source
void decl_digits(std::ostringstream& os, const LowerCtx& c, const std::vector<int>& atoms_major_minor,
                 const std::string& counter, const std::string& indent, const std::string& tag);

// shared by the MatMul and Conv templates
std::string gemm_offset_fn(const LowerCtx& c, const std::string& name, const std::vector<int>& atoms, const Affine& a);
const char* gemm_kernel_body();
std::string gemm_epilogue_source(const LowerCtx& c, const std::vector<int>& batch, const std::vector<int>& rows,
                                 const std::vector<int>& cols, const std::map<int, int>& pslot, const std::string& kparams,
                                 int64_t GN, int row_bias_slot, int64_t GM = 0);   // GM > 0 allows the row-wise vector form

Lowered lower_elementwise(LowerCtx& c);
Lowered lower_reduce(LowerCtx& c);
// norm: the block's second part (a normalisation of the product's rows and what follows it), prepared by
// lower_gemm_norm; norm_in: the tensor it normalises; norm_in_stored: that tensor is also read outside the block
Lowered lower_gemm(LowerCtx& c, LowerCtx* norm = nullptr, int norm_in = -1, bool norm_in_stored = true);
// [GlobalAveragePool ->] 1x1 Conv -> One-to-One operators -> 1x1 Conv on [n, c, 1, 1] vectors as one block (beyond the table)
Lowered lower_squeeze_excite(const Graph& g, const Block& b, const LowerOpts& o);
// MatMul -> One-to-One operators -> normalisation of the last axis as one block (beyond the mapping-type table)
Lowered lower_gemm_norm(const Graph& g, const Block& b, const LowerOpts& o);
Lowered lower_conv(LowerCtx& c);
Lowered lower_conv3d(LowerCtx& c);
Lowered lower_conv_transpose(LowerCtx& c);
Lowered lower_pool(LowerCtx& c);
Lowered lower_scan(LowerCtx& c);
// MatMul -> One-to-One operators -> Softmax -> MatMul (+ successors) as one streaming-softmax kernel
Lowered lower_attention(const Graph& g, const Block& b, const LowerOpts& o);

}  // namespace dnnf
