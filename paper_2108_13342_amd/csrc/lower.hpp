// Fusion blocks and their lowering to one generated HIP kernel each (paper Sec. 4.4).
//
// A block is lowered through a data-flow tree walk (Sec. 4.4.1): starting from each block output
// the walk asks, operator by operator, which value an element depends on, until it reaches the
// block's inputs.  Reorganize and Shuffle operators contribute no code, only a change of index
// (Sec. 4.4.2, intra-block optimisation); common sub-trees are emitted once.
#pragma once
#include <map>
#include <string>
#include <vector>

#include "ir.hpp"

namespace dnnf {

struct Block {
  std::vector<int> ops;   // op ids, topological order
  int fused_type = DNNF_ONE_TO_ONE;
  bool weight_only = false;  // computed once at prepare time
};

enum Family { FAM_EW = 0, FAM_REDUCE = 1, FAM_GEMM = 2, FAM_CONV = 3, FAM_DWCONV = 4, FAM_ALIAS = 5, FAM_ATTENTION = 6, FAM_SE = 7 };

struct Launch {
  std::string name;       // kernel symbol
  std::string source;     // complete HIP translation unit
  unsigned grid[3] = {1, 1, 1}, block[3] = {1, 1, 1};
  unsigned lds_bytes = 0;
  std::vector<int> params;  // tensor ids in kernel-parameter order
  bool scratch = false;     // one more trailing parameter: the block's scratch area (float*)
};

struct Lowered {
  int family = FAM_EW;
  std::vector<int> ext_in, ext_out;  // external tensors read / written
  std::vector<Launch> launches;      // usually one
  int alias_src = -1, alias_dst = -1;  // FAM_ALIAS: dst shares src's storage
  // FAM_ALIAS of a stacking Concat: each listed tensor lives inside alias_dst's storage at the given byte offset
  std::vector<std::pair<int, int64_t>> alias_parts;
  int64_t scratch_bytes = 0;         // device memory the block's launches pass partial results through
  double bytes = 0, flops = 0, irs_removed = 0;
  std::string variant;               // human-readable template choice
};

struct LowerOpts {
  bool intra_block = true;  // fold Reorganize/Shuffle into index maps; when false they copy
  int force_variant = 0;    // 0 auto; template-specific override used by profiling
  bool alias_concat = true; // a Concat that only stacks stored tensors along the outermost axis becomes shared storage
  int pool_op = -1;         // a GlobalAveragePool over one of the block's results, taken inside a depthwise convolution's kernel
};

// Throws Error(DNNF_UNSUPPORTED_OP) when the block's structure has no template; the planner's
// constraint check uses that to refuse a fusion.
Lowered lower_block(const Graph& g, const Block& b, const LowerOpts& o);

void block_io(const Graph& g, const Block& b, std::vector<int>& ext_in, std::vector<int>& ext_out,
              std::vector<int>& removed);

}  // namespace dnnf
