// Fusion plan exploration (paper Sec. 4.3, Listing 1).
#pragma once
#include <functional>
#include <string>
#include <vector>

#include "lower.hpp"

namespace dnnf {

struct PlannerOpts {
  bool fusion = true;
  bool intra_block = true;
  bool check_lowerable = true;   // constraint check also requires a kernel template for the block
  bool successors_first = false; // order of steps II and III of the exploration
  bool attention = false;        // beyond the table: MatMul - One-to-One - Softmax - MatMul as one block
  bool broadcast_prologue = false;   // beyond the table: x * s[n, c, 1, 1] in front of a pointwise convolution joins its block
  int gemm_norm = 0;             // beyond the table: MatMul - One-to-One - Normalize as one block (1 = if measured faster, 2 = always)
  int squeeze_excite = 0;        // beyond the table: [pool -] 1x1 Conv - One-to-One - 1x1 Conv on [n, c, 1, 1] vectors as one block
  int max_block_ops = 64;
  int max_block_operands = 16;
  // Device time of a candidate block in microseconds (Listing 1, step 2.3); empty = no profiling,
  // yellow combinations are then fused.
  std::function<double(const Block&)> latency;
  std::vector<std::string>* log = nullptr;
};

struct PlanStats {
  int seeds = 0, green = 0, yellow_fused = 0, yellow_rejected = 0, red = 0, constraint_rejected = 0,
      profiled = 0;
  int timed = 0, db_hits = 0;   // device measurements taken / answered by the memo or the persisted database
};

// Blocks in an order that respects data dependences.  Weight-only operators form their own blocks
// (flagged), which run once when the plan is prepared.
std::vector<Block> build_fusion_plan(const Graph& g, const PlannerOpts& o, PlanStats* stats);

}  // namespace dnnf
