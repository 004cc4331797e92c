#pragma once
#include <memory>
#include <string>
#include <vector>

#include "lower.hpp"
#include "planner.hpp"

namespace dnnf {

struct PlanBlock {
  Block blk;
  Lowered low;
  std::vector<void*> fn;   // hipFunction_t per launch, loaded lazily
};

struct Plan {
  struct Impl;
  Impl* impl;
  Graph g;
  std::vector<PlanBlock> blocks;
  std::vector<const void*> weight_ptrs;
  std::vector<int64_t> ws_offset;   // per tensor, -1 = none
  std::vector<int> alias_of;        // per tensor, -1 = own storage
  std::vector<int64_t> alias_off;   // byte offset inside the tensor it is kept in (stacking Concat), else 0
  std::vector<int> const_pool;      // compiler-made constants uploaded at prepare time
  size_t ws_bytes = 0;
  std::string cache_dir;
  bool verbose = false;
  bool tune = false;
  bool use_graphs = false;         // replay the run loop as a HIP graph once a set of buffers is seen again
  size_t scratch_offset = 0;       // the blocks' shared scratch area inside the workspace
  int relaid_tensors = 0;          // tensors given a storage order other than the declared one
  LowerOpts lower_opts;
  PlanStats stats;
  std::vector<std::string> log;

  const uint64_t serial;           // unique per plan object of the process (the static workspace remembers its last user by it)

  Plan();
  ~Plan();
  Plan(const Plan&) = delete;
  void layout_workspace();
  void* resolve(int tensor, const void* const* in, void* const* out, void* ws) const;
  void* function_for(const Launch& L);
  void launch_block(size_t b, const void* const* in, void* const* out, void* ws, void* stream);
  void load_kernels();             // every code object of the plan resident on the current device
  void prepare(void* ws, void* stream);
  void run_static(const void* const* in, void* const* out, void* stream);   // run() in the library's static workspace
  void run(const void* const* in, void* const* out, void* ws, void* stream);
  double time_block(size_t b, const void* const* in, void* const* out, void* ws, void* stream, int warmup, int iters);
};

Plan* build_plan(const Graph& g, const dnnf_plan_opts& o, const void* const* weight_ptrs, void* stream);
void precompile(const Lowered& low, const std::string& cache_dir);
// every other tile configuration the block's kernel template offers (empty for most families)
std::vector<Lowered> tile_variants(const Graph& g, const Block& b, const Lowered& chosen, const LowerOpts& lo);

}  // namespace dnnf
