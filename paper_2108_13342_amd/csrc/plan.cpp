// Plan = fusion blocks + their compiled kernels + workspace layout; and the run loop
// (paper Sec. 4.4: one generated operator per fusion block; generated operators are cached and
// reused when the same pattern appears again).
#include "plan.hpp"

#include <hip/hip_runtime.h>
#include <hip/hiprtc.h>
#include <sys/stat.h>
#include <sys/time.h>
#include <unistd.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cstdio>
#include <cstring>
#include <fstream>
#include <functional>
#include <mutex>

namespace dnnf {

#define HIP_OK(expr)                                                                          \
  do {                                                                                        \
    hipError_t e_ = (expr);                                                                   \
    if (e_ != hipSuccess)                                                                     \
      throw Error(DNNF_HIP_ERROR, std::string(#expr) + ": " + hipGetErrorString(e_));         \
  } while (0)

// ------------------------------------------------------------------ kernel cache
namespace {
struct CacheEntry {
  hipModule_t mod = nullptr;
  hipFunction_t fn = nullptr;
};
std::mutex g_cache_mu;
std::map<std::string, std::vector<char>> g_code_cache;  // kernel name -> code object (process-wide)

std::vector<char> compile_to_code(const Launch& L, const std::string& cache_dir, bool verbose) {
  {
    std::lock_guard<std::mutex> lk(g_cache_mu);
    auto it = g_code_cache.find(L.name);
    if (it != g_code_cache.end()) return it->second;
  }
  std::string path;
  if (!cache_dir.empty()) {
    path = cache_dir + "/" + L.name + ".hsaco";
    std::ifstream f(path, std::ios::binary);
    if (f) {
      std::vector<char> code((std::istreambuf_iterator<char>(f)), std::istreambuf_iterator<char>());
      if (!code.empty()) {
        // (a build that prunes the cache directory afterwards marks the code objects it still needs)
        if (getenv("DNNF_CACHE_TOUCH")) (void)utimes(path.c_str(), nullptr);
        std::lock_guard<std::mutex> lk(g_cache_mu);
        g_code_cache[L.name] = code;
        return code;
      }
    }
  }
  hiprtcProgram prog;
  if (hiprtcCreateProgram(&prog, L.source.c_str(), (L.name + ".hip").c_str(), 0, nullptr, nullptr) != HIPRTC_SUCCESS)
    throw Error(DNNF_COMPILE_FAILED, "hiprtcCreateProgram failed");
  // packed-fp32 instruction selection is switched off for all generated code
  const char* opts[] = {"--offload-arch=gfx950", "-O3", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                        "-ffp-contract=fast"};
  hiprtcResult r = hiprtcCompileProgram(prog, 7, opts);
  if (r != HIPRTC_SUCCESS) {
    size_t n = 0;
    hiprtcGetProgramLogSize(prog, &n);
    std::string log(n, '\0');
    if (n) hiprtcGetProgramLog(prog, &log[0]);
    hiprtcDestroyProgram(&prog);
    if (verbose) fprintf(stderr, "---- source of %s ----\n%s\n", L.name.c_str(), L.source.c_str());
    throw Error(DNNF_COMPILE_FAILED, "hiprtc: " + log.substr(0, 4000));
  }
  size_t cs = 0;
  hiprtcGetCodeSize(prog, &cs);
  std::vector<char> code(cs);
  hiprtcGetCode(prog, code.data());
  hiprtcDestroyProgram(&prog);
  if (!path.empty()) {
    mkdir(cache_dir.c_str(), 0755);
    std::string tmp = path + ".tmp" + std::to_string((long)getpid());
    std::ofstream f(tmp, std::ios::binary);
    f.write(code.data(), (std::streamsize)code.size());
    f.close();
    rename(tmp.c_str(), path.c_str());
  }
  std::lock_guard<std::mutex> lk(g_cache_mu);
  g_code_cache[L.name] = code;
  return code;
}
}  // namespace

// One instantiated graph per set of buffers the plan was run with (kernel arguments are part of a graph).
struct RunGraph {
  std::vector<const void*> key;      // input pointers, output pointers, workspace
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;     // null until the set is seen a second time
};

struct Plan::Impl {
  std::map<std::string, CacheEntry> loaded;  // per plan (modules belong to the current context)
  std::vector<RunGraph> graphs;
  hipStream_t capture_stream = nullptr;
  ~Impl() {
    for (auto& rg : graphs) {
      if (rg.exec) (void)hipGraphExecDestroy(rg.exec);
      if (rg.graph) (void)hipGraphDestroy(rg.graph);
    }
    if (capture_stream) (void)hipStreamDestroy(capture_stream);
    for (auto& kv : loaded) if (kv.second.mod) (void)hipModuleUnload(kv.second.mod);
  }
};

static std::atomic<uint64_t> g_plan_serial{0};

Plan::Plan() : impl(new Impl), serial(++g_plan_serial) {}
Plan::~Plan() { delete impl; }

void* Plan::function_for(const Launch& L) {
  auto it = impl->loaded.find(L.name);
  if (it != impl->loaded.end()) return (void*)it->second.fn;
  std::vector<char> code = compile_to_code(L, cache_dir, verbose);
  CacheEntry e;
  HIP_OK(hipModuleLoadData(&e.mod, code.data()));
  HIP_OK(hipModuleGetFunction(&e.fn, e.mod, L.name.c_str()));
  impl->loaded[L.name] = e;
  return (void*)e.fn;
}

void precompile(const Lowered& low, const std::string& cache_dir) {
  for (auto& L : low.launches) compile_to_code(L, cache_dir, false);
}

std::vector<Lowered> tile_variants(const Graph& g, const Block& b, const Lowered& chosen, const LowerOpts& lo) {
  std::vector<Lowered> out;
  if (chosen.family != FAM_GEMM && chosen.family != FAM_CONV && chosen.family != FAM_DWCONV) return out;
  std::set<std::string> seen = {chosen.launches.empty() ? std::string() : chosen.launches[0].name};
  for (int v = 0; v < 32; v++) {
    LowerOpts l2 = lo;
    l2.force_variant = 100 + v;
    try {
      Lowered low = lower_block(g, b, l2);
      if (low.family != chosen.family || low.launches.size() != 1) break;
      if (seen.insert(low.launches[0].name).second) out.push_back(low);      // (two indices may give one kernel)
    } catch (const Error&) {
      break;          // past the last configuration
    }
  }
  return out;
}

// IEEE binary16 from binary32, round to nearest even (host side, for uploaded constants).
static uint16_t float_to_half(float f) {
  uint32_t x;
  memcpy(&x, &f, 4);
  uint32_t sign = (x >> 16) & 0x8000u;
  int32_t e = (int32_t)((x >> 23) & 0xFF) - 127 + 15;
  uint32_t m = x & 0x7FFFFFu;
  if (((x >> 23) & 0xFF) == 0xFF) return (uint16_t)(sign | 0x7C00u | (m ? 0x200u : 0));
  if (e >= 31) return (uint16_t)(sign | 0x7C00u);
  if (e <= 0) {
    if (e < -10) return (uint16_t)sign;
    m |= 0x800000u;
    int shift = 14 - e;
    uint32_t h = m >> shift, rem = m & ((1u << shift) - 1), half = 1u << (shift - 1);
    if (rem > half || (rem == half && (h & 1))) h++;
    return (uint16_t)(sign | h);
  }
  uint32_t h = ((uint32_t)e << 10) | (m >> 13), rem = m & 0x1FFFu;
  if (rem > 0x1000u || (rem == 0x1000u && (h & 1))) h++;
  return (uint16_t)(sign | h);
}

// ------------------------------------------------------------------ workspace layout
static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

void Plan::layout_workspace() {
  ws_offset.assign(g.tensors.size(), -1);
  alias_of.assign(g.tensors.size(), -1);
  alias_off.assign(g.tensors.size(), 0);
  size_t off = 0;
  auto place = [&](int t) {
    if (ws_offset[t] >= 0) return;
    ws_offset[t] = (int64_t)off;
    off = align_up(off + (size_t)std::max<int64_t>(g.tensors[t].bytes(), 1), 256);
  };
  // compiler-made constants (host values, no caller buffer)
  for (size_t t = 0; t < g.tensors.size(); t++) {
    const Tensor& T = g.tensors[t];
    if (T.kind == DNNF_WEIGHT && T.ext_index < 0 && T.has_cval && T.n() > 1) { place((int)t); const_pool.push_back((int)t); }
  }
  for (auto& pb : blocks) {
    if (pb.low.family == FAM_ALIAS && pb.low.alias_parts.empty()) { alias_of[pb.low.alias_dst] = pb.low.alias_src; continue; }
    for (int t : pb.low.ext_out)
      if (g.tensors[t].kind == DNNF_INTERMEDIATE) place(t);
  }
  // stacking Concats: the operands live inside the result (build_plan has made sure no tensor is claimed twice)
  for (auto& pb : blocks)
    if (pb.low.family == FAM_ALIAS && !pb.low.alias_parts.empty())
      for (auto& pr : pb.low.alias_parts) { alias_of[pr.first] = pb.low.alias_dst; alias_off[pr.first] = pr.second; }
  // one scratch area for all blocks (they run one after another on the stream)
  size_t scratch = 0;
  for (auto& pb : blocks) scratch = std::max(scratch, (size_t)pb.low.scratch_bytes);
  scratch_offset = off;
  ws_bytes = align_up(off + scratch, 256);
}

void* Plan::resolve(int t, const void* const* in, void* const* out, void* ws) const {
  int64_t within = 0;
  while (alias_of[t] >= 0) { within += alias_off[t]; t = alias_of[t]; }
  const Tensor& T = g.tensors[t];
  if (T.kind == DNNF_INPUT) {
    DNNF_CHECK(in && in[T.ext_index], DNNF_INVALID_ARG, "missing input pointer for " + T.name);
    return (char*)const_cast<void*>(in[T.ext_index]) + within;
  }
  if (T.kind == DNNF_OUTPUT) {
    DNNF_CHECK(out && out[T.ext_index], DNNF_INVALID_ARG, "missing output pointer for " + T.name);
    return (char*)out[T.ext_index] + within;
  }
  if (T.kind == DNNF_WEIGHT && T.ext_index >= 0) {
    DNNF_CHECK(weight_ptrs[T.ext_index], DNNF_INVALID_ARG, "missing weight pointer for " + T.name);
    return (char*)const_cast<void*>(weight_ptrs[T.ext_index]) + within;
  }
  DNNF_CHECK(ws_offset[t] >= 0, DNNF_INVALID_ARG, "tensor " + T.name + " has no storage");
  DNNF_CHECK(ws, DNNF_INVALID_ARG, "workspace pointer is null");
  return (char*)ws + ws_offset[t] + within;
}

void Plan::launch_block(size_t b, const void* const* in, void* const* out, void* ws, void* stream) {
  PlanBlock& pb = blocks[b];
  DNNF_CHECK(pb.low.family >= 0, DNNF_UNSUPPORTED_OP, "block has no kernel (plan was built for analysis only): " + pb.low.variant);
  for (size_t li = 0; li < pb.low.launches.size(); li++) {
    const Launch& L = pb.low.launches[li];
    if (pb.fn.size() <= li) pb.fn.resize(pb.low.launches.size(), nullptr);
    if (!pb.fn[li]) pb.fn[li] = function_for(L);
    void* ptrs[33];
    void* args[33];
    DNNF_CHECK(L.params.size() <= 32, DNNF_UNSUPPORTED_OP, "too many kernel parameters");
    for (size_t k = 0; k < L.params.size(); k++) {
      ptrs[k] = resolve(L.params[k], in, out, ws);
      args[k] = &ptrs[k];
    }
    if (L.scratch) {
      DNNF_CHECK(ws, DNNF_INVALID_ARG, "workspace pointer is null");
      ptrs[L.params.size()] = (char*)ws + scratch_offset;
      args[L.params.size()] = &ptrs[L.params.size()];
    }
    HIP_OK(hipModuleLaunchKernel((hipFunction_t)pb.fn[li], L.grid[0], L.grid[1], L.grid[2], L.block[0], L.block[1],
                                 L.block[2], L.lds_bytes, (hipStream_t)stream, args, nullptr));
  }
}

// Value of a compiler-made constant in its storage type, as the bytes the device reads.
static std::vector<char> const_bytes(const Tensor& T) {
  std::vector<char> host((size_t)T.bytes());
  for (int64_t i = 0; i < T.n(); i++) {
    double v = T.cval[(size_t)i];
    switch (T.dtype) {
      case DNNF_F32: ((float*)host.data())[i] = (float)v; break;
      case DNNF_F16: ((uint16_t*)host.data())[i] = float_to_half((float)v); break;
      case DNNF_BF16: {
        float f = (float)v;
        uint32_t u;
        memcpy(&u, &f, 4);
        u += 0x7FFFu + ((u >> 16) & 1u);
        ((uint16_t*)host.data())[i] = (uint16_t)(u >> 16);
        break;
      }
      case DNNF_I32: ((int32_t*)host.data())[i] = (int32_t)v; break;
      case DNNF_I64: ((int64_t*)host.data())[i] = (int64_t)v; break;
      default: host[(size_t)i] = (char)v;
    }
  }
  return host;
}

void Plan::load_kernels() {
  for (auto& pb : blocks) {
    if (pb.low.family < 0) continue;
    if (pb.fn.size() < pb.low.launches.size()) pb.fn.resize(pb.low.launches.size(), nullptr);
    for (size_t li = 0; li < pb.low.launches.size(); li++)
      if (!pb.fn[li]) pb.fn[li] = function_for(pb.low.launches[li]);
  }
}

void Plan::prepare(void* ws, void* stream) {
  // every code object of the plan becomes resident here, so that later runs only enqueue launches
  load_kernels();
  if (!ws) return;      // a plan that will only run in the library's static workspace: nothing to fill here
  for (int t : const_pool) {
    const Tensor& T = g.tensors[t];
    std::vector<char> host = const_bytes(T);
    HIP_OK(hipMemcpyAsync((char*)ws + ws_offset[t], host.data(), host.size(), hipMemcpyHostToDevice, (hipStream_t)stream));
    HIP_OK(hipStreamSynchronize((hipStream_t)stream));
  }
  for (size_t b = 0; b < blocks.size(); b++)
    if (blocks[b].blk.weight_only) launch_block(b, nullptr, nullptr, ws, stream);
  HIP_OK(hipStreamSynchronize((hipStream_t)stream));
}

// ------------------------------------------------------------------ the run that allocates nothing
// The workspace of this entry point is a file-scope device array: each GPU the library runs on holds its own copy at
// its own address for the life of the process.  In host code the array's name is only a handle: the device
// address is asked for once per device (hipGetSymbolAddress, with that device current) and everything - kernel
// arguments included - uses that address.
#define DNNF_STATIC_WS_BYTES ((size_t)DNNF_STATIC_WORKSPACE_BYTES)
static __device__ __align__(256) unsigned char scratch[DNNF_STATIC_WS_BYTES];

namespace {
struct StaticSlot {
  void* ptr = nullptr;     // device address of `scratch` on this device
  uint64_t owner = 0;      // serial of the plan whose prepared tensors the array holds (0: none)
};
constexpr int kMaxDevices = 64;
StaticSlot g_static[kMaxDevices];
std::mutex g_static_mu;

// Host bytes reach the array through kernel arguments, 1 KiB per launch: no staging buffer, nothing allocated, and
// the launch may be recorded into a graph like any other.
struct UploadChunk { unsigned char b[1024]; };
// Operand values for profiling launches.  Timing kernels on zeros (or on whatever earlier candidates left behind)
// flatters the matrix cores - the chip's clock follows its power draw, and multiplying zeros draws little - so that
// candidates would be ranked under conditions no inference meets.  Every 16-bit half of a float operand becomes
// s0111xxxxxxxxxxx with pseudo-random s and x: a finite value of ordinary magnitude whether it is read as fp16
// (0.5 .. 2), as bf16 or as the upper half of an fp32 (2^-15 .. 2).
__global__ void dnnf_fill_profile_values(unsigned int* dst, size_t n_words) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_words; i += (size_t)gridDim.x * blockDim.x) {
    unsigned int h = (unsigned int)i * 2654435761u;
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    dst[i] = (0x3800u | (h & 0x87FFu)) | ((0x3800u | ((h >> 16) & 0x87FFu)) << 16);
  }
}

__global__ void dnnf_upload_chunk(unsigned char* dst, UploadChunk c, int n) {
  const int i = (int)(blockIdx.x * blockDim.x + threadIdx.x);
  if (i < n) dst[i] = c.b[i];
}
}  // namespace

void Plan::run_static(const void* const* in, void* const* out, void* stream) {
  DNNF_CHECK(ws_bytes <= DNNF_STATIC_WS_BYTES, DNNF_OUT_OF_MEMORY,
             "the plan needs " + std::to_string(ws_bytes) + " bytes of workspace, the library's static workspace holds " +
                 std::to_string(DNNF_STATIC_WS_BYTES) + ": use dnnf_plan_run with a workspace of the caller's");
  int dev = -1;
  HIP_OK(hipGetDevice(&dev));
  DNNF_CHECK(dev >= 0 && dev < kMaxDevices, DNNF_INVALID_ARG, "device ordinal beyond the static workspace table");
  std::lock_guard<std::mutex> lk(g_static_mu);
  StaticSlot& slot = g_static[dev];
  if (!slot.ptr) {
    void* p = nullptr;
    HIP_OK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    DNNF_CHECK(p, DNNF_HIP_ERROR, "hipGetSymbolAddress returned no address for the static workspace");
    slot.ptr = p;
  }
  // loading a code object allocates: it must have happened before (dnnf_plan_prepare does it)
  for (auto& pb : blocks) {
    DNNF_CHECK(pb.low.family >= 0, DNNF_UNSUPPORTED_OP, "block has no kernel (plan was built for analysis only): " + pb.low.variant);
    for (size_t li = 0; li < pb.low.launches.size(); li++)
      DNNF_CHECK(pb.fn.size() > li && pb.fn[li], DNNF_NOT_FINALIZED,
                 "the plan's kernels are not resident: call dnnf_plan_prepare once (a null workspace is enough) before dnnf_plan_run_static");
  }
  if (slot.owner != serial) {
    // another plan (or nobody) used the array last: its contents are that plan's.  Compiler-made constants and the
    // results of the weight-only blocks are put back; everything else is written by this run before it is read.
    slot.owner = 0;
    for (int t : const_pool) {
      std::vector<char> host = const_bytes(g.tensors[t]);
      for (size_t off = 0; off < host.size(); off += sizeof(UploadChunk)) {
        UploadChunk c;
        const size_t n = std::min(sizeof(UploadChunk), host.size() - off);
        memcpy(c.b, host.data() + off, n);
        hipLaunchKernelGGL(dnnf_upload_chunk, dim3(4), dim3(256), 0, (hipStream_t)stream,
                           (unsigned char*)slot.ptr + ws_offset[t] + off, c, (int)n);
        HIP_OK(hipGetLastError());
      }
    }
    for (size_t b = 0; b < blocks.size(); b++)
      if (blocks[b].blk.weight_only) launch_block(b, nullptr, nullptr, slot.ptr, stream);
    slot.owner = serial;
  }
  for (size_t b = 0; b < blocks.size(); b++)
    if (!blocks[b].blk.weight_only) launch_block(b, in, out, slot.ptr, stream);
}

// Optional graph replay of the run loop (plan option graphs).  The first run with a set of buffers launches
// kernel by kernel (and loads the code objects); when the same set comes again the loop is captured on a
// stream of the plan's own and from then on launched as one graph into the caller's stream.  Measured on
// MI355X: empty kernels follow each other every 1.7 us in a graph against 2.9 us from a stream, but the
// benchmark graphs gain nothing - their launches are issued ahead of the running kernel either way - and
// a one-kernel plan pays the graph's own launch cost, so the option is off by default.
void Plan::run(const void* const* in, void* const* out, void* ws, void* stream) {
  auto plain = [&](void* s) {
    for (size_t b = 0; b < blocks.size(); b++)
      if (!blocks[b].blk.weight_only) launch_block(b, in, out, ws, s);
  };
  if (!use_graphs) { plain(stream); return; }
  std::vector<const void*> key;
  for (size_t i = 0; i < g.inputs.size(); i++) key.push_back(in ? in[i] : nullptr);
  for (size_t i = 0; i < g.outputs.size(); i++) key.push_back(out ? out[i] : nullptr);
  key.push_back(ws);
  RunGraph* rg = nullptr;
  for (auto& e : impl->graphs) if (e.key == key) rg = &e;
  if (rg && rg->exec) { HIP_OK(hipGraphLaunch(rg->exec, (hipStream_t)stream)); return; }
  if (!rg) {
    if (impl->graphs.size() >= 16) {       // callers that never repeat a buffer set gain nothing: stop trying
      use_graphs = false;
    } else {
      RunGraph e;
      e.key = key;
      impl->graphs.push_back(e);
    }
    plain(stream);
    return;
  }
  // second sight of this buffer set: capture (every code object is loaded by now, so nothing but launches happens)
  bool ok = true;
  if (!impl->capture_stream) ok = hipStreamCreateWithFlags(&impl->capture_stream, hipStreamNonBlocking) == hipSuccess;
  if (ok) ok = hipStreamBeginCapture(impl->capture_stream, hipStreamCaptureModeThreadLocal) == hipSuccess;
  if (ok) {
    try {
      plain(impl->capture_stream);
    } catch (const Error&) {
      ok = false;
    }
    hipGraph_t gr = nullptr;
    if (hipStreamEndCapture(impl->capture_stream, &gr) != hipSuccess) ok = false;
    if (ok && hipGraphInstantiate(&rg->exec, gr, nullptr, nullptr, 0) != hipSuccess) { ok = false; rg->exec = nullptr; }
    if (ok) rg->graph = gr;
    else if (gr) (void)hipGraphDestroy(gr);
  }
  if (!ok) {
    (void)hipGetLastError();
    use_graphs = false;                    // this runtime cannot capture the loop: plain launches from now on
    plain(stream);
    return;
  }
  HIP_OK(hipGraphLaunch(rg->exec, (hipStream_t)stream));
}

double Plan::time_block(size_t b, const void* const* in, void* const* out, void* ws, void* stream, int warmup, int iters) {
  hipEvent_t e0, e1;
  HIP_OK(hipEventCreate(&e0));
  HIP_OK(hipEventCreate(&e1));
  for (int i = 0; i < warmup; i++) launch_block(b, in, out, ws, stream);
  HIP_OK(hipEventRecord(e0, (hipStream_t)stream));
  for (int i = 0; i < iters; i++) launch_block(b, in, out, ws, stream);
  HIP_OK(hipEventRecord(e1, (hipStream_t)stream));
  HIP_OK(hipEventSynchronize(e1));
  float ms = 0;
  HIP_OK(hipEventElapsedTime(&ms, e0, e1));
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  return (double)ms * 1000.0 / std::max(iters, 1);
}

// ------------------------------------------------------------------ build
Plan* build_plan(const Graph& g, const dnnf_plan_opts& po, const void* const* weight_ptrs, void* stream) {
  DNNF_CHECK(g.finalized, DNNF_NOT_FINALIZED, "graph is not finalized");
  std::unique_ptr<Plan> P(new Plan);
  P->g = g;
  P->verbose = po.verbose != 0;
  if (po.cache_dir) P->cache_dir = po.cache_dir;
  for (size_t i = 0; i < g.weights.size(); i++) P->weight_ptrs.push_back(weight_ptrs ? weight_ptrs[i] : nullptr);

  // Operators whose results nobody reads (a graph handed over without rewriting keeps them) take no part in the
  // plan: a block made of them would have no output to store.
  for (bool again = true; again;) {
    again = false;
    for (auto& op : P->g.ops) {
      if (!op.alive) continue;
      bool used = false;
      for (int o : op.out) used = used || !P->g.tensors[o].consumers.empty() || P->g.tensors[o].kind == DNNF_OUTPUT;
      if (!used) { op.alive = false; again = true; }
    }
    if (again) P->g.relink();
  }
  P->g.finalized = true;

  if (po.layout) P->relaid_tensors = select_layouts(P->g);

  PlannerOpts o;
  o.fusion = po.fusion != 0;
  o.intra_block = po.intra_block != 0;
  o.successors_first = po.successors_first != 0;
  o.check_lowerable = po.check_lowerable != 0;
  o.attention = po.attention != 0;
  o.broadcast_prologue = po.broadcast_prologue != 0;
  o.gemm_norm = po.gemm_norm;
  o.squeeze_excite = po.squeeze_excite;
  if (po.max_block_ops > 0) o.max_block_ops = po.max_block_ops;
  if (po.max_block_operands > 0) o.max_block_operands = po.max_block_operands;
  std::vector<std::string> log;
  o.log = &log;
  LowerOpts lo;
  lo.intra_block = o.intra_block;
  P->lower_opts = lo;
  P->tune = po.tune != 0;
  P->use_graphs = po.graphs != 0;

  // Step 2.3 of Listing 1: run the candidate on the device.  Operands live in the caller's
  // scratch area (zero-filled, so index tensors are valid); results are memoised by kernel.
  // The paper keeps such measurements in a profiling result database so that a combination is timed
  // once per device (Sec. 4.3): with a cache directory the memo is read from / written back to
  // <cache_dir>/profile_db_<device>.tsv (kernel names are hashes of the generated source, so an entry
  // can never describe different code).
  std::map<std::string, double> memo;
  std::string db_path;
  size_t db_loaded = 0;
  int timed = 0, db_hits = 0;
  bool as_in_network = false;       // set around the tile tuning of GEMM / convolution blocks
  std::function<double(const Lowered&)> time_lowered;
  Plan* raw = P.get();
  if (po.profile && po.fusion && po.profile_scratch && po.profile_scratch_bytes > 0) {
    if (!P->cache_dir.empty()) {
      int dev = 0;
      hipDeviceProp_t prop;
      HIP_OK(hipGetDevice(&dev));
      HIP_OK(hipGetDeviceProperties(&prop, dev));
      std::string tag = prop.gcnArchName;
      for (char& ch : tag) if (!isalnum((unsigned char)ch)) ch = '_';
      db_path = P->cache_dir + "/profile_db_" + tag + "_cu" + std::to_string(prop.multiProcessorCount) + ".tsv";
      std::ifstream in(db_path);
      std::string key;
      double us;
      while (in >> key >> us) memo[key] = us;
      db_loaded = memo.size();
    }
    HIP_OK(hipMemsetAsync(po.profile_scratch, 0, po.profile_scratch_bytes, (hipStream_t)stream));
    time_lowered = [&, raw](const Lowered& low) -> double {
      if (low.family == FAM_ALIAS) return 0.0;
      std::string key;
      for (auto& L : low.launches) key += L.name + ";";
      if (as_in_network) key += "net;";
      auto it = memo.find(key);
      if (it != memo.end()) { db_hits++; return it->second; }
      timed++;
      size_t off = 0;
      double total = 0;
      hipEvent_t e0, e1;
      HIP_OK(hipEventCreate(&e0));
      HIP_OK(hipEventCreate(&e1));
      // the block's scratch area first, shared by its launches
      void* scratch_ptr = po.profile_scratch;
      off = align_up((size_t)low.scratch_bytes, 256);
      for (auto& L : low.launches) {
        void* ptrs[33];
        void* args[33];
        bool fits = L.params.size() <= 32 && off <= po.profile_scratch_bytes;
        for (size_t k = 0; fits && k < L.params.size(); k++) {
          size_t bytes = (size_t)std::max<int64_t>(raw->g.tensors[L.params[k]].bytes(), 1);
          if (off + bytes > po.profile_scratch_bytes) { fits = false; break; }
          ptrs[k] = (char*)po.profile_scratch + off;
          args[k] = &ptrs[k];
          // an index operand (Gather) must hold valid indices: the area was cleared once, but results of candidates
          // timed earlier have been written over it since
          if (!is_float(raw->g.tensors[L.params[k]].dtype)) HIP_OK(hipMemsetAsync(ptrs[k], 0, bytes, (hipStream_t)stream));
          else if (k < low.ext_in.size() && low.launches.size() == 1 && bytes >= 4)      // (operands are 256-byte aligned in the area)
            hipLaunchKernelGGL(dnnf_fill_profile_values, dim3((unsigned)std::min<size_t>(2048, (bytes / 4 + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                               (unsigned int*)ptrs[k], bytes / 4);
          off = align_up(off + bytes, 256);
        }
        if (!fits) { total = -1; break; }
        if (L.scratch) { ptrs[L.params.size()] = scratch_ptr; args[L.params.size()] = &ptrs[L.params.size()]; }
        hipFunction_t fn = (hipFunction_t)raw->function_for(L);
        auto go = [&] {
          HIP_OK(hipModuleLaunchKernel(fn, L.grid[0], L.grid[1], L.grid[2], L.block[0], L.block[1], L.block[2],
                                       L.lds_bytes, (hipStream_t)stream, args, nullptr));
        };
        const int iters = 10;
        // the rest of the profile area serves to push everything out of the caches (the memory-side one is 256 MB)
        const size_t spare = po.profile_scratch_bytes > off ? (po.profile_scratch_bytes - off) / 4 * 4 : 0;
        if (as_in_network && low.launches.size() == 1 && spare >= ((size_t)320 << 20)) {
          // As inside a network: the weights were last read a whole inference ago and come from memory, the activations
          // have just been written by the kernel in front.  In a loop over itself a kernel finds all of its operands in
          // the caches, and the tiles that win that way (operand tiles straight into LDS, one tile ahead) are not the
          // ones that win behind cold weights.
          const size_t thrash = std::min(spare, (size_t)640 << 20);
          go();
          double us = 0;
          for (int i = 0; i < iters; i++) {
            hipLaunchKernelGGL(dnnf_fill_profile_values, dim3(4096), dim3(256), 0, (hipStream_t)stream,
                               (unsigned int*)((char*)po.profile_scratch + off), thrash / 4);
            for (size_t k = 0; k < L.params.size() && k < low.ext_in.size(); k++) {
              const Tensor& T = raw->g.tensors[L.params[k]];
              const size_t bytes = (size_t)std::max<int64_t>(T.bytes(), 1);
              if (is_float(T.dtype) && T.kind != DNNF_WEIGHT && !T.weight_only && bytes >= 4)
                hipLaunchKernelGGL(dnnf_fill_profile_values, dim3((unsigned)std::min<size_t>(2048, (bytes / 4 + 255) / 256)), dim3(256), 0,
                                   (hipStream_t)stream, (unsigned int*)ptrs[k], bytes / 4);
            }
            HIP_OK(hipEventRecord(e0, (hipStream_t)stream));
            go();
            HIP_OK(hipEventRecord(e1, (hipStream_t)stream));
            HIP_OK(hipEventSynchronize(e1));
            float ms = 0;
            HIP_OK(hipEventElapsedTime(&ms, e0, e1));
            us += (double)ms * 1000.0;
          }
          total += us / iters;
        } else {
          for (int i = 0; i < 3; i++) go();
          HIP_OK(hipEventRecord(e0, (hipStream_t)stream));
          for (int i = 0; i < iters; i++) go();
          HIP_OK(hipEventRecord(e1, (hipStream_t)stream));
          HIP_OK(hipEventSynchronize(e1));
          float ms = 0;
          HIP_OK(hipEventElapsedTime(&ms, e0, e1));
          total += (double)ms * 1000.0 / iters;
        }
      }
      (void)hipEventDestroy(e0);
      (void)hipEventDestroy(e1);
      if (total < 0) total = 0;   // did not fit the scratch area: no evidence either way
      memo[key] = total;
      return total;
    };
    o.latency = [&](const Block& b) -> double { return time_lowered(lower_block(raw->g, b, lo)); };
  }

  std::vector<Block> blocks = build_fusion_plan(P->g, o, &P->stats);
  for (auto& b : blocks) {
    PlanBlock pb;
    pb.blk = b;
    try {
      pb.low = lower_block(P->g, b, lo);
      if (P->tune && time_lowered) {
        // the fastest tile configuration on this device (timings are memoised per kernel, so repeated
        // layers are measured once)
        std::vector<Lowered> variants = tile_variants(P->g, b, pb.low, lo);
        as_in_network = !variants.empty() && (pb.low.family == FAM_GEMM || pb.low.family == FAM_CONV);
        double best = time_lowered(pb.low);
        std::string tl = "tune: " + pb.low.variant + " " + std::to_string(best);
        for (Lowered& v : variants) {
          double t = time_lowered(v);
          tl += ", " + v.variant + " " + std::to_string(t);
          if (t > 0 && t < best) { best = t; pb.low = v; }
        }
        as_in_network = false;
        if (pb.low.family == FAM_GEMM || pb.low.family == FAM_CONV || (pb.low.family == FAM_DWCONV && tl.find(", ") != std::string::npos)) log.push_back(tl + " us");
      }
    } catch (const Error& e) {
      if (o.check_lowerable) throw;
      pb.low = Lowered();          // analysis-only plan: the block is reported but cannot run
      pb.low.family = -1;
      pb.low.variant = std::string("no kernel template: ") + e.what();
    }
    P->blocks.push_back(pb);
  }
  // a tensor can be kept inside one stacking Concat only (and not if a lone Reshape already shares its storage out):
  // later claims fall back to copy kernels
  {
    std::set<int> claimed;
    for (auto& pb : P->blocks) if (pb.low.family == FAM_ALIAS && pb.low.alias_parts.empty()) { claimed.insert(pb.low.alias_dst); claimed.insert(pb.low.alias_src); }
    for (auto& pb : P->blocks) {
      if (pb.low.family != FAM_ALIAS || pb.low.alias_parts.empty()) continue;
      bool clash = claimed.count(pb.low.alias_dst) != 0;
      for (auto& pr : pb.low.alias_parts) clash = clash || claimed.count(pr.first);
      if (clash) {
        LowerOpts l2 = lo;
        l2.alias_concat = false;
        pb.low = lower_block(P->g, pb.blk, l2);
      } else {
        for (auto& pr : pb.low.alias_parts) claimed.insert(pr.first);
        claimed.insert(pb.low.alias_dst);
      }
    }
  }
  P->log = log;
  if (P->verbose) {
    for (auto& l : log) fprintf(stderr, "[dnnf plan] %s\n", l.c_str());
    for (auto& pb : P->blocks)
      fprintf(stderr, "[dnnf plan] block: %zu ops, family %d, %s\n", pb.blk.ops.size(), pb.low.family, pb.low.variant.c_str());
  }
  P->stats.timed = timed;
  P->stats.db_hits = db_hits;
  if (!db_path.empty() && memo.size() > db_loaded) {
    // rewritten as a whole through a temporary file, so a concurrent reader never sees half a line
    std::string tmp = db_path + ".tmp" + std::to_string((long)getpid());
    {
      std::ofstream out(tmp);
      out.precision(6);
      for (auto& kv : memo) out << kv.first << "\t" << std::fixed << kv.second << "\n";
    }
    if (rename(tmp.c_str(), db_path.c_str()) != 0) (void)remove(tmp.c_str());
  }
  P->layout_workspace();
  return P.release();
}

}  // namespace dnnf
