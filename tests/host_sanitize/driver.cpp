// Host-side sanitizer driver: feeds graphs (text files written by tests/test_host_sanitizers.py) through the C ABI -
// build, finalize, rewrite, plan under several option sets, read every block's generated source and the JSON dumps -
// in a process whose library and driver are both built with AddressSanitizer and UndefinedBehaviorSanitizer.
// Nothing here touches a GPU: plans are built without profiling and never prepared or run.
//
// File format, one record per line:
//   T <name> <dtype> <kind> <rank> <d0> ...            tensor (enums as integers of include/dnnf.h)
//   C <tensor index> <count> <v0> ...                  host-readable constant values
//   O <kind> <n_in> <in...> <n_out> <out...> <n_attr> { <name> <n> <v...> }*
//   X <expected status of finalize>                    (default 0)
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <fstream>
#include <sstream>
#include <string>
#include <vector>

#include "dnnf.h"

static int fail(const std::string& what) {
  fprintf(stderr, "FAILED: %s: %s\n", what.c_str(), dnnf_last_error());
  return 1;
}

static int run_file(const char* path, bool precompile) {
  std::ifstream f(path);
  if (!f) { fprintf(stderr, "cannot open %s\n", path); return 1; }
  dnnf_graph* g = nullptr;
  if (dnnf_graph_create(&g) != DNNF_OK) return fail("graph_create");
  std::vector<int> ids;
  int n_weights = 0, expect_finalize = 0;
  std::string line;
  while (std::getline(f, line)) {
    std::istringstream s(line);
    std::string tag;
    s >> tag;
    if (tag == "T") {
      std::string name;
      int dtype, kind, rank;
      s >> name >> dtype >> kind >> rank;
      std::vector<int64_t> dims(rank > 0 ? rank : 1, 1);
      for (int i = 0; i < rank; i++) s >> dims[i];
      int id = -1;
      if (dnnf_graph_add_tensor(g, name.c_str(), (dnnf_dtype)dtype, rank, dims.data(), (dnnf_tensor_kind)kind, &id) != DNNF_OK) return fail("add_tensor " + name);
      ids.push_back(id);
      if (kind == DNNF_WEIGHT) n_weights++;
    } else if (tag == "C") {
      int t;
      long long n;
      s >> t >> n;
      std::vector<double> v((size_t)n);
      for (auto& x : v) s >> x;
      if (dnnf_graph_set_const(g, ids.at(t), v.data(), n) != DNNF_OK) return fail("set_const");
    } else if (tag == "O") {
      std::string kind;
      int n_in, n_out, n_attr;
      s >> kind >> n_in;
      std::vector<int> in(n_in > 0 ? n_in : 1), out;
      for (int i = 0; i < n_in; i++) { int t; s >> t; in[i] = ids.at(t); }
      s >> n_out;
      out.resize(n_out > 0 ? n_out : 1);
      for (int i = 0; i < n_out; i++) { int t; s >> t; out[i] = ids.at(t); }
      s >> n_attr;
      std::vector<std::string> names(n_attr);
      std::vector<std::vector<double>> vals(n_attr);
      for (int a = 0; a < n_attr; a++) {
        int n;
        s >> names[a] >> n;
        vals[a].resize(n);
        for (auto& x : vals[a]) s >> x;
      }
      std::vector<dnnf_attr> attrs(n_attr > 0 ? n_attr : 1);
      for (int a = 0; a < n_attr; a++) attrs[a] = dnnf_attr{names[a].c_str(), (int)vals[a].size(), vals[a].data()};
      int op = -1;
      if (dnnf_graph_add_op(g, kind.c_str(), n_in, in.data(), n_out, out.data(), attrs.data(), n_attr, &op) != DNNF_OK) return fail("add_op " + kind);
    } else if (tag == "X") {
      s >> expect_finalize;
    }
  }
  dnnf_status st = dnnf_graph_finalize(g);
  if ((int)st != expect_finalize) return fail("finalize returned " + std::to_string((int)st) + ", expected " + std::to_string(expect_finalize));
  if (st != DNNF_OK) {
    dnnf_graph_destroy(g);
    printf("ok %s (finalize refused as expected)\n", path);
    return 0;
  }
  dnnf_rewrite_stats rs;
  if (dnnf_graph_rewrite(g, &rs) != DNNF_OK) return fail("rewrite");
  size_t need = 0;
  if (dnnf_graph_dump_json(g, nullptr, 0, &need) != DNNF_OK) return fail("graph_dump_json (size query)");
  std::vector<char> buf(need + 1);
  if (dnnf_graph_dump_json(g, buf.data(), buf.size(), &need) != DNNF_OK) return fail("graph_dump_json");
  // weight pointers are never dereferenced while a plan is only built: any non-null value serves
  std::vector<const void*> w((size_t)(n_weights > 0 ? n_weights : 1), (const void*)0x1000);
  int total_blocks = 0;
  for (int variant = 0; variant < 8; variant++) {
    dnnf_plan_opts o;
    dnnf_plan_default_opts(&o);
    o.fusion = variant != 1;
    o.intra_block = variant != 2;
    o.attention = variant == 3;
    o.layout = variant == 4 || variant == 5 || variant == 7;
    o.broadcast_prologue = variant == 5;
    o.successors_first = variant == 2;
    o.gemm_norm = variant == 6 ? 2 : 0;
    o.squeeze_excite = variant == 7 ? 2 : 0;
    dnnf_plan* p = nullptr;
    if (dnnf_plan_build(g, &o, w.data(), nullptr, &p) != DNNF_OK) return fail("plan_build variant " + std::to_string(variant));
    int nb = 0;
    if (dnnf_plan_num_blocks(p, &nb) != DNNF_OK) return fail("num_blocks");
    total_blocks += nb;
    for (int b = 0; b < nb; b++) {
      dnnf_block_info bi;
      if (dnnf_plan_block_info(p, b, &bi) != DNNF_OK) return fail("block_info");
      int ops[256], n = 0;
      if (dnnf_plan_block_ops(p, b, ops, 256, &n) != DNNF_OK) return fail("block_ops");
      size_t sn = 0;
      dnnf_plan_block_source(p, b, nullptr, 0, &sn);
      std::vector<char> src(sn + 1);
      if (sn && dnnf_plan_block_source(p, b, src.data(), src.size(), &sn) != DNNF_OK) return fail("block_source");
    }
    size_t jn = 0;
    dnnf_plan_dump_json(p, nullptr, 0, &jn);
    std::vector<char> js(jn + 1);
    if (dnnf_plan_dump_json(p, js.data(), js.size(), &jn) != DNNF_OK) return fail("plan_dump_json");
    size_t ws = 0;
    if (dnnf_plan_workspace_bytes(p, &ws) != DNNF_OK) return fail("workspace_bytes");
    if (precompile && variant == 0 && dnnf_plan_precompile(p) != DNNF_OK) return fail("precompile");
    dnnf_plan_destroy(p);
  }
  dnnf_graph_destroy(g);
  printf("ok %s ops %d -> %d, %d blocks over 8 plans\n", path, rs.ops_before, rs.ops_after, total_blocks);
  return 0;
}

int main(int argc, char** argv) {
  bool precompile = false;
  int rc = 0;
  for (int i = 1; i < argc; i++) {
    if (!strcmp(argv[i], "--precompile")) { precompile = true; continue; }
    rc |= run_file(argv[i], precompile);
    fflush(stdout);
  }
  return rc;
}
