// extern "C" boundary: argument checking and exception-to-status translation only.
#include <cstring>
#include <set>
#include <string>

#include "plan.hpp"

using namespace dnnf;

struct dnnf_graph {
  Graph g;
};
struct dnnf_plan {
  Plan* p = nullptr;
};

static thread_local std::string g_last_error;

template <class F>
static dnnf_status guard(F&& f) {
  try {
    f();
    return DNNF_OK;
  } catch (const Error& e) {
    g_last_error = e.what();
    return e.code;
  } catch (const std::bad_alloc&) {
    g_last_error = "out of host memory";
    return DNNF_OUT_OF_MEMORY;
  } catch (const std::exception& e) {
    g_last_error = e.what();
    return DNNF_INVALID_ARG;
  } catch (...) {
    g_last_error = "unknown failure";
    return DNNF_INVALID_ARG;
  }
}
#define REQUIRE(c, msg) DNNF_CHECK((c), DNNF_INVALID_ARG, msg)

extern "C" {

const char* dnnf_last_error(void) { return g_last_error.c_str(); }

dnnf_status dnnf_graph_create(dnnf_graph** g) {
  return guard([&] {
    REQUIRE(g, "null out-pointer");
    *g = new dnnf_graph;
  });
}
void dnnf_graph_destroy(dnnf_graph* g) { delete g; }

dnnf_status dnnf_graph_add_tensor(dnnf_graph* g, const char* name, dnnf_dtype dtype, int rank, const int64_t* dims,
                                  dnnf_tensor_kind kind, int* tensor_id) {
  return guard([&] {
    REQUIRE(g && name && tensor_id && rank >= 0 && rank <= 8 && (rank == 0 || dims), "bad argument to dnnf_graph_add_tensor");
    REQUIRE(dtype >= DNNF_F32 && dtype <= DNNF_BOOL && kind >= DNNF_INPUT && kind <= DNNF_OUTPUT, "bad dtype or kind");
    *tensor_id = g->g.add_tensor(name, dtype, Dims(dims, dims + rank), kind);
  });
}

dnnf_status dnnf_graph_set_const(dnnf_graph* g, int t, const double* values, int64_t count) {
  return guard([&] {
    REQUIRE(g && values && t >= 0 && t < (int)g->g.tensors.size(), "bad argument to dnnf_graph_set_const");
    Tensor& T = g->g.tensors[t];
    REQUIRE(T.kind == DNNF_WEIGHT, "constants must be WEIGHT tensors");
    DNNF_CHECK(count == T.n(), DNNF_SHAPE_MISMATCH, "constant element count differs from the tensor's");
    T.cval.assign(values, values + count);
    T.has_cval = true;
  });
}

dnnf_status dnnf_graph_add_op(dnnf_graph* g, const char* kind, int n_in, const int* in_ids, int n_out, const int* out_ids,
                              const dnnf_attr* attrs, int n_attrs, int* op_id) {
  return guard([&] {
    REQUIRE(g && kind && n_in >= 0 && n_out >= 1 && (n_in == 0 || in_ids) && out_ids && n_attrs >= 0 && (n_attrs == 0 || attrs),
            "bad argument to dnnf_graph_add_op");
    Attrs a;
    for (int i = 0; i < n_attrs; i++) {
      REQUIRE(attrs[i].name && attrs[i].n >= 0 && (attrs[i].n == 0 || attrs[i].values), "bad attribute");
      a[attrs[i].name] = std::vector<double>(attrs[i].values, attrs[i].values + attrs[i].n);
    }
    int id = g->g.add_op(kind, std::vector<int>(in_ids, in_ids + n_in), std::vector<int>(out_ids, out_ids + n_out), a);
    if (op_id) *op_id = id;
  });
}

dnnf_status dnnf_graph_finalize(dnnf_graph* g) {
  return guard([&] {
    REQUIRE(g, "null graph");
    g->g.finalize();
  });
}

dnnf_status dnnf_graph_num_ops(const dnnf_graph* g, int* n) {
  return guard([&] {
    REQUIRE(g && n, "null argument");
    *n = g->g.live_ops();
  });
}
dnnf_status dnnf_graph_num_op_slots(const dnnf_graph* g, int* n) {
  return guard([&] {
    REQUIRE(g && n, "null argument");
    *n = (int)g->g.ops.size();
  });
}

dnnf_status dnnf_graph_op_info(const dnnf_graph* g, int op_id, char* kind_buf, int cap, int* alive, int* mapping_type) {
  return guard([&] {
    REQUIRE(g && op_id >= 0 && op_id < (int)g->g.ops.size(), "bad operator id");
    const Op& op = g->g.ops[op_id];
    if (kind_buf && cap > 0) {
      strncpy(kind_buf, op.kind.c_str(), (size_t)cap - 1);
      kind_buf[cap - 1] = 0;
    }
    if (alive) *alive = op.alive;
    if (mapping_type) *mapping_type = op.mapping;
  });
}

dnnf_status dnnf_plan_op_kind(const dnnf_plan* p, int op_id, char* kind_buf, int cap) {
  return guard([&] {
    REQUIRE(p && kind_buf && cap > 0 && op_id >= 0 && op_id < (int)p->p->g.ops.size(), "bad operator id");
    strncpy(kind_buf, p->p->g.ops[op_id].kind.c_str(), (size_t)cap - 1);
    kind_buf[cap - 1] = 0;
  });
}

dnnf_status dnnf_op_mapping_type(const dnnf_graph* g, int op_id, int* type) {
  return guard([&] {
    REQUIRE(g && type && op_id >= 0 && op_id < (int)g->g.ops.size(), "bad operator id");
    DNNF_CHECK(g->g.finalized, DNNF_NOT_FINALIZED, "graph is not finalized");
    *type = g->g.ops[op_id].mapping;
  });
}

dnnf_status dnnf_op_kind_mapping_type(const char* kind, int* type) {
  return guard([&] {
    REQUIRE(kind && type, "null argument");
    const OpKindInfo* k = find_op_kind(kind);
    DNNF_CHECK(k, DNNF_UNSUPPORTED_OP, std::string("unknown operator kind ") + kind);
    *type = k->mapping;
  });
}

dnnf_status dnnf_fuse_relation(int first, int second, int* fused, int* colour) {
  return guard([&] {
    REQUIRE(fused && colour && first >= 0 && first <= 4 && second >= 0 && second <= 4, "bad mapping type");
    fuse_relation(first, second, fused, colour);
  });
}

dnnf_status dnnf_graph_rewrite(dnnf_graph* g, dnnf_rewrite_stats* stats) {
  return guard([&] {
    REQUIRE(g, "null graph");
    DNNF_CHECK(g->g.finalized, DNNF_NOT_FINALIZED, "graph is not finalized");
    RewriteStats st;
    rewrite_graph(g->g, st);
    if (stats) {
      stats->rules_fired = st.rules_fired;
      stats->canonicalisations = st.canonicalisations;
      stats->flops_before = st.flops_before;
      stats->flops_after = st.flops_after;
      stats->ops_before = st.ops_before;
      stats->ops_after = st.ops_after;
      stats->derived_rules_fired = st.derived_rules_fired;
    }
  });
}

dnnf_status dnnf_graph_dump_json(const dnnf_graph* g, char* buf, size_t cap, size_t* needed) {
  return guard([&] {
    REQUIRE(g, "null graph");
    static const char* dts[] = {"f32", "f16", "bf16", "i32", "i64", "bool"};
    static const char* kinds[] = {"input", "weight", "intermediate", "output"};
    std::string s = "{\"tensors\":[";
    char num[64];
    bool first = true;
    std::set<int> used;
    for (auto& op : g->g.ops)
      if (op.alive) { used.insert(op.in.begin(), op.in.end()); used.insert(op.out.begin(), op.out.end()); }
    for (size_t t = 0; t < g->g.tensors.size(); t++) {
      const Tensor& T = g->g.tensors[t];
      if (!used.count((int)t) && T.kind == DNNF_INTERMEDIATE) continue;
      s += first ? "" : ",";
      first = false;
      s += "{\"id\":" + std::to_string(t) + ",\"name\":\"" + T.name + "\",\"dtype\":\"" + dts[T.dtype] + "\",\"kind\":\"" +
           kinds[T.kind] + "\",\"origin\":\"" + T.origin + "\",\"ext\":" + std::to_string(T.ext_index) + ",\"shape\":[";
      for (size_t d = 0; d < T.dims.size(); d++) s += (d ? "," : "") + std::to_string(T.dims[d]);
      s += "]";
      if (T.has_cval) {
        s += ",\"const\":[";
        for (size_t i = 0; i < T.cval.size(); i++) {
          snprintf(num, sizeof num, "%.17g", T.cval[i]);
          s += (i ? "," : "") + std::string(num);
        }
        s += "]";
      }
      s += "}";
    }
    s += "],\"ops\":[";
    first = true;
    for (int oi : g->g.topo) {
      const Op& op = g->g.ops[oi];
      s += first ? "" : ",";
      first = false;
      s += "{\"id\":" + std::to_string(oi) + ",\"kind\":\"" + op.kind + "\",\"mapping\":" + std::to_string(op.mapping) + ",\"flops\":";
      snprintf(num, sizeof num, "%.17g", op.flops);
      s += num;
      s += ",\"in\":[";
      for (size_t k = 0; k < op.in.size(); k++) s += (k ? "," : "") + std::to_string(op.in[k]);
      s += "],\"out\":[";
      for (size_t k = 0; k < op.out.size(); k++) s += (k ? "," : "") + std::to_string(op.out[k]);
      s += "],\"attrs\":{";
      bool fa = true;
      for (auto& kv : op.attrs) {
        s += fa ? "" : ",";
        fa = false;
        s += "\"" + kv.first + "\":[";
        for (size_t i = 0; i < kv.second.size(); i++) {
          snprintf(num, sizeof num, "%.17g", kv.second[i]);
          s += (i ? "," : "") + std::string(num);
        }
        s += "]";
      }
      s += "}}";
    }
    s += "]}";
    if (needed) *needed = s.size() + 1;
    if (buf && cap > 0) {
      strncpy(buf, s.c_str(), cap - 1);
      buf[cap - 1] = 0;
    }
  });
}

void dnnf_plan_default_opts(dnnf_plan_opts* o) {
  if (!o) return;
  memset(o, 0, sizeof *o);
  o->fusion = 1;
  o->profile = 1;
  o->intra_block = 1;
  o->max_block_ops = 64;
  o->max_block_operands = 16;
  o->check_lowerable = 1;
  o->tune = 0;
  o->attention = 0;
  o->layout = 0;
  o->graphs = 0;
  o->broadcast_prologue = 0;
  o->gemm_norm = 0;
  o->squeeze_excite = 0;
}

dnnf_status dnnf_plan_build(const dnnf_graph* g, const dnnf_plan_opts* opts, const void* const* weight_dev_ptrs, void* stream,
                            dnnf_plan** plan) {
  return guard([&] {
    REQUIRE(g && plan, "null argument");
    dnnf_plan_opts o;
    if (opts) o = *opts; else dnnf_plan_default_opts(&o);
    REQUIRE(g->g.weights.empty() || weight_dev_ptrs, "weight pointer array is null");
    Plan* p = build_plan(g->g, o, weight_dev_ptrs, stream);
    *plan = new dnnf_plan;
    (*plan)->p = p;
  });
}

void dnnf_plan_destroy(dnnf_plan* p) {
  if (!p) return;
  delete p->p;
  delete p;
}

dnnf_status dnnf_plan_num_blocks(const dnnf_plan* p, int* n) {
  return guard([&] {
    REQUIRE(p && n, "null argument");
    *n = (int)p->p->blocks.size();
  });
}

dnnf_status dnnf_plan_block_info(const dnnf_plan* p, int b, dnnf_block_info* info) {
  return guard([&] {
    REQUIRE(p && info && b >= 0 && b < (int)p->p->blocks.size(), "bad block index");
    const PlanBlock& pb = p->p->blocks[b];
    memset(info, 0, sizeof *info);
    info->n_ops = (int)pb.blk.ops.size();
    info->fused_type = pb.blk.fused_type;
    info->family = pb.low.family;
    info->bytes = pb.low.bytes;
    info->flops = pb.low.flops;
    info->irs_bytes_removed = pb.low.irs_removed;
    info->n_kernel_launches = (int)pb.low.launches.size();
    std::string nm = pb.low.launches.empty() ? pb.low.variant : pb.low.launches[0].name + ":" + pb.low.variant;
    strncpy(info->kernel_name, nm.c_str(), sizeof info->kernel_name - 1);
    if (pb.blk.weight_only) info->n_kernel_launches = -info->n_kernel_launches;  // negative: runs at prepare time only
  });
}

dnnf_status dnnf_plan_block_ops(const dnnf_plan* p, int b, int* op_ids, int cap, int* n) {
  return guard([&] {
    REQUIRE(p && n && b >= 0 && b < (int)p->p->blocks.size(), "bad block index");
    const auto& ops = p->p->blocks[b].blk.ops;
    *n = (int)ops.size();
    for (int i = 0; i < cap && i < (int)ops.size() && op_ids; i++) op_ids[i] = ops[i];
  });
}

dnnf_status dnnf_plan_block_source(const dnnf_plan* p, int b, char* buf, size_t cap, size_t* needed) {
  return guard([&] {
    REQUIRE(p && b >= 0 && b < (int)p->p->blocks.size(), "bad block index");
    std::string s;
    for (auto& L : p->p->blocks[b].low.launches) s += L.source + "\n";
    if (needed) *needed = s.size() + 1;
    if (buf && cap > 0) {
      strncpy(buf, s.c_str(), cap - 1);
      buf[cap - 1] = 0;
    }
  });
}

dnnf_status dnnf_plan_dump_json(const dnnf_plan* p, char* buf, size_t cap, size_t* needed) {
  return guard([&] {
    REQUIRE(p, "null plan");
    const Plan& P = *p->p;
    static const char* dts[] = {"f32", "f16", "bf16", "i32", "i64", "bool"};
    static const char* kinds[] = {"input", "weight", "intermediate", "output"};
    auto tensor = [&](int t) {
      int root = t;
      int64_t within = 0;
      while (P.alias_of[root] >= 0) { within += P.alias_off[root]; root = P.alias_of[root]; }
      const Tensor& T = P.g.tensors[t];
      const Tensor& R = P.g.tensors[root];
      std::string s = "{\"id\":" + std::to_string(t) + ",\"name\":\"" + T.name + "\",\"origin\":\"" + T.origin + "\",\"dtype\":\"" +
                      dts[T.dtype] + "\",\"kind\":\"" + kinds[R.kind] + "\",\"ext\":" + std::to_string(R.ext_index) +
                      ",\"ws_offset\":" + std::to_string(P.ws_offset[root]) + ",\"alias_offset\":" + std::to_string(within) + ",\"shape\":[";
      for (size_t d = 0; d < T.dims.size(); d++) s += (d ? "," : "") + std::to_string(T.dims[d]);
      s += "],\"perm\":[";                      // storage order chosen by data-format selection (empty: as declared)
      for (size_t d = 0; d < T.perm.size(); d++) s += (d ? "," : "") + std::to_string(T.perm[d]);
      return s + "]}";
    };
    std::string s = "{\"workspace_bytes\":" + std::to_string(P.ws_bytes) + ",\"blocks\":[";
    for (size_t b = 0; b < P.blocks.size(); b++) {
      const PlanBlock& pb = P.blocks[b];
      s += b ? "," : "";
      s += "{\"family\":" + std::to_string(pb.low.family) + ",\"prepare_only\":" + (pb.blk.weight_only ? "true" : "false") +
           ",\"variant\":\"" + pb.low.variant + "\",\"ops\":[";
      for (size_t i = 0; i < pb.blk.ops.size(); i++) s += (i ? "," : "") + std::to_string(pb.blk.ops[i]);
      s += "],\"inputs\":[";
      for (size_t i = 0; i < pb.low.ext_in.size(); i++) s += (i ? "," : "") + tensor(pb.low.ext_in[i]);
      s += "],\"outputs\":[";
      for (size_t i = 0; i < pb.low.ext_out.size(); i++) s += (i ? "," : "") + tensor(pb.low.ext_out[i]);
      // the block's kernel launches: name, grid, workgroup, and the tensors behind the pointer parameters in order
      s += "],\"launches\":[";
      for (size_t i = 0; i < pb.low.launches.size(); i++) {
        const Launch& L = pb.low.launches[i];
        s += std::string(i ? "," : "") + "{\"name\":\"" + L.name + "\",\"grid\":[" + std::to_string(L.grid[0]) + "," + std::to_string(L.grid[1]) + "," +
             std::to_string(L.grid[2]) + "],\"block\":[" + std::to_string(L.block[0]) + "," + std::to_string(L.block[1]) + "," + std::to_string(L.block[2]) +
             "],\"scratch\":" + (L.scratch ? "true" : "false") + ",\"params\":[";
        for (size_t k = 0; k < L.params.size(); k++) s += (k ? "," : "") + tensor(L.params[k]);
        s += "]}";
      }
      s += "]}";
    }
    s += "],\"log\":[";
    for (size_t i = 0; i < P.log.size(); i++) {
      std::string l = P.log[i];
      for (auto& ch : l) if (ch == '"' || ch == '\\') ch = '\'';
      s += (i ? ",\"" : "\"") + l + "\"";
    }
    s += "],\"stats\":{\"seeds\":" + std::to_string(P.stats.seeds) + ",\"green\":" + std::to_string(P.stats.green) +
         ",\"yellow_fused\":" + std::to_string(P.stats.yellow_fused) + ",\"yellow_rejected\":" + std::to_string(P.stats.yellow_rejected) +
         ",\"red\":" + std::to_string(P.stats.red) + ",\"constraint_rejected\":" + std::to_string(P.stats.constraint_rejected) +
         ",\"profiled\":" + std::to_string(P.stats.profiled) + ",\"timed_on_device\":" + std::to_string(P.stats.timed) +
         ",\"answered_by_database\":" + std::to_string(P.stats.db_hits) + ",\"relaid_tensors\":" + std::to_string(P.relaid_tensors) + "}}";
    if (needed) *needed = s.size() + 1;
    if (buf && cap > 0) {
      strncpy(buf, s.c_str(), cap - 1);
      buf[cap - 1] = 0;
    }
  });
}

dnnf_status dnnf_plan_precompile(dnnf_plan* p) {
  return guard([&] {
    REQUIRE(p, "null plan");
    for (auto& pb : p->p->blocks) {
      precompile(pb.low, p->p->cache_dir);
      if (p->p->tune)
        for (const Lowered& v : tile_variants(p->p->g, pb.blk, pb.low, p->p->lower_opts)) precompile(v, p->p->cache_dir);
    }
  });
}

dnnf_status dnnf_plan_workspace_bytes(const dnnf_plan* p, size_t* bytes) {
  return guard([&] {
    REQUIRE(p && bytes, "null argument");
    *bytes = p->p->ws_bytes;
  });
}

dnnf_status dnnf_plan_prepare(dnnf_plan* p, void* ws, void* stream) {
  return guard([&] {
    REQUIRE(p, "null plan");
    p->p->prepare(ws, stream);
  });
}

dnnf_status dnnf_plan_run(dnnf_plan* p, const void* const* in, void* const* out, void* ws, void* stream) {
  return guard([&] {
    REQUIRE(p, "null plan");
    p->p->run(in, out, ws, stream);
  });
}

dnnf_status dnnf_plan_run_static(dnnf_plan* p, const void* const* in, void* const* out, void* stream) {
  return guard([&] {
    REQUIRE(p, "null plan");
    p->p->run_static(in, out, stream);
  });
}

dnnf_status dnnf_plan_run_block(dnnf_plan* p, int b, const void* const* in, void* const* out, void* ws, void* stream) {
  return guard([&] {
    REQUIRE(p && b >= 0 && b < (int)p->p->blocks.size(), "bad block index");
    p->p->launch_block((size_t)b, in, out, ws, stream);
  });
}

dnnf_status dnnf_plan_time_block(dnnf_plan* p, int b, const void* const* in, void* const* out, void* ws, void* stream,
                                 int warmup, int iters, double* usec) {
  return guard([&] {
    REQUIRE(p && usec && b >= 0 && b < (int)p->p->blocks.size() && iters > 0 && warmup >= 0, "bad argument");
    *usec = p->p->time_block((size_t)b, in, out, ws, stream, warmup, iters);
  });
}

}  // extern "C"
