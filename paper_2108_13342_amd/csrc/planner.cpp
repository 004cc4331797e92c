// Fusion plan exploration (paper Sec. 4.3).
//
// The steps are those of Listing 1: pick the One-to-One operator with the smallest intermediate
// result as seed; grow the block along the seed's predecessors and successors, recursively; for
// each candidate consult the mapping-type table (red: stop, green: fuse, yellow: compare the
// measured latency of the fused kernel with that of the two separate kernels) and a constraint
// check.  Points the listing leaves open are read as follows:
//   - the first operand of the table lookup is the current block's fused type when the candidate
//     is a successor, and the candidate's type when it is a predecessor (Fig. 3 rejects the GEMM
//     because the whole block is already Many-to-One);
//   - predecessors are explored before successors (the text allows swapping steps II and III), so
//     a contraction picks up its elementwise epilogue before a following reduction can claim it;
//   - the constraint check bounds block size and operand count, refuses fusions that would make
//     two blocks depend on each other, refuses expensive One-to-One work in front of a contraction
//     (it would be recomputed once per output tile column), and requires a kernel template.
#include "planner.hpp"

#include <algorithm>
#include <set>

namespace dnnf {

namespace {

struct Planner {
  const Graph& g;
  const PlannerOpts& o;
  PlanStats st;
  std::vector<int> group;              // op -> block id, -1 while unfused
  std::vector<std::vector<int>> members;
  std::vector<int> topo_pos;
  std::vector<int> btype;
  std::set<int> sanctioned_prologue;   // broadcast multiplies the extension placed in front of a convolution

  Planner(const Graph& g_, const PlannerOpts& o_) : g(g_), o(o_) {
    group.assign(g.ops.size(), -1);
    topo_pos.assign(g.ops.size(), -1);
    for (size_t i = 0; i < g.topo.size(); i++) topo_pos[g.topo[i]] = (int)i;
  }

  void say(const std::string& s) { if (o.log) o.log->push_back(s); }

  std::vector<int> successors(int op) const {
    std::set<std::pair<int, int>> s;
    for (int t : g.ops[op].out) for (int c : g.tensors[t].consumers) s.insert({topo_pos[c], c});
    std::vector<int> r;
    for (auto& p : s) r.push_back(p.second);
    return r;
  }
  std::vector<int> predecessors(int op) const {
    std::set<std::pair<int, int>> s;
    for (int t : g.ops[op].in) {
      int p = g.tensors[t].producer;
      if (p >= 0) s.insert({topo_pos[p], p});
    }
    std::vector<int> r;
    for (auto& p : s) r.push_back(p.second);
    return r;
  }

  // contracted graph: formed blocks are single nodes, everything else is its own node
  int node_of(int op) const { return group[op] >= 0 ? group[op] : (int)members.size() + op; }
  std::vector<int> node_ops(int node) const {
    if (node < (int)members.size()) return members[node];
    return {node - (int)members.size()};
  }
  // Is `to` reachable from `from` through at least one node other than the two?
  bool reaches_via_others(int from, int to) const {
    std::set<int> seen;
    std::vector<int> stack;
    for (int op : node_ops(from))
      for (int s : successors(op)) {
        int n = node_of(s);
        if (n != from && n != to && !seen.count(n)) { seen.insert(n); stack.push_back(n); }
      }
    int to_min = 1 << 30;
    for (int op : node_ops(to)) to_min = std::min(to_min, topo_pos[op]);
    while (!stack.empty()) {
      int n = stack.back();
      stack.pop_back();
      for (int op : node_ops(n))
        for (int s : successors(op)) {
          int m = node_of(s);
          if (m == to) return true;
          if (m == from || seen.count(m)) continue;
          seen.insert(m);
          stack.push_back(m);
        }
    }
    return false;
  }

  static bool is_contraction(const Op& op) {
    return op.info->cls == OC_CONV || op.info->cls == OC_MATMUL || op.info->cls == OC_GEMM;
  }

  // One-to-One arithmetic placed in front of a contraction is recomputed for every tile that
  // re-reads the operand: allow only a short run of trivial operators there.
  // `joining`: the operator being added as a predecessor of a block that already holds the contraction (-1 otherwise)
  bool prologue_too_heavy(const std::vector<int>& ops, int joining = -1) const {
    int anchor = -1;
    for (int oi : ops) if (is_contraction(g.ops[oi])) anchor = oi;
    if (anchor < 0) return false;
    std::set<int> in(ops.begin(), ops.end()), up;
    std::vector<int> stack = {anchor};
    while (!stack.empty()) {
      int x = stack.back();
      stack.pop_back();
      for (int p : predecessors(x))
        if (in.count(p) && !up.count(p)) { up.insert(p); stack.push_back(p); }
    }
    int cheap = 0;
    for (int p : up) {
      if (sanctioned_prologue.count(p)) continue;      // taken on purpose by the broadcast-prologue extension
      const Op& op = g.ops[p];
      switch (op.info->cls) {
        case OC_UNARY: case OC_BINARY: case OC_WHERE: case OC_BATCHNORM: {
          static const std::set<std::string> trivial = {"Add", "Sub", "Mul", "Neg", "Relu", "Cast", "Identity"};
          if (!trivial.count(op.kind)) return true;
          if (++cheap > 2) return true;
          // an operator that combines two activations computed by operators outside the block would
          // make the contraction read two intermediate results where one suffices: it belongs in
          // its producers' block (as their epilogue)
          int outside = 0;
          for (int t : op.in) {
            const Tensor& T = g.tensors[t];
            if (T.weight_only || T.kind == DNNF_WEIGHT || (T.has_cval && T.n() == 1)) continue;
            if (T.producer >= 0 && !in.count(T.producer)) {
              outside++;
              // an operator reaching back from a contraction's block to the only reader of another operator's result:
              // that reader is better placed behind its producer (an epilogue costs nothing per output tile; a
              // prologue keeps the contraction off its vector operand loaders).  A seed that grows forward into a
              // contraction (the paper's Fig. 3: Add, then Conv) is not affected.
              if (p == joining && T.consumers.size() == 1 && T.kind == DNNF_INTERMEDIATE && group[T.producer] < 0) return true;
            }
          }
          if (outside > 1) return true;
          break;
        }
        default: break;
      }
    }
    return false;
  }

  bool check_constraint(const Block& blk, int cand, bool as_successor = true) {
    if ((int)blk.ops.size() + 1 > o.max_block_ops) return false;
    int cur = group[blk.ops[0]];
    int cn = node_of(cand);
    if (reaches_via_others(cur, cn) || reaches_via_others(cn, cur)) return false;
    Block nb = merged(blk, cand);
    std::vector<int> ein, eout, rem;
    block_io(g, nb, ein, eout, rem);
    int operands = (int)eout.size();
    for (int t : ein) operands += !(g.tensors[t].has_cval && g.tensors[t].n() == 1);  // scalars are inlined
    if (operands > o.max_block_operands) { say("  constraint: too many operands"); return false; }
    if (prologue_too_heavy(nb.ops, as_successor ? -1 : cand)) return false;
    if (as_successor) {
      // A successor reached along a small operand while a much larger operand of it is still waiting for a block
      // (the scores of an attention layer meeting a [B, 1, 1, S] padding term) belongs with the larger operand: taken
      // here it would cut that operand's producer off from its epilogue and cost a pass over the large tensor.
      std::set<int> inb(blk.ops.begin(), blk.ops.end());
      double through = 0, waiting = 0;
      for (int t : g.ops[cand].in) {
        const Tensor& T = g.tensors[t];
        if (T.producer >= 0 && inb.count(T.producer)) through = std::max(through, (double)T.bytes());
        else if (T.producer >= 0 && group[T.producer] < 0 && !T.weight_only && T.kind == DNNF_INTERMEDIATE) waiting = std::max(waiting, (double)T.bytes());
      }
      if (through > 0 && waiting >= 8.0 * through) { say("  constraint: " + g.ops[cand].kind + " is left to the producer of its larger operand"); return false; }
      // A Transpose behind a contraction whose only readers are contractions still to be planned: as an index map on
      // the reader's operand load it costs nothing, as a second, transposed store of this block's epilogue it costs
      // element-wise stores (measured on the QKV projection: 65 us against 40 us).  It is left to its reader.
      if (g.ops[cand].info->cls == OC_TRANSPOSE) {
        bool has_contraction = false, only_contractions = !g.tensors[g.ops[cand].out[0]].consumers.empty();
        for (int oi : blk.ops) has_contraction = has_contraction || is_contraction(g.ops[oi]);
        for (int cidx : g.tensors[g.ops[cand].out[0]].consumers) only_contractions = only_contractions && is_contraction(g.ops[cidx]) && group[cidx] < 0;
        if (g.tensors[g.ops[cand].out[0]].kind == DNNF_OUTPUT) only_contractions = false;
        if (has_contraction && only_contractions) { say("  constraint: Transpose is left to the contraction that reads it"); return false; }
      }
    }
    if (o.check_lowerable) {
      try {
        LowerOpts lo;
        lo.intra_block = o.intra_block;
        lower_block(g, nb, lo);
      } catch (const Error& e) {
        say("  constraint: no template for block + " + g.ops[cand].kind + " (" + e.what() + ")");
        return false;
      }
    }
    return true;
  }

  Block merged(const Block& blk, int cand) const {
    Block nb = blk;
    nb.ops.push_back(cand);
    std::sort(nb.ops.begin(), nb.ops.end(), [&](int a, int b) { return topo_pos[a] < topo_pos[b]; });
    return nb;
  }

  // Steps 2.1 - 2.4 for one candidate; `as_successor` selects the operand order of the lookup.
  void try_fuse(Block& blk, int cand, bool as_successor) {
    if (group[cand] >= 0 || g.tensors[g.ops[cand].out[0]].weight_only != blk.weight_only) return;
    int fused, colour;
    if (as_successor) fuse_relation(blk.fused_type, g.ops[cand].mapping, &fused, &colour);
    else fuse_relation(g.ops[cand].mapping, blk.fused_type, &fused, &colour);
    if (colour == DNNF_RED) { st.red++; return; }                       // fuse_break
    if (!check_constraint(blk, cand, as_successor)) { st.constraint_rejected++; return; }
    if (colour == DNNF_YELLOW && o.latency) {                            // fuse_depend
      Block nb = merged(blk, cand), single;
      single.ops = {cand};
      single.fused_type = g.ops[cand].mapping;
      double t_fused = o.latency(nb), t_sep = o.latency(blk) + o.latency(single);
      st.profiled++;
      say("  profile " + g.ops[cand].kind + ": fused " + std::to_string(t_fused) + " us vs separate " + std::to_string(t_sep) + " us");
      // The listing's test is fused > separate.  Device timings repeat to about a percent, and a candidate that is
      // only a change of index (a Reshape, a Transpose folded into addresses) leaves the kernel what it was: such
      // pairs measure equal up to that noise, and rejecting one on a coin flip splits the block and costs a copy
      // kernel.  A fusion is therefore refused only when it is slower by more than the noise.
      if (t_fused > t_sep * 1.03 + 0.25) { st.yellow_rejected++; return; }
      st.yellow_fused++;
    } else if (colour == DNNF_YELLOW) st.yellow_fused++;
    else st.green++;
    int cur = group[blk.ops[0]];
    blk = merged(blk, cand);
    blk.fused_type = fused;
    group[cand] = cur;
    members[cur] = blk.ops;
    say("  + " + g.ops[cand].kind + (as_successor ? " (successor)" : " (predecessor)"));
    // Step 2.4: continue from the newly fused operator, first in the direction of travel, then
    // towards its other neighbours (an operator's further predecessors may be fused "some, but not
    // all"; the block of Fig. 4 contains a Mul that is reached only through the shared GEMM).
    if (as_successor) {
      for (int s : successors(cand)) try_fuse(blk, s, true);
      for (int p : predecessors(cand)) try_fuse(blk, p, false);
    } else {
      for (int p : predecessors(cand)) try_fuse(blk, p, false);
      for (int s : successors(cand)) try_fuse(blk, s, true);
    }
  }

  void run_partition(bool weight_only, std::vector<Block>& out) {
    auto eligible = [&](int op) { return g.ops[op].alive && group[op] < 0 && g.tensors[g.ops[op].out[0]].weight_only == weight_only; };
    if (o.fusion && o.attention && !weight_only) {
      // Extension beyond the mapping-type table: MatMul -> One-to-One operators -> Softmax -> MatMul
      // becomes one block (a red cell of the table; the streaming-softmax kernel makes it executable).
      // Formed before the seeds are drawn, then grown along the second MatMul's successors as usual.
      for (int sm : g.topo) {
        if (!eligible(sm) || g.ops[sm].info->cls != OC_SOFTMAX) continue;
        const Tensor& P = g.tensors[g.ops[sm].out[0]];
        if (P.consumers.size() != 1 || P.kind != DNNF_INTERMEDIATE) continue;
        int mm2 = P.consumers[0];
        if (!eligible(mm2) || g.ops[mm2].info->cls != OC_MATMUL || g.ops[mm2].in[0] != g.ops[sm].out[0]) continue;
        // walk up from the Softmax input through One-to-One operators to the first MatMul
        std::vector<int> chain;
        int t = g.ops[sm].in[0], mm1 = -1;
        for (int depth = 0; depth < 16; depth++) {
          const Tensor& T = g.tensors[t];
          int p = T.producer;
          if (p < 0 || !eligible(p) || T.consumers.size() != 1 || T.kind != DNNF_INTERMEDIATE) break;
          if (g.ops[p].info->cls == OC_MATMUL) { mm1 = p; break; }
          const OpClass pc = g.ops[p].info->cls;
          if (pc != OC_UNARY && pc != OC_BINARY && pc != OC_WHERE) break;
          // continue along the one activation operand that has the scores' own shape; a second activation that is
          // broadcast against it (a padding mask computed from an input) is an operand of the block like the constant masks
          int next = -1, n_full = 0;
          for (int i : g.ops[p].in) {
            const Tensor& I = g.tensors[i];
            if (I.weight_only || I.kind == DNNF_WEIGHT || I.has_cval) continue;
            if (I.dims != T.dims) continue;
            n_full++;
            next = i;
          }
          if (n_full != 1) break;
          chain.push_back(p);
          t = next;
        }
        if (mm1 < 0) continue;
        Block blk;
        blk.ops = {mm1, sm, mm2};
        blk.ops.insert(blk.ops.end(), chain.begin(), chain.end());
        std::sort(blk.ops.begin(), blk.ops.end(), [&](int a, int b) { return topo_pos[a] < topo_pos[b]; });
        blk.fused_type = DNNF_MANY_TO_MANY;
        blk.weight_only = false;
        try {
          LowerOpts lo;
          lo.intra_block = o.intra_block;
          lower_block(g, blk, lo);
        } catch (const Error& e) {
          say(std::string("attention block refused: ") + e.what());
          continue;
        }
        int id = (int)members.size();
        members.push_back(blk.ops);
        for (int op : blk.ops) group[op] = id;
        say("attention block around " + g.tensors[g.ops[sm].out[0]].name);
        for (int s : successors(mm2)) try_fuse(blk, s, true);
        out.push_back(blk);
        btype.push_back(blk.fused_type);
      }
    }
    if (o.fusion && o.broadcast_prologue && !weight_only) {
      // Second extension beyond the table: a broadcast multiply x * s (s constant over the image plane: the
      // squeeze-excite scaling, One-to-Many) directly in front of a pointwise convolution joins the
      // convolution's block and is applied to the operand as it is loaded - One-to-Many before Many-to-Many
      // is a red cell, because in general the expanded tensor would be recomputed per output tile; here the
      // multiply costs one vector operation per loaded vector and saves writing and re-reading x * s.  Like a
      // yellow cell it is decided by measurement when the plan is built with profiling.
      for (int cv : g.topo) {
        const Op& C = g.ops[cv];
        if (!eligible(cv) || C.info->cls != OC_CONV || C.i("group", 1) != 1) continue;
        const Tensor& W = g.tensors[C.in[1]];
        if (W.dims.size() != 4 || W.dims[2] != 1 || W.dims[3] != 1) continue;
        const Tensor& X = g.tensors[C.in[0]];
        int mul = X.producer;
        if (mul < 0 || !eligible(mul) || g.ops[mul].kind != "Mul" || X.consumers.size() != 1 || X.kind != DNNF_INTERMEDIATE) continue;
        if (X.dims.size() != 4 || X.dims[2] * X.dims[3] == 1) continue;      // a 1x1 map has no plane to broadcast over
        // one operand has the result's shape, the other is constant over the last two axes
        const Op& M = g.ops[mul];
        if (M.in.size() != 2) continue;
        auto plane_const = [&](int t) { const Dims& d = g.tensors[t].dims; return d.size() == 4 && d[2] == 1 && d[3] == 1; };
        if (!((g.tensors[M.in[0]].dims == X.dims && plane_const(M.in[1])) || (g.tensors[M.in[1]].dims == X.dims && plane_const(M.in[0])))) continue;
        Block blk;
        blk.ops = {mul, cv};
        blk.fused_type = DNNF_MANY_TO_MANY;
        blk.weight_only = false;
        LowerOpts lo;
        lo.intra_block = o.intra_block;
        try {
          Lowered low = lower_block(g, blk, lo);
          if (low.variant.find("_pro") == std::string::npos) { say("broadcast prologue refused: no vector operand loader for " + X.name + " (" + low.variant + ")"); continue; }
        } catch (const Error& e) {
          say(std::string("broadcast prologue refused: ") + e.what());
          continue;
        }
        if (o.latency) {
          Block bm, bc;
          bm.ops = {mul};
          bm.fused_type = g.ops[mul].mapping;
          bc.ops = {cv};
          bc.fused_type = DNNF_MANY_TO_MANY;
          st.profiled++;
          const double fused = o.latency(blk), apart = o.latency(bm) + o.latency(bc);
          say("broadcast prologue " + X.name + ": fused " + std::to_string(fused) + " us, separate " + std::to_string(apart) + " us");
          if (fused > apart * 1.03 + 0.25) continue;
        }
        int id = (int)members.size();
        members.push_back(blk.ops);
        for (int op : blk.ops) group[op] = id;
        say("broadcast multiply taken as prologue of convolution " + g.tensors[C.out[0]].name);
        sanctioned_prologue.insert(mul);
        for (int s : successors(cv)) try_fuse(blk, s, true);
        out.push_back(blk);
        btype.push_back(blk.fused_type);
      }
    }
    if (o.fusion && o.squeeze_excite && !weight_only) {
      // Fourth extension beyond the table: the squeeze-excite tail.  From a 1x1 convolution on a [n, c, 1, 1] vector
      // up through the One-to-One operators in front of it to another such convolution, and on to the
      // GlobalAveragePool that feeds that one when its map is small enough for one workgroup per image.
      for (int c2 : g.topo) {
        const Op& C2 = g.ops[c2];
        if (!eligible(c2) || C2.info->cls != OC_CONV) continue;
        auto is_fc = [&](const Op& cv) {
          const Dims& x = g.tensors[cv.in[0]].dims;
          const Dims& w = g.tensors[cv.in[1]].dims;
          return x.size() == 4 && w.size() == 4 && x[2] == 1 && x[3] == 1 && w[2] == 1 && w[3] == 1 && cv.i("group", 1) == 1;
        };
        if (!is_fc(C2)) continue;
        std::set<int> mid;
        int c1 = -1;
        bool ok = true;
        std::vector<int> stack = {C2.in[0]};
        while (!stack.empty() && ok) {
          const int t = stack.back();
          stack.pop_back();
          const Tensor& T = g.tensors[t];
          const int p = T.producer;
          if (p < 0 || T.weight_only || T.kind == DNNF_WEIGHT || T.has_cval) continue;       // an operand of the block
          if (!eligible(p) || T.kind != DNNF_INTERMEDIATE) { ok = false; continue; }
          if (p == c1 || mid.count(p)) continue;
          const OpClass pc = g.ops[p].info->cls;
          if (pc == OC_CONV) {
            if (c1 >= 0 || !is_fc(g.ops[p])) ok = false;
            else c1 = p;
            continue;
          }
          if ((pc != OC_UNARY && pc != OC_BINARY) || mid.size() >= 8) { ok = false; continue; }
          mid.insert(p);
          for (int i : g.ops[p].in) stack.push_back(i);
        }
        if (!ok || c1 < 0) continue;
        int pool = g.tensors[g.ops[c1].in[0]].producer;
        if (pool >= 0 && eligible(pool) && g.ops[pool].info->cls == OC_GAP && g.tensors[g.ops[pool].out[0]].consumers.size() == 1 &&
            g.tensors[g.ops[pool].out[0]].kind == DNNF_INTERMEDIATE) {
          const Dims& m = g.tensors[g.ops[pool].in[0]].dims;
          if (!(m.size() == 4 && m[2] * m[3] <= 256)) pool = -1;
        } else pool = -1;
        // The pool may instead ride on the depthwise convolution that produces its map (convolution, the One-to-One
        // operators up to the pooled tensor, the pool: the convolution's kernel adds up what it stores, one workgroup
        // per image and channel group), which leaves the tail its two layers alone and the map unread.
        Block dwp;
        if (pool >= 0) {
          std::set<int> up;
          int dw = -1;
          bool okd = true;
          std::vector<int> stk = {g.ops[pool].in[0]};
          while (!stk.empty() && okd) {
            const int t = stk.back();
            stk.pop_back();
            const Tensor& T = g.tensors[t];
            const int pr = T.producer;
            if (pr < 0 || T.weight_only || T.kind == DNNF_WEIGHT || T.has_cval) continue;
            if (!eligible(pr)) { okd = false; continue; }
            if (pr == dw || up.count(pr)) continue;
            const OpClass pc = g.ops[pr].info->cls;
            if (pc == OC_CONV) {
              const Dims& w = g.tensors[g.ops[pr].in[1]].dims;
              if (dw >= 0 || w.size() != 4 || g.ops[pr].i("group", 1) != w[0] || w[1] != 1) okd = false;
              else dw = pr;
              continue;
            }
            if ((pc != OC_UNARY && pc != OC_BINARY) || up.size() >= 6) { okd = false; continue; }
            up.insert(pr);
            for (int i : g.ops[pr].in) stk.push_back(i);
          }
          if (okd && dw >= 0) {
            dwp.ops = {dw, pool};
            dwp.ops.insert(dwp.ops.end(), up.begin(), up.end());
            std::sort(dwp.ops.begin(), dwp.ops.end(), [&](int a, int b) { return topo_pos[a] < topo_pos[b]; });
            dwp.fused_type = DNNF_MANY_TO_MANY;
            LowerOpts lo;
            lo.intra_block = o.intra_block;
            try {
              lower_block(g, dwp, lo);
            } catch (const Error& e) {
              say(std::string("pool inside the depthwise convolution refused: ") + e.what());
              dwp.ops.clear();
            }
          }
        }
        // first with the pool (one workgroup per image reads the whole map), then the two layers alone (the pool keeps
        // its own kernel, which spreads a map over many workgroups); without profiling the first form that lowers is taken
        Block blk;
        bool taken = false;
        if (!dwp.ops.empty()) {
          // the tail without its pool + the convolution with it, against the tail with its pool + the convolution alone
          Block tail, tailp, conv_alone;
          tail.ops = {c1, c2};
          tail.ops.insert(tail.ops.end(), mid.begin(), mid.end());
          std::sort(tail.ops.begin(), tail.ops.end(), [&](int a, int b) { return topo_pos[a] < topo_pos[b]; });
          tail.fused_type = DNNF_MANY_TO_MANY;
          tailp = tail;
          tailp.ops.push_back(pool);
          std::sort(tailp.ops.begin(), tailp.ops.end(), [&](int a, int b) { return topo_pos[a] < topo_pos[b]; });
          for (int op : dwp.ops) if (op != pool) conv_alone.ops.push_back(op);
          conv_alone.fused_type = DNNF_MANY_TO_MANY;
          LowerOpts lo;
          lo.intra_block = o.intra_block;
          bool lowers = true;
          try { lower_block(g, tail, lo); } catch (const Error&) { lowers = false; }
          if (lowers) {
            bool take = true;
            if (o.latency && o.squeeze_excite == 1) {
              st.profiled++;
              double with_tail = -1;
              try { lower_block(g, tailp, lo); with_tail = o.latency(tailp) + o.latency(conv_alone); } catch (const Error&) {}
              const double on_conv = o.latency(tail) + o.latency(dwp);
              say("pool of " + g.tensors[C2.out[0]].name + ": inside the depthwise convolution " + std::to_string(on_conv) + " us, inside the tail " +
                  std::to_string(with_tail) + " us (each with the other kernel of the pair)");
              take = with_tail < 0 || on_conv <= with_tail * 1.03 + 0.25;
            }
            if (take) {
              int idd = (int)members.size();
              members.push_back(dwp.ops);
              for (int op : dwp.ops) group[op] = idd;
              say("global average pool taken inside the depthwise convolution " + g.tensors[g.ops[dwp.ops[0]].out[0]].name);
              out.push_back(dwp);
              btype.push_back(dwp.fused_type);
              blk = tail;
              taken = true;
              pool = -1;
            }
          }
        }
        for (int with_pool = pool >= 0 ? 1 : 0; with_pool >= 0 && !taken; with_pool--) {
          blk = Block();
          blk.ops = {c1, c2};
          blk.ops.insert(blk.ops.end(), mid.begin(), mid.end());
          if (with_pool) blk.ops.push_back(pool);
          std::sort(blk.ops.begin(), blk.ops.end(), [&](int a, int b) { return topo_pos[a] < topo_pos[b]; });
          blk.fused_type = DNNF_MANY_TO_MANY;
          blk.weight_only = false;
          LowerOpts lo;
          lo.intra_block = o.intra_block;
          try {
            lower_block(g, blk, lo);
          } catch (const Error& e) {
            say(std::string("squeeze-excite block refused: ") + e.what());
            continue;
          }
          if (o.latency && o.squeeze_excite == 1) {
            // against the table's plan for the same operators: the pool, the first layer with its operators, the second layer
            std::set<int> first(mid.begin(), mid.end());
            first.insert(c1);
            Block bp, b1, b2;
            for (int op : blk.ops) (op == pool ? bp : first.count(op) ? b1 : b2).ops.push_back(op);
            bp.fused_type = b1.fused_type = b2.fused_type = DNNF_MANY_TO_MANY;
            st.profiled++;
            const double fused = o.latency(blk), apart = (with_pool ? o.latency(bp) : 0.0) + o.latency(b1) + o.latency(b2);
            say("squeeze-excite " + g.tensors[C2.out[0]].name + (with_pool ? " with its pool" : "") + ": fused " + std::to_string(fused) +
                " us, separate " + std::to_string(apart) + " us");
            if (fused > apart * 1.03 + 0.25) continue;
          }
          taken = true;
          if (!with_pool) pool = -1;
        }
        if (!taken) continue;
        int id = (int)members.size();
        members.push_back(blk.ops);
        for (int op : blk.ops) group[op] = id;
        say("squeeze-excite block around " + g.tensors[C2.out[0]].name + (pool >= 0 ? " (with its pool)" : ""));
        for (int m : mid) sanctioned_prologue.insert(m);       // operators between the two layers: in front of a convolution on purpose
        for (int s : successors(c2)) try_fuse(blk, s, true);
        out.push_back(blk);
        btype.push_back(blk.fused_type);
      }
    }
    if (o.fusion && o.gemm_norm && !weight_only) {
      // Third extension beyond the table: MatMul -> One-to-One operators -> normalisation of the last axis (the
      // LayerNorm behind a linear layer; Many-to-Many after Many-to-Many, red).  The block's kernel gives a workgroup
      // whole rows of the product, so the statistics are taken before the rows leave the chip - at the price of
      // reading the whole second operand once per 32 rows.  Taken always (gemm_norm = 2), or when measured faster than
      // the MatMul block and the normalisation block side by side.
      for (int mm : g.topo) {
        if (!eligible(mm) || g.ops[mm].info->cls != OC_MATMUL) continue;
        // down from the product through the One-to-One operators that consume it, one after the other, to a normalisation
        // (the last tensor of the chain may have other readers too: the residual stream)
        std::vector<int> mid;
        int nm = -1, t = g.ops[mm].out[0];
        for (int depth = 0; depth < 8 && nm < 0; depth++) {
          int next = -1;
          for (int cns : g.tensors[t].consumers)
            if (eligible(cns) && g.ops[cns].kind == "Normalize" && g.ops[cns].in[0] == t) nm = cns;
          if (nm >= 0) break;
          if (g.tensors[t].consumers.size() != 1 || g.tensors[t].kind != DNNF_INTERMEDIATE) break;
          next = g.tensors[t].consumers[0];
          const OpClass pc = g.ops[next].info->cls;
          if (!eligible(next) || (pc != OC_UNARY && pc != OC_BINARY && pc != OC_RESHAPE)) break;
          mid.push_back(next);
          t = g.ops[next].out[0];
        }
        if (nm < 0) continue;
        Block blk, bmm, bnm;
        blk.ops = {mm, nm};
        blk.ops.insert(blk.ops.end(), mid.begin(), mid.end());
        std::sort(blk.ops.begin(), blk.ops.end(), [&](int a, int b) { return topo_pos[a] < topo_pos[b]; });
        blk.fused_type = DNNF_MANY_TO_MANY;
        blk.weight_only = false;
        LowerOpts lo;
        lo.intra_block = o.intra_block;
        try {
          lower_block(g, blk, lo);
        } catch (const Error& e) {
          say(std::string("MatMul + normalisation block refused: ") + e.what());
          continue;
        }
        if (o.latency && o.gemm_norm == 1) {
          bmm.ops.assign(blk.ops.begin(), blk.ops.end());
          bmm.ops.erase(std::find(bmm.ops.begin(), bmm.ops.end(), nm));
          bmm.fused_type = DNNF_MANY_TO_MANY;
          bnm.ops = {nm};
          bnm.fused_type = DNNF_MANY_TO_MANY;
          st.profiled++;
          const double fused = o.latency(blk), apart = o.latency(bmm) + o.latency(bnm);
          say("MatMul + normalisation " + g.tensors[g.ops[nm].out[0]].name + ": fused " + std::to_string(fused) + " us, separate " + std::to_string(apart) + " us");
          if (fused > apart * 1.03 + 0.25) continue;
        }
        int id = (int)members.size();
        members.push_back(blk.ops);
        for (int op : blk.ops) group[op] = id;
        say("MatMul + normalisation block around " + g.tensors[g.ops[nm].out[0]].name);
        for (int s : successors(nm)) try_fuse(blk, s, true);
        for (int p : predecessors(mm)) try_fuse(blk, p, false);
        out.push_back(blk);
        btype.push_back(blk.fused_type);
      }
    }
    if (o.fusion) {
      for (;;) {
        // Step I: the unfused One-to-One operator with the smallest intermediate result
        int seed = -1;
        int64_t best = 0;
        for (int op : g.topo) {
          if (!eligible(op) || g.ops[op].mapping != DNNF_ONE_TO_ONE) continue;
          int64_t sz = 0;
          for (int t : g.ops[op].out) sz += g.tensors[t].bytes();
          if (seed < 0 || sz < best) { seed = op; best = sz; }
        }
        if (seed < 0) break;
        st.seeds++;
        Block blk;
        blk.ops = {seed};
        blk.fused_type = g.ops[seed].mapping;
        blk.weight_only = weight_only;
        int id = (int)members.size();
        // node ids of unfused operators shift when a block is added; node_of() accounts for it
        members.push_back(blk.ops);
        group[seed] = id;
        say("seed " + g.ops[seed].kind + " (" + g.tensors[g.ops[seed].out[0]].name + ")");
        if (o.successors_first) for (int s : successors(seed)) try_fuse(blk, s, true);   // Step II
        for (int p : predecessors(seed)) try_fuse(blk, p, false);                        // Step III
        if (!o.successors_first) for (int s : successors(seed)) try_fuse(blk, s, true);  // Step II
        out.push_back(blk);
        btype.push_back(blk.fused_type);
      }
    }
    for (int op : g.topo) {
      if (!eligible(op)) continue;
      Block blk;
      blk.ops = {op};
      blk.fused_type = g.ops[op].mapping;
      blk.weight_only = weight_only;
      group[op] = (int)members.size();
      members.push_back(blk.ops);
      out.push_back(blk);
    }
  }
};

}  // namespace

std::vector<Block> build_fusion_plan(const Graph& g, const PlannerOpts& o, PlanStats* stats) {
  DNNF_CHECK(g.finalized, DNNF_NOT_FINALIZED, "graph is not finalized");
  Planner P(g, o);
  std::vector<Block> blocks;
  P.run_partition(true, blocks);
  P.run_partition(false, blocks);
  // Intra-block optimisation (Sec. 4.4.2): a Reorganize / Shuffle / Slice operator left on its own
  // whose result is read by a single block is replaced by a change of that block's data index,
  // i.e. it joins the block.  This also covers index-only operators on weights, which otherwise
  // would be materialised once at prepare time.
  if (o.fusion && o.intra_block) {
    bool changed = true;
    while (changed) {
      changed = false;
      for (size_t bi = 0; bi < blocks.size() && !changed; bi++) {
        Block& blk = blocks[bi];
        if (blk.ops.empty() || blk.weight_only) continue;
        std::vector<int> ein, eout, rem;
        block_io(g, blk, ein, eout, rem);
        for (int t : ein) {
          int p = g.tensors[t].producer;
          if (p < 0) continue;
          const Op& op = g.ops[p];
          if (op.info->cls != OC_RESHAPE && op.info->cls != OC_TRANSPOSE && op.info->cls != OC_SLICE) continue;
          int pb = P.group[p];
          if (pb == (int)bi || blocks[pb].ops.empty()) continue;
          // the producing block must consist of index-only operators whose results only this block reads
          bool index_only = true;
          for (int q : blocks[pb].ops) {
            OpClass cl = g.ops[q].info->cls;
            index_only = index_only && (cl == OC_RESHAPE || cl == OC_TRANSPOSE || cl == OC_SLICE) &&
                         !g.ops[q].has("materialize");   // a layout copy the rewriter asked for stays a copy
          }
          if (!index_only) continue;
          std::vector<int> pin, pout, prem;
          block_io(g, blocks[pb], pin, pout, prem);
          bool only_here = true;
          for (int u : pout) {
            only_here = only_here && g.tensors[u].kind != DNNF_OUTPUT;
            for (int cns : g.tensors[u].consumers) only_here = only_here && P.group[cns] == (int)bi;
          }
          if (!only_here) continue;
          Block nb = blk;
          for (int q : blocks[pb].ops) nb = P.merged(nb, q);
          int fused, colour;
          fuse_relation(op.mapping, blk.fused_type, &fused, &colour);
          nb.fused_type = fused;
          try {
            LowerOpts lo;
            lower_block(g, nb, lo);
          } catch (const Error&) {
            continue;
          }
          if (o.latency) {
            double t_fused = o.latency(nb);
            double t_sep = o.latency(blk) + (blocks[pb].weight_only ? 0.0 : o.latency(blocks[pb]));
            P.st.profiled++;
            P.say("  intra-block " + op.kind + ": folded " + std::to_string(t_fused) + " us vs separate " + std::to_string(t_sep) + " us");
            if (t_fused > t_sep * 1.02) continue;
          }
          P.say("intra-block: " + op.kind + " folded into the index of its consumer block");
          for (int q : blocks[pb].ops) P.group[q] = (int)bi;
          blocks[pb].ops.clear();
          blk = nb;
          changed = true;
          break;
        }
      }
    }
    std::vector<Block> kept;
    std::vector<int> remap(blocks.size(), -1);
    for (size_t b = 0; b < blocks.size(); b++)
      if (!blocks[b].ops.empty()) { remap[b] = (int)kept.size(); kept.push_back(blocks[b]); }
    for (auto& gi : P.group) if (gi >= 0) gi = remap[gi];
    blocks = kept;
  }
  // blocks were appended in creation order; members[] mirrors it.  Order them by dependences.
  size_t nb = blocks.size();
  std::vector<std::set<int>> succ(nb);
  std::vector<int> indeg(nb, 0);
  for (size_t b = 0; b < nb; b++)
    for (int op : blocks[b].ops)
      for (int s : P.successors(op)) {
        int sb = P.group[s];
        if (sb != (int)b && !succ[b].count(sb)) { succ[b].insert(sb); indeg[sb]++; }
      }
  std::set<std::pair<int, int>> ready;  // (first topo position, block)
  auto key = [&](int b) {
    int m = 1 << 30;
    for (int op : blocks[b].ops) m = std::min(m, P.topo_pos[op]);
    return std::make_pair(m, b);
  };
  for (size_t b = 0; b < nb; b++) if (indeg[b] == 0) ready.insert(key((int)b));
  std::vector<Block> ordered;
  while (!ready.empty()) {
    int b = ready.begin()->second;
    ready.erase(ready.begin());
    ordered.push_back(blocks[b]);
    for (int s : succ[b]) if (--indeg[s] == 0) ready.insert(key(s));
  }
  DNNF_CHECK(ordered.size() == nb, DNNF_CYCLE, "fusion plan has mutually dependent blocks");
  // weight-only blocks first (they run at prepare time), keeping relative order
  std::stable_partition(ordered.begin(), ordered.end(), [](const Block& b) { return b.weight_only; });
  if (stats) *stats = P.st;
  return ordered;
}

}  // namespace dnnf
