// Global data-format selection (paper Sec. 4.4.2, inter-block optimisation): the storage order of the
// tensors that travel between fusion blocks is chosen for the dominant operators that touch them.
//
// On this GPU the dominant operators of a convolutional graph are its convolutions, and both kernel
// templates they lower to want the channel axis innermost: a pointwise convolution then reads its
// activation operand K-contiguous (16-byte vectors straight into the MFMA operand tile, for any
// spatial extent, where NCHW needs pixel rows that are multiples of the vector width), and a depthwise
// convolution runs one lane per 8 channels with every tap a full-width vector load.  One-to-One
// operators, broadcasts and pooling follow whatever order their operands have, so the pass gives every
// activation of a convolutional region the same order and no reformatting kernel is ever inserted;
// only the caller's tensors (graph inputs and outputs) keep the declared NCHW order, and the kernels
// that read or write them absorb the change in their address functions.
//
// Depthwise filters are re-laid once, when the plan is prepared, as [kh, kw, 1, c] so that a tap's
// coefficients for 8 neighbouring channels are one vector as well: an Identity operator on the weight
// (a weight-only block) whose result carries the new order.  Dense filters with a window are re-laid
// [co, kh, kw, ci] the same way: the implicit GEMM then walks K tap by tap, and within a tap the operand's
// channels are contiguous (16-byte vectors straight into the MFMA operand tile, zero vectors for padding).
#include <algorithm>

#include "ir.hpp"

namespace dnnf {

int select_layouts(Graph& g) {
  const std::vector<int> kChannelsLast = {0, 2, 3, 1};
  auto vec_of = [&](const Tensor& T) { return 16 / dtype_bytes(T.dtype); };
  // candidates: rank-4 float intermediates whose channel count fills whole vectors and that no
  // Reorganize operator reinterprets as a flat buffer
  auto eligible = [&](int t) {
    const Tensor& T = g.tensors[t];
    if (T.kind != DNNF_INTERMEDIATE || T.weight_only || T.dims.size() != 4 || !is_float(T.dtype)) return false;
    if (T.dims[1] % vec_of(T)) return false;
    auto flat = [&](int oi) { return g.ops[oi].info->cls == OC_RESHAPE; };
    if (T.producer >= 0 && flat(T.producer)) return false;
    for (int oi : T.consumers) if (flat(oi)) return false;
    return true;
  };
  std::vector<char> chosen(g.tensors.size(), 0);
  bool any_conv = false;
  for (int oi : g.topo) {
    const Op& op = g.ops[oi];
    if (op.info->cls != OC_CONV) continue;
    any_conv = true;
    for (int t : {op.in[0], op.out[0]}) if (eligible(t)) chosen[t] = 1;
  }
  if (!any_conv) return 0;
  // the region grows through operators that are indifferent to the order of their operands
  bool again = true;
  while (again) {
    again = false;
    for (int oi : g.topo) {
      const Op& op = g.ops[oi];
      const OpClass cl = op.info->cls;
      if (cl != OC_UNARY && cl != OC_BINARY && cl != OC_WHERE && cl != OC_BATCHNORM && cl != OC_GAP && cl != OC_POOL && cl != OC_CONV) continue;
      bool touches = false;
      for (int t : op.in) touches = touches || chosen[t];
      for (int t : op.out) touches = touches || chosen[t];
      if (!touches) continue;
      auto grow = [&](int t) {
        if (!chosen[t] && eligible(t)) { chosen[t] = 1; again = true; }
      };
      for (int t : op.in) grow(t);
      for (int t : op.out) grow(t);
    }
  }
  int n = 0;
  for (size_t t = 0; t < g.tensors.size(); t++)
    if (chosen[t]) { g.tensors[t].perm = kChannelsLast; n++; }

  // depthwise filters whose activation operand is channels-last
  std::vector<std::pair<int, int>> relay;   // (conv op, weight tensor)
  for (int oi : g.topo) {
    const Op& op = g.ops[oi];
    if (op.info->cls != OC_CONV) continue;
    const Tensor& X = g.tensors[op.in[0]];
    const Tensor& W = g.tensors[op.in[1]];
    const int64_t grp = op.i("group", 1);
    const bool depthwise = grp > 1 && grp == X.dims[1] && W.dims[1] == 1 && W.dims[0] == X.dims[1];
    if (!depthwise || X.dims[1] % vec_of(W)) continue;
    if (!chosen[op.in[0]] && !chosen[op.out[0]]) continue;
    if (W.kind != DNNF_WEIGHT && !W.weight_only) continue;
    relay.push_back({oi, op.in[1]});
  }
  // dense filters with a window (3x3, 5x5, ...) whose activation operand is channels-last: [co, kh, kw, ci], the K
  // order in which a tap's channels are one contiguous run of the operand
  std::vector<std::pair<int, int>> relay_dense;
  for (int oi : g.topo) {
    const Op& op = g.ops[oi];
    if (op.info->cls != OC_CONV || op.i("group", 1) != 1) continue;
    const Tensor& X = g.tensors[op.in[0]];
    const Tensor& W = g.tensors[op.in[1]];
    if (W.dims.size() != 4 || W.dims[2] * W.dims[3] == 1 || !chosen[op.in[0]] || X.dims[1] % vec_of(W)) continue;
    if (W.kind != DNNF_WEIGHT && !W.weight_only) continue;
    relay_dense.push_back({oi, op.in[1]});
  }
  for (auto& r : relay_dense) {
    const Tensor W = g.tensors[r.second];
    int w2 = g.new_tensor_like(W.name + ".ohwi", W.dtype, W.dims);
    g.tensors[w2].perm = {0, 2, 3, 1};
    g.add_op("Identity", {r.second}, {w2}, {});
    g.ops[r.first].in[1] = w2;
    n++;
  }
  for (auto& r : relay) {
    const Tensor W = g.tensors[r.second];
    int w2 = g.new_tensor_like(W.name + ".hwc", W.dtype, W.dims);
    g.tensors[w2].perm = {2, 3, 1, 0};
    g.add_op("Identity", {r.second}, {w2}, {});
    g.ops[r.first].in[1] = w2;
    n++;
  }
  if (!relay.empty() || !relay_dense.empty()) {
    g.relink();
    g.finalized = true;
  }
  return n;
}

}  // namespace dnnf
