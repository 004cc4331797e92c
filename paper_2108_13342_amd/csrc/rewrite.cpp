#include "ir.hpp"
namespace dnnf {
void rewrite_graph(Graph& g, RewriteStats& st) {
  st.ops_before = st.ops_after = g.live_ops();
  st.flops_before = st.flops_after = g.total_flops();
}
}  // namespace dnnf
