#include "lower_ctx.hpp"
namespace dnnf {
Lowered lower_reduce(LowerCtx& c) { throw Error(DNNF_UNSUPPORTED_OP, "row-reduction template not built yet"); }
}  // namespace dnnf
