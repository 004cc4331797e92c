#include "lower_ctx.hpp"
namespace dnnf {
Lowered lower_conv(LowerCtx& c) { throw Error(DNNF_UNSUPPORTED_OP, "conv template not built yet"); }
}  // namespace dnnf
