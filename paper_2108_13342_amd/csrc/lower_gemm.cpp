#include "lower_ctx.hpp"
namespace dnnf {
Lowered lower_gemm(LowerCtx& c) { throw Error(DNNF_UNSUPPORTED_OP, "gemm template not built yet"); }
}  // namespace dnnf
