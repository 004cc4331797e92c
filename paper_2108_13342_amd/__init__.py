"""MI355X-native fused-block executor (hot path of the DNNFusion method, arxiv 2108.13342).

The product is the C-ABI library `libdnnf.so` (include/dnnf.h); `api` is its thin binding.
"""
