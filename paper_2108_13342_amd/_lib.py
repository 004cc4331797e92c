"""ctypes loader for libdnnf.so.  Fails loudly when the library is missing: there is no fallback."""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libdnnf.so")

_lib = None


class Attr(C.Structure):
    _fields_ = [("name", C.c_char_p), ("n", C.c_int), ("values", C.POINTER(C.c_double))]


class RewriteStats(C.Structure):
    _fields_ = [("rules_fired", C.c_int), ("canonicalisations", C.c_int), ("flops_before", C.c_double),
                ("flops_after", C.c_double), ("ops_before", C.c_int), ("ops_after", C.c_int), ("derived_rules_fired", C.c_int)]


class PlanOpts(C.Structure):
    _fields_ = [("fusion", C.c_int), ("profile", C.c_int), ("intra_block", C.c_int), ("max_block_ops", C.c_int),
                ("max_block_operands", C.c_int), ("profile_scratch", C.c_void_p), ("profile_scratch_bytes", C.c_size_t),
                ("cache_dir", C.c_char_p), ("verbose", C.c_int), ("successors_first", C.c_int),
                ("check_lowerable", C.c_int), ("tune", C.c_int), ("attention", C.c_int), ("layout", C.c_int), ("broadcast_prologue", C.c_int), ("graphs", C.c_int), ("gemm_norm", C.c_int), ("squeeze_excite", C.c_int)]


class BlockInfo(C.Structure):
    _fields_ = [("n_ops", C.c_int), ("fused_type", C.c_int), ("family", C.c_int), ("bytes", C.c_double),
                ("flops", C.c_double), ("irs_bytes_removed", C.c_double), ("n_kernel_launches", C.c_int),
                ("kernel_name", C.c_char * 96)]


EXPORTS = {
    "dnnf_last_error": (C.c_char_p, []),
    "dnnf_graph_create": (C.c_int, [C.POINTER(C.c_void_p)]),
    "dnnf_graph_destroy": (None, [C.c_void_p]),
    "dnnf_graph_add_tensor": (C.c_int, [C.c_void_p, C.c_char_p, C.c_int, C.c_int, C.POINTER(C.c_int64), C.c_int, C.POINTER(C.c_int)]),
    "dnnf_graph_set_const": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_double), C.c_int64]),
    "dnnf_graph_add_op": (C.c_int, [C.c_void_p, C.c_char_p, C.c_int, C.POINTER(C.c_int), C.c_int, C.POINTER(C.c_int),
                                    C.POINTER(Attr), C.c_int, C.POINTER(C.c_int)]),
    "dnnf_graph_finalize": (C.c_int, [C.c_void_p]),
    "dnnf_graph_num_ops": (C.c_int, [C.c_void_p, C.POINTER(C.c_int)]),
    "dnnf_graph_num_op_slots": (C.c_int, [C.c_void_p, C.POINTER(C.c_int)]),
    "dnnf_graph_op_info": (C.c_int, [C.c_void_p, C.c_int, C.c_char_p, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int)]),
    "dnnf_plan_op_kind": (C.c_int, [C.c_void_p, C.c_int, C.c_char_p, C.c_int]),
    "dnnf_op_mapping_type": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_int)]),
    "dnnf_op_kind_mapping_type": (C.c_int, [C.c_char_p, C.POINTER(C.c_int)]),
    "dnnf_fuse_relation": (C.c_int, [C.c_int, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int)]),
    "dnnf_graph_rewrite": (C.c_int, [C.c_void_p, C.POINTER(RewriteStats)]),
    "dnnf_graph_dump_json": (C.c_int, [C.c_void_p, C.c_char_p, C.c_size_t, C.POINTER(C.c_size_t)]),
    "dnnf_plan_default_opts": (None, [C.POINTER(PlanOpts)]),
    "dnnf_plan_build": (C.c_int, [C.c_void_p, C.POINTER(PlanOpts), C.POINTER(C.c_void_p), C.c_void_p, C.POINTER(C.c_void_p)]),
    "dnnf_plan_destroy": (None, [C.c_void_p]),
    "dnnf_plan_num_blocks": (C.c_int, [C.c_void_p, C.POINTER(C.c_int)]),
    "dnnf_plan_block_info": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(BlockInfo)]),
    "dnnf_plan_block_ops": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_int), C.c_int, C.POINTER(C.c_int)]),
    "dnnf_plan_block_source": (C.c_int, [C.c_void_p, C.c_int, C.c_char_p, C.c_size_t, C.POINTER(C.c_size_t)]),
    "dnnf_plan_dump_json": (C.c_int, [C.c_void_p, C.c_char_p, C.c_size_t, C.POINTER(C.c_size_t)]),
    "dnnf_plan_precompile": (C.c_int, [C.c_void_p]),
    "dnnf_plan_workspace_bytes": (C.c_int, [C.c_void_p, C.POINTER(C.c_size_t)]),
    "dnnf_plan_prepare": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "dnnf_plan_run": (C.c_int, [C.c_void_p, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_void_p, C.c_void_p]),
    "dnnf_plan_run_static": (C.c_int, [C.c_void_p, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_void_p]),
    "dnnf_plan_run_block": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_void_p, C.c_void_p]),
    "dnnf_plan_time_block": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_void_p,
                                       C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_double)]),
}


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`. "
                "There is no CPU fallback for the fused-block executor.")
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(l, name)   # AttributeError if a declared symbol is not exported
            fn.restype = res
            fn.argtypes = args
        _lib = l
    return _lib
