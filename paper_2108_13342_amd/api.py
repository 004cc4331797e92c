"""Thin Python binding over the C ABI (include/dnnf.h): argument marshalling only.

`Graph` and `Plan` mirror the dnnf_graph_* / dnnf_plan_* calls one to one.
`Session` is a convenience that feeds a workload description through those
calls and owns the torch tensors whose device pointers are handed to the
library (PyTorch provides device memory and streams, nothing else).
"""
from __future__ import annotations

import ctypes as C
from typing import Dict, List, Optional, Sequence

import numpy as np

from . import _lib
from ._lib import Attr, BlockInfo, PlanOpts, RewriteStats

DTYPES = {"f32": 0, "f16": 1, "bf16": 2, "i32": 3, "i64": 4, "bool": 5}
KINDS = {"input": 0, "weight": 1, "intermediate": 2, "output": 3}
MAPPING_NAMES = ["One-to-One", "Reorganize", "Shuffle", "One-to-Many", "Many-to-Many"]
COLOUR_NAMES = ["green", "yellow", "red"]
FAMILY_NAMES = ["elementwise", "row-reduction", "gemm", "conv", "depthwise-conv", "alias", "attention", "squeeze-excite"]


class DnnfError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"dnnf error {code}: {msg}")
        self.code = code


def _check(rc):
    if rc != 0:
        raise DnnfError(rc, _lib.lib().dnnf_last_error().decode(errors="replace"))


def fuse_relation(first: int, second: int):
    f, c = C.c_int(), C.c_int()
    _check(_lib.lib().dnnf_fuse_relation(first, second, C.byref(f), C.byref(c)))
    return f.value, c.value


def op_kind_mapping_type(kind: str) -> int:
    t = C.c_int()
    _check(_lib.lib().dnnf_op_kind_mapping_type(kind.encode(), C.byref(t)))
    return t.value


class Graph:
    def __init__(self):
        self._h = C.c_void_p()
        _check(_lib.lib().dnnf_graph_create(C.byref(self._h)))

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:      # (module globals are gone when the interpreter shuts down)
            _lib.lib().dnnf_graph_destroy(self._h)
            self._h = None

    def add_tensor(self, name, dtype, dims, kind) -> int:
        arr = (C.c_int64 * max(len(dims), 1))(*[int(d) for d in dims])
        tid = C.c_int()
        _check(_lib.lib().dnnf_graph_add_tensor(self._h, name.encode(), DTYPES[dtype], len(dims), arr, KINDS[kind], C.byref(tid)))
        return tid.value

    def set_const(self, tensor_id, values):
        v = np.ascontiguousarray(np.asarray(values, dtype=np.float64).ravel())
        _check(_lib.lib().dnnf_graph_set_const(self._h, tensor_id, v.ctypes.data_as(C.POINTER(C.c_double)), v.size))

    def add_op(self, kind, in_ids, out_ids, attrs=None) -> int:
        attrs = attrs or {}
        keep = []
        arr = (Attr * max(len(attrs), 1))()
        for i, (k, v) in enumerate(attrs.items()):
            if isinstance(v, str):          # a string attribute (Einsum's equation) travels as its character codes
                v = [ord(ch) for ch in v]
            vals = np.atleast_1d(np.asarray(v, dtype=np.float64)).ravel()
            buf = (C.c_double * max(vals.size, 1))(*vals.tolist())
            keep.append(buf)
            arr[i] = Attr(k.encode(), int(vals.size), C.cast(buf, C.POINTER(C.c_double)))
        ins = (C.c_int * max(len(in_ids), 1))(*in_ids)
        outs = (C.c_int * max(len(out_ids), 1))(*out_ids)
        oid = C.c_int()
        _check(_lib.lib().dnnf_graph_add_op(self._h, kind.encode(), len(in_ids), ins, len(out_ids), outs, arr, len(attrs), C.byref(oid)))
        return oid.value

    def finalize(self):
        _check(_lib.lib().dnnf_graph_finalize(self._h))

    def num_ops(self) -> int:
        n = C.c_int()
        _check(_lib.lib().dnnf_graph_num_ops(self._h, C.byref(n)))
        return n.value

    def num_op_slots(self) -> int:
        n = C.c_int()
        _check(_lib.lib().dnnf_graph_num_op_slots(self._h, C.byref(n)))
        return n.value

    def op_info(self, op_id):
        buf = C.create_string_buffer(64)
        alive, mt = C.c_int(), C.c_int()
        _check(_lib.lib().dnnf_graph_op_info(self._h, op_id, buf, 64, C.byref(alive), C.byref(mt)))
        return buf.value.decode(), bool(alive.value), mt.value

    def op_mapping_type(self, op_id) -> int:
        t = C.c_int()
        _check(_lib.lib().dnnf_op_mapping_type(self._h, op_id, C.byref(t)))
        return t.value

    def live_ops(self):
        return [(i,) + self.op_info(i)[0:1] + self.op_info(i)[2:3] for i in range(self.num_op_slots()) if self.op_info(i)[1]]

    def dump_json(self) -> dict:
        import json
        need = C.c_size_t()
        _check(_lib.lib().dnnf_graph_dump_json(self._h, None, 0, C.byref(need)))
        buf = C.create_string_buffer(need.value + 1)
        _check(_lib.lib().dnnf_graph_dump_json(self._h, buf, need.value + 1, C.byref(need)))
        return json.loads(buf.value.decode())

    def rewrite(self) -> Dict[str, float]:
        st = RewriteStats()
        _check(_lib.lib().dnnf_graph_rewrite(self._h, C.byref(st)))
        return {f: getattr(st, f) for f, _ in RewriteStats._fields_}


def graph_from_spec(spec, finalize=True):
    """Feeds a workloads.graph.GraphSpec through the C ABI.  Returns (Graph, {tensor name: id})."""
    g = Graph()
    ids = {}
    for t in spec.tensors.values():
        ids[t.name] = g.add_tensor(t.name, t.dtype, t.shape, t.kind)
        if t.kind == "weight" and t.data is not None and (t.const or t.data.size <= 4096):
            g.set_const(ids[t.name], t.data)
    for op in spec.ops:
        g.add_op(op.kind, [ids[i] for i in op.inputs], [ids[o] for o in op.outputs], op.attrs)
    if finalize:
        g.finalize()
    return g, ids


class Plan:
    def __init__(self, graph: Graph, weight_ptrs: Sequence[int], stream: int = 0, fusion=1, profile=0, intra_block=1,
                 max_block_ops=0, max_block_operands=0, profile_scratch: int = 0, profile_scratch_bytes: int = 0,
                 cache_dir: Optional[str] = None, verbose=0, successors_first=0, check_lowerable=1, tune=0, attention=0, layout=0, graphs=0, broadcast_prologue=0,
                 gemm_norm=0, squeeze_excite=0):
        L = _lib.lib()
        o = PlanOpts()
        L.dnnf_plan_default_opts(C.byref(o))
        o.fusion, o.profile, o.intra_block = int(fusion), int(profile), int(intra_block)
        o.max_block_ops, o.max_block_operands = int(max_block_ops), int(max_block_operands)
        o.profile_scratch, o.profile_scratch_bytes = profile_scratch or None, int(profile_scratch_bytes)
        self._cache_dir = cache_dir.encode() if cache_dir else None
        o.cache_dir = self._cache_dir
        o.verbose = int(verbose)
        o.successors_first, o.check_lowerable = int(successors_first), int(check_lowerable)
        o.tune, o.attention = int(tune), int(attention)
        o.layout = int(layout)
        o.graphs = int(graphs)
        o.broadcast_prologue = int(broadcast_prologue)
        o.gemm_norm = int(gemm_norm)
        o.squeeze_excite = int(squeeze_excite)
        wp = (C.c_void_p * max(len(weight_ptrs), 1))(*[p or None for p in weight_ptrs])
        self._h = C.c_void_p()
        self._graph = graph
        _check(L.dnnf_plan_build(graph._h, C.byref(o), wp, stream or None, C.byref(self._h)))

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.lib().dnnf_plan_destroy(self._h)
            self._h = None

    def num_blocks(self) -> int:
        n = C.c_int()
        _check(_lib.lib().dnnf_plan_num_blocks(self._h, C.byref(n)))
        return n.value

    def block_info(self, b) -> Dict[str, object]:
        bi = BlockInfo()
        _check(_lib.lib().dnnf_plan_block_info(self._h, b, C.byref(bi)))
        d = {f: getattr(bi, f) for f, _ in BlockInfo._fields_}
        d["kernel_name"] = bi.kernel_name.decode()
        d["prepare_only"] = bi.n_kernel_launches < 0
        d["n_kernel_launches"] = abs(bi.n_kernel_launches)
        return d

    def block_ops(self, b) -> List[int]:
        n = C.c_int()
        _check(_lib.lib().dnnf_plan_block_ops(self._h, b, None, 0, C.byref(n)))
        arr = (C.c_int * max(n.value, 1))()
        _check(_lib.lib().dnnf_plan_block_ops(self._h, b, arr, n.value, C.byref(n)))
        return list(arr[:n.value])

    def block_source(self, b) -> str:
        need = C.c_size_t()
        _check(_lib.lib().dnnf_plan_block_source(self._h, b, None, 0, C.byref(need)))
        buf = C.create_string_buffer(need.value + 1)
        _check(_lib.lib().dnnf_plan_block_source(self._h, b, buf, need.value + 1, C.byref(need)))
        return buf.value.decode()

    def dump_json(self) -> dict:
        import json
        need = C.c_size_t()
        _check(_lib.lib().dnnf_plan_dump_json(self._h, None, 0, C.byref(need)))
        buf = C.create_string_buffer(need.value + 1)
        _check(_lib.lib().dnnf_plan_dump_json(self._h, buf, need.value + 1, C.byref(need)))
        return json.loads(buf.value.decode())

    def precompile(self):
        _check(_lib.lib().dnnf_plan_precompile(self._h))

    def workspace_bytes(self) -> int:
        n = C.c_size_t()
        _check(_lib.lib().dnnf_plan_workspace_bytes(self._h, C.byref(n)))
        return n.value

    @staticmethod
    def _ptrs(ps):
        return (C.c_void_p * max(len(ps), 1))(*[p or None for p in ps])

    def prepare(self, workspace: int, stream: int = 0):
        _check(_lib.lib().dnnf_plan_prepare(self._h, workspace or None, stream or None))

    def run(self, inputs, outputs, workspace: int, stream: int = 0):
        _check(_lib.lib().dnnf_plan_run(self._h, self._ptrs(inputs), self._ptrs(outputs), workspace or None, stream or None))

    def run_static(self, inputs, outputs, stream: int = 0):
        _check(_lib.lib().dnnf_plan_run_static(self._h, self._ptrs(inputs), self._ptrs(outputs), stream or None))

    def run_block(self, b, inputs, outputs, workspace: int, stream: int = 0):
        _check(_lib.lib().dnnf_plan_run_block(self._h, b, self._ptrs(inputs), self._ptrs(outputs), workspace or None, stream or None))

    def time_block(self, b, inputs, outputs, workspace: int, stream: int = 0, warmup=3, iters=20) -> float:
        us = C.c_double()
        _check(_lib.lib().dnnf_plan_time_block(self._h, b, self._ptrs(inputs), self._ptrs(outputs), workspace or None,
                                               stream or None, warmup, iters, C.byref(us)))
        return us.value

    def op_kind(self, op_id) -> str:
        buf = C.create_string_buffer(64)
        _check(_lib.lib().dnnf_plan_op_kind(self._h, op_id, buf, 64))
        return buf.value.decode()

    def describe(self) -> List[Dict[str, object]]:
        out = []
        for b in range(self.num_blocks()):
            d = self.block_info(b)
            d["ops"] = [self.op_kind(i) for i in self.block_ops(b)]
            out.append(d)
        return out


def precompile_spec(spec, fusion=1, rewrite=True, cache_dir=None, tune=0, attention=0, layout=0, broadcast_prologue=0, gemm_norm=0, squeeze_excite=0) -> int:
    """Host-only: build the plan for `spec` (no profiling) and compile its kernels into cache_dir."""
    g, _ = graph_from_spec(spec)
    if rewrite:
        g.rewrite()
    nw = len([t for t in spec.tensors.values() if t.kind == "weight"])
    p = Plan(g, [1] * nw, fusion=fusion, profile=0, cache_dir=cache_dir, tune=tune, attention=attention, layout=layout,
             broadcast_prologue=broadcast_prologue, gemm_norm=gemm_norm, squeeze_excite=squeeze_excite)   # pointers are never dereferenced here
    p.precompile()
    return p.num_blocks()


class Session:
    """Owns device tensors (torch) for one workload and drives a Plan over them."""

    def __init__(self, spec, fusion=1, rewrite=True, profile=0, intra_block=1, device="cuda:0", cache_dir="default",
                 verbose=0, n_buffer_sets=1, tune=0, attention=0, layout=0, graphs=0, broadcast_prologue=0, guard_bytes=0,
                 gemm_norm=0, squeeze_excite=0):
        """guard_bytes > 0 surrounds every output buffer and the workspace with that many bytes of a fixed pattern
        (a multiple of 256, so the buffers keep their alignment); guards_intact() tells whether any kernel wrote there."""
        import torch

        self.torch = torch
        self.spec = spec
        self.device = torch.device(device)
        self.guard_bytes = int(guard_bytes)
        assert self.guard_bytes % 256 == 0
        self._guards = []
        tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16, "i32": torch.int32, "i64": torch.int64, "bool": torch.bool}
        self.graph, self.ids = graph_from_spec(spec)
        self.rewrite_stats = self.graph.rewrite() if rewrite else None

        def up(t):
            a = t.data
            if t.dtype in ("i32", "i64", "bool"):
                return torch.from_numpy(np.ascontiguousarray(a)).to(tdt[t.dtype]).to(self.device)
            return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.device).to(tdt[t.dtype]).contiguous()

        self.weights = [up(t) for t in spec.tensors.values() if t.kind == "weight"]
        self.n_sets = n_buffer_sets
        self.inputs = [[up(t) for t in spec.tensors.values() if t.kind == "input"] for _ in range(n_buffer_sets)]
        self.out_specs = [t for t in spec.tensors.values() if t.kind == "output"]
        self.outputs = [[self._alloc(t.shape, tdt[t.dtype]) for t in self.out_specs] for _ in range(n_buffer_sets)]
        self.stream = torch.cuda.current_stream(self.device).cuda_stream
        scratch = None
        if profile:
            total = sum(int(np.prod(t.shape)) * 8 for t in spec.tensors.values())
            nbytes = int(min(max(total // 4, 1 << 26), 8 << 30))
            scratch = torch.zeros(nbytes, dtype=torch.uint8, device=self.device)
        if cache_dir == "default":
            from .build import CACHE
            cache_dir = CACHE
        self.plan = Plan(self.graph, [w.data_ptr() for w in self.weights], stream=self.stream, fusion=fusion, profile=profile,
                         intra_block=intra_block, profile_scratch=scratch.data_ptr() if scratch is not None else 0,
                         profile_scratch_bytes=scratch.numel() if scratch is not None else 0, cache_dir=cache_dir,
                         verbose=verbose, tune=tune, attention=attention, layout=layout, graphs=graphs,
                         broadcast_prologue=broadcast_prologue, gemm_norm=gemm_norm, squeeze_excite=squeeze_excite)
        del scratch
        self.workspace = self._alloc((max(self.plan.workspace_bytes(), 256),), torch.uint8)
        self.plan.prepare(self.workspace.data_ptr(), self.stream)

    GUARD_PATTERN = 0xA5

    def _alloc(self, shape, dtype):
        torch = self.torch
        n = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
        if not self.guard_bytes or n == 0:
            return torch.empty(shape, dtype=dtype, device=self.device)
        g = self.guard_bytes
        raw = torch.full((n + 2 * g,), self.GUARD_PATTERN, dtype=torch.uint8, device=self.device)
        self._guards.append((raw, n))
        return raw[g:g + n].view(dtype).view(tuple(shape))

    def guards_intact(self) -> bool:
        """True if no byte of the guard areas around the outputs and the workspace has changed."""
        self.torch.cuda.synchronize(self.device)
        g = self.guard_bytes
        return all(bool((raw[:g] == self.GUARD_PATTERN).all()) and bool((raw[g + n:] == self.GUARD_PATTERN).all())
                   for raw, n in self._guards)

    def in_ptrs(self, s=0):
        return [t.data_ptr() for t in self.inputs[s]]

    def out_ptrs(self, s=0):
        return [t.data_ptr() for t in self.outputs[s]]

    def run(self, s=0):
        self.plan.run(self.in_ptrs(s), self.out_ptrs(s), self.workspace.data_ptr(), self.stream)

    def result(self, s=0) -> Dict[str, np.ndarray]:
        self.torch.cuda.synchronize(self.device)
        return {t.name: o.to(self.torch.float64).cpu().numpy() for t, o in zip(self.out_specs, self.outputs[s])}
