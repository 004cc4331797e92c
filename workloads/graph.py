"""A neutral description of an operator graph: tensors, operators, attributes.

Plain data only.  The fp64 oracle interprets it; the GPU binding feeds it to the
C-ABI library call by call.  Operators are at the granularity of the ONNX
vocabulary the paper classifies (its Table 2); composite layers (LayerNorm,
GELU, channel shuffle, ...) appear only as their decompositions.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np

INPUT, WEIGHT, INTERMEDIATE, OUTPUT = "input", "weight", "intermediate", "output"


@dataclass
class TensorSpec:
    name: str
    dtype: str                 # "f32" | "f16" | "bf16" | "i32" | "i64"
    shape: tuple
    kind: str                  # input | weight | intermediate | output
    data: Optional[np.ndarray] = None   # inputs and weights: values already rounded to `dtype`
    const: bool = False        # small constant whose values the compiler may read on the host


@dataclass
class OpSpec:
    kind: str
    inputs: List[str]
    outputs: List[str]
    attrs: Dict[str, object] = field(default_factory=dict)


@dataclass
class GraphSpec:
    name: str
    dtype: str
    tensors: Dict[str, TensorSpec] = field(default_factory=dict)
    ops: List[OpSpec] = field(default_factory=list)
    meta: Dict[str, object] = field(default_factory=dict)

    def inputs(self):
        return [t for t in self.tensors.values() if t.kind == INPUT]

    def weights(self):
        return [t for t in self.tensors.values() if t.kind == WEIGHT]

    def outputs(self):
        return [t for t in self.tensors.values() if t.kind == OUTPUT]


class GraphBuilder:
    """Records tensors and operators; computes nothing."""

    def __init__(self, name: str, dtype: str):
        self.g = GraphSpec(name=name, dtype=dtype)
        self._n = 0

    # -- tensors ---------------------------------------------------------
    def _add(self, name, dtype, shape, kind, data=None, const=False):
        if name in self.g.tensors:
            raise ValueError(f"duplicate tensor {name}")
        shape = tuple(int(s) for s in shape)
        if data is not None:
            data = np.asarray(data, order="C")
            if tuple(data.shape) != shape:
                raise ValueError(f"{name}: data shape {data.shape} != {shape}")
        self.g.tensors[name] = TensorSpec(name, dtype, shape, kind, data, const)
        return name

    def input(self, name, shape, data, dtype=None):
        return self._add(name, dtype or self.g.dtype, shape, INPUT, data)

    def weight(self, name, shape, data, dtype=None):
        return self._add(name, dtype or self.g.dtype, shape, WEIGHT, data)

    def const(self, name, value, dtype=None, shape=()):
        """A small constant (scalar by default) that lives in the graph as a weight."""
        from .rng import round_to
        dtype = dtype or self.g.dtype
        arr = np.full(shape, value, dtype=np.float64) if np.isscalar(value) else np.asarray(value, dtype=np.float64)
        return self._add(name, dtype, arr.shape, WEIGHT, round_to(arr, dtype), const=True)

    def fresh(self, stem):
        self._n += 1
        return f"{stem}_{self._n}"

    # -- operators -------------------------------------------------------
    def op(self, kind, inputs: Sequence[str], out_shapes, attrs=None, out_names=None, out_dtype=None):
        """Append one operator; returns its output name (or list of names)."""
        single = not (isinstance(out_shapes, list))
        shapes = [out_shapes] if single else out_shapes
        names = []
        for i, s in enumerate(shapes):
            nm = out_names[i] if out_names else self.fresh(kind.lower())
            self._add(nm, out_dtype or self.g.dtype, s, INTERMEDIATE)
            names.append(nm)
        self.g.ops.append(OpSpec(kind, list(inputs), names, dict(attrs or {})))
        return names[0] if single else names

    def shape(self, name):
        return self.g.tensors[name].shape

    def mark_output(self, name):
        self.g.tensors[name].kind = OUTPUT

    def finish(self) -> GraphSpec:
        return self.g


def bcast_shape(a, b):
    r = max(len(a), len(b))
    a = (1,) * (r - len(a)) + tuple(a)
    b = (1,) * (r - len(b)) + tuple(b)
    out = []
    for x, y in zip(a, b):
        if x != y and x != 1 and y != 1:
            raise ValueError(f"cannot broadcast {a} with {b}")
        out.append(max(x, y))
    return tuple(out)
