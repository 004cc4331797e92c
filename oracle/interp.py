"""fp64 CPU oracle: evaluates the ORIGINAL operator graph one operator at a time.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this module;
only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg use it.
It shares no code with the HIP path.

What it computes: fusion and graph rewriting are result-preserving
transformations (paper Sec. 1, benefits (i)-(iii) concern materialisation and
scans only; Sec. 5 states model accuracy is identical across frameworks), so
the value of a fused plan is by definition the value of the un-rewritten,
unfused graph.  The oracle is that definition written out: every tensor is
float64, every operator is the textbook definition of the ONNX operator the
paper's Table 2 names, no blocking, no fusion, no reordering.  Inputs and
weights arrive already rounded to the storage type; nothing is rounded
afterwards.

Library primitives used as steps: numpy elementwise functions, numpy.einsum /
matmul for contractions, scipy.special.erf.  Each is pinned by tests against
closed forms, brute-force loops and invariants (tests/test_oracle_ops.py).
"""
from __future__ import annotations

import numpy as np
from scipy import special as _sp

F64 = np.float64


# ------------------------------------------------------------------ elementwise (One-to-One, Table 2)
def _clip(x, attrs):
    return np.minimum(np.maximum(x, attrs.get("min", -np.inf)), attrs.get("max", np.inf))


_UNARY = {
    "Relu": lambda x, a: np.maximum(x, 0.0),
    "Sigmoid": lambda x, a: 1.0 / (1.0 + np.exp(-x)),
    "Tanh": lambda x, a: np.tanh(x),
    "Exp": lambda x, a: np.exp(x),
    "Log": lambda x, a: np.log(x),
    "Sqrt": lambda x, a: np.sqrt(x),
    "Abs": lambda x, a: np.abs(x),
    "Neg": lambda x, a: -x,
    "Reciprocal": lambda x, a: 1.0 / x,
    "Erf": lambda x, a: _sp.erf(x),
    "Square": lambda x, a: x * x,
    "Clip": _clip,
    "LeakyRelu": lambda x, a: np.where(x >= 0, x, a.get("alpha", 0.01) * x),
    "Identity": lambda x, a: x,
    "Floor": lambda x, a: np.floor(x),
    "Ceil": lambda x, a: np.ceil(x),
    "Round": lambda x, a: np.rint(x),          # halves to the nearest even integer
    "Not": lambda x, a: (x == 0).astype(F64),          # truth values are 0 / 1 numbers here, as Greater produces them
    "Sin": lambda x, a: np.sin(x),
    "Cos": lambda x, a: np.cos(x),
    "Asin": lambda x, a: np.arcsin(x),
    "Cast": lambda x, a: x,   # value-preserving between float types inside an fp64 evaluation
}

_BINARY = {
    "Add": np.add, "Sub": np.subtract, "Mul": np.multiply, "Div": np.divide,
    "Pow": np.power, "Max": np.maximum, "Min": np.minimum,
    "PRelu": lambda x, slope: np.where(x >= 0, x, slope * x),
    # integer left shift (the direction for which Table 4's ReduceSum/BitShift swap is exact)
    "BitShift": lambda a, b: np.left_shift(a.astype(np.int64), b.astype(np.int64)),
}


def batch_norm(x, gamma, beta, mean, var, eps):
    """Inference BatchNormalization over axis 1: gamma*(x-mean)/sqrt(var+eps)+beta."""
    sh = (1, -1) + (1,) * (x.ndim - 2)
    return gamma.reshape(sh) * (x - mean.reshape(sh)) / np.sqrt(var.reshape(sh) + eps) + beta.reshape(sh)


# ------------------------------------------------------------------ Many-to-Many (Table 2)
def conv2d(x, w, bias, strides, pads, group):
    """Direct 2-D cross-correlation, NCHW / OIHW, zero padding, groups.

    out[n,o,p,q] = bias[o] + sum_{c,i,j} x[n, g(o)*Cg + c, p*sh + i - pt, q*sw + j - pl] * w[o,c,i,j]
    """
    n, c, h, wd = x.shape
    co, cg, kh, kw = w.shape
    sh, sw = strides
    pt, pl, pb, pr = pads
    assert cg * group == c and co % group == 0
    ho = (h + pt + pb - kh) // sh + 1
    wo = (wd + pl + pr - kw) // sw + 1
    xp = np.zeros((n, c, h + pt + pb, wd + pl + pr), dtype=F64)
    xp[:, :, pt:pt + h, pl:pl + wd] = x
    out = np.zeros((n, co, ho, wo), dtype=F64)
    og = co // group
    for i in range(kh):
        for j in range(kw):
            xs = xp[:, :, i:i + sh * (ho - 1) + 1:sh, j:j + sw * (wo - 1) + 1:sw]
            if group == 1:
                out += np.einsum("nchw,oc->nohw", xs, w[:, :, i, j])
            elif cg == 1 and og == 1:
                out += xs * w[:, 0, i, j].reshape(1, -1, 1, 1)
            else:
                for g in range(group):
                    out[:, g * og:(g + 1) * og] += np.einsum(
                        "nchw,oc->nohw", xs[:, g * cg:(g + 1) * cg], w[g * og:(g + 1) * og, :, i, j])
    if bias is not None:
        out += bias.reshape(1, -1, 1, 1)
    return out


def softmax(x, axis):
    """exp(x - max) / sum exp(x - max) along `axis`."""
    m = np.max(x, axis=axis, keepdims=True)
    e = np.exp(x - m)
    return e / np.sum(e, axis=axis, keepdims=True)


def conv3d(x, w, bias, strides, pads):
    """Direct 3-d cross-correlation, NCDHW / OIDHW, zero padding, group 1.

    out[n,o,d,p,q] = bias[o] + sum_{c,a,i,j} x[n, c, d*sd + a - pf, p*sh + i - pt, q*sw + j - pl] * w[o,c,a,i,j]
    """
    n, c, dd, h, wd = x.shape
    co, ci, kd, kh, kw = w.shape
    assert ci == c
    sd, sh, sw = (int(v) for v in strides)
    pf, pt, pl, pb_, pbt, pr = (int(v) for v in pads)
    do = (dd + pf + pb_ - kd) // sd + 1
    ho = (h + pt + pbt - kh) // sh + 1
    wo = (wd + pl + pr - kw) // sw + 1
    xp = np.zeros((n, c, dd + pf + pb_, h + pt + pbt, wd + pl + pr), dtype=F64)
    xp[:, :, pf:pf + dd, pt:pt + h, pl:pl + wd] = x
    out = np.zeros((n, co, do, ho, wo), dtype=F64)
    for a in range(kd):
        for i in range(kh):
            for j in range(kw):
                xs = xp[:, :, a:a + sd * (do - 1) + 1:sd, i:i + sh * (ho - 1) + 1:sh, j:j + sw * (wo - 1) + 1:sw]
                out += np.einsum("ncdhw,oc->nodhw", xs, w[:, :, a, i, j])
    if bias is not None:
        out += bias.reshape(1, -1, 1, 1, 1)
    return out


def conv_transpose2d(x, w, bias, strides, pads, output_padding):
    """Transposed 2-d convolution, NCHW input, [C, CO, KH, KW] filter, group 1, in its scatter form: every input
    element adds x[n, c, h, w] * w[c, o, i, j] to out[n, o, h*sh + i - pad_top, w*sw + j - pad_left]; the result
    has (H - 1)*sh - pad_top - pad_bottom + KH + output_padding rows (columns likewise)."""
    n, c, h, wd = x.shape
    ci, co, kh, kw = w.shape
    assert ci == c
    sh, sw = (int(v) for v in strides)
    pt, pl, pb, pr = (int(v) for v in pads)
    oph, opw = (int(v) for v in output_padding)
    ho = (h - 1) * sh - pt - pb + kh + oph
    wo = (wd - 1) * sw - pl - pr + kw + opw
    full = np.zeros((n, co, (h - 1) * sh + kh + oph, (wd - 1) * sw + kw + opw), dtype=F64)
    for i in range(kh):
        for j in range(kw):
            full[:, :, i:i + sh * (h - 1) + 1:sh, j:j + sw * (wd - 1) + 1:sw] += np.einsum("nchw,co->nohw", x, w[:, :, i, j])
    out = full[:, :, pt:pt + ho, pl:pl + wo].copy()
    if bias is not None:
        out += bias.reshape(1, -1, 1, 1)
    return out


def einsum(equation, a, b):
    """Two-operand Einsum (a Many-to-Many operator of Table 2) by its definition: the result element at an
    assignment of the result's labels is the sum, over every assignment of the remaining labels, of the product of
    the two operand elements those labels select.  Written as broadcasting: each operand is laid out over the full
    label space (size-1 axes where it lacks a label), the product is formed, and the labels absent from the result
    are summed."""
    lhs, out = equation.replace(" ", "").split("->")
    ta, tb = lhs.split(",")
    labels = sorted(set(ta) | set(tb))

    def spread(x, term):
        x = np.asarray(x, dtype=F64)
        assert x.ndim == len(term) and len(set(term)) == len(term), (equation, x.shape)
        x = np.transpose(x, [term.index(l) for l in labels if l in term])      # the term's labels in the common order
        dims = iter(x.shape)
        return x.reshape([next(dims) if l in term else 1 for l in labels])

    prod = spread(a, ta) * spread(b, tb)
    summed = tuple(i for i, l in enumerate(labels) if l not in out)
    res = prod.sum(axis=summed) if summed else prod
    rest = [l for l in labels if l in out]
    return np.transpose(res, [rest.index(l) for l in out])


def cumsum(x, axis, exclusive=False, reverse=False):
    """CumSum (a Many-to-Many operator of Table 2; the definition of a prefix sum): out[.., i, ..] = sum of
    x[.., j, ..] over j <= i along `axis`; `exclusive` leaves x[i] itself out (j < i), `reverse` sums from the
    far end (j >= i, resp. j > i)."""
    x = np.asarray(x)
    axis = axis % x.ndim
    out = np.empty_like(x)
    n = x.shape[axis]
    run = np.zeros(x.shape[:axis] + x.shape[axis + 1:], dtype=x.dtype)
    sel = [slice(None)] * x.ndim
    for step in range(n):
        i = n - 1 - step if reverse else step
        sel[axis] = i
        if exclusive:
            out[tuple(sel)] = run
            run = run + x[tuple(sel)]
        else:
            run = run + x[tuple(sel)]
            out[tuple(sel)] = run
    return out


def pool2d(x, kind, kernel, strides, pads, count_include_pad=False):
    """MaxPool / AveragePool over a 2-d window of an NCHW tensor (Table 2 operators; textbook definition):
    out[n, c, p, q] = max resp. mean of x[n, c, p * sh + i - pad_top, q * sw + j - pad_left] over the window
    positions (i, j) that fall inside the map; the mean divides by the number of such positions unless
    count_include_pad, which divides by the window size (padding counted as zeros)."""
    n, c, h, w = x.shape
    kh, kw = (int(v) for v in kernel)
    sh, sw = (int(v) for v in strides)
    pt, pl, pb, pr = (int(v) for v in pads)
    ho = (h + pt + pb - kh) // sh + 1
    wo = (w + pl + pr - kw) // sw + 1
    out = np.empty((n, c, ho, wo), dtype=F64)
    for p in range(ho):
        h0, h1 = max(p * sh - pt, 0), min(p * sh - pt + kh, h)
        for q in range(wo):
            w0, w1 = max(q * sw - pl, 0), min(q * sw - pl + kw, w)
            win = x[:, :, h0:h1, w0:w1]
            if kind == "MaxPool":
                out[:, :, p, q] = np.max(win, axis=(2, 3))
            else:
                denom = kh * kw if count_include_pad else (h1 - h0) * (w1 - w0)
                out[:, :, p, q] = np.sum(win, axis=(2, 3)) / denom
    return out


def _reduce(fn, x, attrs):
    axes = tuple(int(a) % x.ndim for a in attrs["axes"])
    return fn(x, axis=axes, keepdims=bool(attrs.get("keepdims", 1)))


# ------------------------------------------------------------------ index-only operators
def _slice(x, attrs):
    sl = [slice(None)] * x.ndim
    steps = attrs.get("steps", [1] * len(attrs["axes"]))
    for ax, s, e, st in zip(attrs["axes"], attrs["starts"], attrs["ends"], steps):
        sl[int(ax) % x.ndim] = slice(int(s), int(e), int(st))
    return x[tuple(sl)]


def _split(x, attrs):
    ax = int(attrs["axis"]) % x.ndim
    pts = np.cumsum(attrs["split"])[:-1]
    return np.split(x, pts, axis=ax)


def eval_op(kind, ins, attrs):
    """Value(s) of one operator given its fp64 (or integer index) operands."""
    if kind in _UNARY:
        return _UNARY[kind](ins[0], attrs)
    if kind == "BitShift" and int(attrs.get("direction_right", 0)):
        # the other direction of the integer shift (Table 2 lists the operator; the direction is its attribute)
        return np.right_shift(np.asarray(ins[0]).astype(np.int64), np.asarray(ins[1]).astype(np.int64))
    if kind in _BINARY:
        return _BINARY[kind](ins[0], ins[1])
    if kind == "Where":
        return np.where(ins[0] != 0, ins[1], ins[2])
    if kind == "Greater":
        return (ins[0] > ins[1]).astype(F64)
    if kind == "BatchNormalization":
        return batch_norm(*ins, float(attrs.get("epsilon", 1e-5)))
    if kind == "Conv" and ins[0].ndim == 5:
        return conv3d(ins[0], ins[1], ins[2] if len(ins) > 2 else None, attrs.get("strides", [1, 1, 1]), attrs.get("pads", [0] * 6))
    if kind == "Conv":
        return conv2d(ins[0], ins[1], ins[2] if len(ins) > 2 else None,
                      attrs.get("strides", [1, 1]), attrs.get("pads", [0, 0, 0, 0]), int(attrs.get("group", 1)))
    if kind == "ConvTranspose":
        return conv_transpose2d(ins[0], ins[1], ins[2] if len(ins) > 2 else None, attrs.get("strides", [1, 1]),
                                attrs.get("pads", [0, 0, 0, 0]), attrs.get("output_padding", [0, 0]))
    if kind == "MatMul":
        return np.matmul(ins[0], ins[1])
    if kind == "Gemm":
        a = ins[0].T if attrs.get("transA", 0) else ins[0]
        b = ins[1].T if attrs.get("transB", 0) else ins[1]
        y = attrs.get("alpha", 1.0) * (a @ b)
        return y + attrs.get("beta", 1.0) * ins[2] if len(ins) > 2 else y
    if kind == "ReduceMean":
        return _reduce(np.mean, ins[0], attrs)
    if kind == "ReduceSum":
        return _reduce(np.sum, ins[0], attrs)
    if kind == "ReduceMax":
        return _reduce(np.max, ins[0], attrs)
    if kind == "ReduceProd":
        return _reduce(np.prod, ins[0], attrs)
    if kind == "Softmax":
        return softmax(ins[0], int(attrs.get("axis", -1)))
    if kind == "Normalize":
        # not an ONNX operator: the name the library gives to the LayerNorm statistics chain
        # ReduceMean, Sub, Pow 2, ReduceMean, Add eps, Sqrt, Div over the last axis.  Written as that chain.
        x = ins[0]
        d = x - np.mean(x, axis=-1, keepdims=True)
        return d / np.sqrt(np.mean(d * d, axis=-1, keepdims=True) + float(attrs.get("epsilon", 1e-5)))
    if kind == "GlobalAveragePool":
        return np.mean(ins[0], axis=tuple(range(2, ins[0].ndim)), keepdims=True)
    if kind == "InstanceNormalization":
        # per (n, c): (x - mean) / sqrt(var + eps) over the axes behind the channel axis, then scale[c], bias[c]
        x = ins[0]
        ax = tuple(range(2, x.ndim))
        d = x - np.mean(x, axis=ax, keepdims=True)
        sh = (1, -1) + (1,) * (x.ndim - 2)
        return d / np.sqrt(np.mean(d * d, axis=ax, keepdims=True) + float(attrs.get("epsilon", 1e-5))) * ins[1].reshape(sh) + ins[2].reshape(sh)
    if kind in ("DepthToSpace", "SpaceToDepth"):
        # element by element from the operators' index definition (block size b):
        #   DepthToSpace, depth-column-row: y[n, c, h*b + i, w*b + j] = x[n, (i*b + j)*C' + c, h, w]
        #   DepthToSpace, column-row-depth: y[n, c, h*b + i, w*b + j] = x[n, c*b*b + i*b + j, h, w]
        #   SpaceToDepth:                   y[n, (i*b + j)*C + c, h, w] = x[n, c, h*b + i, w*b + j]
        x = ins[0]
        b = int(attrs["blocksize"])
        n, c, h, w = x.shape
        if kind == "DepthToSpace":
            cp = c // (b * b)
            y = np.empty((n, cp, h * b, w * b), dtype=x.dtype)
            for i in range(b):
                for j in range(b):
                    for cc in range(cp):
                        src = cc * b * b + i * b + j if int(attrs.get("mode_crd", 0)) else (i * b + j) * cp + cc
                        y[:, cc, i::b, j::b] = x[:, src, :, :]
            return y
        y = np.empty((n, c * b * b, h // b, w // b), dtype=x.dtype)
        for i in range(b):
            for j in range(b):
                for cc in range(c):
                    y[:, (i * b + j) * c + cc, :, :] = x[:, cc, i::b, j::b]
        return y
    if kind == "Einsum":
        return einsum(attrs["equation"], ins[0], ins[1])
    if kind == "CumSum":
        return cumsum(ins[0], int(attrs.get("axis", 0)), bool(attrs.get("exclusive", 0)), bool(attrs.get("reverse", 0)))
    if kind in ("MaxPool", "AveragePool"):
        return pool2d(ins[0], kind, attrs["kernel_shape"], attrs.get("strides", [1, 1]), attrs.get("pads", [0, 0, 0, 0]),
                      bool(attrs.get("count_include_pad", 0)))
    if kind == "Gather":
        return np.take(ins[0], ins[1].astype(np.int64), axis=int(attrs.get("axis", 0)))
    if kind == "Unsqueeze" and "axes" in attrs:
        # axes name positions in the RESULT that become extent-1 dimensions; the element order is untouched
        y = ins[0]
        for ax in sorted(int(a) % (y.ndim + len(attrs["axes"])) for a in attrs["axes"]):
            y = np.expand_dims(y, ax)
        return y
    if kind == "Squeeze" and "axes" in attrs:
        return np.squeeze(ins[0], axis=tuple(int(a) % ins[0].ndim for a in attrs["axes"]))
    if kind in ("Reshape", "Flatten", "Squeeze", "Unsqueeze"):
        return ins[0].reshape(attrs["shape"]) if "shape" in attrs else ins[0].reshape(attrs["out_shape"])
    if kind == "Transpose":
        return np.transpose(ins[0], attrs["perm"])
    if kind == "Slice":
        return _slice(ins[0], attrs)
    if kind == "Split":
        return _split(ins[0], attrs)
    if kind == "Concat":
        return np.concatenate(ins, axis=int(attrs["axis"]))
    if kind == "Expand":
        return np.broadcast_to(ins[0], attrs["shape"]).copy()
    if kind in ("Resize", "Upsample"):
        # nearest neighbour, integer factors: out[i] = in[floor(i / s)] along every axis
        y = ins[0]
        for ax, sc in enumerate(attrs["scales"]):
            if int(sc) != 1:
                y = np.repeat(y, int(sc), axis=ax)
        return y
    raise NotImplementedError(f"oracle: operator {kind}")


def run_graph(spec, feeds=None, keep=None):
    """Evaluate `spec` (a workloads.graph.GraphSpec-shaped object) operator by operator.

    feeds: optional {input name: array} overriding the recorded input data.
    keep:  None -> return graph outputs only; "all" -> every tensor; or an iterable of names.
    Returns {name: float64 ndarray}.
    """
    env = {}
    for t in spec.tensors.values():
        if t.kind in ("input", "weight"):
            src = feeds[t.name] if feeds and t.name in feeds else t.data
            if src is None:
                raise ValueError(f"no data for {t.name}")
            env[t.name] = np.asarray(src).astype(np.int64 if t.dtype in ("i32", "i64") else F64)
    outs = {t.name for t in spec.tensors.values() if t.kind == "output"}
    want = set(spec.tensors) if keep == "all" else outs | set(keep or ())
    uses = {}
    for op in spec.ops:
        for i in op.inputs:
            uses[i] = uses.get(i, 0) + 1
    for op in spec.ops:
        res = eval_op(op.kind, [env[i] for i in op.inputs], op.attrs)
        res = res if isinstance(res, (list, tuple)) else [res]
        assert len(res) == len(op.outputs), op.kind
        for nm, val in zip(op.outputs, res):
            val = np.asarray(val, dtype=F64)
            assert tuple(val.shape) == tuple(spec.tensors[nm].shape), (op.kind, nm, val.shape, spec.tensors[nm].shape)
            env[nm] = val
        for i in op.inputs:
            uses[i] -= 1
            if uses[i] == 0 and i not in want and spec.tensors[i].kind == "intermediate":
                env.pop(i, None)
    return {k: env[k] for k in want if k in env}
