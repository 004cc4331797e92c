"""The five synthetic workloads (graph + seeded inputs/weights).

Each builder returns a GraphSpec at ONNX-operator granularity.  Sizes default to
the full benchmark configuration; every builder takes keyword overrides so the
same recipe can be instantiated small enough for the fp64 oracle to run in
seconds.  The graphs stand in for the paper's trained models (its Tables 5/6:
EfficientNet-B0, BERT-like encoders, GPT-2): latency does not depend on the
values, so seeded random weights of the published layer shapes are used.

Nothing here evaluates the graph: values are drawn, rounded once to the
storage type, and recorded.
"""
from __future__ import annotations

import math

import numpy as np

from . import rng
from .graph import GraphBuilder, bcast_shape

BASE_SEED = 210813342


class _Streams:
    """Hands out one RNG stream id per tensor, in creation order."""

    def __init__(self, seed):
        self.seed = seed
        self.k = 0

    def normal(self, shape, mean=0.0, std=1.0, dtype="f32"):
        self.k += 1
        return rng.round_to(rng.normal(self.seed, self.k, shape, mean, std), dtype)

    def uniform(self, shape, lo, hi, dtype="f32"):
        self.k += 1
        return rng.round_to(rng.uniform(self.seed, self.k, shape, lo, hi), dtype)

    def integers(self, shape, lo, hi):
        self.k += 1
        return rng.integers(self.seed, self.k, shape, lo, hi)


# ---------------------------------------------------------------- helpers
def _bin(b, kind, x, y):
    return b.op(kind, [x, y], bcast_shape(b.shape(x), b.shape(y)))


def _un(b, kind, x, attrs=None):
    return b.op(kind, [x], b.shape(x), attrs)


def _matmul(b, x, w):
    sx, sw = b.shape(x), b.shape(w)
    assert sx[-1] == sw[-2], (sx, sw)
    batch = bcast_shape(sx[:-2], sw[:-2])
    return b.op("MatMul", [x, w], batch + (sx[-2], sw[-1]))


def _reshape(b, x, shape):
    assert int(np.prod(shape)) == int(np.prod(b.shape(x)))
    return b.op("Reshape", [x], tuple(shape), {"shape": [int(s) for s in shape]})


def _transpose(b, x, perm):
    s = b.shape(x)
    return b.op("Transpose", [x], tuple(s[p] for p in perm), {"perm": [int(p) for p in perm]})


def _reduce(b, kind, x, axes, keepdims=1):
    s = list(b.shape(x))
    axes = [a % len(s) for a in axes]
    out = [1 if i in axes else d for i, d in enumerate(s)] if keepdims else [d for i, d in enumerate(s) if i not in axes]
    return b.op(kind, [x], tuple(out), {"axes": axes, "keepdims": int(keepdims)})


def _conv(b, x, w, bias, stride, pad, group=1):
    n, c, h, wd = b.shape(x)
    co, cig, kh, kw = b.shape(w)
    assert cig * group == c, (b.shape(x), b.shape(w), group)
    ho = (h + 2 * pad - kh) // stride + 1
    wo = (wd + 2 * pad - kw) // stride + 1
    ins = [x, w] + ([bias] if bias else [])
    return b.op("Conv", ins, (n, co, ho, wo),
                {"strides": [stride, stride], "pads": [pad, pad, pad, pad], "group": group})


def _layernorm(b, st, x, width, dtype, tag, eps=1e-5, affine_std=0.02):
    """LayerNorm over the last axis as the usual exporter decomposition (9 ops)."""
    g = b.weight(f"{tag}_gamma", (width,), st.normal((width,), 1.0, affine_std, dtype), dtype)
    be = b.weight(f"{tag}_beta", (width,), st.normal((width,), 0.0, affine_std, dtype), dtype)
    two = b.const(f"{tag}_two", 2.0, dtype=dtype)
    epsc = b.const(f"{tag}_eps", eps)
    mu = _reduce(b, "ReduceMean", x, [-1])
    d = _bin(b, "Sub", x, mu)
    if b.g.dtype != dtype:       # the fp32 region of a 16-bit export: the exponent constant is cast like the operand
        two = b.op("Cast", [two], (), {"to": 1})
    sq = _bin(b, "Pow", d, two)
    var = _reduce(b, "ReduceMean", sq, [-1])
    ve = _bin(b, "Add", var, epsc)
    sd = _un(b, "Sqrt", ve)
    nrm = _bin(b, "Div", d, sd)
    sc = _bin(b, "Mul", nrm, g)
    return _bin(b, "Add", sc, be)


def _gelu_erf(b, x, tag):
    """0.5 * x * (1 + erf(x / sqrt(2))) as five operators."""
    r2 = b.const(f"{tag}_sqrt2", math.sqrt(2.0))
    one = b.const(f"{tag}_one", 1.0)
    half = b.const(f"{tag}_half", 0.5)
    t = _bin(b, "Div", x, r2)
    t = _un(b, "Erf", t)
    t = _bin(b, "Add", t, one)
    t = _bin(b, "Mul", x, t)
    return _bin(b, "Mul", t, half)


def _gelu_tanh(b, x, tag, pow_in_fp32=False):
    """0.5 * x * (1 + tanh(sqrt(2/pi) * (x + 0.044715 x^3))) as eight operators (ten with the Cast pair a 16-bit
    export puts around Pow)."""
    three = b.const(f"{tag}_three", 3.0)
    c0 = b.const(f"{tag}_c0", 0.044715)
    c1 = b.const(f"{tag}_c1", math.sqrt(2.0 / math.pi))
    one = b.const(f"{tag}_one", 1.0)
    half = b.const(f"{tag}_half", 0.5)
    if pow_in_fp32:
        t = b.op("Cast", [x], b.shape(x), {"to": 1}, out_dtype="f32")
        t = b.op("Pow", [t, b.op("Cast", [three], (), {"to": 1}, out_dtype="f32")], b.shape(x), out_dtype="f32")
        t = b.op("Cast", [t], b.shape(x), {"to": 16})
    else:
        t = _bin(b, "Pow", x, three)
    t = _bin(b, "Mul", t, c0)
    t = _bin(b, "Add", x, t)
    t = _bin(b, "Mul", t, c1)
    t = _un(b, "Tanh", t)
    t = _bin(b, "Add", t, one)
    t = _bin(b, "Mul", x, t)
    return _bin(b, "Mul", t, half)


def _swish(b, x):
    return _bin(b, "Mul", x, _un(b, "Sigmoid", x))


# ---------------------------------------------------------------- config 1
def residual_block(N=1, C=64, H=56, W=56, K=3, seed=BASE_SEED + 1):
    """conv KxK (stride 1, same padding) -> BatchNormalization -> Relu -> Add identity -> Relu, fp32."""
    st = _Streams(seed)
    b = GraphBuilder("residual_block", "f32")
    x = b.input("x", (N, C, H, W), st.normal((N, C, H, W)))
    w = b.weight("conv_w", (C, C, K, K), st.normal((C, C, K, K), 0.0, math.sqrt(2.0 / (C * K * K))))
    gamma = b.weight("bn_gamma", (C,), st.uniform((C,), 0.5, 1.5))
    beta = b.weight("bn_beta", (C,), st.normal((C,), 0.0, 0.1))
    mean = b.weight("bn_mean", (C,), st.normal((C,), 0.0, 0.1))
    var = b.weight("bn_var", (C,), st.uniform((C,), 0.5, 1.5))
    y = _conv(b, x, w, None, 1, K // 2)
    y = b.op("BatchNormalization", [y, gamma, beta, mean, var], b.shape(y), {"epsilon": 1e-5})
    y = _un(b, "Relu", y)
    y = _bin(b, "Add", y, x)
    y = _un(b, "Relu", y)
    b.mark_output(y)
    return b.finish()


# ---------------------------------------------------------------- config 2
def memory_bound_chain(N=16, C=256, H=64, W=64, groups=8, rounds=3, seed=BASE_SEED + 2):
    """rounds x 8 One-to-One layers, then NCHW->NHWC, reshape, channel shuffle; fp32.

    One round = add c1, mul c2 (per-channel constants), exp(clip(x,-4,4)), sigmoid, tanh,
    GELU (erf form), square, sqrt(|x|+1): 8 layers = 15 ONNX-granularity operators.
    """
    st = _Streams(seed)
    b = GraphBuilder("memory_bound_chain", "f32")
    x = b.input("x", (N, C, H, W), st.normal((N, C, H, W)))
    y = x
    for r in range(rounds):
        c1 = b.weight(f"r{r}_c1", (1, C, 1, 1), st.uniform((1, C, 1, 1), -1.0, 1.0))
        c2 = b.weight(f"r{r}_c2", (1, C, 1, 1), st.uniform((1, C, 1, 1), -1.0, 1.0))
        y = _bin(b, "Add", y, c1)
        y = _bin(b, "Mul", y, c2)
        y = _un(b, "Clip", y, {"min": -4.0, "max": 4.0})
        y = _un(b, "Exp", y)
        y = _un(b, "Sigmoid", y)
        y = _un(b, "Tanh", y)
        y = _gelu_erf(b, y, f"r{r}_gelu")
        y = _bin(b, "Pow", y, b.const(f"r{r}_two", 2.0))
        y = _un(b, "Abs", y)
        y = _bin(b, "Add", y, b.const(f"r{r}_one", 1.0))
        y = _un(b, "Sqrt", y)
    y = _transpose(b, y, (0, 2, 3, 1))                       # NCHW -> NHWC
    y = _reshape(b, y, (N, H * W, C))
    y = _reshape(b, y, (N, H * W, groups, C // groups))     # channel shuffle
    y = _transpose(b, y, (0, 1, 3, 2))
    y = _reshape(b, y, (N, H * W, C))
    b.mark_output(y)
    g = b.finish()
    g.meta.update(layers=8 * rounds, elements=N * C * H * W)
    return g


# ---------------------------------------------------------------- config 3
def transformer_encoder_layer(B=8, S=384, D=768, NH=12, F=3072, dtype="f16", seed=BASE_SEED + 3):
    """Post-LayerNorm encoder layer (BERT-base shaped), 16-bit storage."""
    st = _Streams(seed)
    b = GraphBuilder("transformer_encoder_layer", dtype)
    hd = D // NH
    x = b.input("x", (B, S, D), st.normal((B, S, D), dtype=dtype))
    nmask = int(math.floor(0.1 * S))
    mvals = np.zeros((B, 1, 1, S), dtype=np.float32)
    mvals[..., S - nmask:] = -1e4
    mask = b.weight("attn_mask", (B, 1, 1, S), rng.round_to(mvals.astype(np.float64), dtype))

    def lin(name, inp, k, n):
        w = b.weight(f"{name}_w", (k, n), st.normal((k, n), 0.0, 0.02, dtype))
        bias = b.weight(f"{name}_b", (n,), st.normal((n,), 0.0, 0.02, dtype))
        return _bin(b, "Add", _matmul(b, inp, w), bias)

    qkv = lin("qkv", x, D, 3 * D)
    q, k, v = b.op("Split", [qkv], [(B, S, D)] * 3, {"axis": 2, "split": [D, D, D]})
    q = _transpose(b, _reshape(b, q, (B, S, NH, hd)), (0, 2, 1, 3))
    k = _transpose(b, _reshape(b, k, (B, S, NH, hd)), (0, 2, 3, 1))
    v = _transpose(b, _reshape(b, v, (B, S, NH, hd)), (0, 2, 1, 3))
    s = _matmul(b, q, k)
    s = _bin(b, "Mul", s, b.const("attn_scale", 1.0 / math.sqrt(hd)))
    s = _bin(b, "Add", s, mask)
    p = b.op("Softmax", [s], b.shape(s), {"axis": -1})
    o = _matmul(b, p, v)
    o = _reshape(b, _transpose(b, o, (0, 2, 1, 3)), (B, S, D))
    o = lin("attn_out", o, D, D)
    h = _bin(b, "Add", o, x)
    h = _layernorm(b, st, h, D, dtype, "ln1")
    f = lin("ffn1", h, D, F)
    f = _gelu_erf(b, f, "ffn_gelu")
    f = lin("ffn2", f, F, D)
    y = _bin(b, "Add", f, h)
    y = _layernorm(b, st, y, D, dtype, "ln2")
    b.mark_output(y)
    return b.finish()


# ---------------------------------------------------------------- config 4
EFFNET_B0_STAGES = [  # (expand, kernel, out channels, repeats, first stride)
    (1, 3, 16, 1, 1), (6, 3, 24, 2, 2), (6, 5, 40, 2, 2), (6, 3, 80, 3, 2),
    (6, 5, 112, 3, 1), (6, 5, 192, 4, 2), (6, 3, 320, 1, 1)]


def efficientnet_b0(N=32, R=224, stages=None, stem=32, dtype="f16", seed=BASE_SEED + 4):
    """Stem + MBConv blocks with squeeze-excite; BatchNorm already folded into conv weight + bias."""
    st = _Streams(seed)
    b = GraphBuilder("efficientnet_b0", dtype)
    stages = EFFNET_B0_STAGES if stages is None else stages
    x = b.input("x", (N, 3, R, R), st.normal((N, 3, R, R), dtype=dtype))

    def conv_bn(name, inp, cout, k, stride, group=1):
        cin = b.shape(inp)[1]
        fan = (cin // group) * k * k
        w = st.normal((cout, cin // group, k, k), 0.0, math.sqrt(2.0 / fan)).astype(np.float64)
        gamma = st.uniform((cout,), 0.5, 1.5).astype(np.float64)
        beta = st.normal((cout,), 0.0, 0.1).astype(np.float64)
        mean = st.normal((cout,), 0.0, 0.1).astype(np.float64)
        var = st.uniform((cout,), 0.5, 1.5).astype(np.float64)
        scale = gamma / np.sqrt(var + 1e-5)
        wn = b.weight(f"{name}_w", w.shape, rng.round_to(w * scale[:, None, None, None], dtype))
        bn = b.weight(f"{name}_b", (cout,), rng.round_to(beta - mean * scale, dtype))
        return _conv(b, inp, wn, bn, stride, k // 2, group)

    y = _swish(b, conv_bn("stem", x, stem, 3, 2))
    bi = 0
    for (e, k, cout, reps, s0) in stages:
        for r in range(reps):
            bi += 1
            cin = b.shape(y)[1]
            stride = s0 if r == 0 else 1
            inp = y
            t = y
            if e != 1:
                t = _swish(b, conv_bn(f"mb{bi}_expand", t, cin * e, 1, 1))
            cexp = b.shape(t)[1]
            t = _swish(b, conv_bn(f"mb{bi}_dw", t, cexp, k, stride, group=cexp))
            se = max(1, cin // 4)
            n_, c_, h_, w_ = b.shape(t)
            sq = b.op("GlobalAveragePool", [t], (n_, c_, 1, 1))
            w1 = b.weight(f"mb{bi}_se1_w", (se, cexp, 1, 1), st.normal((se, cexp, 1, 1), 0.0, math.sqrt(2.0 / cexp), dtype))
            b1 = b.weight(f"mb{bi}_se1_b", (se,), st.normal((se,), 0.0, 0.1, dtype))
            sq = _swish(b, _conv(b, sq, w1, b1, 1, 0))
            w2 = b.weight(f"mb{bi}_se2_w", (cexp, se, 1, 1), st.normal((cexp, se, 1, 1), 0.0, math.sqrt(2.0 / se), dtype))
            b2 = b.weight(f"mb{bi}_se2_b", (cexp,), st.normal((cexp,), 0.0, 0.1, dtype))
            sq = _un(b, "Sigmoid", _conv(b, sq, w2, b2, 1, 0))
            t = _bin(b, "Mul", t, sq)
            t = conv_bn(f"mb{bi}_project", t, cout, 1, 1)
            if stride == 1 and cin == cout:
                t = _bin(b, "Add", t, inp)
            y = t
    b.mark_output(y)
    return b.finish()


# ---------------------------------------------------------------- config 5
def _cast(b, x, to):
    return b.op("Cast", [x], b.shape(x), {"to": {"f32": 1, "f16": 10, "bf16": 16, "i64": 7, "bool": 9}[to]}, out_dtype=to)


def _unsqueeze(b, x, axis):
    s = list(b.shape(x))
    s.insert(axis, 1)
    return b.op("Unsqueeze", [x], tuple(s), {"axes": [axis], "out_shape": s}, out_dtype=b.g.tensors[x].dtype)


def _layernorm_fp32(b, st, x, width, dtype, tag):
    """LayerNorm as a 16-bit export keeps it: the operand is cast up, the nine operators of the decomposition run on
    fp32 tensors, the result is cast back."""
    if dtype == "f32":
        return _layernorm(b, st, x, width, dtype, tag)
    keep = b.g.dtype
    b.g.dtype = "f32"                      # operators created below declare fp32 results
    try:
        y = _layernorm(b, st, _cast(b, x, "f32"), width, dtype, tag)
    finally:
        b.g.dtype = keep
    return _cast(b, y, dtype)


def gpt2_decoder(B=4, S=1024, D=768, NH=12, F=3072, L=12, V=50257, P=1024, dtype="bf16", seed=BASE_SEED + 5):
    """Pre-LayerNorm causal decoder stack (GPT-2-small shaped) with tied vocabulary projection, at the granularity a
    static-shape export of the published model code has: every linear layer as view / MatMul / Add / view, heads split
    by Reshape + Transpose per tensor, the causal mask selected with Where from a sliced boolean buffer, the padding mask
    (an input of ones here) turned into an additive term once and added in every layer, the attention scale as
    Sqrt(Cast(head size)), LayerNorm / softmax / Pow kept in fp32 between Cast pairs, LayerNorm, softmax and the tanh
    GELU in their decompositions, and the layer's key / value returned stacked ("present").  84 operators per layer."""
    st = _Streams(seed)
    b = GraphBuilder("gpt2_decoder", dtype)
    hd = D // NH
    f32 = "f32"
    ids = b.input("input_ids", (B, S), st.integers((B, S), 0, V), dtype="i64")
    amask = b.input("attention_mask", (B, S), np.ones((B, S), dtype=np.int64), dtype="i64")
    wte = b.weight("wte", (V, D), st.normal((V, D), 0.0, 0.02, dtype))
    wpe = b.weight("wpe", (P, D), st.normal((P, D), 0.0, 0.02, dtype))
    allowed = np.tril(np.ones((P, P), dtype=np.uint8)).reshape(1, 1, P, P)        # 1 where key j <= query i
    maskbuf = b._add("causal_bias", "bool", (1, 1, P, P), "weight", allowed)
    pos_ids = b._add("position_ids", "i64", (1, S), "weight", np.arange(S, dtype=np.int64).reshape(1, S), const=True)
    mask_value = b.const("mask_value", -1e4)

    def lin(name, inp, k, n):
        """Conv1D of the published code: x.view(-1, k) @ W + bias, viewed back."""
        w = b.weight(f"{name}_w", (k, n), st.normal((k, n), 0.0, 0.02, dtype))
        bias = b.weight(f"{name}_b", (n,), st.normal((n,), 0.0, 0.02, dtype))
        lead = b.shape(inp)[:-1]
        x2 = _reshape(b, inp, (int(np.prod(lead)), k))
        return _reshape(b, _bin(b, "Add", _matmul(b, x2, w), bias), tuple(lead) + (n,))

    tok = b.op("Gather", [wte, b.op("Reshape", [ids], (B, S), {"shape": [B, S]}, out_dtype="i64")], (B, S, D), {"axis": 0})
    pos = b.op("Gather", [wpe, pos_ids], (1, S, D), {"axis": 0})
    h = _bin(b, "Add", tok, pos)
    # padding mask [B, S] -> additive [B, 1, 1, S]: (1 - m) * -1e4
    em = _cast(b, _unsqueeze(b, _unsqueeze(b, amask, 1), 2), dtype)
    em = _bin(b, "Mul", _bin(b, "Sub", b.const("pad_one", 1.0), em), b.const("pad_value", -1e4))
    for l in range(L):
        a = _layernorm_fp32(b, st, h, D, dtype, f"l{l}_ln1")
        qkv = lin(f"l{l}_attn", a, D, 3 * D)
        q, k, v = b.op("Split", [qkv], [(B, S, D)] * 3, {"axis": 2, "split": [D, D, D]})
        q = _transpose(b, _reshape(b, q, (B, S, NH, hd)), (0, 2, 1, 3))
        k = _transpose(b, _reshape(b, k, (B, S, NH, hd)), (0, 2, 3, 1))
        v = _transpose(b, _reshape(b, v, (B, S, NH, hd)), (0, 2, 1, 3))
        present = b.op("Concat", [_unsqueeze(b, _transpose(b, k, (0, 1, 3, 2)), 0), _unsqueeze(b, v, 0)], (2, B, NH, S, hd), {"axis": 0},
                       out_names=[f"present_{l}"])
        b.mark_output(present)
        s = _matmul(b, q, k)
        hd_c = b._add(f"l{l}_head_size", "i64", (), "weight", np.asarray(hd, dtype=np.int64), const=True)
        s = _bin(b, "Div", s, _un(b, "Sqrt", _cast(b, hd_c, dtype)))
        m = b.op("Slice", [maskbuf], (1, 1, S, P), {"starts": [0], "ends": [S], "axes": [2]}, out_dtype="bool")
        m = b.op("Slice", [m], (1, 1, S, S), {"starts": [0], "ends": [S], "axes": [3]}, out_dtype="bool")
        s = b.op("Where", [_cast(b, m, "bool"), _cast(b, s, dtype), mask_value], b.shape(s))
        s = _bin(b, "Add", s, em)
        if dtype != f32:
            keep, b.g.dtype = b.g.dtype, f32
            s = _cast(b, s, f32)
        mx = _reduce(b, "ReduceMax", s, [-1])          # softmax, decomposed
        e = _un(b, "Exp", _bin(b, "Sub", s, mx))
        p = _bin(b, "Div", e, _reduce(b, "ReduceSum", e, [-1]))
        if dtype != f32:
            b.g.dtype = keep
            p = _cast(b, p, dtype)
        o = _matmul(b, p, v)
        o = _reshape(b, _transpose(b, o, (0, 2, 1, 3)), (B, S, D))
        h = _bin(b, "Add", h, lin(f"l{l}_proj", o, D, D))
        f = _layernorm_fp32(b, st, h, D, dtype, f"l{l}_ln2")
        f = lin(f"l{l}_fc", f, D, F)
        f = _gelu_tanh(b, f, f"l{l}_gelu", pow_in_fp32=dtype != f32)
        h = _bin(b, "Add", h, lin(f"l{l}_fcproj", f, F, D))
    h = _layernorm_fp32(b, st, h, D, dtype, "lnf")
    logits = _matmul(b, h, _transpose(b, wte, (1, 0)))
    b.mark_output(logits)
    return b.finish()


def copy_calibration(N=16, C=256, H=64, W=64, seed=BASE_SEED + 9):
    """One elementwise operator over a tensor of the chain config's size: a plain streaming kernel of
    known traffic (64 MiB read, 64 MiB written) used to calibrate HBM byte counters."""
    st = _Streams(seed)
    b = GraphBuilder("copy_calibration", "f32")
    x = b.input("x", (N, C, H, W), st.normal((N, C, H, W)))
    y = _un(b, "Neg", x)
    b.mark_output(y)
    return b.finish()


def unet_decoder(N=8, C=256, R=16, steps=3, dtype="f16", seed=BASE_SEED + 6):
    """The decoder half of a U-Net / YOLO-neck-shaped model: per step a pointwise convolution halves the channels,
    the map is enlarged 2x by nearest-neighbour Resize (Conv -> Resize: One-to-Many behind Many-to-Many, a yellow
    cell of the paper's mapping-type table), concatenated with a skip tensor of the same size and mixed by a 3x3
    convolution + ReLU.  Not one of the five benchmark configurations: a second workload for the One-to-Many cases."""
    st = _Streams(seed)
    b = GraphBuilder("unet_decoder", dtype)
    x = b.input("x", (N, C, R, R), st.normal((N, C, R, R), 0.0, 1.0, dtype))
    c, r = C, R
    for i in range(steps):
        half = c // 2
        skip = b.input(f"skip{i}", (N, half, 2 * r, 2 * r), st.normal((N, half, 2 * r, 2 * r), 0.0, 1.0, dtype))
        w1 = b.weight(f"up{i}_w", (half, c, 1, 1), st.normal((half, c, 1, 1), 0.0, math.sqrt(2.0 / c), dtype))
        b1 = b.weight(f"up{i}_b", (half,), st.normal((half,), 0.0, 0.1, dtype))
        t = _un(b, "Relu", _conv(b, x, w1, b1, 1, 0))
        t = b.op("Resize", [t], (N, half, 2 * r, 2 * r), {"scales": [1, 1, 2, 2]})
        t = b.op("Concat", [t, skip], (N, c, 2 * r, 2 * r), {"axis": 1})
        w2 = b.weight(f"mix{i}_w", (half, c, 3, 3), st.normal((half, c, 3, 3), 0.0, math.sqrt(2.0 / (c * 9)), dtype))
        b2 = b.weight(f"mix{i}_b", (half,), st.normal((half,), 0.0, 0.1, dtype))
        x = _un(b, "Relu", _conv(b, t, w2, b2, 1, 1))
        c, r = half, 2 * r
    b.mark_output(x)
    return b.finish()


# Reduced instances used by parity tests: several kernel tiles plus ragged tails, small enough for
# the fp64 oracle to finish in seconds.
SMALL = {
    "residual_block": dict(N=2, C=24, H=19, W=13),
    "memory_bound_chain": dict(N=2, C=48, H=20, W=13, groups=4),
    "transformer_encoder_layer": dict(B=2, S=72, D=96, NH=4, F=200),
    "efficientnet_b0": dict(N=2, R=64),
    "gpt2_decoder": dict(B=2, S=80, D=96, NH=4, F=200, L=2, V=1003, P=96),
}

# Mid-sized EfficientNet-shaped stacks for the parity tests of data-format selection: maps large enough for
# the MFMA convolution template, both depthwise kernel sizes and strides.  Stages are (expand, kernel,
# out channels, repeats, first stride) as in EFFNET_B0_STAGES.
_MID_STAGES = [(1, 3, 16, 1, 1), (6, 3, 24, 2, 2), (6, 5, 40, 2, 2), (6, 3, 80, 1, 2)]
MID_EFFICIENTNET = [
    dict(N=3, R=96, stages=_MID_STAGES, dtype="f16"),
    dict(N=3, R=96, stages=_MID_STAGES[:3], dtype="bf16"),
    dict(N=2, R=64, stages=_MID_STAGES[:3], dtype="f32"),
    dict(N=2, R=64, stages=_MID_STAGES[:2], dtype="f16"),
    dict(N=4, R=128, stages=_MID_STAGES[:3], dtype="f16"),       # squeeze-excite scaled maps large enough for the MFMA template
]

# Reduced transformer instances with a head dimension of 32 (a multiple of the MFMA K step), for the
# parity tests of the fused attention block.
SMALL_HEAD32 = {
    "transformer_encoder_layer": dict(B=2, S=72, D=128, NH=4, F=200),
    "gpt2_decoder": dict(B=2, S=48, D=64, NH=2, F=160, L=2, V=211, P=64),
}

# workloads beyond the five benchmark configurations (bench.py --workload NAME)
EXTRA = {"unet_decoder": unet_decoder}
SMALL_EXTRA = {"unet_decoder": dict(N=2, C=32, R=6, steps=2)}

CONFIGS = {
    "residual_block": residual_block,
    "memory_bound_chain": memory_bound_chain,
    "transformer_encoder_layer": transformer_encoder_layer,
    "efficientnet_b0": efficientnet_b0,
    "gpt2_decoder": gpt2_decoder,
}
