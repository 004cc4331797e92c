"""Small single-purpose graphs for kernel-family tests (seeded, no arithmetic here)."""
import math

import numpy as np

from workloads import configs, rng
from workloads.graph import GraphBuilder


def _st(seed):
    return configs._Streams(seed)


def softmax_block(shape, dtype="f32", scale=0.125, masked_tail=3, seed=11):
    """scores * scale + mask -> Softmax -> * 2 (an epilogue), over the last axis."""
    st = _st(seed)
    b = GraphBuilder("softmax_block", dtype)
    x = b.input("x", shape, st.normal(shape, 0.0, 3.0, dtype))
    m = np.zeros((1,) * (len(shape) - 1) + (shape[-1],), dtype=np.float64)
    if masked_tail:
        m[..., -masked_tail:] = -1e4
    mask = b.weight("mask", m.shape, rng.round_to(m, dtype))
    s = configs._bin(b, "Mul", x, b.const("scale", scale))
    s = configs._bin(b, "Add", s, mask)
    p = b.op("Softmax", [s], shape, {"axis": -1})
    y = configs._bin(b, "Mul", p, b.const("two", 2.0))
    b.mark_output(y)
    return b.finish()


def layernorm_block(rows, width, dtype="f32", residual=True, seed=12):
    """(x + r) -> LayerNorm (decomposed, 9 operators) over the last axis."""
    st = _st(seed)
    b = GraphBuilder("layernorm_block", dtype)
    x = b.input("x", (rows, width), st.normal((rows, width), 0.5, 2.0, dtype))
    h = x
    if residual:
        r = b.input("r", (rows, width), st.normal((rows, width), 0.0, 1.0, dtype))
        h = configs._bin(b, "Add", x, r)
    y = configs._layernorm(b, st, h, width, dtype, "ln")
    b.mark_output(y)
    return b.finish()


def reduce_block(kind, shape, axes, keepdims=1, dtype="f32", seed=13):
    """|x| + 0.5 -> Reduce* -> sqrt (the Sub+Pow+ReduceMean+Add+Sqrt style chain of the paper's Sec. 6)."""
    st = _st(seed)
    b = GraphBuilder("reduce_block", dtype)
    x = b.input("x", shape, st.normal(shape, 0.0, 1.0 if kind != "ReduceProd" else 0.1, dtype))
    t = configs._un(b, "Abs", x)
    t = configs._bin(b, "Add", t, b.const("half", 0.5 if kind != "ReduceProd" else 0.95))
    r = configs._reduce(b, kind, t, axes, keepdims)
    y = configs._un(b, "Sqrt", r)
    b.mark_output(y)
    return b.finish()


def gap_block(shape, dtype="f32", seed=14):
    """swish -> GlobalAveragePool (squeeze step of squeeze-excite)."""
    st = _st(seed)
    b = GraphBuilder("gap_block", dtype)
    x = b.input("x", shape, st.normal(shape, 0.0, 1.0, dtype))
    t = configs._swish(b, x)
    n, c = shape[0], shape[1]
    y = b.op("GlobalAveragePool", [t], (n, c, 1, 1))
    b.mark_output(y)
    return b.finish()


def gemm_block(M, K, N, dtype="f16", batch=(), bias=True, gelu=False, residual=False, seed=15, w_std=None, w_transposed=False):
    """x @ w (+ bias, GELU, residual).  w_transposed: the weight is stored [N, K] and transposed in the graph, so
    both operands of the product are contiguous along K."""
    st = _st(seed)
    b = GraphBuilder("gemm_block", dtype)
    x = b.input("x", batch + (M, K), st.normal(batch + (M, K), 0.0, 1.0, dtype))
    if w_transposed:
        w = configs._transpose(b, b.weight("w", (N, K), st.normal((N, K), 0.0, w_std or 1.0 / math.sqrt(K), dtype)), (1, 0))
    else:
        w = b.weight("w", (K, N), st.normal((K, N), 0.0, w_std or 1.0 / math.sqrt(K), dtype))
    y = configs._matmul(b, x, w)
    if bias:
        y = configs._bin(b, "Add", y, b.weight("bias", (N,), st.normal((N,), 0.0, 0.5, dtype)))
    if gelu:
        y = configs._gelu_erf(b, y, "g")
    if residual:
        r = b.input("r", batch + (M, N), st.normal(batch + (M, N), 0.0, 1.0, dtype))
        y = configs._bin(b, "Add", y, r)
    b.mark_output(y)
    return b.finish()


def linear_layernorm_block(M, K, N, dtype="bf16", batch=(), residual=True, keep_sum=True, w_transposed=True, seed=37):
    """x @ w + bias (+ residual) -> LayerNorm over the last axis (decomposed) -> gamma, beta: a linear layer with the
    normalisation that follows it.  keep_sum: the sum in front of the normalisation is a graph output too (the
    residual stream of a pre-LayerNorm network), otherwise it exists only inside the block."""
    st = _st(seed)
    b = GraphBuilder("linear_layernorm_block", dtype)
    x = b.input("x", batch + (M, K), st.normal(batch + (M, K), 0.0, 1.0, dtype))
    if w_transposed:
        w = configs._transpose(b, b.weight("w", (N, K), st.normal((N, K), 0.0, 1.0 / math.sqrt(K), dtype)), (1, 0))
    else:
        w = b.weight("w", (K, N), st.normal((K, N), 0.0, 1.0 / math.sqrt(K), dtype))
    y = configs._bin(b, "Add", configs._matmul(b, x, w), b.weight("bias", (N,), st.normal((N,), 0.0, 0.5, dtype)))
    if residual:
        y = configs._bin(b, "Add", y, b.input("r", batch + (M, N), st.normal(batch + (M, N), 0.0, 1.0, dtype)))
    z = configs._layernorm(b, st, y, N, dtype, "ln", affine_std=0.2)
    if keep_sum:
        b.mark_output(y)
    b.mark_output(z)
    return b.finish()


def se_tail_block(N, C, H, W, CR, dtype="f16", scale=True, bias=True, act="swish", seed=38, dw=None):
    """The squeeze-excite tail of a mobile-network block: GlobalAveragePool -> 1x1 Conv (C -> CR) -> swish (or Relu) ->
    1x1 Conv (CR -> C) -> Sigmoid [-> x * s].  H = W = 1: the first layer reads an already pooled vector.
    dw = (kernel, stride): the map is the swish of a depthwise convolution of the input (after a pointwise one, so
    that it lives inside the channels-last region) instead of the input itself; H, W are the input's."""
    st = _st(seed)
    b = GraphBuilder("se_tail_block", dtype)
    x = b.input("x", (N, C, H, W), st.normal((N, C, H, W), 0.3, 1.0, dtype))
    if dw:
        kk, stride = dw
        wp = b.weight("pw_w", (C, C, 1, 1), st.normal((C, C, 1, 1), 0.0, math.sqrt(1.0 / C), dtype))
        x = configs._swish(b, configs._conv(b, x, wp, None, 1, 0))
        wd = b.weight("dw_w", (C, 1, kk, kk), st.normal((C, 1, kk, kk), 0.0, math.sqrt(2.0 / (kk * kk)), dtype))
        bd = b.weight("dw_b", (C,), st.normal((C,), 0.0, 0.2, dtype))
        x = configs._swish(b, configs._conv(b, x, wd, bd, stride, kk // 2, C))
        H, W = (H + 2 * (kk // 2) - kk) // stride + 1, (W + 2 * (kk // 2) - kk) // stride + 1
    sq = b.op("GlobalAveragePool", [x], (N, C, 1, 1)) if H * W > 1 else x
    w1 = b.weight("se1_w", (CR, C, 1, 1), st.normal((CR, C, 1, 1), 0.0, math.sqrt(2.0 / C), dtype))
    b1 = b.weight("se1_b", (CR,), st.normal((CR,), 0.0, 0.1, dtype)) if bias else None
    h = configs._conv(b, sq, w1, b1, 1, 0)
    h = configs._swish(b, h) if act == "swish" else configs._un(b, "Relu", h)
    w2 = b.weight("se2_w", (C, CR, 1, 1), st.normal((C, CR, 1, 1), 0.0, math.sqrt(2.0 / CR), dtype))
    b2 = b.weight("se2_b", (C,), st.normal((C,), 0.0, 0.1, dtype)) if bias else None
    s = configs._un(b, "Sigmoid", configs._conv(b, h, w2, b2, 1, 0))
    if scale and H * W > 1:
        b.mark_output(configs._bin(b, "Mul", x, s))
    else:
        b.mark_output(s)
    return b.finish()


def attention_block(B, H, SQ, SK, D, dtype="f16", mask="add", kt_stored=True, merge_heads=True, seed=21):
    """softmax(Q K^T / sqrt(D) + mask) V per (batch, head).  Q [B,H,SQ,D]; K is handed over as K^T [B,H,D,SK]
    (kt_stored) or as K [B,H,SK,D] with a Transpose in the graph; V [B,H,SK,D]; the result is written
    [B,SQ,H*D] (merge_heads) or [B,H,SQ,D]."""
    st = _st(seed)
    b = GraphBuilder("attention_block", dtype)
    q = b.input("q", (B, H, SQ, D), st.normal((B, H, SQ, D), 0.0, 1.0, dtype))
    if kt_stored:
        kt = b.input("kt", (B, H, D, SK), st.normal((B, H, D, SK), 0.0, 1.0, dtype))
    else:
        kt = configs._transpose(b, b.input("k", (B, H, SK, D), st.normal((B, H, SK, D), 0.0, 1.0, dtype)), (0, 1, 3, 2))
    v = b.input("v", (B, H, SK, D), st.normal((B, H, SK, D), 0.0, 1.0, dtype))
    s = configs._matmul(b, q, kt)
    s = configs._bin(b, "Div", s, b.const("sqrt_d", math.sqrt(D)))
    if mask == "add":          # additive key mask per batch entry, -1e4 on the masked keys
        m = np.where(st.uniform((B, 1, 1, SK), 0.0, 1.0, "f32") < 0.2, -1e4, 0.0)
        s = configs._bin(b, "Add", s, b.weight("mask", (B, 1, 1, SK), rng.round_to(m, dtype)))
    elif mask == "causal":
        m = np.triu(np.full((SQ, SK), -1e4), k=1 + SK - SQ).reshape(1, 1, SQ, SK)
        s = configs._bin(b, "Add", s, b.weight("mask", (1, 1, SQ, SK), rng.round_to(m, dtype)))
    p = b.op("Softmax", [s], (B, H, SQ, SK), {"axis": -1})
    o = configs._matmul(b, p, v)
    if merge_heads:
        o = configs._reshape(b, configs._transpose(b, o, (0, 2, 1, 3)), (B, SQ, H * D))
    b.mark_output(o)
    return b.finish()


def upsample_concat_block(N, C1, C2, H, W, dtype="f16", scale=2, conv=False, seed=23):
    """A decoder step of a U-Net-shaped model: the low-resolution path (optionally behind a 1x1 Conv) is
    enlarged by nearest-neighbour Resize, scaled, and concatenated along the channels with a skip
    tensor that passes through a Sigmoid; optionally a 3x3 Conv + Relu follows."""
    st = _st(seed)
    b = GraphBuilder("upsample_concat", dtype)
    x = b.input("x", (N, C1, H, W), st.normal((N, C1, H, W), 0.0, 1.0, dtype))
    skip = b.input("skip", (N, C2, H * scale, W * scale), st.normal((N, C2, H * scale, W * scale), 0.0, 1.0, dtype))
    t = x
    if conv:
        w = b.weight("w1", (C1, C1, 1, 1), st.normal((C1, C1, 1, 1), 0.0, math.sqrt(2.0 / C1), dtype))
        t = configs._conv(b, t, w, None, 1, 0)
    t = configs._un(b, "Relu", t)
    t = b.op("Resize", [t], (N, C1, H * scale, W * scale), {"scales": [1, 1, scale, scale]})
    t = configs._bin(b, "Mul", t, b.weight("g", (1, C1, 1, 1), st.uniform((1, C1, 1, 1), 0.5, 1.5, dtype)))
    s2 = configs._un(b, "Sigmoid", skip)
    y = b.op("Concat", [t, s2], (N, C1 + C2, H * scale, W * scale), {"axis": 1})
    if conv:
        w2 = b.weight("w2", (C1, C1 + C2, 3, 3), st.normal((C1, C1 + C2, 3, 3), 0.0, math.sqrt(2.0 / ((C1 + C2) * 9)), dtype))
        y = configs._un(b, "Relu", configs._conv(b, y, w2, None, 1, 1))
    b.mark_output(y)
    return b.finish()


def expand_transpose_block(N, H, W, dtype="f32", seed=24):
    """Expand (One-to-Many) followed by Transpose (Shuffle) and an Add: one of the table's yellow pairs."""
    st = _st(seed)
    b = GraphBuilder("expand_transpose", dtype)
    x = b.input("x", (N, 1, W), st.normal((N, 1, W), 0.0, 1.0, dtype))
    r = b.input("r", (N, W, H), st.normal((N, W, H), 0.0, 1.0, dtype))
    t = b.op("Expand", [x], (N, H, W), {"shape": [N, H, W]})
    t = configs._transpose(b, t, (0, 2, 1))
    y = configs._bin(b, "Add", t, r)
    b.mark_output(y)
    return b.finish()


def conv_block(N, C, H, W, CO, K, stride=1, group=1, dtype="f32", bias=True, act=None, residual=False, seed=16):
    st = _st(seed)
    b = GraphBuilder("conv_block", dtype)
    x = b.input("x", (N, C, H, W), st.normal((N, C, H, W), 0.0, 1.0, dtype))
    w = b.weight("w", (CO, C // group, K, K), st.normal((CO, C // group, K, K), 0.0, math.sqrt(2.0 / (C // group * K * K)), dtype))
    bs = b.weight("b", (CO,), st.normal((CO,), 0.0, 0.2, dtype)) if bias else None
    y = configs._conv(b, x, w, bs, stride, K // 2, group)
    if act == "relu":
        y = configs._un(b, "Relu", y)
    if act == "swish":
        y = configs._swish(b, y)
    if act == "sigmoid":
        y = configs._un(b, "Sigmoid", y)
    if residual:
        y = configs._bin(b, "Add", y, x)
    b.mark_output(y)
    return b.finish()


def pool_block(kind, N, C, H, W, k, stride, pad=0, dtype="f16", include_pad=0, prologue=False, seed=25):
    """[Relu ->] MaxPool / AveragePool -> per-channel affine: the pooling operator with a One-to-One operator in
    front of it and two behind it."""
    st = _st(seed)
    b = GraphBuilder("pool_block", dtype)
    x = b.input("x", (N, C, H, W), st.normal((N, C, H, W), 0.0, 1.0, dtype))
    t = configs._un(b, "Relu", x) if prologue else x
    ho, wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    y = b.op(kind, [t], (N, C, ho, wo), {"kernel_shape": [k, k], "strides": [stride, stride], "pads": [pad] * 4,
                                        "count_include_pad": include_pad})
    sc = b.weight("scale", (1, C, 1, 1), st.uniform((1, C, 1, 1), 0.5, 1.5, dtype))
    sh = b.weight("shift", (1, C, 1, 1), st.normal((1, C, 1, 1), 0.0, 0.2, dtype))
    y = configs._bin(b, "Add", configs._bin(b, "Mul", y, sc), sh)
    b.mark_output(y)
    return b.finish()


def cumsum_block(shape, axis, dtype="f32", exclusive=0, reverse=0, prologue=False, epilogue=True, reshape=False, residual=False, seed=33):
    """[Abs ->] CumSum along `axis` [-> * scale + shift] [-> Reshape that splits the scanned axis]: the prefix sum
    with a One-to-One operator in front of it, two behind it, and an index map on its result."""
    st = _st(seed)
    b = GraphBuilder("cumsum_block", dtype)
    x = b.input("x", shape, st.normal(shape, 0.0, 1.0, dtype))
    t = configs._un(b, "Abs", x) if prologue else x
    y = b.op("CumSum", [t], shape, {"axis": axis, "exclusive": exclusive, "reverse": reverse})
    if epilogue:
        bshape = tuple(d if i == len(shape) - 1 else 1 for i, d in enumerate(shape))
        sc = b.weight("scale", bshape, st.uniform(bshape, 0.5, 1.5, dtype))
        y = configs._bin(b, "Add", configs._bin(b, "Mul", y, sc), b.const("shift", 0.25))
        if residual:
            y = configs._bin(b, "Add", y, x)          # the scan's own operand again, behind it
    if reshape:
        ax = axis % len(shape)
        assert shape[ax] % 2 == 0
        y = configs._reshape(b, y, shape[:ax] + (2, shape[ax] // 2) + shape[ax + 1:])
    b.mark_output(y)
    return b.finish()


def conv_pool_net(N=2, C=16, R=48, dtype="f16", seed=26):
    """A small encoder-decoder in the shape of the pooling CNNs: (conv 3x3 + bias + Relu -> MaxPool 2x2) twice,
    a pointwise bottleneck, AveragePool 3x3 s1, Upsample x2, Concat with the skip tensor, pointwise head."""
    st = _st(seed)
    b = GraphBuilder("conv_pool_net", dtype)
    x = b.input("x", (N, 8, R, R), st.normal((N, 8, R, R), 0.0, 1.0, dtype))

    def conv(t, cout, k, name):
        cin = b.shape(t)[1]
        w = b.weight(name + "_w", (cout, cin, k, k), st.normal((cout, cin, k, k), 0.0, math.sqrt(2.0 / (cin * k * k)), dtype))
        bs = b.weight(name + "_b", (cout,), st.normal((cout,), 0.0, 0.1, dtype))
        return configs._conv(b, t, w, bs, 1, k // 2, 1)

    def pool(t, kind, k, s, pad):
        n, c, h, w = b.shape(t)
        return b.op(kind, [t], (n, c, (h + 2 * pad - k) // s + 1, (w + 2 * pad - k) // s + 1),
                    {"kernel_shape": [k, k], "strides": [s, s], "pads": [pad] * 4})

    e1 = configs._un(b, "Relu", conv(x, C, 3, "e1"))
    p1 = pool(e1, "MaxPool", 2, 2, 0)
    e2 = configs._un(b, "Relu", conv(p1, 2 * C, 3, "e2"))
    p2 = pool(e2, "MaxPool", 2, 2, 0)
    mid = configs._un(b, "Relu", conv(p2, 2 * C, 1, "mid"))
    sm = pool(mid, "AveragePool", 3, 1, 1)
    n, c, h, w = b.shape(sm)
    up = b.op("Upsample", [sm], (n, c, 2 * h, 2 * w), {"scales": [1, 1, 2, 2]})
    cat = b.op("Concat", [up, e2], (n, c + 2 * C, 2 * h, 2 * w), {"axis": 1})
    y = conv(cat, C, 1, "head")
    b.mark_output(y)
    return b.finish()


def resnet_stage(N=2, C=32, R=40, dtype="f16", k=3, seed=27):
    """Stem conv -> basic block (conv - Relu - conv - add - Relu) -> strided conv -> basic block: dense k x k
    convolutions whose operands are intermediate tensors (channels-last under data-format selection)."""
    st = _st(seed)
    b = GraphBuilder("resnet_stage", dtype)
    x = b.input("x", (N, 3, R, R), st.normal((N, 3, R, R), 0.0, 1.0, dtype))
    cnt = [0]

    def conv(t, cout, kk, stride=1):
        cin = b.shape(t)[1]
        cnt[0] += 1
        w = b.weight(f"w{cnt[0]}", (cout, cin, kk, kk), st.normal((cout, cin, kk, kk), 0.0, math.sqrt(1.0 / (cin * kk * kk)), dtype))
        bs = b.weight(f"b{cnt[0]}", (cout,), st.normal((cout,), 0.0, 0.1, dtype))
        return configs._conv(b, t, w, bs, stride, kk // 2, 1)

    def basic(t):
        ch = b.shape(t)[1]
        y = configs._un(b, "Relu", conv(t, ch, k))
        y = conv(y, ch, k)
        return configs._un(b, "Relu", configs._bin(b, "Add", y, t))

    t = configs._un(b, "Relu", conv(x, C, 3))
    t = basic(t)
    t = configs._un(b, "Relu", conv(t, 2 * C, k, 2))
    t = basic(t)
    b.mark_output(t)
    return b.finish()


def pixel_shuffle_block(N=2, C=8, H=12, W=10, b=2, dtype="f16", crd=0, seed=28):
    """SpaceToDepth -> pointwise conv -> Relu -> DepthToSpace -> Mul const: both Shuffle operators of Table 2 around a
    convolution (the sub-pixel upsampling pattern); they fold into the convolution's operand and result index maps."""
    st = _st(seed)
    bld = GraphBuilder("pixel_shuffle_block", dtype)
    x = bld.input("x", (N, C, H, W), st.normal((N, C, H, W), 0.0, 1.0, dtype))
    s2d = bld.op("SpaceToDepth", [x], (N, C * b * b, H // b, W // b), {"blocksize": b})
    cin = C * b * b
    w = bld.weight("w", (cin, cin, 1, 1), st.normal((cin, cin, 1, 1), 0.0, math.sqrt(2.0 / cin), dtype))
    y = configs._un(bld, "Relu", configs._conv(bld, s2d, w, None, 1, 0, 1))
    d2s = bld.op("DepthToSpace", [y], (N, C, H, W), {"blocksize": b, "mode_crd": crd})
    out = configs._bin(bld, "Mul", d2s, bld.const("gain", 1.5))
    bld.mark_output(out)
    return bld.finish()


def shuffle_only_block(N=2, C=12, H=6, W=10, b=2, dtype="f32", seed=29):
    """Exp -> DepthToSpace -> Add const and a SpaceToDepth of the same input: index maps without an anchor."""
    st = _st(seed)
    bld = GraphBuilder("shuffle_only_block", dtype)
    x = bld.input("x", (N, C, H, W), st.normal((N, C, H, W), 0.0, 1.0, dtype))
    e = configs._un(bld, "Exp", x)
    d = bld.op("DepthToSpace", [e], (N, C // (b * b), H * b, W * b), {"blocksize": b})
    bld.mark_output(configs._bin(bld, "Add", d, bld.const("one", 1.0)))
    s = bld.op("SpaceToDepth", [x], (N, C * b * b, H // b, W // b), {"blocksize": b})
    bld.mark_output(configs._un(bld, "Neg", s))
    return bld.finish()


def instance_norm_block(N=2, C=6, H=9, W=11, dtype="f32", seed=30):
    """Mul const -> InstanceNormalization (scale, bias per channel) -> Relu."""
    st = _st(seed)
    bld = GraphBuilder("instance_norm_block", dtype)
    x = bld.input("x", (N, C, H, W), st.normal((N, C, H, W), 0.3, 1.2, dtype))
    sc = bld.weight("scale", (C,), st.uniform((C,), 0.5, 1.5, dtype))
    bs = bld.weight("bias", (C,), st.normal((C,), 0.0, 0.3, dtype))
    t = configs._bin(bld, "Mul", x, bld.const("two", 2.0))
    y = bld.op("InstanceNormalization", [t, sc, bs], (N, C, H, W), {"epsilon": 1e-5})
    bld.mark_output(configs._un(bld, "Relu", y))
    return bld.finish()


def more_unary_block(shape=(3, 7, 50), dtype="f32", seed=31):
    """Sin, Cos, Asin, Round, Floor, Ceil and PRelu in one chain (the One-to-One operators of Table 2 beyond the
    ones the benchmark graphs use)."""
    st = _st(seed)
    bld = GraphBuilder("more_unary_block", dtype)
    x = bld.input("x", shape, st.normal(shape, 0.0, 2.0, dtype))
    slope = bld.weight("slope", (shape[-1],), st.uniform((shape[-1],), 0.05, 0.4, dtype))
    s, co = configs._un(bld, "Sin", x), configs._un(bld, "Cos", x)
    a = configs._un(bld, "Asin", configs._bin(bld, "Mul", s, bld.const("c9", 0.9)))
    # integer-valued pieces from a value that is never within rounding of a tie
    r = configs._un(bld, "Round", configs._bin(bld, "Add", configs._bin(bld, "Mul", co, bld.const("c3", 3.0)), bld.const("off", 0.25)))
    f = configs._un(bld, "Floor", configs._bin(bld, "Add", configs._bin(bld, "Mul", s, bld.const("c4", 4.0)), bld.const("off2", 0.3)))
    ce = configs._un(bld, "Ceil", configs._bin(bld, "Add", configs._bin(bld, "Mul", co, bld.const("c5", 5.0)), bld.const("off3", 0.4)))
    t = configs._bin(bld, "Add", configs._bin(bld, "Add", a, r), configs._bin(bld, "Add", f, ce))
    bld.mark_output(bld.op("PRelu", [t, slope], shape))
    return bld.finish()


def einsum_block(equation, shape_a, shape_b, dtype="f16", b_weight=False, epilogue=True, seed=35):
    """Einsum(a, b) [-> * 0.5 -> Tanh]: a contraction written as an Einsum, with One-to-One operators behind it."""
    st = _st(seed)
    bld = GraphBuilder("einsum_block", dtype)
    lhs, out = equation.split("->")
    ta, tb = lhs.split(",")
    ext = {l: shape_a[i] for i, l in enumerate(ta)}
    ext.update({l: shape_b[i] for i, l in enumerate(tb)})
    k = 1
    for l in set(ta) & set(tb) - set(out):
        k *= ext[l]
    a = bld.input("a", shape_a, st.normal(shape_a, 0.0, 1.0, dtype))
    if b_weight:
        b = bld.weight("b", shape_b, st.normal(shape_b, 0.0, 1.0 / math.sqrt(k), dtype))
    else:
        b = bld.input("b", shape_b, st.normal(shape_b, 0.0, 1.0 / math.sqrt(k), dtype))
    y = bld.op("Einsum", [a, b], tuple(ext[l] for l in out), {"equation": equation})
    if epilogue:
        y = configs._un(bld, "Tanh", configs._bin(bld, "Mul", y, bld.const("half", 0.5)))
    bld.mark_output(y)
    return bld.finish()


def bitshift_block(shape=(7, 50), right=0, seed=36):
    """BitShift of an int64 tensor by a per-column amount (the one integer operator of Table 2)."""
    st = _st(seed)
    b = GraphBuilder("bitshift_block", "f32")
    x = b.input("x", shape, st.integers(shape, 0, 1 << 20), dtype="i64")
    sh = b.weight("shift", (shape[-1],), st.integers((shape[-1],), 0, 9), dtype="i64")
    y = b.op("BitShift", [x, sh], shape, {"direction_right": right}, out_dtype="i64")
    b.mark_output(y)
    return b.finish()


def logic_block(shape=(5, 9, 40), dtype="f32", seed=34):
    """Greater -> Not -> Where: out = Where(Not(x > y), 2 x, y - 1) + Where(x > y, 1, 0)."""
    st = _st(seed)
    b = GraphBuilder("logic_block", dtype)
    x = b.input("x", shape, st.normal(shape, 0.0, 1.0, dtype))
    y = b.input("y", shape, st.normal(shape, 0.0, 1.0, dtype))
    m = b.op("Greater", [x, y], shape)
    n = configs._un(b, "Not", m)
    w1 = b.op("Where", [n, configs._bin(b, "Mul", x, b.const("two", 2.0)), configs._bin(b, "Sub", y, b.const("one", 1.0))], shape)
    w2 = b.op("Where", [m, b.const("t", 1.0), b.const("f", 0.0)], shape)
    b.mark_output(configs._bin(b, "Add", w1, w2))
    return b.finish()


def conv3d_block(N=2, C=8, D=6, H=10, W=12, CO=16, k=(3, 3, 3), stride=(1, 1, 1), pad=(1, 1, 1), dtype="f16", act="relu",
                 residual=False, prologue=False, seed=32):
    """[Relu ->] 3-d Conv + bias -> per-channel affine -> Relu [-> Add x]: the building block of the C3D / S3D-shaped
    video models (a separable S3D pair is a (1, 3, 3) convolution followed by a (3, 1, 1) one)."""
    st = _st(seed)
    b = GraphBuilder("conv3d_block", dtype)
    x = b.input("x", (N, C, D, H, W), st.normal((N, C, D, H, W), 0.0, 1.0, dtype))
    w = b.weight("w", (CO, C) + tuple(k), st.normal((CO, C) + tuple(k), 0.0, math.sqrt(2.0 / (C * k[0] * k[1] * k[2])), dtype))
    bs = b.weight("b", (CO,), st.normal((CO,), 0.0, 0.2, dtype))
    t = configs._un(b, "Relu", x) if prologue else x
    od = [(s_ + 2 * p_ - k_) // st_ + 1 for s_, p_, k_, st_ in zip((D, H, W), pad, k, stride)]
    y = b.op("Conv", [t, w, bs], (N, CO, od[0], od[1], od[2]), {"strides": list(stride), "pads": list(pad) + list(pad), "group": 1})
    sc = b.weight("scale", (1, CO, 1, 1, 1), st.uniform((1, CO, 1, 1, 1), 0.5, 1.5, dtype))
    y = configs._bin(b, "Mul", y, sc)
    if act == "relu":
        y = configs._un(b, "Relu", y)
    if residual:
        y = configs._bin(b, "Add", y, x)
    b.mark_output(y)
    return b.finish()


def s3d_unit(N=2, C=16, D=8, R=16, dtype="f16", seed=33):
    """A separable spatio-temporal unit: (1,3,3) convolution + Relu, then (3,1,1) convolution + Relu, then a
    pointwise (1,1,1) projection added to the unit's input."""
    st = _st(seed)
    b = GraphBuilder("s3d_unit", dtype)
    x = b.input("x", (N, C, D, R, R), st.normal((N, C, D, R, R), 0.0, 1.0, dtype))

    def conv(t, cout, k, name):
        cin = b.shape(t)[1]
        w = b.weight(name + "_w", (cout, cin) + k, st.normal((cout, cin) + k, 0.0, math.sqrt(2.0 / (cin * k[0] * k[1] * k[2])), dtype))
        bs = b.weight(name + "_b", (cout,), st.normal((cout,), 0.0, 0.1, dtype))
        pad = [kk // 2 for kk in k]
        n, _, d, h, w_ = b.shape(t)
        return b.op("Conv", [t, w, bs], (n, cout, d, h, w_), {"strides": [1, 1, 1], "pads": pad + pad, "group": 1})

    t = configs._un(b, "Relu", conv(x, 2 * C, (1, 3, 3), "sp"))
    t = configs._un(b, "Relu", conv(t, 2 * C, (3, 1, 1), "tm"))
    y = configs._bin(b, "Add", conv(t, C, (1, 1, 1), "pw"), x)
    b.mark_output(y)
    return b.finish()


def conv_transpose_block(N=2, C=16, H=12, W=10, CO=8, k=4, stride=2, pad=1, out_pad=0, dtype="f16", prologue=False, skip=False, seed=34):
    """[Relu ->] ConvTranspose + bias -> LeakyRelu [-> Add skip]: the learned upsampling step of encoder-decoder models."""
    st = _st(seed)
    b = GraphBuilder("conv_transpose_block", dtype)
    x = b.input("x", (N, C, H, W), st.normal((N, C, H, W), 0.0, 1.0, dtype))
    w = b.weight("w", (C, CO, k, k), st.normal((C, CO, k, k), 0.0, math.sqrt(2.0 * stride * stride / (C * k * k)), dtype))
    bs = b.weight("b", (CO,), st.normal((CO,), 0.0, 0.2, dtype))
    t = configs._un(b, "Relu", x) if prologue else x
    ho, wo = (H - 1) * stride - 2 * pad + k + out_pad, (W - 1) * stride - 2 * pad + k + out_pad
    y = b.op("ConvTranspose", [t, w, bs], (N, CO, ho, wo), {"strides": [stride, stride], "pads": [pad] * 4, "output_padding": [out_pad, out_pad], "group": 1})
    y = b.op("LeakyRelu", [y], (N, CO, ho, wo), {"alpha": 0.1})
    if skip:
        sk = b.input("skip", (N, CO, ho, wo), st.normal((N, CO, ho, wo), 0.0, 1.0, dtype))
        y = configs._bin(b, "Add", y, sk)
    b.mark_output(y)
    return b.finish()


def random_graph(seed, dtype="f32", n_ops=14, wide=False):
    """A seeded random DAG over the operator kinds the planner mixes: One-to-One (unary, binary with broadcast
    operands), Reorganize (Reshape, Transpose), Shuffle (Slice, Concat), One-to-Many (Expand) and Many-to-Many
    (row reductions, Softmax, MatMul with a constant matrix).  Values stay bounded (every growing operator is followed
    by a squashing one), so fp16 runs stay finite."""
    r = np.random.RandomState(seed)
    st = _st(1000 + seed)
    b = GraphBuilder(f"random_graph_{seed}", dtype)
    rank = int(r.choice([2, 3, 4]))
    dims = tuple(int(r.choice([2, 3, 4, 6, 8, 12, 20])) for _ in range(rank - 1)) + (int(r.choice([8, 16, 24, 40])),)
    live = [b.input("x0", dims, st.normal(dims, 0.0, 1.0, dtype)), b.input("x1", dims, st.normal(dims, 0.0, 1.0, dtype))]
    n_w = 0

    def weight(shape, std=1.0):
        nonlocal n_w
        n_w += 1
        return b.weight(f"w{n_w}", shape, st.normal(shape, 0.0, std, dtype))

    used = []

    def pick():
        t = live[int(r.randint(len(live)))]
        used.append(t)
        return t

    for _ in range(n_ops):
        x = pick()
        s = b.shape(x)
        kinds = ["unary", "binary", "bcast", "reshape", "transpose", "slice", "concat", "expand", "reduce", "softmax", "matmul"]
        probs = [0.2, 0.16, 0.1, 0.1, 0.1, 0.07, 0.06, 0.04, 0.07, 0.04, 0.06]
        if wide:      # the rarer operators of Table 2 as well
            kinds += ["split", "gather", "where", "cumsum", "resize", "einsum"]
            probs = [q * 0.7 for q in probs] + [0.06, 0.04, 0.06, 0.04, 0.04, 0.06]
        kind = r.choice(kinds, p=probs)
        if kind == "unary":
            y = configs._un(b, str(r.choice(["Relu", "Sigmoid", "Tanh", "Abs", "Neg", "Sin", "Cos"])), x)
        elif kind == "binary":
            others = [t for t in live if b.shape(t) == s and t is not x]
            if not others:
                continue
            o = others[int(r.randint(len(others)))]
            used.append(o)
            y = configs._bin(b, str(r.choice(["Add", "Sub", "Mul", "Max"])), x, o)
            y = configs._un(b, "Tanh", y)
        elif kind == "bcast":
            ws = tuple(d if r.rand() < 0.5 else 1 for d in s)
            y = configs._bin(b, str(r.choice(["Add", "Mul"])), x, weight(ws, 0.5))
        elif kind == "reshape":
            n = int(np.prod(s))
            cands = [(n,), (s[0], n // s[0])] + ([(s[0] * s[1],) + tuple(s[2:])] if len(s) > 2 else []) + \
                    ([tuple(s[:-1]) + (2, s[-1] // 2)] if s[-1] % 2 == 0 and len(s) < 4 else [])
            y = configs._reshape(b, x, cands[int(r.randint(len(cands)))])
        elif kind == "transpose":
            if len(s) < 2:
                continue
            perm = list(r.permutation(len(s)))
            y = configs._transpose(b, x, perm)
        elif kind == "slice":
            ax = int(r.randint(len(s)))
            if s[ax] < 2:
                continue
            lo = int(r.randint(0, s[ax] - 1))
            hi = int(r.randint(lo + 1, s[ax] + 1))
            y = b.op("Slice", [x], tuple(hi - lo if i == ax else d for i, d in enumerate(s)), {"starts": [lo], "ends": [hi], "axes": [ax]})
        elif kind == "concat":
            ax = int(r.randint(len(s)))
            others = [t for t in live if len(b.shape(t)) == len(s) and all(b.shape(t)[i] == s[i] for i in range(len(s)) if i != ax)]
            o = others[int(r.randint(len(others)))]
            used.append(o)
            y = b.op("Concat", [x, o], tuple(d + b.shape(o)[ax] if i == ax else d for i, d in enumerate(s)), {"axis": ax})
        elif kind == "expand":
            if len(s) >= 4 or int(np.prod(s)) > 4096:
                continue
            k = int(r.choice([2, 3]))
            y = b.op("Expand", [configs._reshape(b, x, (1,) + tuple(s))], (k,) + tuple(s), {"shape": [k] + list(s)})
        elif kind == "reduce":
            if len(s) < 2:
                continue
            y = configs._reduce(b, str(r.choice(["ReduceSum", "ReduceMean", "ReduceMax"])), x, [-1], keepdims=int(r.rand() < 0.5))
            y = configs._un(b, "Tanh", y)
        elif kind == "softmax":
            y = b.op("Softmax", [x], s, {"axis": -1})
        elif kind == "split":
            ax = int(r.randint(len(s)))
            if s[ax] % 2:
                continue
            half = tuple(d // 2 if i == ax else d for i, d in enumerate(s))
            p0, p1 = b.op("Split", [x], [half, half], {"axis": ax, "split": [s[ax] // 2, s[ax] // 2]})
            live.append(configs._un(b, "Tanh", p0))
            y = configs._un(b, "Abs", p1)
        elif kind == "gather":
            ax = int(r.randint(len(s)))
            m = int(r.choice([1, 3, 5]))
            n_w += 1
            idx = b.weight(f"idx{n_w}", (m,), st.integers((m,), 0, s[ax]), dtype="i64")
            y = b.op("Gather", [x, idx], tuple(s[:ax]) + (m,) + tuple(s[ax + 1:]), {"axis": ax})
        elif kind == "where":
            others = [t for t in live if b.shape(t) == s and t is not x]
            if not others:
                continue
            o = others[int(r.randint(len(others)))]
            used.append(o)
            m = b.op("Greater", [x, o], s)
            if r.rand() < 0.5:
                m = configs._un(b, "Not", m)
            y = b.op("Where", [m, configs._un(b, "Tanh", x), o], s)
        elif kind == "cumsum":
            ax = int(r.randint(len(s)))
            y = b.op("CumSum", [x], s, {"axis": ax, "exclusive": int(r.rand() < 0.3), "reverse": int(r.rand() < 0.3)})
            cname = f"cs{len(live)}"
            while cname in b.g.tensors:          # (two scans drawn while the same number of tensors is live)
                cname += "_"
            y = configs._un(b, "Tanh", configs._bin(b, "Mul", y, b.const(cname, 1.0 / s[ax])))
        elif kind == "resize":
            if len(s) != 4 or int(np.prod(s)) * 4 > 1 << 15:
                continue
            y = b.op("Resize", [x], (s[0], s[1], s[2] * 2, s[3] * 2), {"scales": [1, 1, 2, 2]})
        elif kind == "einsum":
            if len(s) != 3:
                continue
            others = [t for t in live if b.shape(t) == s and t is not x]
            if not others:
                continue
            o = others[int(r.randint(len(others)))]
            used.append(o)
            # scores-like (contract the last axis) or values-like (contract the middle one)
            if r.rand() < 0.5:
                y = b.op("Einsum", [x, o], (s[0], s[1], s[1]), {"equation": "bid,bjd->bij"})
            else:
                y = b.op("Einsum", [x, o], (s[0], s[2], s[2]), {"equation": "bki,bkj->bij"})
            y = configs._un(b, "Tanh", configs._bin(b, "Mul", y, b.const(f"es{len(live)}", 0.2)))
        else:
            if len(s) < 2:
                continue
            n = int(r.choice([8, 16, 24]))
            y = configs._un(b, "Tanh", configs._matmul(b, x, weight((s[-1], n), 1.0 / math.sqrt(s[-1]))))
        if int(np.prod(b.shape(y))) > 1 << 16:
            continue
        live.append(y)
    # outputs: every tensor nothing else reads (so no operator is dead), and one from the middle, which is then both a
    # graph output and an operand of later operators
    outs = [t for t in live[2:] if not any(t is u for u in used)] or [live[-1]]
    mid = live[2 + (len(live) - 2) // 2] if len(live) > 4 else None
    if mid is not None and not any(mid is t for t in outs):
        outs.append(mid)
    for t in outs:
        b.mark_output(t)
    return b.finish()


def random_cnn(seed, dtype="f16", n_ops=12, wide=False, big=False):
    """A seeded random NCHW network from the pieces of the CNN workloads: pointwise / 3x3 / strided / depthwise
    convolutions with bias, ReLU and swish, residual adds, window pooling, squeeze-excite gates (GlobalAveragePool ->
    1x1 conv -> Sigmoid -> Mul), channel Split / Concat, the ShuffleNet channel shuffle (Reshape - Transpose -
    Reshape), nearest upsampling.  Exercises the planner and, with layout selection, the channels-last kernels on
    structures no hand-written test has."""
    r = np.random.RandomState(7000 + seed)
    st = _st(2000 + seed)
    b = GraphBuilder(f"random_cnn_{seed}", dtype)
    N = int(r.choice([1, 2, 3]))
    C = int(r.choice([8, 16, 24, 32]))
    R = int(r.choice([8, 12, 14, 16]))
    if big:       # maps and channel counts that reach the larger tiles, the LDS-staged depthwise kernel, split pooling
        N, C, R = int(r.choice([4, 8])), int(r.choice([32, 64, 96])), int(r.choice([28, 40, 56]))
    x = b.input("x", (N, C, R, R), st.normal((N, C, R, R), 0.0, 1.0, dtype))
    live = [x]
    used = []
    n_w = 0

    def weight(shape, std):
        nonlocal n_w
        n_w += 1
        return b.weight(f"w{n_w}", shape, st.normal(shape, 0.0, std, dtype))

    def conv(t, co, k, stride=1, group=1):
        c = b.shape(t)[1]
        w = weight((co, c // group, k, k), math.sqrt(2.0 / (c // group * k * k)))
        bias = weight((co,), 0.1) if r.rand() < 0.7 else None
        return configs._conv(b, t, w, bias, stride, k // 2, group)

    for _ in range(n_ops):
        t = live[int(r.randint(max(0, len(live) - 4), len(live)))]       # mostly recent tensors: chains with a few branches
        used.append(t)
        n, c, h, w_ = b.shape(t)
        kinds = ["pw", "c3", "dw", "act", "res", "pool", "se", "split", "shuffle", "up", "affine"]
        probs = [0.2, 0.12, 0.14, 0.12, 0.1, 0.07, 0.07, 0.05, 0.05, 0.03, 0.05]
        if wide:      # decoder and style-transfer pieces as well
            kinds += ["convt", "inorm", "d2s", "s2d", "cslice"]
            probs = [q * 0.75 for q in probs] + [0.05, 0.06, 0.04, 0.04, 0.06]
        kind = r.choice(kinds, p=probs)
        if kind == "pw":
            y = conv(t, int(r.choice([64, 96, 128, 192] if big else [8, 16, 24, 32, 48])), 1)
        elif kind == "c3":
            s = 2 if h >= 8 and r.rand() < 0.3 else 1
            y = conv(t, int(r.choice([32, 64] if big else [8, 16, 32])), 3, stride=s)
        elif kind == "dw":
            k = int(r.choice([3, 5]))
            s = 2 if h >= 8 and r.rand() < 0.25 else 1
            y = conv(t, c, k, stride=s, group=c)
        elif kind == "act":
            y = configs._un(b, "Relu", t) if r.rand() < 0.5 else configs._swish(b, t)
        elif kind == "res":
            others = [o for o in live if b.shape(o) == (n, c, h, w_) and o is not t]
            if not others:
                continue
            o = others[int(r.randint(len(others)))]
            used.append(o)
            y = configs._bin(b, "Add", t, o)
        elif kind == "pool":
            if h < 4:
                continue
            k, s, p = [(2, 2, 0), (3, 2, 1), (3, 1, 1)][int(r.randint(3))]
            ho = (h + 2 * p - k) // s + 1
            y = b.op(str(r.choice(["MaxPool", "AveragePool"])), [t], (n, c, ho, ho), {"kernel_shape": [k, k], "strides": [s, s], "pads": [p] * 4})
        elif kind == "se":
            g = b.op("GlobalAveragePool", [t], (n, c, 1, 1))
            cm = max(4, c // 4)
            g = configs._un(b, "Relu", conv(g, cm, 1))
            g = configs._un(b, "Sigmoid", conv(g, c, 1))
            y = configs._bin(b, "Mul", t, g)
        elif kind == "split":
            if c % 16:
                continue
            p0, p1 = b.op("Split", [t], [(n, c // 2, h, w_)] * 2, {"axis": 1, "split": [c // 2, c // 2]})
            y = b.op("Concat", [configs._un(b, "Relu", conv(p1, c // 2, 1)), p0], (n, c, h, w_), {"axis": 1})
        elif kind == "shuffle":
            if c % 2:
                continue
            y = configs._reshape(b, configs._transpose(b, configs._reshape(b, t, (n, 2, c // 2, h, w_)), (0, 2, 1, 3, 4)), (n, c, h, w_))
        elif kind == "up":
            if h > 8 or n * c * h * w_ * 4 > 1 << 16:
                continue
            y = b.op("Resize", [t], (n, c, 2 * h, 2 * w_), {"scales": [1, 1, 2, 2]})
        elif kind == "convt":
            if h > 8:
                continue
            co = int(r.choice([8, 16]))
            wt = weight((c, co, 4, 4), math.sqrt(8.0 / (c * 16)))
            y = b.op("ConvTranspose", [t, wt, weight((co,), 0.1)], (n, co, 2 * h, 2 * w_), {"strides": [2, 2], "pads": [1] * 4, "output_padding": [0, 0], "group": 1})
            y = b.op("LeakyRelu", [y], (n, co, 2 * h, 2 * w_), {"alpha": 0.1})
        elif kind == "inorm":
            if h * w_ < 4:
                continue
            sc = b.weight(f"isc{len(live)}", (c,), st.uniform((c,), 0.5, 1.5, dtype))
            sh = b.weight(f"ish{len(live)}", (c,), st.normal((c,), 0.0, 0.3, dtype))
            y = configs._un(b, "Relu", b.op("InstanceNormalization", [t, sc, sh], (n, c, h, w_), {"epsilon": 1e-5}))
        elif kind == "d2s":
            if c % 4 or h > 8:
                continue
            y = b.op("DepthToSpace", [t], (n, c // 4, 2 * h, 2 * w_), {"blocksize": 2, "mode_crd": int(r.rand() < 0.5)})
        elif kind == "s2d":
            if h % 2 or w_ % 2:
                continue
            y = b.op("SpaceToDepth", [t], (n, c * 4, h // 2, w_ // 2), {"blocksize": 2})
        elif kind == "cslice":
            if c < 16:
                continue
            lo = int(r.choice([0, 8]))
            y = b.op("Slice", [t], (n, 8, h, w_), {"starts": [lo], "ends": [lo + 8], "axes": [1]})
        else:
            sc = b.weight(f"sc{len(live)}", (1, c, 1, 1), st.uniform((1, c, 1, 1), 0.5, 1.5, dtype))
            sh = b.weight(f"sh{len(live)}", (1, c, 1, 1), st.normal((1, c, 1, 1), 0.0, 0.2, dtype))
            y = configs._bin(b, "Add", configs._bin(b, "Mul", t, sc), sh)
        live.append(y)
    outs = [t for t in live[1:] if not any(t is u for u in used)] or [live[-1]]
    for t in outs:
        b.mark_output(t)
    return b.finish()


def random_seq(seed, dtype="f16", n_ops=8, big=False):
    """A seeded random sequence model over [B, S, D] activations from the pieces of the transformer workloads: an
    optional embedding Gather, linear layers (bias, GELU / ReLU / none), LayerNorm in its exported decomposition,
    residual adds, attention (fused QKV or separate projections, K transposed by the head split or by an extra
    Transpose, scale as Mul or Div, padding / causal / no mask, optionally written as Einsum), Split / Concat
    along the feature axis and a CumSum."""
    r = np.random.RandomState(9000 + seed)
    st = _st(3000 + seed)
    b = GraphBuilder(f"random_seq_{seed}", dtype)
    B, S = int(r.choice([1, 2, 3])), int(r.choice([8, 24, 40, 72]))
    NH = int(r.choice([1, 2, 4]))
    hd = int(r.choice([8, 16, 32]))
    if big:       # several key tiles per attention row, GEMMs that reach the larger tiles
        B, S, NH, hd = int(r.choice([2, 4])), int(r.choice([136, 200, 384])), int(r.choice([4, 6])), int(r.choice([32, 64]))
    D = NH * hd
    n_w = 0

    def weight(shape, std, name=None):
        nonlocal n_w
        n_w += 1
        return b.weight(name or f"w{n_w}", shape, st.normal(shape, 0.0, std, dtype))

    def lin(t, n, act=None, bias=True):
        k = b.shape(t)[-1]
        y = configs._matmul(b, t, weight((k, n), 1.0 / math.sqrt(k)))
        if bias:
            y = configs._bin(b, "Add", y, weight((n,), 0.1))
        if act == "gelu":
            y = configs._gelu_erf(b, y, f"g{n_w}")
        elif act == "relu":
            y = configs._un(b, "Relu", y)
        return y

    if r.rand() < 0.4:
        V = int(r.choice([50, 128]))
        ids = b.input("ids", (B, S), st.integers((B, S), 0, V), dtype="i64")
        x = b.op("Gather", [weight((V, D), 1.0, "wte"), ids], (B, S, D), {"axis": 0})
        x = configs._bin(b, "Add", x, weight((S, D), 0.3, "wpe"))
    else:
        x = b.input("x", (B, S, D), st.normal((B, S, D), 0.0, 1.0, dtype))
    live = [x]
    used = []
    for i in range(n_ops):
        t = live[int(r.randint(max(0, len(live) - 3), len(live)))]
        used.append(t)
        kind = r.choice(["lin", "ln", "res", "attn", "ffn", "splitcat", "cumsum"], p=[0.2, 0.18, 0.14, 0.22, 0.14, 0.08, 0.04])
        if kind == "lin":
            y = lin(t, D, act=[None, "relu", "gelu"][int(r.randint(3))], bias=r.rand() < 0.8)
        elif kind == "ln":
            y = configs._layernorm(b, configs._Streams(4000 + seed * 50 + i), t, D, dtype, f"ln{i}")
        elif kind == "res":
            others = [o for o in live if o is not t]
            if not others:
                continue
            o = others[int(r.randint(len(others)))]
            used.append(o)
            y = configs._bin(b, "Add", t, o)
        elif kind == "ffn":
            F = int(r.choice([2, 4])) * D
            y = configs._bin(b, "Add", lin(lin(t, F, act="gelu"), D), t)
        elif kind == "splitcat":
            p0, p1 = b.op("Split", [t], [(B, S, D // 2)] * 2, {"axis": 2, "split": [D // 2, D // 2]})
            y = b.op("Concat", [configs._un(b, "Tanh", p1), p0], (B, S, D), {"axis": 2})
        elif kind == "cumsum":
            y = configs._bin(b, "Mul", b.op("CumSum", [t], (B, S, D), {"axis": 1}), b.const(f"inv{i}", 1.0 / S))
        else:
            if r.rand() < 0.5:
                q, k, v = b.op("Split", [lin(t, 3 * D)], [(B, S, D)] * 3, {"axis": 2, "split": [D, D, D]})
            else:
                q, k, v = lin(t, D), lin(t, D, bias=False), lin(t, D)
            q = configs._transpose(b, configs._reshape(b, q, (B, S, NH, hd)), (0, 2, 1, 3))
            v = configs._transpose(b, configs._reshape(b, v, (B, S, NH, hd)), (0, 2, 1, 3))
            form = int(r.randint(3))
            if form == 0:
                k = configs._transpose(b, configs._reshape(b, k, (B, S, NH, hd)), (0, 2, 3, 1))
                s = configs._matmul(b, q, k)
            elif form == 1:
                k = configs._transpose(b, configs._reshape(b, k, (B, S, NH, hd)), (0, 2, 1, 3))
                s = configs._matmul(b, q, configs._transpose(b, k, (0, 1, 3, 2)))
            else:
                k = configs._transpose(b, configs._reshape(b, k, (B, S, NH, hd)), (0, 2, 1, 3))
                s = b.op("Einsum", [q, k], (B, NH, S, S), {"equation": "bhid,bhjd->bhij"})
            s = configs._bin(b, "Mul", s, b.const(f"sc{i}", 1.0 / math.sqrt(hd))) if r.rand() < 0.5 else \
                configs._bin(b, "Div", s, b.const(f"sd{i}", math.sqrt(hd)))
            mk = int(r.randint(3))
            if mk == 0:
                mv = np.zeros((B, 1, 1, S), dtype=np.float64)
                mv[..., S - max(1, S // 8):] = -1e4
                s = configs._bin(b, "Add", s, b.weight(f"pad{i}", (B, 1, 1, S), rng.round_to(mv, dtype)))
            elif mk == 1:
                cm = np.triu(np.full((S, S), -1e4), k=1).reshape(1, 1, S, S)
                s = configs._bin(b, "Add", s, b.weight(f"causal{i}", (1, 1, S, S), rng.round_to(cm, dtype)))
            p = b.op("Softmax", [s], (B, NH, S, S), {"axis": -1})
            o = configs._matmul(b, p, v)
            y = lin(configs._reshape(b, configs._transpose(b, o, (0, 2, 1, 3)), (B, S, D)), D)
            if r.rand() < 0.6:
                y = configs._bin(b, "Add", y, t)
        live.append(y)
    outs = [t for t in live[1:] if not any(t is u for u in used)] or [live[-1]]
    for t in outs:
        b.mark_output(t)
    return b.finish()


def gather_block(ids, table_shape=(23, 40), axis=0, dtype="f32", ids_dtype="i64", const_ids=False, seed=41):
    """table[..., ids, ...] * 2 + 1: an embedding-style Gather along `axis` with a One-to-One epilogue.  `ids` may hold
    negative values (they count from the end of the axis, as the operator is defined)."""
    st = _st(seed)
    b = GraphBuilder("gather_block", dtype)
    ids = np.asarray(ids)
    table = b.weight("table", table_shape, st.normal(table_shape, 0.0, 1.0, dtype))
    if const_ids:
        i = b._add("ids", ids_dtype, ids.shape, "weight", ids.astype(np.int64), const=True)
    else:
        i = b.input("ids", ids.shape, ids.astype(np.int64), dtype=ids_dtype)
    out = tuple(table_shape[:axis]) + tuple(ids.shape) + tuple(table_shape[axis + 1:])
    y = b.op("Gather", [table, i], out, {"axis": axis})
    y = configs._bin(b, "Add", configs._bin(b, "Mul", y, b.const("two", 2.0)), b.const("one", 1.0))
    b.mark_output(y)
    return b.finish()
