"""Pins for the fp64 oracle: closed forms, brute-force loops, invariants.

None of these re-types an oracle formula: each compares the oracle with a
value fixed by mathematics (a closed form, a quadrature, an identity) or with
a literal nested-loop evaluation of the operator's definition on a tiny input.
"""
import itertools
import math

import numpy as np
import pytest

from oracle.interp import eval_op, run_graph
from workloads import configs, rng
from workloads.graph import GraphBuilder

R = np.random.default_rng(7)


def ev(kind, ins, **attrs):
    return eval_op(kind, [np.asarray(i, dtype=np.float64) for i in ins], attrs)


# ----------------------------------------------------------------- One-to-One operators
def test_elementwise_closed_forms():
    assert ev("Exp", [[0.0, 1.0, -1.0]]) == pytest.approx([1.0, math.e, 1 / math.e], rel=1e-15)
    assert ev("Tanh", [[0.0]])[0] == 0.0
    assert ev("Sigmoid", [[0.0]])[0] == 0.5
    assert ev("Erf", [[0.0]])[0] == 0.0
    assert ev("Erf", [[6.0]])[0] == pytest.approx(1.0, abs=1e-15)
    assert ev("Log", [[math.e ** 3]])[0] == pytest.approx(3.0, rel=1e-15)
    assert ev("Sqrt", [[2.25]])[0] == 1.5
    assert ev("Reciprocal", [[4.0]])[0] == 0.25
    assert list(ev("Relu", [[-2.0, 0.0, 3.0]])) == [0.0, 0.0, 3.0]
    assert list(ev("Abs", [[-2.0, 3.0]])) == [2.0, 3.0]
    assert list(ev("Neg", [[-2.0, 3.0]])) == [2.0, -3.0]
    assert list(ev("Clip", [[-9.0, 0.5, 9.0]], min=-4.0, max=4.0)) == [-4.0, 0.5, 4.0]
    assert list(ev("Square", [[-3.0, 0.5]])) == [9.0, 0.25]
    assert list(ev("Pow", [[2.0, 3.0], 3.0])) == [8.0, 27.0]
    assert list(ev("LeakyRelu", [[-2.0, 2.0]], alpha=0.1)) == [-0.2, 2.0]
    assert list(ev("Sub", [[5.0], [3.0]])) == [2.0] and list(ev("Div", [[6.0], [3.0]])) == [2.0]
    assert list(ev("Max", [[1.0, 5.0], [3.0, 2.0]])) == [3.0, 5.0]
    assert list(ev("Where", [[1.0, 0.0], [10.0, 11.0], [20.0, 21.0]])) == [10.0, 21.0]


def test_elementwise_identities():
    x = R.normal(size=1000) * 3
    # odd / even symmetry
    for k in ("Tanh", "Erf"):
        assert np.allclose(ev(k, [x]), -ev(k, [-x]), rtol=0, atol=1e-16)
    # sigmoid(x) = (1 + tanh(x/2)) / 2 ; sigmoid(x) + sigmoid(-x) = 1
    assert np.allclose(ev("Sigmoid", [x]), 0.5 * (1 + np.tanh(x / 2)), rtol=1e-14)
    assert np.allclose(ev("Sigmoid", [x]) + ev("Sigmoid", [-x]), 1.0, rtol=1e-15)
    # tanh = (e^2x - 1)/(e^2x + 1)
    e2 = np.exp(2 * x)
    assert np.allclose(ev("Tanh", [x]), (e2 - 1) / (e2 + 1), rtol=1e-12, atol=1e-15)
    # exp(a+b) = exp(a)exp(b)
    assert np.allclose(ev("Exp", [x + 1.0]), ev("Exp", [x]) * math.e, rtol=1e-14)


def _simpson(f, a, b, n=4000):
    t = np.linspace(a, b, n + 1)
    w = np.ones(n + 1)
    w[1:-1:2], w[2:-1:2] = 4, 2
    return (b - a) / (3 * n) * np.sum(w * f(t))


def test_erf_against_quadrature():
    for x in (0.1, 0.5, 1.0, 1.7, 2.5, -0.8):
        ref = 2 / math.sqrt(math.pi) * _simpson(lambda t: np.exp(-t * t), 0.0, x)
        assert ev("Erf", [[x]])[0] == pytest.approx(ref, rel=1e-11)


def test_gelu_graphs_against_normal_cdf():
    """The erf-form GELU subgraph equals x * Phi(x), Phi by quadrature of the normal density;
    the tanh-form subgraph equals its closed expression."""
    xs = np.array([-2.0, -0.5, 0.3, 1.0, 2.2])
    b = GraphBuilder("g", "f32")
    x = b.input("x", xs.shape, xs)
    y = configs._gelu_erf(b, x, "ge")
    z = configs._gelu_tanh(b, x, "gt")
    b.mark_output(y), b.mark_output(z)
    g = b.finish()
    # constants were rounded to f32 in the graph; evaluate with exact ones for this pin
    for t in g.tensors.values():
        if t.const:
            t.data = {"ge_sqrt2": math.sqrt(2), "gt_c1": math.sqrt(2 / math.pi), "gt_c0": 0.044715}.get(t.name, float(t.data))
            t.data = np.array(t.data, dtype=np.float64)
    out = run_graph(g)
    for i, xv in enumerate(xs):
        phi = 0.5 + _simpson(lambda t: np.exp(-t * t / 2) / math.sqrt(2 * math.pi), 0.0, xv)
        assert out[y][i] == pytest.approx(xv * phi, rel=1e-10)
        ref = 0.5 * xv * (1 + math.tanh(math.sqrt(2 / math.pi) * (xv + 0.044715 * xv ** 3)))
        assert out[z][i] == pytest.approx(ref, rel=1e-14)


def test_broadcasting_follows_trailing_axis_alignment():
    a = R.normal(size=(2, 3, 4, 5))
    c = R.normal(size=(1, 3, 1, 1))
    v = R.normal(size=(5,))
    got = ev("Add", [a, c])
    got2 = ev("Mul", [a, v])
    for n, ch, h, w in itertools.product(range(2), range(3), range(4), range(5)):
        assert got[n, ch, h, w] == a[n, ch, h, w] + c[0, ch, 0, 0]
        assert got2[n, ch, h, w] == a[n, ch, h, w] * v[w]


def test_batchnorm_closed_form_and_affine_equivalence():
    x = R.normal(size=(2, 3, 4, 4))
    g, b_, m, v = R.uniform(0.5, 1.5, 3), R.normal(size=3), R.normal(size=3), R.uniform(0.5, 1.5, 3)
    got = ev("BatchNormalization", [x, g, b_, m, v], epsilon=1e-5)
    for c in range(3):
        s = g[c] / math.sqrt(v[c] + 1e-5)
        assert np.allclose(got[:, c], x[:, c] * s + (b_[c] - m[c] * s), rtol=1e-13, atol=1e-13)
    # x == mean maps to beta exactly
    xm = np.broadcast_to(m.reshape(1, 3, 1, 1), x.shape)
    assert np.array_equal(ev("BatchNormalization", [xm, g, b_, m, v], epsilon=1e-5)[0, :, 0, 0], b_)


# ----------------------------------------------------------------- Many-to-Many operators
def _conv_loops(x, w, bias, s, p, group):
    n, c, h, wd = x.shape
    co, cg, kh, kw = w.shape
    ho, wo = (h + 2 * p - kh) // s + 1, (wd + 2 * p - kw) // s + 1
    out = np.zeros((n, co, ho, wo))
    og = co // group
    for b in range(n):
        for o in range(co):
            g = o // og
            for y in range(ho):
                for xx in range(wo):
                    acc = 0.0 if bias is None else bias[o]
                    for ci in range(cg):
                        for i in range(kh):
                            for j in range(kw):
                                yy, xj = y * s + i - p, xx * s + j - p
                                if 0 <= yy < h and 0 <= xj < wd:
                                    acc += x[b, g * cg + ci, yy, xj] * w[o, ci, i, j]
                    out[b, o, y, xx] = acc
    return out


@pytest.mark.parametrize("c,co,k,s,p,group,bias", [
    (3, 4, 3, 1, 1, 1, True), (4, 6, 3, 2, 1, 2, False), (4, 4, 5, 2, 2, 4, True), (2, 3, 1, 1, 0, 1, True),
    (3, 2, 3, 2, 1, 1, False)])
def test_conv_against_seven_deep_loops(c, co, k, s, p, group, bias):
    x = R.normal(size=(2, c, 6, 5))
    w = R.normal(size=(co, c // group, k, k))
    b_ = R.normal(size=co) if bias else None
    got = eval_op("Conv", [x, w] + ([b_] if bias else []), {"strides": [s, s], "pads": [p] * 4, "group": group})
    assert np.allclose(got, _conv_loops(x, w, b_, s, p, group), rtol=1e-13, atol=1e-13)


def test_conv_special_cases():
    x = R.normal(size=(2, 5, 6, 7))
    # 1x1 convolution is a matrix product over channels
    w = R.normal(size=(4, 5, 1, 1))
    got = eval_op("Conv", [x, w], {"strides": [1, 1], "pads": [0] * 4, "group": 1})
    ref = np.einsum("oc,nchw->nohw", w[:, :, 0, 0], x)
    assert np.allclose(got, ref, rtol=1e-13)
    # a delta kernel at tap (0, 2) with padding 1 shifts the image left by one, zero filled
    d = np.zeros((5, 1, 3, 3))
    d[:, 0, 1, 2] = 1.0
    got = eval_op("Conv", [x, d], {"strides": [1, 1], "pads": [1] * 4, "group": 5})
    ref = np.zeros_like(x)
    ref[..., :-1] = x[..., 1:]
    assert np.array_equal(got, ref)
    # linearity in the input
    w3 = R.normal(size=(3, 5, 3, 3))
    a = {"strides": [2, 2], "pads": [1] * 4, "group": 1}
    x2 = R.normal(size=x.shape)
    assert np.allclose(eval_op("Conv", [2 * x + x2, w3], a), 2 * eval_op("Conv", [x, w3], a) + eval_op("Conv", [x2, w3], a), rtol=1e-12, atol=1e-12)


def test_matmul_against_triple_loop_and_batch_broadcast():
    a = R.normal(size=(2, 3, 4, 5))
    b_ = R.normal(size=(5, 6))
    got = eval_op("MatMul", [a, b_], {})
    for i, j, m, n in itertools.product(range(2), range(3), range(4), range(6)):
        assert got[i, j, m, n] == pytest.approx(sum(a[i, j, m, k] * b_[k, n] for k in range(5)), rel=1e-13, abs=1e-14)
    c = R.normal(size=(2, 3, 5, 4))
    got = eval_op("MatMul", [a, c], {})
    for i, j in itertools.product(range(2), range(3)):
        assert np.allclose(got[i, j], a[i, j] @ c[i, j], rtol=1e-13)
    # identity and operand order (a transposed operand would fail here)
    assert np.array_equal(eval_op("MatMul", [a[0, 0], np.eye(5)], {}), a[0, 0])
    u, v = np.array([[1.0, 2.0]]), np.array([[3.0], [4.0]])
    assert eval_op("MatMul", [u, v], {}).shape == (1, 1) and eval_op("MatMul", [v, u], {}).tolist() == [[3.0, 6.0], [4.0, 8.0]]


def test_gemm_flags():
    a, b_, c = R.normal(size=(4, 3)), R.normal(size=(5, 4)), R.normal(size=(5,))
    got = eval_op("Gemm", [a, b_, c], {"transA": 1, "transB": 1, "alpha": 0.5, "beta": 2.0})
    assert np.allclose(got, 0.5 * a.T @ b_.T + 2.0 * c, rtol=1e-14)


def test_reductions_and_pooling():
    x = R.normal(size=(2, 3, 4, 5))
    assert np.allclose(eval_op("ReduceMean", [x], {"axes": [-1], "keepdims": 1})[1, 2, 3, 0], sum(x[1, 2, 3]) / 5, rtol=1e-14)
    assert eval_op("ReduceSum", [x], {"axes": [1, 3], "keepdims": 0}).shape == (2, 4)
    assert eval_op("ReduceMax", [x], {"axes": [-1], "keepdims": 1})[0, 0, 0, 0] == max(x[0, 0, 0])
    assert eval_op("ReduceProd", [x], {"axes": [3], "keepdims": 0})[0, 1, 2] == pytest.approx(math.prod(x[0, 1, 2]), rel=1e-13)
    gap = eval_op("GlobalAveragePool", [x], {})
    assert gap.shape == (2, 3, 1, 1) and gap[1, 2, 0, 0] == pytest.approx(x[1, 2].sum() / 20, rel=1e-14)
    assert np.array_equal(eval_op("GlobalAveragePool", [np.full((1, 2, 3, 3), 1.25)], {}), np.full((1, 2, 1, 1), 1.25))


def test_softmax_invariants():
    x = R.normal(size=(3, 4, 17)) * 5
    p = eval_op("Softmax", [x], {"axis": -1})
    assert np.allclose(p.sum(-1), 1.0, rtol=1e-14)
    assert np.allclose(eval_op("Softmax", [x + 123.0], {"axis": -1}), p, rtol=1e-12)
    # ratio of two entries is exp of the difference
    assert p[0, 0, 3] / p[0, 0, 5] == pytest.approx(math.exp(x[0, 0, 3] - x[0, 0, 5]), rel=1e-12)
    # additive -1e4 mask: masked probabilities are exactly zero
    xm = x.copy()
    xm[..., 12:] += -1e4
    pm = eval_op("Softmax", [xm], {"axis": -1})
    assert np.all(pm[..., 12:] == 0.0) and np.allclose(pm[..., :12].sum(-1), 1.0)
    # two-class softmax is the logistic function
    z = np.array([[0.7, -0.4]])
    assert eval_op("Softmax", [z], {"axis": -1})[0, 0] == pytest.approx(1 / (1 + math.exp(-1.1)), rel=1e-14)


def test_decomposed_softmax_equals_primitive():
    g = configs.gpt2_decoder(B=1, S=8, D=16, NH=2, F=32, L=1, V=50, P=8)
    out = run_graph(g, keep="all")
    # locate the decomposed softmax: Div whose second operand is a ReduceSum
    prod = {o.outputs[0]: o for o in g.ops}
    hits = 0
    for o in g.ops:
        if o.kind == "Div" and prod.get(o.inputs[1]) is not None and prod[o.inputs[1]].kind == "ReduceSum":
            sub = prod[prod[o.inputs[0]].inputs[0]]
            scores = out[sub.inputs[0]]
            assert np.allclose(out[o.outputs[0]], eval_op("Softmax", [scores], {"axis": -1}), rtol=1e-13)
            # causal: strictly upper triangle is exactly zero
            assert np.all(np.triu(out[o.outputs[0]][0, 0], k=1) == 0.0)
            hits += 1
    assert hits == 1


def test_layernorm_decomposition_moments():
    b = GraphBuilder("ln", "f32")
    xs = R.normal(size=(5, 48)) * 3 + 1
    x = b.input("x", xs.shape, xs)
    st = configs._Streams(3)
    y = configs._layernorm(b, st, x, 48, "f32", "t", eps=1e-5)
    b.mark_output(y)
    g = b.finish()
    out = run_graph(g, keep="all")
    div = [o for o in g.ops if o.kind == "Div"][0].outputs[0]
    n = out[div]
    var = xs.var(axis=1)
    assert np.allclose(n.mean(axis=1), 0.0, atol=1e-14)
    assert np.allclose(n.var(axis=1), var / (var + np.float64(np.float32(1e-5))), rtol=1e-12)
    gam, bet = g.tensors["t_gamma"].data.astype(np.float64), g.tensors["t_beta"].data.astype(np.float64)
    assert np.allclose(out[y], n * gam + bet, rtol=1e-14)


def test_conv_bn_folding_equivalence():
    """conv -> BatchNormalization equals a conv with per-output-channel scaled weights plus a bias."""
    g = configs.residual_block(N=1, C=4, H=6, W=6)
    out = run_graph(g, keep="all")
    bn = [o for o in g.ops if o.kind == "BatchNormalization"][0]
    T = {k: v.data.astype(np.float64) for k, v in g.tensors.items() if v.data is not None}
    s = T["bn_gamma"] / np.sqrt(T["bn_var"] + 1e-5)
    folded = eval_op("Conv", [T["x"], T["conv_w"] * s[:, None, None, None], T["bn_beta"] - T["bn_mean"] * s],
                     {"strides": [1, 1], "pads": [1] * 4, "group": 1})
    assert np.allclose(out[bn.outputs[0]], folded, rtol=1e-12, atol=1e-13)


# ----------------------------------------------------------------- Reorganize / Shuffle / One-to-Many
def _unravel(i, shape):
    idx = []
    for d in reversed(shape):
        idx.append(i % d)
        i //= d
    return tuple(reversed(idx))


def test_transpose_and_reshape_on_iota():
    shape, perm = (2, 3, 4, 5), (0, 2, 3, 1)
    x = np.arange(120, dtype=np.float64).reshape(shape)
    t = eval_op("Transpose", [x], {"perm": list(perm)})
    oshape = tuple(shape[p] for p in perm)
    for o in range(120):
        oi = _unravel(o, oshape)
        ii = [0] * 4
        for k, p in enumerate(perm):
            ii[p] = oi[k]
        assert t[oi] == x[tuple(ii)]
    r = eval_op("Reshape", [t], {"shape": [6, 20]})
    assert np.array_equal(r.ravel(), t.ravel())


def test_channel_shuffle_permutation_of_chain_config():
    """Composite index map of config 2's tail: out[n, hw, c'] = in[n, (c' mod g)*(C/g) + c' div g, hw]."""
    N, C, H, W, G = 2, 16, 3, 5, 4
    g = configs.memory_bound_chain(N=N, C=C, H=H, W=W, groups=G, rounds=0)
    iota = np.arange(N * C * H * W, dtype=np.float64).reshape(N, C, H, W)
    out = list(run_graph(g, feeds={"x": iota}).values())[0]
    assert out.shape == (N, H * W, C)
    for n, hw, cp in itertools.product(range(N), range(H * W), range(C)):
        c = (cp % G) * (C // G) + cp // G
        assert out[n, hw, cp] == iota[n, c, hw // W, hw % W]
    # shuffling with (g, C/g) and then (C/g, g) is the identity
    x = np.arange(C, dtype=np.float64)
    s1 = x.reshape(G, C // G).T.reshape(C)
    s2 = eval_op("Transpose", [s1.reshape(C // G, G)], {"perm": [1, 0]}).reshape(C)
    assert np.array_equal(s2, x)


def test_gather_slice_split_concat_expand():
    table = R.normal(size=(7, 3))
    ids = np.array([[6, 0], [2, 2]])
    got = eval_op("Gather", [table, ids], {"axis": 0})
    assert got.shape == (2, 2, 3)
    for i, j in itertools.product(range(2), range(2)):
        assert np.array_equal(got[i, j], table[ids[i, j]])
    x = np.arange(24, dtype=np.float64).reshape(2, 3, 4)
    assert eval_op("Slice", [x], {"starts": [1], "ends": [3], "axes": [2]}).tolist() == [[[1, 2], [5, 6], [9, 10]], [[13, 14], [17, 18], [21, 22]]]
    a, b_ = eval_op("Split", [x], {"axis": 2, "split": [1, 3]})
    assert a.shape == (2, 3, 1) and b_[1, 2].tolist() == [21, 22, 23]
    assert np.array_equal(eval_op("Concat", [a, b_], {"axis": 2}), x)
    e = eval_op("Expand", [np.array([[1.0], [2.0]])], {"shape": [2, 3]})
    assert e.tolist() == [[1, 1, 1], [2, 2, 2]]


# ----------------------------------------------------------------- whole graphs
def test_residual_block_graph_against_loops():
    g = configs.residual_block(N=1, C=3, H=5, W=4)
    T = {k: v.data.astype(np.float64) for k, v in g.tensors.items() if v.data is not None}
    y = _conv_loops(T["x"], T["conv_w"], None, 1, 1, 1)
    ref = np.zeros_like(y)
    for c in range(3):
        bn = T["bn_gamma"][c] * (y[0, c] - T["bn_mean"][c]) / np.sqrt(T["bn_var"][c] + 1e-5) + T["bn_beta"][c]
        ref[0, c] = np.maximum(np.maximum(bn, 0) + T["x"][0, c], 0)
    out = list(run_graph(g).values())[0]
    assert np.allclose(out, ref, rtol=1e-12, atol=1e-13)


def test_chain_graph_against_scalar_python():
    g = configs.memory_bound_chain(N=1, C=4, H=2, W=3, groups=2, rounds=2)
    T = {k: v.data.astype(np.float64) for k, v in g.tensors.items() if v.data is not None}
    out = list(run_graph(g).values())[0]
    for c, h, w in itertools.product(range(4), range(2), range(3)):
        v = T["x"][0, c, h, w]
        for r in range(2):
            v = (v + T[f"r{r}_c1"][0, c, 0, 0]) * T[f"r{r}_c2"][0, c, 0, 0]
            v = math.exp(min(max(v, -4.0), 4.0))
            v = math.tanh(1 / (1 + math.exp(-v)))
            v = v * (math.erf(v / float(T[f"r{r}_gelu_sqrt2"])) + 1.0) * 0.5
            v = math.sqrt(abs(v * v) + 1.0)
        cp = [k for k in range(4) if (k % 2) * 2 + k // 2 == c][0]
        assert out[0, h * 3 + w, cp] == pytest.approx(v, rel=1e-13)


def test_attention_rows_of_encoder_layer():
    """Scores, mask and softmax of the encoder config: masked keys get zero weight, rows sum to one,
    and one attention output entry equals its scalar definition."""
    B, S, D, NH = 2, 20, 16, 2
    g = configs.transformer_encoder_layer(B=B, S=S, D=D, NH=NH, F=32, dtype="f32")
    out = run_graph(g, keep="all")
    sm = [o for o in g.ops if o.kind == "Softmax"][0]
    p = out[sm.outputs[0]]
    assert p.shape == (B, NH, S, S)
    assert np.all(p[..., S - 2:] == 0.0) and np.allclose(p.sum(-1), 1.0)
    T = {k: v.data.astype(np.float64) for k, v in g.tensors.items() if v.data is not None}
    qkv = T["x"] @ T["qkv_w"] + T["qkv_b"]
    hd = D // NH
    b_, h, i = 1, 1, 7
    q = qkv[b_, i, h * hd:(h + 1) * hd]
    sc = np.array([q @ qkv[b_, j, D + h * hd:D + (h + 1) * hd] for j in range(S)]) * float(T["attn_scale"]) + T["attn_mask"][b_, 0, 0]
    w = np.exp(sc - sc.max())
    w /= w.sum()
    assert np.allclose(p[b_, h, i], w, rtol=1e-12)
    o = sum(w[j] * qkv[b_, j, 2 * D + h * hd:2 * D + (h + 1) * hd] for j in range(S))
    pv = [x for x in g.ops if x.kind == "MatMul"][2].outputs[0]
    assert np.allclose(out[pv][b_, h, i], o, rtol=1e-12)


def test_all_configs_evaluate_small():
    small = {
        "residual_block": dict(N=1, C=8, H=9, W=7),
        "memory_bound_chain": dict(N=2, C=16, H=5, W=6, groups=4),
        "transformer_encoder_layer": dict(B=2, S=24, D=32, NH=4, F=64),
        "efficientnet_b0": dict(N=1, R=32),
        "gpt2_decoder": dict(B=1, S=16, D=32, NH=4, F=64, L=2, V=97, P=16),
    }
    for name, kw in small.items():
        g = configs.CONFIGS[name](**kw)
        out = run_graph(g)
        assert len(out) == (1 + kw["L"] if name == "gpt2_decoder" else 1)      # the decoder also returns every layer's key / value
        for v in out.values():
            assert np.all(np.isfinite(v))


def test_rng_is_counter_based_and_storage_rounding_is_rne():
    a = rng.normal(5, 1, (1000,))
    assert np.array_equal(a[100:200], np.sqrt(-2 * np.log(1 - rng.uniform01(5, 1_000_005, 100, 100))) * np.cos(2 * np.pi * rng.uniform01(5, 1_000_006, 100, 100)))
    assert abs(a.mean()) < 0.15 and 0.85 < a.std() < 1.15
    # bf16 RNE: 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even (1.0); 1 + 3*2^-8 ties to 1 + 2^-6
    assert rng.round_to(np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -20]), "bf16").tolist() == [1.0, 1 + 2.0 ** -6, 1 + 2.0 ** -7]
    assert rng.round_to(np.array([2049.0]), "f16").tolist() == [2048.0]


def test_resize_nearest_by_index_formula():
    """Resize / Upsample with integer factors: out[n, c, i, j] = in[n, c, i // sh, j // sw] (brute force)."""
    x = np.arange(2 * 3 * 4 * 5, dtype=np.float64).reshape(2, 3, 4, 5)
    for kind, sc in (("Resize", [1, 1, 2, 3]), ("Upsample", [1, 2, 1, 2])):
        y = eval_op(kind, [x], {"scales": sc})
        assert y.shape == tuple(d * s for d, s in zip(x.shape, sc))
        for idx in itertools.product(*[range(d) for d in y.shape]):
            assert y[idx] == x[tuple(i // s for i, s in zip(idx, sc))]
    # factor 1 everywhere is the identity; values are copied, never interpolated
    assert np.array_equal(eval_op("Resize", [x], {"scales": [1, 1, 1, 1]}), x)


def test_window_pooling_against_scalar_loops_and_special_cases():
    """MaxPool / AveragePool: every output element against a scalar loop over its window (padding excluded,
    or counted as zeros with count_include_pad); a window covering the whole map is the global pool; a 1x1
    window is the identity; pooling a constant map gives the constant."""
    rs = np.random.default_rng(7)
    x = rs.normal(size=(2, 3, 7, 6))
    for kind in ("MaxPool", "AveragePool"):
        for (kh, kw), (sh, sw), pads, inc in [((3, 3), (2, 2), (1, 1, 1, 1), 0), ((2, 3), (1, 2), (0, 1, 1, 0), 1), ((2, 2), (2, 2), (0, 0, 0, 0), 0)]:
            y = eval_op(kind, [x], {"kernel_shape": [kh, kw], "strides": [sh, sw], "pads": list(pads), "count_include_pad": inc})
            ho = (7 + pads[0] + pads[2] - kh) // sh + 1
            wo = (6 + pads[1] + pads[3] - kw) // sw + 1
            assert y.shape == (2, 3, ho, wo)
            for n, c, p, q in itertools.product(range(2), range(3), range(ho), range(wo)):
                vals = []
                for i, j in itertools.product(range(kh), range(kw)):
                    ih, iw = p * sh + i - pads[0], q * sw + j - pads[1]
                    if 0 <= ih < 7 and 0 <= iw < 6:
                        vals.append(x[n, c, ih, iw])
                want = max(vals) if kind == "MaxPool" else sum(vals) / (kh * kw if inc else len(vals))
                assert y[n, c, p, q] == pytest.approx(want, rel=1e-14, abs=1e-15)
    whole = {"kernel_shape": [7, 6], "strides": [1, 1], "pads": [0, 0, 0, 0]}
    assert np.allclose(eval_op("AveragePool", [x], whole), eval_op("GlobalAveragePool", [x], {}), rtol=1e-14)
    assert np.array_equal(eval_op("MaxPool", [x], whole)[:, :, 0, 0], x.max(axis=(2, 3)))
    one = {"kernel_shape": [1, 1], "strides": [1, 1], "pads": [0, 0, 0, 0]}
    assert np.array_equal(eval_op("MaxPool", [x], one), x) and np.array_equal(eval_op("AveragePool", [x], one), x)
    const = np.full((1, 2, 5, 5), 3.25)
    pad = {"kernel_shape": [3, 3], "strides": [1, 1], "pads": [1, 1, 1, 1]}
    assert np.array_equal(eval_op("MaxPool", [const], pad), const) and np.allclose(eval_op("AveragePool", [const], pad), const, rtol=1e-15)


def test_einsum_against_scalar_loops_and_matrix_products():
    """Einsum: every result element of small cases against nested scalar loops over the summed labels; the matrix
    product, the batched product with a transposed operand and the outer product as special cases."""
    rs = np.random.default_rng(21)
    cases = [("ik,kj->ij", (3, 4), (4, 5)), ("bhid,bhjd->bhij", (2, 2, 3, 4), (2, 2, 5, 4)), ("bij,bjk->bki", (2, 3, 4), (2, 4, 2)),
             ("i,j->ji", (3,), (4,)), ("abc,cbd->ad", (2, 3, 4), (4, 3, 2)), ("nchw,oc->nohw", (2, 3, 2, 2), (4, 3))]
    for eq, sa, sb in cases:
        a, b = rs.normal(size=sa), rs.normal(size=sb)
        got = eval_op("Einsum", [a, b], {"equation": eq})
        lhs, out = eq.split("->")
        ta, tb = lhs.split(",")
        ext = {l: a.shape[i] for i, l in enumerate(ta)}
        ext.update({l: b.shape[i] for i, l in enumerate(tb)})
        summed = [l for l in sorted(ext) if l not in out]
        assert got.shape == tuple(ext[l] for l in out), eq
        for oidx in itertools.product(*[range(ext[l]) for l in out]):
            env = dict(zip(out, oidx))
            acc = 0.0
            for sidx in itertools.product(*[range(ext[l]) for l in summed]):
                env.update(zip(summed, sidx))
                acc += a[tuple(env[l] for l in ta)] * b[tuple(env[l] for l in tb)]
            assert got[oidx] == pytest.approx(acc, rel=1e-12, abs=1e-12), (eq, oidx)
    a, b = rs.normal(size=(3, 4)), rs.normal(size=(4, 5))
    np.testing.assert_allclose(eval_op("Einsum", [a, b], {"equation": "ik,kj->ij"}), a @ b, rtol=1e-13)
    np.testing.assert_allclose(eval_op("Einsum", [a, b.T], {"equation": "ik,jk->ji"}), (a @ b).T, rtol=1e-13)
    np.testing.assert_array_equal(eval_op("Einsum", [a[0], b[0]], {"equation": "i,j->ij"}), np.outer(a[0], b[0]))


def test_bitshift_both_directions_by_hand():
    """BitShift: worked values, the doubling / halving identities and right-after-left being the identity."""
    x = np.array([5, 1, 12, 1023], dtype=np.int64)
    s = np.array([2, 10, 0, 3], dtype=np.int64)
    left = eval_op("BitShift", [x, s], {})
    assert np.asarray(left).astype(np.int64).tolist() == [20, 1024, 12, 8184]
    right = eval_op("BitShift", [x, s], {"direction_right": 1})
    assert np.asarray(right).astype(np.int64).tolist() == [1, 0, 12, 127]
    assert np.asarray(left).astype(np.int64).tolist() == (x * 2 ** s).tolist()
    assert np.asarray(right).astype(np.int64).tolist() == (x // 2 ** s).tolist()
    back = eval_op("BitShift", [np.asarray(left).astype(np.int64), s], {"direction_right": 1})
    assert np.asarray(back).astype(np.int64).tolist() == x.tolist()


def test_truth_value_operators():
    """Greater / Not / Where on 0 / 1 truth values: a worked example by hand, De Morgan through Where."""
    x, y = np.array([1.0, -2.0, 3.0, 0.5]), np.array([0.0, 0.0, 4.0, 0.5])
    m = eval_op("Greater", [x, y], {})
    assert m.tolist() == [1.0, 0.0, 0.0, 0.0]
    n = eval_op("Not", [m], {})
    assert n.tolist() == [0.0, 1.0, 1.0, 1.0]
    assert eval_op("Not", [n], {}).tolist() == m.tolist()
    assert eval_op("Where", [n, x, y], {}).tolist() == [0.0, -2.0, 3.0, 0.5]
    assert eval_op("Where", [m, x, y], {}).tolist() == [1.0, 0.0, 4.0, 0.5]


def test_cumsum_against_scalar_loops_closed_forms_and_differences():
    """Prefix sums: scalar loops on a small tensor for every axis and flag, the closed form on a constant and on
    1..n (triangular numbers), and the inverse relation out[i] - out[i-1] = x[i]."""
    rs = np.random.RandomState(5)
    x = rs.standard_normal((3, 4, 5))
    for axis in (0, 1, 2, -1):
        for excl in (False, True):
            for rev in (False, True):
                got = eval_op("CumSum", [x], {"axis": axis, "exclusive": int(excl), "reverse": int(rev)})
                xm = np.moveaxis(x, axis, -1)
                want = np.zeros_like(xm)
                n = xm.shape[-1]
                for i in range(xm.shape[0]):
                    for j in range(xm.shape[1]):
                        for k in range(n):
                            js = [q for q in range(n) if (q > k if excl else q >= k)] if rev else [q for q in range(n) if (q < k if excl else q <= k)]
                            want[i, j, k] = sum(xm[i, j, q] for q in js)
                np.testing.assert_allclose(got, np.moveaxis(want, -1, axis), rtol=1e-12, atol=1e-12)
    cs = lambda v, axis, **kw: eval_op("CumSum", [np.asarray(v)], dict(axis=axis, **kw))
    np.testing.assert_array_equal(cs(np.full((2, 6), 2.0), 1), np.tile(2.0 * np.arange(1, 7), (2, 1)))
    np.testing.assert_array_equal(cs(np.arange(1.0, 9.0), 0), [k * (k + 1) / 2 for k in range(1, 9)])
    np.testing.assert_array_equal(cs(np.arange(1.0, 9.0), 0, exclusive=1), [k * (k - 1) / 2 for k in range(1, 9)])
    np.testing.assert_array_equal(cs(np.arange(1.0, 5.0), 0, reverse=1), [10.0, 9.0, 7.0, 4.0])
    np.testing.assert_allclose(np.diff(cs(x, 1), axis=1), x[:, 1:, :], rtol=1e-12, atol=1e-12)
    # inclusive = exclusive + x; the last inclusive element is the plain sum
    np.testing.assert_allclose(cs(x, 2), cs(x, 2, exclusive=1) + x, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(cs(x, 2)[..., -1], x.sum(axis=2), rtol=1e-12)


def test_depth_space_shuffles_against_their_reshape_transpose_definition():
    """DepthToSpace / SpaceToDepth: the oracle evaluates the index formula; the operators are defined as a
    Reshape - Transpose - Reshape chain, which numpy spells out independently here.  The two are inverse to each
    other (depth-column-row order), and a block size of 1 is the identity."""
    rs = np.random.default_rng(3)
    x = rs.normal(size=(2, 12, 3, 5))
    b, cp = 2, 3
    d = eval_op("DepthToSpace", [x], {"blocksize": b})
    want = x.reshape(2, b, b, cp, 3, 5).transpose(0, 3, 4, 1, 5, 2).reshape(2, cp, 3 * b, 5 * b)
    assert np.array_equal(d, want)
    dc = eval_op("DepthToSpace", [x], {"blocksize": b, "mode_crd": 1})
    assert np.array_equal(dc, x.reshape(2, cp, b, b, 3, 5).transpose(0, 1, 4, 2, 5, 3).reshape(2, cp, 3 * b, 5 * b))
    assert not np.array_equal(d, dc)
    y = rs.normal(size=(2, 3, 6, 10))
    s = eval_op("SpaceToDepth", [y], {"blocksize": b})
    assert np.array_equal(s, y.reshape(2, 3, 3, b, 5, b).transpose(0, 3, 5, 1, 2, 4).reshape(2, 12, 3, 5))
    assert np.array_equal(eval_op("DepthToSpace", [s], {"blocksize": b}), y)
    assert np.array_equal(eval_op("SpaceToDepth", [y], {"blocksize": 1}), y)
    # single elements through the printed index formula
    assert d[1, 2, 2 * b + 1, 4 * b + 0] == x[1, (1 * b + 0) * cp + 2, 2, 4]


def test_instance_normalization_statistics_and_affine():
    """Per (n, c): zero mean and variance var / (var + eps) before the affine step; scale and bias act per channel;
    a single-image, single-channel map equals the LayerNorm statistics chain over the flattened map."""
    rs = np.random.default_rng(4)
    x = rs.normal(1.0, 3.0, size=(3, 4, 5, 7))
    one, zero = np.ones(4), np.zeros(4)
    y = eval_op("InstanceNormalization", [x, one, zero], {"epsilon": 1e-3})
    assert np.allclose(y.mean(axis=(2, 3)), 0.0, atol=1e-14)
    v = x.var(axis=(2, 3))
    assert np.allclose(y.var(axis=(2, 3)), v / (v + 1e-3), rtol=1e-12)
    sc, bs = rs.uniform(0.5, 2.0, 4), rs.normal(size=4)
    z = eval_op("InstanceNormalization", [x, sc, bs], {"epsilon": 1e-3})
    assert np.allclose(z, y * sc[None, :, None, None] + bs[None, :, None, None], rtol=1e-13, atol=1e-13)
    flat = eval_op("Normalize", [x[:1, :1].reshape(1, 35)], {"epsilon": 1e-3})
    assert np.allclose(y[0, 0].reshape(1, 35), flat, rtol=1e-13, atol=1e-14)


def test_more_elementwise_operators():
    x = np.array([-2.5, -1.5, -0.5, 0.5, 1.5, 2.5, 0.49999, -0.50001])
    assert eval_op("Round", [x], {}).tolist() == [-2.0, -2.0, -0.0, 0.0, 2.0, 2.0, 0.0, -1.0]      # ties to even
    t = np.linspace(-3, 3, 41)
    assert np.allclose(eval_op("Sin", [t], {}) ** 2 + eval_op("Cos", [t], {}) ** 2, 1.0, rtol=1e-15)
    assert eval_op("Sin", [np.array([0.0, math.pi / 2])], {}).tolist() == pytest.approx([0.0, 1.0])
    u = np.linspace(-1.5, 1.5, 31)
    assert np.allclose(eval_op("Asin", [eval_op("Sin", [u], {})], {}), u, rtol=1e-13, atol=1e-15)
    assert eval_op("Floor", [x], {}).tolist() == [-3.0, -2.0, -1.0, 0.0, 1.0, 2.0, 0.0, -1.0]
    assert eval_op("Ceil", [x], {}).tolist() == [-2.0, -1.0, -0.0, 1.0, 2.0, 3.0, 1.0, -0.0]
    slope = np.full(8, 0.1)
    assert np.array_equal(eval_op("PRelu", [x, slope], {}), eval_op("LeakyRelu", [x], {"alpha": 0.1}))
    assert eval_op("PRelu", [np.array([-2.0, 3.0]), np.array([0.5, 7.0])], {}).tolist() == [-1.0, 3.0]


def test_conv3d_against_scalar_loops_and_the_2d_convolution():
    """3-d convolution: every output element of a small case against the eight-deep scalar loop; a kernel of depth 1
    is the 2-d convolution of every depth slice; a one-hot kernel shifts the input; the bias is added per channel."""
    rs = np.random.default_rng(11)
    x = rs.normal(size=(2, 3, 4, 5, 6))
    w = rs.normal(size=(4, 3, 2, 3, 2))
    bias = rs.normal(size=4)
    strides, pads = [1, 2, 1], [1, 1, 0, 0, 1, 1]
    y = eval_op("Conv", [x, w, bias], {"strides": strides, "pads": pads})
    do, ho, wo = (4 + 1 + 0 - 2) // 1 + 1, (5 + 1 + 1 - 3) // 2 + 1, (6 + 0 + 1 - 2) // 1 + 1
    assert y.shape == (2, 4, do, ho, wo)
    for n, o, d, p, q in itertools.product(range(2), range(4), range(do), range(ho), range(wo)):
        acc = bias[o]
        for c, a, i, j in itertools.product(range(3), range(2), range(3), range(2)):
            zd, zh, zw = d * 1 + a - 1, p * 2 + i - 1, q * 1 + j - 0
            if 0 <= zd < 4 and 0 <= zh < 5 and 0 <= zw < 6:
                acc += x[n, c, zd, zh, zw] * w[o, c, a, i, j]
        assert y[n, o, d, p, q] == pytest.approx(acc, rel=1e-12, abs=1e-12)
    w1 = rs.normal(size=(4, 3, 1, 3, 3))
    y3 = eval_op("Conv", [x, w1], {"strides": [1, 1, 1], "pads": [0, 1, 1, 0, 1, 1]})
    for d in range(4):
        y2 = eval_op("Conv", [x[:, :, d], w1[:, :, 0]], {"strides": [1, 1], "pads": [1, 1, 1, 1]})
        assert np.allclose(y3[:, :, d], y2, rtol=1e-13, atol=1e-13)
    hot = np.zeros((3, 3, 3, 3, 3))
    for c in range(3):
        hot[c, c, 0, 1, 2] = 1.0        # reads x[d - 1, p, q + 1]
    ys = eval_op("Conv", [x, hot], {"strides": [1, 1, 1], "pads": [1, 1, 1, 1, 1, 1]})
    assert np.array_equal(ys[:, :, 1:, :, :-1], x[:, :, :-1, :, 1:]) and np.all(ys[:, :, 0] == 0) and np.all(ys[:, :, :, :, -1] == 0)


def test_conv_transpose_against_gather_loops_the_adjoint_identity_and_the_flipped_convolution():
    """ConvTranspose (the oracle scatters): every output element of a small case against the gather-form scalar loop;
    <ConvTranspose(x), y> = <x, Conv(y)> with the same filter read as [O = C, I = CO] (the operator is the adjoint of
    the convolution); at stride 1 it equals a convolution with the filter flipped and its channel axes exchanged."""
    rs = np.random.default_rng(12)
    x = rs.normal(size=(2, 3, 4, 5))
    w = rs.normal(size=(3, 2, 3, 4))
    bias = rs.normal(size=2)
    for strides, pads, opad in (([2, 3], [1, 0, 0, 2], [1, 0]), ([1, 1], [0, 1, 2, 0], [0, 0]), ([2, 2], [1, 1, 1, 1], [1, 1])):
        y = eval_op("ConvTranspose", [x, w, bias], {"strides": strides, "pads": pads, "output_padding": opad})
        ho = (4 - 1) * strides[0] - pads[0] - pads[2] + 3 + opad[0]
        wo = (5 - 1) * strides[1] - pads[1] - pads[3] + 4 + opad[1]
        assert y.shape == (2, 2, ho, wo)
        for n, o, p, q in itertools.product(range(2), range(2), range(ho), range(wo)):
            acc = bias[o]
            for c, i, j in itertools.product(range(3), range(3), range(4)):
                th, tw = p + pads[0] - i, q + pads[1] - j
                if th >= 0 and tw >= 0 and th % strides[0] == 0 and tw % strides[1] == 0 and th // strides[0] < 4 and tw // strides[1] < 5:
                    acc += x[n, c, th // strides[0], tw // strides[1]] * w[c, o, i, j]
            assert y[n, o, p, q] == pytest.approx(acc, rel=1e-12, abs=1e-12)
    # adjoint of Conv with strides / pads alike
    strides, pads = [2, 2], [1, 1, 1, 1]
    yt = eval_op("ConvTranspose", [x, w], {"strides": strides, "pads": pads})
    z = rs.normal(size=yt.shape)
    back = eval_op("Conv", [z, w], {"strides": strides, "pads": pads})      # w read as [O = 3, I = 2, kh, kw]
    assert back.shape == x.shape
    assert float(np.sum(yt * z)) == pytest.approx(float(np.sum(x * back)), rel=1e-12)
    # stride 1: a convolution with the flipped, channel-exchanged filter and pads k - 1 - p
    y1 = eval_op("ConvTranspose", [x, w], {"strides": [1, 1], "pads": [1, 2, 1, 2]})
    wf = np.ascontiguousarray(w[:, :, ::-1, ::-1].transpose(1, 0, 2, 3))
    y2 = eval_op("Conv", [x, wf], {"strides": [1, 1], "pads": [3 - 1 - 1, 4 - 1 - 2, 3 - 1 - 1, 4 - 1 - 2]})
    assert np.allclose(y1, y2, rtol=1e-13, atol=1e-13)


def test_attention_unit_graph_rows_against_scalar_python():
    """The attention unit graph (Q K^T / sqrt(D) + mask -> Softmax -> V, heads merged) evaluated by the
    oracle equals a scalar-loop evaluation of a few output elements."""
    import sys, os
    sys.path.insert(0, os.path.dirname(__file__))
    import unit_graphs as U

    spec = U.attention_block(1, 2, 5, 8, 4, dtype="f32", mask="causal")
    (name, out), = run_graph(spec).items()
    q, kt, v, m = (spec.tensors[n].data.astype(np.float64) for n in ("q", "kt", "v", "mask"))
    for (h, i, d) in ((0, 0, 0), (1, 3, 2), (1, 4, 3)):
        s = [sum(q[0, h, i, e] * kt[0, h, e, j] for e in range(4)) / math.sqrt(4.0) + m[0, 0, i, j] for j in range(8)]
        mx = max(s)
        p = [math.exp(a - mx) for a in s]
        want = sum(p[j] / sum(p) * v[0, h, j, d] for j in range(8))
        assert abs(out[0, i, h * 4 + d] - want) <= 1e-12 * max(1.0, abs(want))


def test_min_max_worked_values_and_lattice_identities():
    """Min / Max: values worked by hand (broadcast included), then the identities that a swapped or sign-flipped
    implementation breaks: min + max = a + b, min = -max(-a, -b), min <= both operands."""
    a = np.array([[1.0, -2.0, 3.5], [0.0, 7.0, -7.0]])
    b = np.array([0.5, -1.0, 4.0])
    assert eval_op("Min", [a, b], {}).tolist() == [[0.5, -2.0, 3.5], [0.0, -1.0, -7.0]]
    assert eval_op("Max", [a, b], {}).tolist() == [[1.0, -1.0, 4.0], [0.5, 7.0, 4.0]]
    rs = np.random.default_rng(5)
    x, y = rs.normal(size=(4, 9)), rs.normal(size=(4, 9))
    mn, mx = eval_op("Min", [x, y], {}), eval_op("Max", [x, y], {})
    assert np.array_equal(mn + mx, x + y) or np.allclose(mn + mx, x + y, rtol=0, atol=1e-15)
    assert np.array_equal(mn, -eval_op("Max", [-x, -y], {}))
    assert np.all(mn <= x) and np.all(mn <= y) and np.all((mn == x) | (mn == y))


def test_cos_values_sign_and_phase():
    """Cos: exact points (a result of -cos or sin would fail them), evenness, and the quarter-period shift of Sin."""
    pts = eval_op("Cos", [np.array([0.0, math.pi, math.pi / 3, 2 * math.pi / 3])], {})
    assert pts[0] == 1.0 and pts[1] == -1.0
    assert pts[2] == pytest.approx(0.5, abs=1e-15) and pts[3] == pytest.approx(-0.5, abs=1e-15)
    t = np.linspace(-4, 4, 81)
    assert np.array_equal(eval_op("Cos", [t], {}), eval_op("Cos", [-t], {}))
    assert np.allclose(eval_op("Cos", [t], {}), eval_op("Sin", [t + math.pi / 2], {}), rtol=0, atol=1e-15)
    # derivative check against the series: cos t ~ 1 - t^2/2 + t^4/24 near 0
    s = np.array([1e-3, -2e-3])
    assert np.allclose(eval_op("Cos", [s], {}), 1 - s ** 2 / 2 + s ** 4 / 24, rtol=0, atol=3e-16)


def test_gather_along_inner_axes_against_nested_loops():
    """Gather with axis 1 and axis -1 (and negative indices, which count from the end): element by element
    out[i, j.., k] = data[i, ids[j..], k], the index tensor's axes standing where the gathered axis stood."""
    rs = np.random.default_rng(6)
    data = rs.normal(size=(3, 5, 4))
    ids = np.array([[4, 0, 0], [-1, 2, -5]])
    g1 = eval_op("Gather", [data, ids], {"axis": 1})
    assert g1.shape == (3, 2, 3, 4)
    for i, p, q, k in itertools.product(range(3), range(2), range(3), range(4)):
        j = int(ids[p, q])
        j = j + 5 if j < 0 else j
        assert g1[i, p, q, k] == data[i, j, k]
    ids2 = np.array([3, -4, 1, 1, 0])
    g2 = eval_op("Gather", [data, ids2], {"axis": -1})
    assert g2.shape == (3, 5, 5)
    for i, j, p in itertools.product(range(3), range(5), range(5)):
        k = int(ids2[p])
        k = k + 4 if k < 0 else k
        assert g2[i, j, p] == data[i, j, k]
    # axis 2 written positively is the same operator
    assert np.array_equal(g2, eval_op("Gather", [data, ids2], {"axis": 2}))


def test_slice_with_steps_and_offsets_against_index_loops():
    """Slice with steps: out[i] = x[start + i * step] for as long as the index stays before `end`; several axes at
    once; a start in the middle; a step that does not divide the range."""
    x = np.arange(2 * 9 * 7, dtype=np.float64).reshape(2, 9, 7)
    y = eval_op("Slice", [x], {"starts": [1, 2], "ends": [9, 7], "axes": [1, 2], "steps": [3, 2]})
    rows = list(range(1, 9, 3))          # 1, 4, 7
    cols = list(range(2, 7, 2))          # 2, 4, 6
    assert y.shape == (2, len(rows), len(cols)) == (2, 3, 3)
    for n, i, j in itertools.product(range(2), range(3), range(3)):
        assert y[n, i, j] == x[n, 1 + 3 * i, 2 + 2 * j]
    z = eval_op("Slice", [x], {"starts": [0], "ends": [8], "axes": [1], "steps": [5]})      # 0, 5: the range is not a multiple of the step
    assert z.shape == (2, 2, 7) and np.array_equal(z[:, 1], x[:, 5])
    one = eval_op("Slice", [x], {"starts": [3], "ends": [6], "axes": [2], "steps": [1]})
    assert np.array_equal(one, eval_op("Slice", [x], {"starts": [3], "ends": [6], "axes": [2]}))
    assert one[1, 8].tolist() == [x[1, 8, 3], x[1, 8, 4], x[1, 8, 5]]


def test_unsqueeze_and_squeeze_by_axes():
    """Unsqueeze inserts extent-1 dimensions at the named positions of the result, Squeeze removes the named ones;
    neither moves an element (checked on iota against the flat order and against hand-written shapes)."""
    x = np.arange(24, dtype=np.float64).reshape(2, 3, 4)
    u = eval_op("Unsqueeze", [x], {"axes": [0, 3]})
    assert u.shape == (1, 2, 3, 1, 4) and np.array_equal(u.ravel(), x.ravel())
    assert u[0, 1, 2, 0, 3] == x[1, 2, 3]
    assert eval_op("Unsqueeze", [x], {"axes": [-1]}).shape == (2, 3, 4, 1)
    assert eval_op("Unsqueeze", [x], {"axes": [1]}).shape == (2, 1, 3, 4)
    q = eval_op("Squeeze", [u], {"axes": [0, 3]})
    assert q.shape == x.shape and np.array_equal(q, x)
    assert eval_op("Squeeze", [u], {"axes": [3]}).shape == (1, 2, 3, 4)
    # stacking two tensors the way a key / value pair is returned: Unsqueeze each at 0, Concat along 0
    a, b_ = x, x + 100
    st = eval_op("Concat", [eval_op("Unsqueeze", [a], {"axes": [0]}), eval_op("Unsqueeze", [b_], {"axes": [0]})], {"axis": 0})
    assert st.shape == (2, 2, 3, 4) and st[1, 1, 2, 3] == x[1, 2, 3] + 100 and st[0, 0, 0, 1] == 1


def test_where_and_cast_on_a_causal_mask():
    """Where(mask, x, c) keeps x where the mask is set and takes c elsewhere (a swapped pair of branches fails);
    Cast changes no value.  On a lower-triangular boolean mask the result is x on and below the diagonal."""
    n = 5
    mask = np.tril(np.ones((n, n)))
    x = np.arange(n * n, dtype=np.float64).reshape(n, n) + 1
    y = eval_op("Where", [eval_op("Cast", [mask], {"to": 9}), x, np.array(-1e4)], {})
    for i in range(n):
        for j in range(n):
            assert y[i, j] == (x[i, j] if j <= i else -1e4)
    assert np.array_equal(eval_op("Cast", [x], {"to": 1}), x)
