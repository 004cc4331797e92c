"""Fusion-plan exploration against the paper's worked examples (Sec. 4.3 Fig. 3, Sec. 4.4.1 Fig. 4,
the chains named in Sec. 6) and the plans of the five workloads.  Host only: plans are built
without profiling, no kernel is launched."""
import numpy as np
import pytest

from paper_2108_13342_amd import api
from workloads import configs
from workloads.graph import GraphBuilder

O2O, REORG, SHUF, O2M, M2M = range(5)


def _plan(spec, rewrite=False, **kw):
    g, ids = api.graph_from_spec(spec)
    if rewrite:
        g.rewrite()
    nw = len([t for t in spec.tensors.values() if t.kind == "weight"])
    p = api.Plan(g, [1] * nw, profile=0, **kw)
    blocks = [d for d in p.describe() if not d["prepare_only"]]
    return g, p, blocks


def _z(shape):
    return np.zeros(shape, dtype=np.float32)


def fig3_graph():
    """GEMM -> Add -> Conv -> Relu -> Mul -> Sub, all results of one shape (Fig. 3's assumption)."""
    b = GraphBuilder("fig3", "f32")
    sh = (1, 8, 12, 12)
    a = b.input("a", (1, 8, 12, 16), _z((1, 8, 12, 16)))
    w = b.weight("w", (16, 12), _z((16, 12)))
    x2 = b.input("x2", sh, _z(sh))
    m = b.input("m", sh, _z(sh))
    s = b.input("s", sh, _z(sh))
    cw = b.weight("cw", (8, 8, 3, 3), _z((8, 8, 3, 3)))
    g = configs._matmul(b, a, w)
    t = configs._bin(b, "Add", g, x2)
    t = configs._conv(b, t, cw, None, 1, 1)
    t = configs._un(b, "Relu", t)
    t = configs._bin(b, "Mul", t, m)
    t = configs._bin(b, "Sub", t, s)
    b.mark_output(t)
    return b.finish()


def test_fig3_worked_example():
    """Seed Add; successors Conv, Relu, Mul, Sub join: a five-operator block of type Many-to-Many
    (the paper says Many-to-One, which it folds into Many-to-Many); the preceding GEMM is refused
    because block and GEMM are both Many-to-Many (fuse_break)."""
    _, p, blocks = _plan(fig3_graph(), successors_first=1)
    assert [b["ops"] for b in blocks] == [["MatMul"], ["Add", "Conv", "Relu", "Mul", "Sub"]]
    assert blocks[1]["fused_type"] == M2M
    # with predecessors explored first (this build's default; Sec. 4.3 allows swapping the two steps)
    # the GEMM takes the Add as its epilogue and the red cell then falls between Add and Conv
    _, _, blocks = _plan(fig3_graph(), successors_first=0)
    assert [b["ops"] for b in blocks] == [["MatMul", "Add"], ["Conv", "Relu", "Mul", "Sub"]]


def fig4_graph():
    """Out = IRS3 + IRS5 with IRS3 = Recip(IRS2), IRS2 = IRS1 * C, IRS5 = IRS1 * D... both Mul read
    IRS1 = GEMM(A, B): the common sub-tree of the data-flow tree."""
    b = GraphBuilder("fig4", "f32")
    A = b.input("A", (24, 16), _z((24, 16)))
    B = b.weight("B", (16, 20), _z((16, 20)))
    C = b.input("C", (24, 20), _z((24, 20)))
    D = b.input("D", (24, 20), _z((24, 20)))
    irs1 = configs._matmul(b, A, B)
    irs2 = configs._bin(b, "Mul", irs1, C)
    irs3 = configs._un(b, "Reciprocal", irs2)
    irs5 = configs._bin(b, "Mul", irs1, D)
    out = configs._bin(b, "Add", irs3, irs5)
    b.mark_output(out)
    return b.finish()


def test_fig4_code_generation_example():
    """All five operators end in one Many-to-Many block (Add+Recip -> One-to-One, +Mul -> One-to-One,
    +GEMM -> Many-to-One); the GEMM result shared by both Mul is evaluated once."""
    for order in (0, 1):
        _, p, blocks = _plan(fig4_graph(), successors_first=order)
        assert len(blocks) == 1 and sorted(blocks[0]["ops"]) == ["Add", "MatMul", "Mul", "Mul", "Reciprocal"]
        assert blocks[0]["fused_type"] == M2M and blocks[0]["family"] == 2
        src = p.block_source(0)
        epi = src[src.index("DEV void epilogue("):src.index("#define EPI_VEC")]
        assert epi.count("= anchor_v;") == 1           # one read of the shared sub-tree
        assert epi.count("cvt_out(") == 1


def test_gemm_div_transpose_example():
    """Sec. 4.4.1: GEMM + Div + Transpose - Transpose and Div fuse to a Shuffle-typed operator and the
    GEMM writes each output element to the destination that operator decides."""
    b = GraphBuilder("gdt", "f32")
    A = b.input("A", (40, 16), _z((40, 16)))
    B = b.weight("B", (16, 24), _z((16, 24)))
    d = b.input("d", (40, 24), _z((40, 24)))
    y = configs._transpose(b, configs._bin(b, "Div", configs._matmul(b, A, B), d), (1, 0))
    b.mark_output(y)
    assert api.fuse_relation(O2O, SHUF) == (SHUF, 0)
    assert api.fuse_relation(M2M, SHUF)[0] == M2M
    _, p, blocks = _plan(b.finish())
    assert len(blocks) == 1 and blocks[0]["ops"] == ["MatMul", "Div", "Transpose"] and blocks[0]["family"] == 2
    src = p.block_source(0)
    epi = src[src.index("DEV void epilogue"):src.index("#define KPARAMS")]
    # row r of the GEMM lands in column r of the [24, 40] result: stride 1 on the row atom, 40 on the column atom
    store = [l for l in epi.splitlines() if "cvt_out(" in l][0]
    assert "* 40" in store and "* 24" not in store


def test_named_chains_fuse_into_one_block():
    """Sec. 6: MatMul + Reshape + Transpose + Add (GPT-2) and Sub + Pow + ReduceMean + Add + Sqrt (TinyBERT)."""
    b = GraphBuilder("gpt2_chain", "f32")
    x = b.input("x", (2, 16, 32), _z((2, 16, 32)))
    w = b.weight("w", (32, 32), _z((32, 32)))
    r = b.input("r", (2, 4, 16, 8), _z((2, 4, 16, 8)))
    y = configs._matmul(b, x, w)
    y = configs._transpose(b, configs._reshape(b, y, (2, 16, 4, 8)), (0, 2, 1, 3))
    y = configs._bin(b, "Add", y, r)
    b.mark_output(y)
    _, _, blocks = _plan(b.finish())
    assert len(blocks) == 1 and blocks[0]["ops"] == ["MatMul", "Reshape", "Transpose", "Add"]

    def chain(mu_kind):
        b = GraphBuilder("tinybert_chain", "f32")
        x = b.input("x", (6, 48), _z((6, 48)))
        mu = b.weight("mu", (6, 1), _z((6, 1))) if mu_kind == "weight" else b.input("mu", (6, 1), _z((6, 1)))
        t = configs._bin(b, "Sub", x, mu)
        t = configs._bin(b, "Pow", t, b.const("two", 2.0))
        t = configs._reduce(b, "ReduceMean", t, [-1])
        t = configs._bin(b, "Add", t, b.const("eps", 1e-5))
        t = configs._un(b, "Sqrt", t)
        b.mark_output(t)
        return b.finish()

    _, _, blocks = _plan(chain("weight"))
    assert len(blocks) == 1 and blocks[0]["ops"] == ["Sub", "Pow", "ReduceMean", "Add", "Sqrt"]
    assert blocks[0]["family"] == 1 and blocks[0]["fused_type"] == M2M
    # When the subtrahend is a broadcast ACTIVATION the Sub is "elementwise with broadcast", i.e.
    # One-to-Many by Table 2, and One-to-Many -> Many-to-Many is one of the two red cells: by the
    # table the Sub stays outside, although Sec. 6 lists the chain as fusable.  In LayerNorm graphs the
    # whole statistics chain is recognised as one Normalize operator before planning, so it still
    # ends in a single block there (test_rewrite_* and the workload plans).
    _, _, blocks = _plan(chain("activation"))
    assert [b["ops"] for b in blocks] == [["Sub"], ["Pow", "ReduceMean", "Add", "Sqrt"]]


def test_seed_is_smallest_one_to_one_result():
    """Step I: the One-to-One operator with the smallest intermediate result seeds first; here the
    [4, 1] Sqrt, not the earlier and larger Relu."""
    b = GraphBuilder("seed", "f32")
    x = b.input("x", (4, 64), _z((4, 64)))
    t = configs._un(b, "Relu", x)
    r = configs._reduce(b, "ReduceSum", t, [-1])
    y = configs._un(b, "Sqrt", r)
    b.mark_output(y)
    g, ids = api.graph_from_spec(b.finish())
    p = api.Plan(g, [], profile=0)
    log = p.dump_json()["log"]
    seeds = [l for l in log if l.startswith("seed")]
    assert seeds[0].startswith("seed Sqrt")
    assert [d["ops"] for d in p.describe()] == [["Relu", "ReduceSum", "Sqrt"]]


def test_red_cell_keeps_two_contractions_apart_and_blocks_stay_acyclic():
    spec = configs.transformer_encoder_layer(**configs.SMALL["transformer_encoder_layer"])
    g, p, blocks = _plan(spec, rewrite=True)
    ops = [b["ops"] for b in blocks]
    for o in ops:
        heavy = [k for k in o if k in ("MatMul", "Softmax", "Normalize", "Conv")]
        assert len(heavy) <= 1, o
    assert len(blocks) == 9
    # (a leading Transpose is the folded half of the weight re-layout: see test_weight_layout_rewrite)
    # the head-splitting Transposes are not stored transposed by the QKV projection: each is left to the contraction that
    # reads it, where it is an index map on the operand load (Q K^T then reads K contiguous along the head dimension)
    assert ops[0] == ["Transpose", "MatMul", "Add", "Split", "Reshape", "Reshape", "Reshape"]
    assert ["Transpose", "Transpose", "MatMul", "Mul", "Add"] in ops and ["Transpose", "MatMul"] in ops
    assert ["Softmax"] in ops and ["Transpose", "MatMul", "Add", "Mul", "Erf", "Add", "Mul", "Mul"] in ops
    # the GELU chain is not pulled in front of the second FFN GEMM (it would be recomputed per tile column)
    assert ["Transpose", "MatMul", "Add", "Add"] in ops
    # every block's inputs are produced by earlier blocks
    d = p.dump_json()
    seen = set()
    for blk in d["blocks"]:
        for t in blk["inputs"]:
            assert t["kind"] in ("input", "weight") or t["name"] in seen or t["ws_offset"] >= 0
        seen |= {t["name"] for t in blk["outputs"]}


@pytest.mark.parametrize("name,max_blocks", [("residual_block", 1), ("memory_bound_chain", 1), ("efficientnet_b0", 115),
                                             ("gpt2_decoder", 24)])
def test_workload_fusion_rates(name, max_blocks):
    spec = configs.CONFIGS[name](**configs.SMALL[name])
    _, p, blocks = _plan(spec, rewrite=True)
    kernels = [b for b in blocks if b["family"] != 5]
    assert len(kernels) <= max_blocks, [b["ops"] for b in kernels]
    assert sum(b["irs_bytes_removed"] for b in blocks) > 0


def test_unfused_plan_is_one_block_per_operator():
    spec = configs.transformer_encoder_layer(**configs.SMALL["transformer_encoder_layer"])
    _, p, blocks = _plan(spec, fusion=0)
    assert len(blocks) == len(spec.ops) and all(b["n_ops"] == 1 for b in blocks)


def test_constraint_check_limits_block_size():
    spec = configs.memory_bound_chain(**configs.SMALL["memory_bound_chain"])
    _, _, blocks = _plan(spec, max_block_ops=10)
    assert max(b["n_ops"] for b in blocks) <= 10 and len(blocks) >= 5


def test_intra_block_folding_of_index_operators():
    """Sec. 4.4.2: a Transpose / Slice read by one consumer becomes a change of index.  The tied
    vocabulary projection reads the embedding table through a Transpose: no transposed copy is made."""
    spec = configs.gpt2_decoder(**configs.SMALL["gpt2_decoder"])
    _, p, blocks = _plan(spec, rewrite=True)
    assert blocks[-1]["ops"] == ["Transpose", "MatMul"]
    # the only work left to do on weights at prepare time: the re-layout the rewriter asked for, the position rows
    # gathered by the constant position ids, and the slice of the causal buffer the layers select with
    assert all(d["ops"] in (["Transpose"], ["Gather"], ["Slice", "Slice", "Cast"]) for d in p.describe() if d["prepare_only"])
    _, p2, blocks2 = _plan(spec, rewrite=True, intra_block=0)
    assert any(d["ops"] != ["Transpose"] for d in p2.describe() if d["prepare_only"])


def test_weight_layout_rewrite():
    """Sec. 4.4.2, inter-block: the block's dominant operator decides the data format.  A constant
    [K, N] MatMul operand is re-laid out once as [N, K] (a weight-only Transpose that runs at prepare
    time) and read through a folded Transpose, so the GEMM kernel gets both operands K-contiguous."""
    spec = configs.transformer_encoder_layer(**configs.SMALL["transformer_encoder_layer"])
    g, p, blocks = _plan(spec, rewrite=True)
    prep = [d for d in p.describe() if d["prepare_only"]]
    assert len(prep) == 4 and all(d["ops"] == ["Transpose"] for d in prep)      # qkv, out-proj, ffn1, ffn2
    gemm = [b for b in blocks if b["family"] == 2 and b["ops"][0] == "Transpose" and b["ops"][1] == "MatMul"]
    # (the fourth is P V, which reads V through its head-splitting Transpose)
    assert len(gemm) == 4 and sum("_a0b0" in b["kernel_name"] for b in gemm) == 3
    # the activation x activation products (QK^T, PV) are untouched
    assert sum(1 for b in blocks if b["family"] == 2) == 6


def test_attention_block_is_an_option_beyond_the_table():
    """MatMul - Div - Add - Softmax - MatMul: the table keeps the three Many-to-Many operators apart (red
    cells); with the extension switched on they and the head-merging Transpose / Reshape form one block."""
    import sys, os
    sys.path.insert(0, os.path.dirname(__file__))
    import unit_graphs as U

    spec = U.attention_block(2, 3, 128, 128, 64, dtype="f16", mask="add")
    _, _, blocks = _plan(spec, rewrite=True)
    assert sorted(b["family"] for b in blocks if b["family"] in (1, 2)) == [1, 2, 2]
    _, p, blocks = _plan(spec, rewrite=True, attention=1)
    assert [b["family"] for b in blocks] == [6] and blocks[0]["fused_type"] == M2M
    assert sorted(blocks[0]["ops"]) == ["Add", "MatMul", "MatMul", "Mul", "Reshape", "Softmax", "Transpose"]
    src = p.block_source(0)
    assert "score4" in src and "epilogue_vec" in src
    # a head dimension the MFMA step does not divide: the template refuses, the table's plan stands
    _, _, blocks = _plan(U.attention_block(1, 2, 64, 64, 24, dtype="f16", mask=None), rewrite=True, attention=1)
    assert 6 not in [b["family"] for b in blocks]


def test_one_to_many_operators_plan():
    """Resize is One-to-Many (Table 2); Relu -> Resize -> Mul -> Concat(.., Sigmoid(skip)) forms one block that
    is lowered operand by operand; behind a Conv (a yellow pair) the Resize, and the Concat behind it, join the
    convolution's block: its epilogue stores every result at its 2 x 2 destinations inside the Concat result."""
    import sys, os
    sys.path.insert(0, os.path.dirname(__file__))
    import unit_graphs as U

    g, p, blocks = _plan(U.upsample_concat_block(2, 8, 6, 10, 12, "f16"), rewrite=True)
    kinds = {kind: mt for _, kind, mt in g.live_ops()}
    assert kinds["Resize"] == O2M and kinds["Concat"] == O2O
    assert len(blocks) == 1 and blocks[0]["kernel_name"].endswith("concat_parts")
    src = p.block_source(0)
    assert src.count("extern \"C\" __global__") == 2          # one kernel per Concat operand
    _, _, blocks = _plan(U.upsample_concat_block(2, 16, 8, 10, 12, "f16", conv=True), rewrite=True)
    assert [b["family"] for b in blocks] == [3, 3]
    assert blocks[0]["ops"] == ["Conv", "Relu", "Resize", "Mul", "Sigmoid", "Concat"]
    assert api.fuse_relation(M2M, O2M)[1] == 1                # yellow: Conv -> Resize is decided by profiling


def test_dead_operators_are_left_out_of_the_plan():
    """A graph handed over without rewriting may hold operators nobody reads (here a pooling chain and a gate): the
    plan is built over the live ones and says nothing of the rest."""
    import os, sys
    sys.path.insert(0, os.path.dirname(__file__))
    import unit_graphs as U
    from paper_2108_13342_amd import api

    spec = U.random_cnn(936, "f16", n_ops=8, wide=True)
    live_outputs = {t.name for t in spec.tensors.values() if t.kind == "output"}
    assert live_outputs == {"relu_1", "maxpool_4"} and len(spec.ops) == 11
    g, _ = api.graph_from_spec(spec)
    nw = len([t for t in spec.tensors.values() if t.kind == "weight"])
    p = api.Plan(g, [1] * nw, fusion=1, profile=0)
    stored = {t["name"] for blk in p.dump_json()["blocks"] for t in blk["outputs"]}
    assert stored == live_outputs


def test_matmul_layernorm_option_forms_row_owning_blocks():
    """Plan option gemm_norm (beyond the table): MatMul -> bias -> residual -> LayerNorm becomes one block; by default the
    red cell keeps the normalisation a block of its own.  A LayerNorm that follows no MatMul (the decoder's first one,
    behind the embedding sum) is untouched."""
    from workloads import configs
    kw = configs.SMALL["gpt2_decoder"]
    spec = configs.CONFIGS["gpt2_decoder"](**kw)
    g, _ = api.graph_from_spec(spec)
    g.rewrite()
    nw = len([t for t in spec.tensors.values() if t.kind == "weight"])
    plans = {}
    for opt in (0, 2):
        p = api.Plan(g, [1] * nw, fusion=1, profile=0, gemm_norm=opt)
        plans[opt] = [d for d in p.describe() if not d["prepare_only"]]
    assert not any("Normalize" in d["ops"] and "MatMul" in d["ops"] for d in plans[0])
    fused = [d for d in plans[2] if "Normalize" in d["ops"] and "MatMul" in d["ops"]]
    assert len(fused) == 2 * kw["L"] and all(d["kernel_name"].endswith("_rownorm") and d["family"] == 2 for d in fused)
    assert len(plans[2]) == len(plans[0]) - 2 * kw["L"]
    alone = [d for d in plans[2] if d["ops"][0] == "Normalize"]
    assert len(alone) == 1


@pytest.mark.parametrize("fusion", [0, 1])
def test_split_into_parts_of_length_one_gets_a_kernel_per_part(fusion):
    """A part of length 1 leaves no index along the split axis, so a kernel whose index space is one part cannot
    reach the other: each part is stored by a kernel of its own, and no store hides behind a predicate on a constant."""
    import re
    b = GraphBuilder("split1", "f32")
    x = b.input("x", (2, 8), _z((2, 8)))
    p0, p1 = b.op("Split", [x], [(1, 8), (1, 8)], {"axis": 0, "split": [1, 1]})
    b.mark_output(configs._un(b, "Tanh", p0))
    b.mark_output(configs._un(b, "Abs", p1))
    _, p, blocks = _plan(b.finish(), fusion=fusion)
    stores = 0
    for i in range(p.num_blocks()):
        src = p.block_source(i)
        body = src[src.find('extern "C"'):]
        assert not re.search(r"if \(\(\d+\) == \d+\)", body), body
        stores += len(re.findall(r"\*\(sv\d+_t\*\)|\bp\d+\[[^\]]*\] = ", body))
    assert stores == (2 if fusion else 4)
