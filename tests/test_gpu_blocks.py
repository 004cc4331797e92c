"""GPU parity of single fusion blocks, one kernel family at a time, against the fp64 oracle."""
import numpy as np
import pytest

import unit_graphs as U
from parity import check_against_oracle

pytestmark = pytest.mark.gpu


def _families(s):
    return [d["family"] for d in s.plan.describe() if not d["prepare_only"]]


# ----------------------------------------------------------------- row reductions
@pytest.mark.parametrize("shape,dtype", [((3, 5, 40), "f32"), ((2, 4, 70, 384), "f16"), ((5, 1024), "bf16"), ((7, 2500), "f32"),
                                         ((1, 1), "f32")])
def test_softmax_block(shape, dtype):
    s, _ = check_against_oracle(U.softmax_block(shape, dtype, masked_tail=min(3, shape[-1] - 1)))
    assert _families(s) == [1]


@pytest.mark.parametrize("rows,width,dtype", [(10, 96, "f32"), (37, 768, "f16"), (6, 768, "bf16"), (3, 4100, "f32")])
def test_layernorm_block(rows, width, dtype):
    spec = U.layernorm_block(rows, width, dtype)
    s, _ = check_against_oracle(spec)
    assert _families(s) == [1] and s.rewrite_stats["ops_after"] == 4


@pytest.mark.parametrize("kind", ["ReduceSum", "ReduceMean", "ReduceMax", "ReduceProd"])
@pytest.mark.parametrize("shape,axes,keep", [((6, 7, 50), [-1], 1), ((4, 9, 11), [1, 2], 0), ((3, 3000), [1], 1)])
def test_reduce_block(kind, shape, axes, keep):
    if kind == "ReduceProd" and np.prod([shape[a] for a in axes]) > 200:
        pytest.skip("product of thousands of factors under/overflows fp32 by construction")
    check_against_oracle(U.reduce_block(kind, shape, axes, keep))


@pytest.mark.parametrize("shape,dtype", [((2, 6, 9, 9), "f32"), ((3, 40, 14, 14), "f16"), ((2, 5, 112, 112), "f16")])
def test_gap_block(shape, dtype):
    check_against_oracle(U.gap_block(shape, dtype))


def test_unfused_reductions_match_too():
    check_against_oracle(U.layernorm_block(9, 200, "f32"), fusion=0, rewrite=False)
    check_against_oracle(U.softmax_block((4, 33), "f32"), fusion=0)


# ----------------------------------------------------------------- contractions
@pytest.mark.parametrize("M,K,N,dtype,kw", [
    (200, 96, 136, "f16", dict(gelu=True, residual=True)),       # ragged M and N tiles, full epilogue
    (100, 64, 72, "bf16", dict(batch=(3,))),                     # batch folded into rows
    (70, 33, 50, "f32", dict()),                                 # odd K: scalar loaders, fp32 MFMA
    (256, 512, 384, "f16", dict(bias=False)),                    # exact tiles, several K steps
    (300, 768, 768, "bf16", dict(residual=True)),
    (129, 40, 8, "f32", dict()),
    (1, 64, 64, "f16", dict()),
    # rows of odd length: no destination row starts on a 16-byte boundary, each is stored from its own first aligned column on
    (200, 96, 137, "f16", dict(gelu=True, residual=True)),
    (300, 768, 521, "bf16", dict()),
    (70, 64, 67, "f32", dict()),
    (100, 64, 75, "bf16", dict(batch=(3,))),
    (64, 128, 1003, "bf16", dict(bias=False)),
])
def test_gemm_block(M, K, N, dtype, kw):
    s, _ = check_against_oracle(U.gemm_block(M, K, N, dtype, **kw))
    assert _families(s) == [2], s.plan.describe()


@pytest.mark.parametrize("tile", [
    "128,128,64,2,2,1,2", "128,64,64,2,2,1,2", "64,128,64,2,2,1,2", "64,64,64,2,2,1,2", "64,64,64,2,2,2,3",
    "256,128,64,4,2,1,2", "256,256,64,4,2,2,2",          # eight wavefronts
    "128,128,64,2,4,2,2", "128,128,64,2,4,1,2",          # eight wavefronts on a 128x128 tile
    "256,256,64,4,4,2,2", "128,128,64,4,4,2,2",          # sixteen wavefronts
    "32,32,64,1,1,1,2",                                  # four wavefronts splitting K
    "32,768,64,1,8,1",                                   # a workgroup owning whole rows of 768 (what a fused LayerNorm would need)
])
def test_gemm_tile_configurations(tile, monkeypatch):
    """Every tile configuration the tuner may pick, on a problem with ragged rows and columns."""
    monkeypatch.setenv("DNNF_GEMM_TILE", tile)
    s, _ = check_against_oracle(U.gemm_block(300, 768, 520, "bf16", residual=True))
    bm, bn = tile.split(",")[:2]
    assert [d["kernel_name"].split(":")[1] for d in s.plan.describe() if d["family"] == 2][0].startswith(f"mfma_{bm}x{bn}x64")


@pytest.mark.parametrize("tile", ["64,64,64,2,2,2,1,1", "128,64,64,2,2,2,1,1", "128,128,64,2,2,2,1,1", "256,128,64,4,2,2,1,1", "256,256,64,4,2,2,1,1",
                                  "128,128,64,2,4,2,1,1", "64,128,64,2,4,2,1,1", "128,64,64,4,2,2,1,1", "256,256,64,4,4,2,1,1"])
@pytest.mark.parametrize("dtype,N", [("bf16", 520), ("f16", 520), ("bf16", 777)])
def test_gemm_tiles_loaded_straight_into_lds(tile, dtype, N, monkeypatch):
    """The tile configurations whose operand tiles bypass the registers (both operands contiguous along K, K a whole
    number of tiles), with ragged rows and columns: edge rows are clamped, never skipped.  N = 777: rows of odd length,
    stored row by row from their first aligned column."""
    monkeypatch.setenv("DNNF_GEMM_TILE", tile)
    s, _ = check_against_oracle(U.gemm_block(300, 768, N, dtype, residual=True, w_transposed=True))
    bm, bn = tile.split(",")[:2]
    names = [d["kernel_name"].split(":")[1] for d in s.plan.describe() if d["family"] == 2 and not d["prepare_only"]]
    assert names[0].startswith(f"mfma_{bm}x{bn}x64") and names[0].endswith("_dma"), names


@pytest.mark.parametrize("tile,K", [("64,64,64,2,2,3,1,1", 768), ("128,64,64,4,2,4,1,1", 768), ("128,128,64,2,4,3,1,1", 768),
                                    ("64,64,64,2,2,4,1,1", 128), ("64,64,64,2,2,3,1,1", 64), ("128,128,64,4,4,4,1,1", 192)])
def test_gemm_direct_to_lds_on_three_and_four_buffers(tile, K, monkeypatch):
    """The direct-to-LDS loop with loads two and three tiles ahead, also on products with fewer K tiles than buffers."""
    monkeypatch.setenv("DNNF_GEMM_TILE", tile)
    s, _ = check_against_oracle(U.gemm_block(300, K, 520, "bf16", residual=True, w_transposed=True))
    names = [d["kernel_name"].split(":")[1] for d in s.plan.describe() if d["family"] == 2 and not d["prepare_only"]]
    assert names[0].endswith("_dma" + tile.split(",")[5]), names


@pytest.mark.parametrize("M,K,N,dtype,kw", [
    (300, 768, 520, "bf16", dict(residual=True, w_transposed=True)),       # 16-byte vectors of eight
    (300, 768, 777, "bf16", dict(residual=True, w_transposed=True)),       # rows of odd length: shifted slab, aligned groups
    (130, 96, 200, "f32", dict(gelu=True)),                                # 16-byte vectors of four
    (64, 40, 36, "f16", dict(batch=(3,))),                                 # batched, 8-byte vectors
])
def test_gemm_streaming_stores(M, K, N, dtype, kw, monkeypatch):
    """Results large enough to pass the caches by leave through non-temporal vector stores; here every result does."""
    monkeypatch.setenv("DNNF_STREAM_MB", "0")
    s, _ = check_against_oracle(U.gemm_block(M, K, N, dtype, **kw))
    src = [s.plan.block_source(b) for b, d in enumerate(s.plan.describe()) if d["family"] == 2 and not d["prepare_only"]]
    assert src and all("dn_store_stream((" in x for x in src)          # (a call with a cast pointer, not the helper's definition)


@pytest.mark.parametrize("args,kw", [
    ((100, 64, 200), dict()),                                              # ragged rows and columns, the sum is an output too
    ((70, 96, 768), dict(keep_sum=False, dtype="f16")),                    # the widest row one workgroup holds; the sum stays on chip
    ((45, 64, 130), dict(dtype="f32", residual=False, w_transposed=False)),
    ((40, 64, 96), dict(batch=(3,))),
    ((300, 768, 768), dict()),                                             # the decoder's attention-output projection, fewer rows
])
def test_linear_layernorm_block(args, kw):
    """Extension beyond the table (plan option gemm_norm): MatMul -> bias / residual -> LayerNorm as one block whose
    workgroups own whole rows of the product."""
    spec = U.linear_layernorm_block(*args, **kw)
    s, _ = check_against_oracle(spec, gemm_norm=2)
    names = [d["kernel_name"].split(":")[1] for d in s.plan.describe() if not d["prepare_only"]]
    assert len(names) == 1 and names[0].endswith("_rownorm"), names
    # the table's plan for comparison, and the measured decision between the two (either outcome must be right)
    s0, _ = check_against_oracle(spec)
    assert _families(s0) == [2, 1], s0.plan.describe()
    check_against_oracle(spec, gemm_norm=1, profile=1)


def test_linear_layernorm_rows_too_long_for_one_workgroup():
    s, _ = check_against_oracle(U.linear_layernorm_block(50, 64, 1000), gemm_norm=2)
    assert _families(s) == [2, 1] and any("refused" in l and "768" in l for l in s.plan.dump_json()["log"])


@pytest.mark.parametrize("args,kw,layout,variant", [
    ((3, 240, 14, 14, 10), dict(), 1, "pool196_fc240x10x240"),              # (a graph input keeps its declared NCHW order)
    ((5, 1152, 7, 7, 48), dict(), 1, "pool49_fc1152x48x1152"),              # the widest tail of config 4
    ((2, 96, 9, 11, 4), dict(dtype="bf16"), 0, "pool99_fc96x4x96"),         # declared NCHW order: element-wise pooling
    ((4, 100, 5, 6, 6), dict(dtype="f32", act="relu", bias=False), 1, "pool30_fc100x6x100"),
    ((3, 70, 1, 1, 14), dict(scale=False), 0, "fc70x14x70"),                # the two layers alone, on an already pooled vector
    ((2, 200, 8, 8, 50), dict(scale=False), 1, "pool64_fc200x50x200"),      # 200 output rows: a ragged last group of 64
])
def test_squeeze_excite_tail_block(args, kw, layout, variant):
    """Extension beyond the table (plan option squeeze_excite): pool, first layer, activation, second layer, sigmoid as one
    kernel, one workgroup per image."""
    spec = U.se_tail_block(*args, **kw)
    s, _ = check_against_oracle(spec, squeeze_excite=2, layout=layout)
    se = [d["kernel_name"].split(":")[1] for d in s.plan.describe() if d["family"] == 7]
    assert se == [variant], [d["kernel_name"] for d in s.plan.describe()]
    # the table's plan: pool, layer, layer (and the multiply) apart; and the measured decision between the two
    s0, _ = check_against_oracle(spec, layout=layout)
    assert 7 not in _families(s0) and len(_families(s0)) >= len(_families(s)) + 1
    check_against_oracle(spec, squeeze_excite=1, profile=1, layout=layout)


@pytest.mark.parametrize("args,kw,variant", [
    ((3, 64, 14, 14, 16), dict(dw=(5, 1)), "dw_lds14x14c32_5x5s1_pool"),              # whole 14x14 planes, 32 channels per workgroup
    ((5, 192, 7, 7, 48), dict(dw=(3, 1)), "dw_lds7x7c64_3x3s1_pool"),                 # 64 channels per workgroup
    ((2, 40, 13, 13, 10), dict(dw=(5, 2), dtype="bf16"), "dw_lds7x7c32_5x5s2_pool"),  # stride 2, a last channel group of 8
    ((2, 32, 9, 12, 8), dict(dw=(3, 1), dtype="f32"), "dw_lds9x12c32_3x3s1_pool"),    # fp32: vectors of four channels
])
def test_pool_inside_the_depthwise_convolution(args, kw, variant):
    """With the squeeze-excite option, the global average pool over a map of up to 256 positions rides on the depthwise
    convolution that produces the map (one workgroup per image and channel group adds up what it stores); the tail
    keeps its two layers."""
    spec = U.se_tail_block(*args, **kw)
    s, _ = check_against_oracle(spec, squeeze_excite=2, layout=1)
    names = [d["kernel_name"].split(":")[1] for d in s.plan.describe() if not d["prepare_only"]]
    assert variant in names and any(x.startswith("fc") for x in names) and not any(x.startswith("pool") for x in names), names
    from parity import check_blocks_against_oracle
    checked, skipped, worst = check_blocks_against_oracle(spec, layout=1, squeeze_excite=2)
    assert checked >= 3, (checked, skipped)
    check_against_oracle(spec, squeeze_excite=1, profile=1, layout=1)


def test_squeeze_excite_tail_leaves_large_maps_their_pooling_kernel():
    s, _ = check_against_oracle(U.se_tail_block(2, 32, 40, 40, 8), squeeze_excite=2, layout=1)
    fams = _families(s)
    assert fams.count(7) == 1 and fams.count(1) == 1, s.plan.describe()
    assert [d["kernel_name"].split(":")[1] for d in s.plan.describe() if d["family"] == 7] == ["fc32x8x32"]


@pytest.mark.parametrize("eq,sa,sb,kw", [
    ("ik,kj->ij", (100, 64), (64, 72), dict(dtype="f32")),                         # the plain matrix product
    ("bhid,bhjd->bhij", (2, 3, 40, 32), (2, 3, 56, 32), dict(dtype="f16")),        # attention scores: both operands K-contiguous
    ("bhij,bhjd->bihd", (2, 3, 40, 56), (2, 3, 56, 32), dict(dtype="f16")),        # probabilities x values, heads merged by the result order
    ("nchw,oc->nohw", (2, 24, 9, 10), (16, 24), dict(dtype="f16", b_weight=True)),  # a pointwise convolution written as an Einsum
    ("abc,cbd->da", (20, 6, 8), (8, 6, 12), dict(dtype="bf16", epilogue=False)),   # two summed labels, transposed result
])
def test_einsum_block(eq, sa, sb, kw):
    """Einsum runs as the GEMM block its expansion (Transpose / Reshape / MatMul) fuses into: one kernel."""
    s, _ = check_against_oracle(U.einsum_block(eq, sa, sb, **kw))
    fams = [d["family"] for d in s.plan.describe() if not d["prepare_only"] and d["family"] != 5]
    # (the planner may leave the transposition of a bare result to a kernel of its own)
    assert fams == [2] or (fams == [2, 0] and not kw.get("epilogue", True)), s.plan.describe()


@pytest.mark.parametrize("right", [0, 1])
def test_bitshift_block(right):
    """Integer arithmetic is exact: the shifted int64 values must equal the oracle's bit for bit."""
    from oracle.interp import run_graph
    from paper_2108_13342_amd import api

    spec = U.bitshift_block(right=right)
    want = run_graph(spec)
    s = api.Session(spec, fusion=1)
    s.run()
    got = s.result()
    for name, w in want.items():
        assert np.array_equal(got[name].astype(np.int64), np.asarray(w).astype(np.int64)), name


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_logic_block(dtype):
    """Greater, Not and Where (truth values as 0 / 1) in one elementwise block."""
    s, _ = check_against_oracle(U.logic_block(dtype=dtype))
    assert _families(s) == [0], s.plan.describe()


# ----------------------------------------------------------------- prefix sums
@pytest.mark.parametrize("shape,axis,dtype,kw", [
    ((6, 200), 1, "f32", dict()),                                            # a wavefront per line, ragged last chunk
    ((3, 130, 70), 1, "f32", dict(prologue=True)),                           # a lane per line (inner axis contiguous)
    ((4, 8, 96), -1, "f16", dict(exclusive=1)),
    ((2, 64, 40), 0, "f32", dict(reverse=1)),                                # two-element scan
    ((5, 128), 1, "bf16", dict(reverse=1, exclusive=1, prologue=True)),
    ((2, 48, 32), 1, "f32", dict(reshape=True)),                             # the result's Reshape splits the scanned axis
    ((1, 1, 1000), 2, "f32", dict(epilogue=False)),                          # one long line
    ((70, 3), 1, "f32", dict()),                                             # very short lines
    ((4, 96, 16), 1, "f32", dict(residual=True)),                            # the operand is read again behind the scan
    ((6, 130), 1, "f16", dict(residual=True, prologue=True)),
])
def test_cumsum_block(shape, axis, dtype, kw):
    # bf16 / fp16 storage rounds the inputs; sums of up to 1000 terms in fp32 against fp64
    s, _ = check_against_oracle(U.cumsum_block(shape, axis, dtype, **kw), tol=4e-2 if dtype == "bf16" else 2e-2)
    assert _families(s) == [1], s.plan.describe()
    assert len([d for d in s.plan.describe() if not d["prepare_only"]]) == 1


def test_gemm_unfused_matches():
    # the unfused executor rounds every intermediate to fp16 (1 + erf cancels): it is the baseline, not held to 2e-2
    check_against_oracle(U.gemm_block(150, 96, 80, "f16", gelu=True), fusion=0, tol=0.25)
    check_against_oracle(U.gemm_block(150, 96, 80, "f32", gelu=True), fusion=0)


# ----------------------------------------------------------------- convolutions
@pytest.mark.parametrize("args,kw", [
    ((2, 8, 13, 11, 12, 3), dict(dtype="f32", act="relu")),                     # im2col gather, ragged everything
    ((1, 64, 20, 20, 64, 3), dict(dtype="f32", act="relu", residual=True)),     # the residual-block shape, smaller map
    ((2, 20, 33, 31, 40, 3), dict(dtype="f32", act="relu")),                   # registers-only loop: channels, rows, columns all ragged
    ((2, 12, 30, 30, 70, 5), dict(dtype="f32", act="relu")),                    # the same with 25 taps
    ((4, 20, 45, 45, 40, 3), dict(dtype="f32", stride=2, residual=False)),      # the same with stride 2
    ((2, 32, 16, 16, 24, 1), dict(dtype="f16")),                                # few outputs: one wavefront per output
    ((8, 32, 16, 16, 48, 1), dict(dtype="f16")),                                # pointwise: affine operand, 16-byte pixel vectors
    ((2, 24, 14, 14, 144, 1), dict(dtype="f16", act="swish")),                  # pointwise, 196 pixels: scalar loader
    ((2, 3, 33, 33, 32, 3), dict(dtype="f16", stride=2, act="swish")),          # stem-like, Cin = 3
    ((3, 40, 9, 9, 40, 1), dict(dtype="bf16", residual=True)),
    ((4, 24, 14, 14, 144, 1), dict(dtype="f16", act="swish")),                  # pointwise, 196 pixels: 8-byte pixel vectors
    ((8, 32, 7, 7, 192, 1), dict(dtype="f16", act="swish")),                    # pointwise, 49 pixels: gathering loader
    ((32, 192, 1, 1, 12, 1), dict(dtype="f16", act="swish")),                   # squeeze-excite FC: one wavefront per output
    ((32, 48, 1, 1, 12, 1), dict(dtype="f16", act="swish")),                    # a short K: one lane per output
    ((32, 10, 1, 1, 240, 1), dict(dtype="f16", act="sigmoid")),                 # the second squeeze-excite FC: K of 10, ragged against every vector width
])
def test_conv_block(args, kw):
    s, _ = check_against_oracle(U.conv_block(*args, **kw))
    assert _families(s) == [3], s.plan.describe()


def test_conv_variants_chosen():
    """The shapes above reach the loaders they are meant to exercise."""
    def variant(*args, **kw):
        from paper_2108_13342_amd import api
        s = api.Session(U.conv_block(*args, **kw), fusion=1)
        return [d["kernel_name"].split(":")[1] for d in s.plan.describe() if d["family"] in (3, 4)][0]
    assert variant(1, 64, 20, 20, 64, 3, dtype="f32").startswith("direct_32x32")
    assert variant(2, 20, 33, 31, 40, 3, dtype="f32").startswith("direct_32x32")
    assert variant(2, 12, 30, 30, 70, 5, dtype="f32").startswith("direct_32x32")
    assert variant(8, 32, 16, 16, 48, 1, dtype="f16").endswith("b1")
    assert variant(4, 24, 14, 14, 144, 1, dtype="f16").endswith("b1")
    assert variant(8, 32, 7, 7, 192, 1, dtype="f16").endswith("b3")
    assert variant(32, 192, 1, 1, 12, 1, dtype="f16").startswith("dot_wave")
    assert variant(32, 48, 1, 1, 12, 1, dtype="f16").startswith("dot_lane")
    assert variant(2, 16, 18, 32, 16, 3, stride=1, group=16, dtype="f16").startswith("dw_tile4x8")
    assert variant(2, 12, 22, 56, 12, 5, stride=2, group=12, dtype="bf16").startswith("dw_tile4x4")
    assert variant(2, 16, 14, 14, 16, 5, stride=2, group=16, dtype="f16").startswith("dw_rows")


@pytest.mark.parametrize("args,kw", [
    ((2, 16, 14, 14, 16, 5), dict(stride=2, group=16, dtype="f16", act="swish")),
    ((2, 24, 17, 13, 24, 3), dict(stride=1, group=24, dtype="f32", act="relu")),
    ((1, 96, 28, 28, 96, 3), dict(stride=2, group=96, dtype="bf16", act="swish")),    # 4 rows x 2 columns per lane
    ((2, 16, 18, 32, 16, 3), dict(stride=1, group=16, dtype="f16", act="swish")),     # 4 x 8 tile, ragged row tiles
    ((1, 8, 20, 24, 8, 5), dict(stride=1, group=8, dtype="f32", act="relu")),         # 4 x 4 tile, fp32, 5x5 halo
    ((2, 12, 22, 56, 12, 5), dict(stride=2, group=12, dtype="bf16", act="swish")),    # stride 2: 8 inputs per 4 outputs
    ((1, 8, 12, 12, 8, 3), dict(stride=1, group=8, dtype="f16")),
])
def test_depthwise_conv_block(args, kw):
    s, _ = check_against_oracle(U.conv_block(*args, **kw))
    assert _families(s) == [4], s.plan.describe()


def test_conv_unfused_matches():
    check_against_oracle(U.conv_block(2, 8, 13, 11, 12, 3, dtype="f32", act="relu"), fusion=0)


# ----------------------------------------------------------------- One-to-Many operators: Resize, Expand, Concat
@pytest.mark.parametrize("args,kw", [
    ((2, 8, 6, 10, 12), dict(dtype="f16")),                  # channel counts and widths that vectorise
    ((2, 8, 8, 9, 7), dict(dtype="f32", scale=3)),           # odd sizes, factor 3
    ((1, 5, 3, 17, 13), dict(dtype="bf16")),                 # parts whose offsets are not vector-aligned
])
def test_upsample_concat_block(args, kw):
    """Relu -> Resize (nearest) -> Mul and Sigmoid(skip) -> Concat: one block, one kernel per Concat operand,
    the enlarged tensor never exists in memory."""
    s, _ = check_against_oracle(U.upsample_concat_block(*args, **kw))
    d = [x for x in s.plan.describe() if not x["prepare_only"]]
    assert len(d) == 1 and d[0]["kernel_name"].endswith("concat_parts") and sorted(d[0]["ops"]) == ["Concat", "Mul", "Relu", "Resize", "Sigmoid"]


def test_decoder_step_with_convs():
    """Conv -> Resize is one of the table's yellow pairs: the enlarged tensor is written by the convolution's own
    epilogue (every result stored at its 2 x 2 destinations), so the small map never reaches memory; the Concat behind
    it is One-to-One and joins as well.  Without profiling
    yellow is fused; with profiling the planner times both forms and either outcome must reproduce the oracle."""
    s, _ = check_against_oracle(U.upsample_concat_block(2, 16, 8, 10, 12, dtype="f16", conv=True))
    d = [x for x in s.plan.describe() if not x["prepare_only"]]
    # the convolution's kernel writes the enlarged, scaled map straight into its channel range of the Concat result; a
    # second kernel of the same block fills the skip tensor's range
    assert [x["family"] for x in d] == [3, 3]
    assert d[0]["ops"] == ["Conv", "Relu", "Resize", "Mul", "Sigmoid", "Concat"] and d[0]["n_kernel_launches"] == 2, d[0]
    s, _ = check_against_oracle(U.upsample_concat_block(2, 16, 8, 10, 12, dtype="f16", conv=True), profile=1)
    assert any("profile Resize" in l for l in s.plan.dump_json()["log"])       # the yellow cell was decided by measurement
    for dtype, scale in (("f32", 3), ("bf16", 2)):
        check_against_oracle(U.upsample_concat_block(3, 24, 8, 9, 7, dtype=dtype, scale=scale, conv=True))


@pytest.mark.parametrize("layout", [0, 1])
def test_unet_decoder_small(layout):
    """Two decoder steps (pointwise Conv + ReLU -> Resize -> Concat -> 3x3 Conv + ReLU) against the oracle, planned with
    on-device profiling of the yellow Conv -> Resize cells, in both data formats."""
    from workloads import configs

    spec = configs.unet_decoder(**configs.SMALL_EXTRA["unet_decoder"])
    s, _ = check_against_oracle(spec, profile=1, layout=layout)
    assert any("Resize" in x["ops"] and "Conv" in x["ops"] for x in s.plan.describe()) or any("profile Resize" in l for l in s.plan.dump_json()["log"])


def test_expand_transpose_block():
    s, _ = check_against_oracle(U.expand_transpose_block(3, 20, 24))
    d = [x for x in s.plan.describe() if not x["prepare_only"]]
    assert len(d) == 1 and d[0]["ops"] == ["Expand", "Transpose", "Add"]


# ----------------------------------------------------------------- window pooling
@pytest.mark.parametrize("kind,args,kw", [
    ("MaxPool", (2, 16, 14, 14, 2, 2), dict(dtype="f16")),
    ("MaxPool", (2, 12, 15, 13, 3, 2), dict(pad=1, dtype="f32", prologue=True)),             # ragged map, padding, Relu in front
    ("AveragePool", (3, 8, 12, 12, 3, 1), dict(pad=1, dtype="bf16")),                        # divides by the valid count at the edges
    ("AveragePool", (2, 24, 9, 9, 3, 2), dict(pad=1, dtype="f16", include_pad=1)),
    ("AveragePool", (1, 5, 8, 8, 8, 1), dict(dtype="f32")),                                  # window = whole map: a global pool
])
def test_pool_block(kind, args, kw):
    s, _ = check_against_oracle(U.pool_block(kind, *args, **kw))
    names = [d["kernel_name"] for d in s.plan.describe() if not d["prepare_only"]]
    assert len(names) == 1 and ("maxpool" in names[0] or "avgpool" in names[0]), names      # prologue and epilogue fused into the pooling kernel
    check_against_oracle(U.pool_block(kind, *args, **kw), fusion=0, tol=None if kw.get("dtype") == "f32" else 0.05)


@pytest.mark.parametrize("layout", [0, 1])
def test_conv_pool_net(layout):
    """Convolutions, both pooling operators, Upsample and Concat in one graph; with data-format selection the
    pooling kernels move 8 channels per lane."""
    s, _ = check_against_oracle(U.conv_pool_net(N=4, R=64), fusion=1, layout=layout)
    v = [d["kernel_name"].split(":")[1] for d in s.plan.describe() if not d["prepare_only"]]
    assert sum("pool" in x for x in v) == 3, v
    assert any("pool_chan8" in x for x in v) == bool(layout), v
    # the second 3x3 convolution reads a channels-last intermediate: tap-by-tap vector operand loads
    assert any(x.endswith("b4") for x in v) == bool(layout), v
    check_against_oracle(U.conv_pool_net(), fusion=1, layout=layout)        # small maps: one wavefront per output


@pytest.mark.parametrize("kw,tol", [(dict(dtype="f16"), None), (dict(dtype="f32", C=32, N=3), 2e-5), (dict(dtype="bf16", k=5, R=24), 4e-2),
                                    (dict(dtype="f16", N=1, C=40, R=19), None)])
@pytest.mark.parametrize("layout", [1, 0])
def test_resnet_stage(kw, tol, layout):
    """Dense 3x3 / 5x5 convolutions over intermediate tensors, strides 1 and 2, zero padding, residual adds: with
    data-format selection the filters are re-laid [co, kh, kw, ci] and the operand is read tap by tap in 16-byte
    channel vectors (or gathered in that K order where the map is too small for the MFMA template)."""
    s, _ = check_against_oracle(U.resnet_stage(**kw), fusion=1, layout=layout, tol=tol)
    v = [d["kernel_name"].split(":")[1] for d in s.plan.describe() if not d["prepare_only"]]
    if layout and kw.get("N", 2) > 1:
        assert sum(x.endswith("b4") for x in v) >= 2, v      # (the N = 1 case is all one-wavefront-per-output kernels)
    else:
        assert not any(x.endswith("b4") for x in v), v


# ----------------------------------------------------------------- more operators of Table 2
@pytest.mark.parametrize("kw", [dict(), dict(crd=1, dtype="f32"), dict(N=4, C=16, H=64, W=64), dict(b=3, C=4, H=9, W=12, dtype="bf16")])
def test_pixel_shuffle_block(kw):
    """SpaceToDepth in front of a pointwise convolution (folded into the operand's index function), DepthToSpace
    behind it (its own elementwise block: the convolution template does not take a result whose channel axis is cut)."""
    s, _ = check_against_oracle(U.pixel_shuffle_block(**kw))
    ops = [d["ops"] for d in s.plan.describe() if not d["prepare_only"]]
    assert ops[0][:2] == ["SpaceToDepth", "Conv"], ops
    check_against_oracle(U.pixel_shuffle_block(**kw), fusion=0, tol=None if kw.get("dtype") == "f32" else 0.05)


def test_shuffle_only_block():
    s, _ = check_against_oracle(U.shuffle_only_block())
    assert sorted(len(d["ops"]) for d in s.plan.describe()) == [2, 3]       # both shuffles fused with their neighbours
    check_against_oracle(U.shuffle_only_block(dtype="f16", C=16, H=8, W=16))


@pytest.mark.parametrize("kw", [dict(), dict(N=3, C=16, H=40, W=60, dtype="f16"), dict(N=1, C=3, H=64, W=64, dtype="bf16")])
def test_instance_norm_block(kw):
    s, _ = check_against_oracle(U.instance_norm_block(**kw))
    assert len([d for d in s.plan.describe() if not d["prepare_only"]]) == 1
    check_against_oracle(U.instance_norm_block(**kw), fusion=0, tol=None if kw.get("dtype", "f32") == "f32" else 0.05)


def test_more_unary_block():
    s, _ = check_against_oracle(U.more_unary_block(), tol=2e-5)
    assert len(s.plan.describe()) == 1
    check_against_oracle(U.more_unary_block(), fusion=0, tol=2e-5)


# ----------------------------------------------------------------- 3-d convolution (C3D / S3D-shaped blocks)
@pytest.mark.parametrize("kw", [
    dict(N=4, C=8, D=8, H=16, W=16, CO=32),                                              # 3x3x3 on the MFMA template
    dict(N=1, C=3, D=5, H=9, W=7, CO=8, dtype="f32", k=(3, 3, 3), pad=(1, 1, 1)),       # ragged everything, one wavefront per output
    dict(N=2, C=16, D=8, H=14, W=14, CO=32, stride=(1, 2, 2), dtype="bf16"),             # spatial stride
    dict(N=2, C=8, D=7, H=12, W=12, CO=8, k=(3, 1, 1), pad=(1, 0, 0), residual=True),    # temporal convolution + residual
    dict(N=4, C=8, D=4, H=24, W=24, CO=24, k=(1, 3, 3), pad=(0, 1, 1), prologue=True, dtype="f32"),   # spatial convolution, Relu in front, fp32 MFMA
    dict(N=2, C=12, D=6, H=10, W=10, CO=12, k=(2, 2, 2), stride=(2, 2, 2), pad=(0, 0, 0)),            # even window, stride = window
])
def test_conv3d_block(kw):
    s, _ = check_against_oracle(U.conv3d_block(**kw), tol=2e-5 if kw.get("dtype") == "f32" else None)
    d = [x for x in s.plan.describe() if not x["prepare_only"]]
    assert len(d) == 1 and "3d" in d[0]["kernel_name"], d          # prologue, bias, affine, activation, residual: one kernel
    if kw.get("N") == 4:
        assert "igemm3d" in d[0]["kernel_name"], d
    check_against_oracle(U.conv3d_block(**kw), fusion=0, tol=2e-5 if kw.get("dtype") == "f32" else 0.05)


def test_s3d_unit():
    s, _ = check_against_oracle(U.s3d_unit())
    ops = [x["ops"] for x in s.plan.describe() if not x["prepare_only"]]
    assert ops == [["Conv", "Relu"], ["Conv", "Relu"], ["Conv", "Add"]], ops
    check_against_oracle(U.s3d_unit(N=1, C=8, D=5, R=11, dtype="f32"), tol=2e-5)


# ----------------------------------------------------------------- transposed convolution
@pytest.mark.parametrize("kw", [
    dict(),                                                                     # 4x4 stride 2: the usual learned 2x upsampling
    dict(N=4, C=32, H=24, W=24, CO=16),                                         # large enough for the MFMA template
    dict(N=1, C=5, H=7, W=9, CO=3, k=3, stride=2, pad=0, out_pad=1, dtype="f32"),   # output padding, ragged
    dict(N=2, C=8, H=9, W=9, CO=8, k=3, stride=1, pad=1, dtype="bf16", prologue=True),
    dict(N=3, C=24, H=16, W=16, CO=12, k=2, stride=2, pad=0, skip=True, dtype="f32"),  # stride = window, skip connection added
    dict(N=2, C=6, H=5, W=6, CO=4, k=5, stride=3, pad=2, dtype="f16"),
])
def test_conv_transpose_block(kw):
    s, _ = check_against_oracle(U.conv_transpose_block(**kw), tol=2e-5 if kw.get("dtype") == "f32" else None)
    d = [x for x in s.plan.describe() if not x["prepare_only"]]
    assert len(d) == 1 and ("igemmT" in d[0]["kernel_name"] or "dotT" in d[0]["kernel_name"]), d
    if kw.get("N") == 4:
        assert "igemmT" in d[0]["kernel_name"], d
    check_against_oracle(U.conv_transpose_block(**kw), fusion=0, tol=2e-5 if kw.get("dtype") == "f32" else 0.05)


# ----------------------------------------------------------------- gathered indices
@pytest.mark.parametrize("axis,shape,dtype", [(0, (23, 40), "f32"), (1, (6, 17, 8), "f16"), (2, (3, 5, 64), "bf16")])
def test_gather_with_negative_indices(axis, shape, dtype):
    """Indices in [-n, n): negative ones count from the end of the axis, as the operator is defined (the oracle's
    definition is pinned for them on the host).  The generated code wraps them before they enter the address."""
    n = shape[axis]
    ids = np.array([[0, -1, n - 1, -n, 3], [-2, 1, -n + 1, n - 2, 0]])
    check_against_oracle(U.gather_block(ids, table_shape=shape, axis=axis, dtype=dtype))
    check_against_oracle(U.gather_block(ids, table_shape=shape, axis=axis, dtype=dtype, ids_dtype="i32"), fusion=0)
