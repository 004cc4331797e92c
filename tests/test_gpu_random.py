"""Seeded random graphs: the fused plan, the plan without intra-block index folding and the unfused executor all
reproduce the oracle.  The graphs mix every mapping type, so the planner's choices (what joins a block, which index
maps fold into which loads and stores) vary from seed to seed."""
import os
import sys

import pytest

sys.path.insert(0, os.path.dirname(__file__))
import unit_graphs as U
from parity import check_against_oracle, check_blocks_against_oracle

pytestmark = pytest.mark.gpu


def check(spec, tol, **kw):
    """End to end against the oracle at `tol` (rounding accumulates over the blocks of a plan, and the unfused executor
    rounds every intermediate), and - for fused plans - every block on its own, from the oracle's values rounded once,
    at the tolerance a single block has to meet: 1e-5 for fp32, 2e-2 for the 16-bit types."""
    check_against_oracle(spec, tol=tol, **kw)
    if kw.get("fusion", 1):
        check_blocks_against_oracle(spec, **{k: v for k, v in kw.items() if k != "fusion"})


@pytest.mark.parametrize("seed", range(24))
def test_random_graph_f32(seed):
    spec = U.random_graph(seed, "f32")
    check(spec, 2e-4)
    check(spec, 2e-4, fusion=0)


@pytest.mark.parametrize("seed", range(24, 36))
def test_random_graph_f16(seed):
    spec = U.random_graph(seed, "f16")
    check(spec, 3e-2)
    check(spec, 3e-2, intra_block=0)


@pytest.mark.parametrize("seed", range(36, 44))
def test_random_graph_profiled_plan(seed):
    check(U.random_graph(seed, "f32", n_ops=20), 2e-4, profile=1)


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("seed", list(range(20)) + [76, 244, 300])
def test_random_cnn(seed, layout):
    """Random convolutional networks (depthwise / pointwise / 3x3 convolutions, pooling, squeeze-excite gates, channel
    split / concat / shuffle, upsampling), in the declared NCHW order and with data-format selection."""
    dtype = ["f16", "f32", "bf16"][seed % 3]
    tol = {"f32": 5e-4, "f16": 3e-2, "bf16": 8e-2}[dtype]
    check(U.random_cnn(seed, dtype, n_ops=10 + seed % 7), tol, layout=layout, profile=seed % 2)


@pytest.mark.parametrize("attention", [0, 1])
@pytest.mark.parametrize("seed", list(range(12)) + [119])
def test_random_seq(seed, attention):
    """Random sequence models (embedding Gather, linear layers, decomposed LayerNorm, attention in several spellings,
    Split / Concat, CumSum), planned by the table alone and with the attention block allowed."""
    dtype = ["f16", "f32", "bf16"][seed % 3]
    tol = {"f32": 1e-3, "f16": 4e-2, "bf16": 1e-1}[dtype]
    check(U.random_seq(seed, dtype, n_ops=6 + seed % 5), tol, attention=attention, profile=seed % 2)


@pytest.mark.parametrize("seed", [7001, 7012, 7033, 7050, 7056])
def test_random_seq_with_every_result_streamed(seed, monkeypatch):
    """The same sequence models with every MatMul result leaving through non-temporal stores (threshold forced to
    zero): the store sits in front of whatever code follows each epilogue, at many tile shapes and row lengths."""
    monkeypatch.setenv("DNNF_STREAM_MB", "0")
    dtype = ["f16", "bf16", "f32"][seed % 3]
    check_against_oracle(U.random_seq(seed, dtype, n_ops=6 + seed % 5), tol={"f32": 1e-3, "f16": 4e-2, "bf16": 1.5e-1}[dtype],
                         attention=seed % 2)


@pytest.mark.parametrize("seed", list(range(100, 112)) + [85, 119, 187, 216, 217, 7008, 7014, 7057, 10012])
def test_random_graph_wide(seed):
    """Random DAGs that also draw the rarer operators of Table 2: multi-output Split, Gather along any axis,
    Greater / Not / Where, CumSum, Resize, Einsum.  Odd seeds build their plan with on-device profiling."""
    dtype = ["f32", "f16", "bf16"][seed % 3]
    tol = {"f32": 3e-4, "f16": 3e-2, "bf16": 1e-1}[dtype]
    check(U.random_graph(seed, dtype, n_ops=14 + seed % 9, wide=True), tol, profile=seed % 2)


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("seed", range(30, 40))
def test_random_cnn_wide(seed, layout):
    """Random convolutional networks that also draw ConvTranspose, InstanceNormalization, DepthToSpace / SpaceToDepth and
    channel Slices."""
    dtype = ["f16", "f32", "bf16"][seed % 3]
    tol = {"f32": 5e-4, "f16": 3e-2, "bf16": 8e-2}[dtype]
    check(U.random_cnn(seed, dtype, n_ops=10 + seed % 7, wide=True), tol, layout=layout, profile=seed % 2)


@pytest.mark.parametrize("seed", range(4))
def test_random_networks_at_larger_shapes(seed):
    """The same generators at shapes that reach the larger GEMM / convolution tiles, the LDS-staged depthwise kernel,
    split pooling and several key tiles per attention row; plans built as bench.py builds them (profiled, tuned on
    odd seeds, data-format selection for the convolutional ones)."""
    dtype = ["f16", "bf16", "f32"][seed % 3]
    check(U.random_cnn(seed, dtype, n_ops=8 + seed % 5, wide=seed % 2 == 1, big=True), {"f32": 1e-3, "f16": 3e-2, "bf16": 8e-2}[dtype],
                         layout=1, profile=1, tune=seed % 2, broadcast_prologue=(seed // 2) % 2)
    check(U.random_seq(seed, dtype, n_ops=4 + seed % 4, big=True), {"f32": 2e-3, "f16": 4e-2, "bf16": 1.5e-1}[dtype],
                         attention=seed % 2, profile=1, tune=(seed // 2) % 2)
