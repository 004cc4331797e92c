"""GPU parity of the streaming-softmax attention block (the extension beyond the paper's table:
MatMul -> One-to-One operators -> Softmax -> MatMul in one kernel) against the fp64 oracle, which
evaluates the same operators one by one with a plain row softmax."""
import numpy as np
import pytest

import unit_graphs as U
from parity import TOL, check_against_oracle, check_blocks_against_oracle, rel_err
from workloads import configs

pytestmark = pytest.mark.gpu


def _attention_blocks(s):
    return [d for d in s.plan.describe() if d["family"] == 6]


@pytest.mark.parametrize("args,kw", [
    ((2, 3, 128, 128, 64), dict(dtype="f16", mask="add")),                       # exact tiles
    ((1, 2, 200, 200, 64), dict(dtype="bf16", mask="causal")),                   # ragged queries and keys, causal mask tensor
    ((2, 2, 72, 328, 64), dict(dtype="f16", mask="add", merge_heads=False)),     # cross-attention shape, plain output layout
    ((1, 4, 256, 192, 32), dict(dtype="bf16", mask=None, kt_stored=False)),      # K handed over untransposed, head dimension 32
    ((1, 1, 40, 64, 128), dict(dtype="f16", mask="add")),                        # head dimension 128, fewer queries than a tile
])
def test_attention_block(args, kw):
    spec = U.attention_block(*args, **kw)
    s, _ = check_against_oracle(spec, attention=1)
    blocks = _attention_blocks(s)
    assert len(blocks) == 1 and len([d for d in s.plan.describe() if not d["prepare_only"] and d["family"] != 5]) == 1, s.plan.describe()


def test_attention_off_by_default():
    """Without the option the table decides: Many-to-Many + Many-to-Many stays split."""
    from paper_2108_13342_amd import api
    s = api.Session(U.attention_block(2, 3, 128, 128, 64), fusion=1)
    assert not _attention_blocks(s)
    assert len([d for d in s.plan.describe() if d["family"] in (1, 2)]) == 3


def test_fully_masked_tiles_and_large_scores():
    """Whole key tiles at -1e4 (their probabilities underflow to exactly 0) and scores whose running
    maximum changes late in the row: the rescaling of the partial sums must reproduce the row softmax."""
    spec = U.attention_block(1, 2, 192, 256, 64, dtype="f16", mask="causal")
    q = spec.tensors["q"].data
    q[..., 150:, :] *= 6.0          # rows whose largest score sits in their last key tile
    check_against_oracle(spec, attention=1)


def test_transformer_layers_with_attention_block():
    # reduced variants whose head dimension (32) the template supports
    for name, kw in configs.SMALL_HEAD32.items():
        spec = configs.CONFIGS[name](**kw)
        s, _ = check_against_oracle(spec, attention=1)
        assert len(_attention_blocks(s)) == kw.get("L", 1), name


def test_gpt2_full_size_attention_plan():
    """The benchmark's configuration (tuned plan, attention blocks) at full size against the oracle on one
    sequence; 12 layers of bf16 rounding accumulate as in the plan without the extension."""
    from oracle.interp import run_graph
    from paper_2108_13342_amd import api

    spec = configs.CONFIGS["gpt2_decoder"]()
    s = api.Session(spec, fusion=1, profile=1, tune=1, attention=1)
    assert len(_attention_blocks(s)) == 12
    s.run()
    got = s.result()
    ids = spec.tensors["input_ids"].data
    sub = configs.CONFIGS["gpt2_decoder"](B=1)
    for nm, t in sub.tensors.items():
        if t.kind == "weight" and nm in spec.tensors and spec.tensors[nm].data.shape == t.data.shape:
            t.data = spec.tensors[nm].data
    want = run_graph(sub, feeds={"input_ids": ids[1:2]})
    for name, w in want.items():
        g = got[name][:, 1:2] if name.startswith("present_") else got[name][1:2]
        assert rel_err(g, w) <= TOL["bf16"] * np.sqrt(12), name
