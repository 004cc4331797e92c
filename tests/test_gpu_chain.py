"""GPU parity: One-to-One chains with Reorganize/Shuffle tails (config 2), fused and unfused."""
import numpy as np
import pytest

from parity import check_against_oracle, rel_err
from workloads import configs

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("kw", [
    dict(N=2, C=48, H=20, W=13, groups=4),      # several 64x64 tiles with ragged edges on both tile axes
    dict(N=1, C=8, H=3, W=5, groups=2),         # smaller than one tile
    dict(N=3, C=256, H=9, W=7, groups=8),       # full channel count, odd spatial extent
])
@pytest.mark.parametrize("fusion", [1, 0])
def test_chain_matches_oracle(kw, fusion):
    spec = configs.memory_bound_chain(**kw)
    s, errs = check_against_oracle(spec, fusion=fusion, floor="max")
    if fusion:
        assert s.plan.num_blocks() == 1, s.plan.describe()
    else:
        assert sum(1 for d in s.plan.describe() if d["family"] != 5) >= 45


@pytest.mark.parametrize("kw", [dict(N=2, C=48, H=20, W=13, groups=4), dict(N=2, C=256, H=64, W=64, groups=8)])
def test_index_remap_is_bit_exact(kw):
    """With no arithmetic in the block (rounds=0) the fused kernel is a pure permutation:
    NCHW->NHWC, reshape and channel shuffle folded into one index map.  Must be exact."""
    from oracle.interp import run_graph
    from paper_2108_13342_amd import api

    spec = configs.memory_bound_chain(rounds=0, **kw)
    want = list(run_graph(spec).values())[0]
    for fusion in (1, 0):
        s = api.Session(spec, fusion=fusion)
        s.run()
        got = list(s.result().values())[0]
        assert np.array_equal(got, want.astype(np.float32).astype(np.float64))


def test_chain_full_size_sampled():
    """Config 2 at benchmark size in the launch configuration bench.py times; the oracle evaluates
    a batch sub-range (the chain is elementwise, so a sub-range is computed independently)."""
    from oracle.interp import run_graph
    from paper_2108_13342_amd import api

    spec = configs.memory_bound_chain()
    s = api.Session(spec, fusion=1)
    assert s.plan.num_blocks() == 1
    s.run()
    got = list(s.result().values())[0]
    assert np.all(np.isfinite(got))
    x = spec.tensors["x"].data
    for n0 in (0, 15):
        sub = configs.memory_bound_chain(N=1)
        for name, t in sub.tensors.items():       # same weights as the full graph, one image of its input
            if t.kind == "weight":
                t.data = spec.tensors[name].data
        want = list(run_graph(sub, feeds={"x": x[n0:n0 + 1]}).values())[0]
        assert rel_err(got[n0:n0 + 1], want, floor="max") <= 1e-5
