"""dnnf_plan_run_static: the run that allocates nothing (its workspace is a device array inside the library) gives bit
for bit what dnnf_plan_run gives with a caller-owned workspace - on two calls in a row that share the array, the second
with a smaller input, and again after the array has changed hands."""
import pytest
import torch

from paper_2108_13342_amd import api
from workloads import configs

pytestmark = pytest.mark.gpu

STAGES = [(1, 3, 16, 1, 1), (6, 3, 24, 2, 2), (6, 5, 40, 2, 2)]


def _both_ways(sess):
    """Outputs of the ordinary run (buffer set 0) and of the static-workspace run (buffer set 1)."""
    sess.run(0)
    sess.plan.run_static(sess.in_ptrs(1), sess.out_ptrs(1), sess.stream)
    torch.cuda.synchronize()
    return sess.outputs[0], sess.outputs[1]


def test_static_workspace_run_matches_the_ordinary_run():
    # convolutional plans with data-format selection: weight-only blocks (re-laid filters, folded constants) whose results
    # live in the workspace, and pooling kernels that pass partial sums through the blocks' scratch area
    big = api.Session(configs.efficientnet_b0(N=3, R=96, stages=STAGES, dtype="f16"), fusion=1, layout=1, n_buffer_sets=2)
    small = api.Session(configs.efficientnet_b0(N=2, R=64, stages=STAGES[:2], dtype="f16"), fusion=1, layout=1, n_buffer_sets=2)
    seq = api.Session(configs.gpt2_decoder(**configs.SMALL["gpt2_decoder"]), fusion=1, n_buffer_sets=2)
    assert max(s.plan.workspace_bytes() for s in (big, small, seq)) <= 64 << 20
    assert any(d["prepare_only"] for d in big.plan.describe())
    for sess in (big, small, big, seq, small):          # the array changes hands every time
        for o in sess.outputs[1]:
            o.zero_()
        want, got = _both_ways(sess)
        for w, g in zip(want, got):
            assert torch.isfinite(w.float()).all()
            assert torch.equal(w, g), f"{sess.spec.name}: static-workspace run differs from the ordinary run"
    # and twice in a row without a change of hands (no re-preparation in between)
    want, got = _both_ways(small)
    assert all(torch.equal(w, g) for w, g in zip(want, got))


def test_static_workspace_refuses_what_it_cannot_hold_or_has_not_loaded():
    spec = configs.transformer_encoder_layer()                       # full size: far more than the static area
    g, _ = api.graph_from_spec(spec)
    g.rewrite()
    nw = len([t for t in spec.tensors.values() if t.kind == "weight"])
    p = api.Plan(g, [1] * nw, fusion=1)
    assert p.workspace_bytes() > 64 << 20
    with pytest.raises(api.DnnfError) as e:
        p.run_static([1], [1])
    assert e.value.code == -5 and "static workspace holds" in str(e.value)
    # kernels not resident: refused, nothing is loaded behind the caller's back
    spec = configs.residual_block(**configs.SMALL["residual_block"])
    g, _ = api.graph_from_spec(spec)
    g.rewrite()
    p = api.Plan(g, [1] * len([t for t in spec.tensors.values() if t.kind == "weight"]), fusion=1)
    with pytest.raises(api.DnnfError) as e:
        p.run_static([1], [1])
    assert e.value.code == -8 and "dnnf_plan_prepare" in str(e.value)
