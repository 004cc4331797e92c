"""Host side of dnnf_plan_run_static: a plan larger than the library's static workspace is refused before any device
call is made (so this runs without a GPU)."""
import pytest

from paper_2108_13342_amd import api
from workloads import configs


def test_oversized_plan_is_refused_with_both_sizes_named():
    spec = configs.transformer_encoder_layer()
    g, _ = api.graph_from_spec(spec)
    g.rewrite()
    nw = len([t for t in spec.tensors.values() if t.kind == "weight"])
    p = api.Plan(g, [1] * nw, fusion=1)
    need = p.workspace_bytes()
    assert need > 64 << 20
    with pytest.raises(api.DnnfError) as e:
        p.run_static([1], [1])
    assert e.value.code == -5
    assert str(need) in str(e.value) and str(64 << 20) in str(e.value)
