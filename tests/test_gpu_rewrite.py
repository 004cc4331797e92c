"""The Table 4 rule graphs on the GPU: each graph is rewritten (its rule fires), planned, lowered and run, and
the result is compared with the oracle's evaluation of the graph as first written - the rewrites are exact-
result transformations, so rewriting may change cost but never the values (paper Sec. 4.2)."""
import numpy as np
import pytest

from parity import check_against_oracle
from test_host_rewrite import TABLE4, rule_graph

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("rule", list(TABLE4))
@pytest.mark.parametrize("m,n", [(37, 200), (130, 70)])
def test_table4_rule_graph_runs_rewritten(rule, m, n):
    spec = rule_graph(rule, m, n)
    if rule == "comm_exp":
        # a product of n exponentials: keep it in range for fp32 at these widths
        spec.tensors["A"].data = (spec.tensors["A"].data * 0.25).astype(np.float32)
    # the integer rule (ReduceSum over a shifted int64 tensor) is exact: bit for bit; the two rules whose rewritten form
    # changes the order of a long fp32 accumulation (a product of exponentials, a squared row sum) get a wider margin
    tol = 0.0 if rule == "comm_bitshift" else 5e-5 if rule in ("comm_exp", "assoc_rsum") else 1e-5
    s, _ = check_against_oracle(spec, fusion=1, rewrite=True, tol=tol)
    assert s.rewrite_stats["rules_fired"] >= 1
    # and the graph as written gives the same values (more work, same result)
    check_against_oracle(spec, fusion=1, rewrite=False, tol=tol)
