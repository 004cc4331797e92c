"""Seeded random graphs: the fused plan, the plan without intra-block index folding and the unfused executor all
reproduce the oracle.  The graphs mix every mapping type, so the planner's choices (what joins a block, which index
maps fold into which loads and stores) vary from seed to seed."""
import os
import sys

import pytest

sys.path.insert(0, os.path.dirname(__file__))
import unit_graphs as U
from parity import check_against_oracle

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", range(24))
def test_random_graph_f32(seed):
    spec = U.random_graph(seed, "f32")
    check_against_oracle(spec, tol=2e-4)
    check_against_oracle(spec, tol=2e-4, fusion=0)


@pytest.mark.parametrize("seed", range(24, 36))
def test_random_graph_f16(seed):
    spec = U.random_graph(seed, "f16")
    check_against_oracle(spec, tol=3e-2)
    check_against_oracle(spec, tol=3e-2, intra_block=0)


@pytest.mark.parametrize("seed", range(36, 44))
def test_random_graph_profiled_plan(seed):
    check_against_oracle(U.random_graph(seed, "f32", n_ops=20), tol=2e-4, profile=1)
