"""Shared helpers of the GPU parity tests."""
import numpy as np

TOL = {"f32": 1e-5, "f16": 2e-2, "bf16": 2e-2}


def rel_err(got, want):
    """max_i |g_i - o_i| / max(|o_i|, 1e-3 * max_j |o_j|): relative error with a floor, so outputs
    that cross zero do not blow the figure up."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    if want.size == 0:
        return 0.0
    floor = 1e-3 * float(np.max(np.abs(want)))
    return float(np.max(np.abs(got - want) / np.maximum(np.abs(want), max(floor, 1e-300))))


def check_against_oracle(spec, fusion=1, rewrite=True, profile=0, tol=None, intra_block=1):
    from oracle.interp import run_graph
    from paper_2108_13342_amd import api

    want = run_graph(spec)
    s = api.Session(spec, fusion=fusion, rewrite=rewrite, profile=profile, intra_block=intra_block)
    s.run()
    got = s.result()
    tol = tol if tol is not None else TOL[spec.dtype]
    errs = {}
    for name, w in want.items():
        assert np.all(np.isfinite(got[name])), f"{name}: non-finite values from the GPU"
        errs[name] = rel_err(got[name], w)
        assert errs[name] <= tol, f"{spec.name} {name}: max rel err {errs[name]:.3e} > {tol} (fusion={fusion})"
    return s, errs
