"""Shared helpers of the GPU parity tests."""
import numpy as np

TOL = {"f32": 1e-5, "f16": 2e-2, "bf16": 2e-2}


def rel_err(got, want, floor="rms"):
    """max_i |g_i - o_i| / max(|o_i|, floor).

    floor="rms":  the root-mean-square of the expected tensor, i.e. errors of elements smaller than
                  the tensor's own scale are measured against that scale.  This is the asserted metric:
                  a sum of K fp32 terms carries an absolute error of about sqrt(K)*2^-24 times the
                  magnitude of the terms however small the sum itself comes out, so an element that
                  cancels to near zero cannot be held to a relative bound (test_fp32_metric.py shows
                  the numbers for the residual-block config).
    floor="max":  1e-3 * max|o|, the stricter floor; asserted where no long fp32 sum feeds the output.
    """
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    if want.size == 0:
        return 0.0
    if floor == "rms":
        fl = float(np.sqrt(np.mean(want * want)))
    else:
        fl = 1e-3 * float(np.max(np.abs(want)))
    return float(np.max(np.abs(got - want) / np.maximum(np.abs(want), max(fl, 1e-300))))


def check_against_oracle(spec, fusion=1, rewrite=True, profile=0, tol=None, intra_block=1, floor="rms"):
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
        errs[name] = rel_err(got[name], w, floor)
        assert errs[name] <= tol, f"{spec.name} {name}: max rel err {errs[name]:.3e} > {tol} (fusion={fusion})"
    return s, errs
