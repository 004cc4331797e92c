"""Why the asserted error metric floors the denominator at the tensor's rms.

A plain float32 evaluation of the residual-block config (sequential fp32 accumulation over the
576 products of each output, fp32 epilogue) is compared with the fp64 oracle.  Its largest
absolute error is a few ulps of the intermediate sums; measured against a floor of 1e-3*max|o|
that is far above 1e-5 for the outputs that cancel to near zero, so no fp32 kernel could meet
1e-5 under that floor.  Measured against the output's own scale (rms) it is a few 1e-6.
"""
import numpy as np

from oracle.interp import run_graph
from parity import rel_err
from workloads import configs


def test_fp32_arithmetic_resolution_on_residual_block():
    spec = configs.residual_block(N=1, C=64, H=20, W=20)
    want = list(run_graph(spec).values())[0]
    T = {k: v.data for k, v in spec.tensors.items() if v.data is not None}
    x, w = T["x"].astype(np.float32), T["conv_w"].astype(np.float32)
    xp = np.zeros((1, 64, 22, 22), np.float32)
    xp[:, :, 1:21, 1:21] = x
    acc = np.zeros((1, 64, 20, 20), np.float32)
    for ci in range(64):
        for i in range(3):
            for j in range(3):
                acc += xp[:, ci:ci + 1, i:i + 20, j:j + 20] * w[:, ci, i, j].reshape(1, 64, 1, 1)
    s = (T["bn_gamma"] / np.sqrt(T["bn_var"] + np.float32(1e-5))).astype(np.float32)
    sh = (T["bn_beta"] - T["bn_mean"] * s).astype(np.float32)
    y = np.maximum(np.maximum(acc * s.reshape(1, -1, 1, 1) + sh.reshape(1, -1, 1, 1), 0) + x, 0)
    strict, scaled = rel_err(y, want, floor="max"), rel_err(y, want, floor="rms")
    assert strict > 1e-5, "fp32 arithmetic itself exceeds 1e-5 under the 1e-3*max floor"
    assert scaled < 1e-5, "and sits well inside 1e-5 at the tensor's scale"
