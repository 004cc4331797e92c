"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer.

`paper_2108_13342_amd.build.build_sanitizer_driver()` compiles csrc/*.cpp a second time with the host pass
instrumented (device code is never instrumented) and links tests/host_sanitize/driver.cpp against it.  The driver
feeds every graph below through the C ABI - build, finalize, rewrite, eight plans per graph (unfused, fused, no index
folding, attention block, data-format selection, broadcast prologue, MatMul + LayerNorm blocks, squeeze-excite tails), every block's generated source, the JSON dumps -
and one graph through hipRTC as well.  No GPU is involved.  A report from either sanitizer ends the driver with a
non-zero status (undefined behaviour is built as non-recoverable).
"""
import os
import subprocess
import sys

import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(__file__))
import unit_graphs as U                                   # noqa: E402
from paper_2108_13342_amd import api, build              # noqa: E402
from workloads import configs                            # noqa: E402


def write_spec(spec, path, expect_finalize=0):
    """GraphSpec -> the driver's text format (see tests/host_sanitize/driver.cpp)."""
    idx = {}
    lines = []
    for t in spec.tensors.values():
        idx[t.name] = len(idx)
        lines.append(" ".join(["T", t.name.replace(" ", "_"), str(api.DTYPES[t.dtype]), str(api.KINDS[t.kind]), str(len(t.shape)),
                               *[str(int(d)) for d in t.shape]]))
        if t.kind == "weight" and t.data is not None and (t.const or t.data.size <= 4096):
            v = np.asarray(t.data, dtype=np.float64).ravel()
            lines.append(" ".join(["C", str(idx[t.name]), str(v.size), *[repr(float(x)) for x in v]]))
    for op in spec.ops:
        rec = ["O", op.kind, str(len(op.inputs)), *[str(idx[i]) for i in op.inputs], str(len(op.outputs)), *[str(idx[o]) for o in op.outputs],
               str(len(op.attrs))]
        for k, v in op.attrs.items():
            if isinstance(v, str):
                v = [ord(ch) for ch in v]
            vals = np.atleast_1d(np.asarray(v, dtype=np.float64)).ravel()
            rec += [k, str(vals.size), *[repr(float(x)) for x in vals]]
        lines.append(" ".join(rec))
    lines.append(f"X {expect_finalize}")
    with open(path, "w") as f:
        f.write("\n".join(lines) + "\n")


def graphs():
    g = {name: configs.CONFIGS[name](**kw) for name, kw in configs.SMALL.items()}
    g["unet_decoder"] = configs.EXTRA["unet_decoder"](**configs.SMALL_EXTRA["unet_decoder"])
    g["head32_decoder"] = configs.CONFIGS["gpt2_decoder"](**configs.SMALL_HEAD32["gpt2_decoder"])
    g["mid_efficientnet"] = configs.CONFIGS["efficientnet_b0"](**configs.MID_EFFICIENTNET[0])
    g["conv_direct"] = U.conv_block(2, 20, 33, 31, 40, 3, dtype="f32", act="relu")
    g["conv_dw"] = U.conv_block(2, 16, 18, 32, 16, 3, group=16, dtype="f16", act="swish")
    g["gemm_odd"] = U.gemm_block(150, 96, 81, "bf16", gelu=True)
    g["attention"] = U.attention_block(2, 3, 40, 56, 32)
    g["linear_layernorm"] = U.linear_layernorm_block(40, 64, 96, batch=(3,))
    g["se_tail"] = U.se_tail_block(3, 240, 14, 14, 10)
    g["upsample_concat"] = U.upsample_concat_block(2, 8, 8, 9, 7, dtype="f32", scale=3, conv=True)
    g["conv3d"] = U.conv3d_block()
    g["conv_transpose"] = U.conv_transpose_block()
    g["cumsum"] = U.cumsum_block((3, 50, 7), 1)
    g["einsum"] = U.einsum_block("bij,bjk->bik", (2, 9, 12), (2, 12, 10))
    g["bitshift"] = U.bitshift_block()
    g["gather_const"] = U.gather_block(np.array([[0, -1, 22]]), const_ids=True)
    for seed in (3, 4):
        g[f"random_graph_{seed}"] = U.random_graph(seed)
        g[f"random_cnn_{seed}"] = U.random_cnn(seed)
        g[f"random_seq_{seed}"] = U.random_seq(seed)
    return g


@pytest.fixture(scope="module")
def driver():
    return build.build_sanitizer_driver()


def run(driver, args):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    return subprocess.run([driver, *args], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, env=env, timeout=900)


def test_host_code_under_address_and_undefined_behaviour_sanitizers(driver, tmp_path):
    files = []
    for name, spec in graphs().items():
        p = str(tmp_path / (name + ".txt"))
        write_spec(spec, p)
        files.append(p)
    # a constant Gather index outside the axis is refused when the graph is finalized (DNNF_INVALID_ARG = -1)
    bad = str(tmp_path / "gather_bad.txt")
    write_spec(U.gather_block(np.array([[0, 23]]), const_ids=True), bad, expect_finalize=-1)
    files.append(bad)
    r = run(driver, files)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-6000:])
    assert "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr and "LeakSanitizer" not in r.stderr, r.stderr[-6000:]
    assert r.stdout.count("\nok ") + r.stdout.startswith("ok ") == len(files), r.stdout


def test_kernel_compilation_path_under_sanitizers(driver, tmp_path):
    """hipRTC compilation of one small plan's kernels (code objects kept in memory only)."""
    p = str(tmp_path / "gemm.txt")
    write_spec(U.gemm_block(70, 64, 48, "f16", gelu=True), p)
    r = run(driver, ["--precompile", p])
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-6000:])
    assert "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-6000:]
