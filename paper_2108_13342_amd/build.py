"""Builds libdnnf.so in-tree and (optionally) pre-compiles the generated kernels.

The library's own sources are host C++: every device kernel is generated at
plan-build time and compiled for gfx950 with hipRTC, which works without a
GPU.  `prewarm()` runs that generation for the benchmark graphs so that the
code objects travel with the tree in `kernel_cache/`.
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libdnnf.so")
CACHE = os.path.join(HERE, "kernel_cache")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def build_library(verbose: bool = False) -> str:
    srcs = sorted(glob.glob(os.path.join(HERE, "csrc", "*.cpp")))
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    cxx = os.path.join(ROCM, "bin", "hipcc")
    common = ["-std=c++17", "-O2", "-fPIC", "-Wall", "-Wno-unused-function", f"-I{ROCM}/include",
              "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-x", "hip"]
    procs = []
    objs = []
    for s in srcs:
        o = os.path.join(objdir, os.path.basename(s)[:-4] + ".o")
        objs.append(o)
        procs.append((s, subprocess.Popen([cxx, *common, "-c", s, "-o", o], stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
    for s, p in procs:
        out = p.communicate()[0].decode()
        if p.returncode != 0:
            raise RuntimeError(f"compiling {s} failed:\n{out}")
        if verbose and out.strip():
            print(out)
    link = [cxx, "-shared", "-o", LIB, *objs, f"-L{ROCM}/lib", "-lhiprtc", f"-Wl,-rpath,{ROCM}/lib"]
    r = subprocess.run(link, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    if r.returncode != 0:
        raise RuntimeError("linking libdnnf.so failed:\n" + r.stdout.decode())
    return LIB


def prewarm(verbose: bool = False) -> int:
    """Generate and compile the kernels of the benchmark graphs (fused and unfused plans)."""
    sys.path.insert(0, ROOT)
    from paper_2108_13342_amd import api
    from workloads import configs

    # kernels are keyed by a hash of their source: drop the ones earlier generator versions left behind
    if os.path.isdir(CACHE):
        for f in glob.glob(os.path.join(CACHE, "*.hsaco")):
            os.remove(f)
    n = 0
    for name, kw in configs.SMALL_HEAD32.items():
        n += api.precompile_spec(configs.CONFIGS[name](**kw), fusion=1, cache_dir=CACHE, attention=1)
    for kw in configs.MID_EFFICIENTNET:
        for layout in (0, 1):
            n += api.precompile_spec(configs.efficientnet_b0(**kw), fusion=1, cache_dir=CACHE, layout=layout)
        n += api.precompile_spec(configs.efficientnet_b0(**kw), fusion=1, cache_dir=CACHE, layout=1, broadcast_prologue=1)
    for name, variants in ((n, [dict(), configs.SMALL[n]]) for n in configs.CONFIGS):
        for kw in variants:
            spec = configs.CONFIGS[name](**kw)
            for fusion in (1, 0):
                try:
                    # the full-size fused plans are the ones bench.py tunes on the device
                    n += api.precompile_spec(spec, fusion=fusion, cache_dir=CACHE, tune=int(fusion == 1 and not kw))
                    if fusion == 1 and name in ("transformer_encoder_layer", "gpt2_decoder"):
                        n += api.precompile_spec(spec, fusion=1, cache_dir=CACHE, tune=int(not kw), attention=1)
                    if name == "efficientnet_b0":     # the channels-last plans (data-format selection)
                        n += api.precompile_spec(spec, fusion=fusion, rewrite=bool(fusion), cache_dir=CACHE, tune=int(fusion == 1 and not kw), layout=1)
                        if fusion == 1:
                            n += api.precompile_spec(spec, fusion=1, cache_dir=CACHE, tune=int(not kw), layout=1, broadcast_prologue=1)
                except api.DnnfError as e:   # a family not built yet must not break the build
                    if verbose:
                        print(f"prewarm {name} fusion={fusion}: {e}")
    return n


if __name__ == "__main__":
    print(build_library(verbose=True))
    if "--prewarm" in sys.argv:
        print("kernels:", prewarm(verbose=True))
