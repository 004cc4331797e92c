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


# host-side sanitizers: each -fsanitize goes to the host pass only (device code is never instrumented)
SANITIZE = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined",
            "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


def build_library(verbose: bool = False, sanitize: bool = False) -> str:
    """Compiles csrc/*.cpp into libdnnf.so.  sanitize=True builds a second library instead, _build/asan/libdnnf_asan.so,
    whose host code carries AddressSanitizer and UndefinedBehaviorSanitizer instrumentation (for tests/host_sanitize/)."""
    srcs = sorted(glob.glob(os.path.join(HERE, "csrc", "*.cpp")))
    objdir = os.path.join(HERE, "_build", "asan") if sanitize else os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    cxx = os.path.join(ROCM, "bin", "hipcc")
    common = ["-std=c++17", "-O1" if sanitize else "-O2", "-fPIC", "-Wall", "-Wno-unused-function", f"-I{ROCM}/include",
              "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", *(SANITIZE if sanitize else []), "-x", "hip"]
    lib = os.path.join(objdir, "libdnnf_asan.so") if sanitize else LIB
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
    link = [cxx, "-shared", "-o", lib, *objs, *(SANITIZE if sanitize else []), f"-L{ROCM}/lib", "-lhiprtc", f"-Wl,-rpath,{ROCM}/lib"]
    r = subprocess.run(link, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    if r.returncode != 0:
        raise RuntimeError("linking " + os.path.basename(lib) + " failed:\n" + r.stdout.decode())
    return lib


def build_sanitizer_driver(verbose: bool = False) -> str:
    """The sanitizer build of the library plus tests/host_sanitize/driver.cpp linked against it; returns the executable."""
    lib = build_library(verbose, sanitize=True)
    exe = os.path.join(os.path.dirname(lib), "host_sanitize")
    # the driver is plain C++ (no device pass): the same clang that hipcc drives, called directly
    cxx = os.path.join(ROCM, "lib", "llvm", "bin", "clang++")
    cmd = [cxx, "-std=c++17", "-O1", "-g", f"-I{os.path.join(ROOT, 'include')}", "-fsanitize=address", "-fsanitize=undefined",
           "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
           os.path.join(ROOT, "tests", "host_sanitize", "driver.cpp"), "-o", exe, lib, f"-Wl,-rpath,{os.path.dirname(lib)}",
           f"-L{ROCM}/lib", "-lhiprtc", f"-Wl,-rpath,{ROCM}/lib"]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    if r.returncode != 0:
        raise RuntimeError("building the sanitizer driver failed:\n" + r.stdout.decode())
    return exe


def _prewarm_jobs():
    """(workload name, keyword overrides, plan options) of every plan whose kernels ship in kernel_cache/."""
    from workloads import configs

    jobs = []
    for name, kw in configs.SMALL_HEAD32.items():
        jobs.append((name, kw, dict(fusion=1, attention=1)))
    for kw in configs.MID_EFFICIENTNET:
        for layout in (0, 1):
            jobs.append(("efficientnet_b0", kw, dict(fusion=1, layout=layout)))
        jobs.append(("efficientnet_b0", kw, dict(fusion=1, layout=1, broadcast_prologue=1)))
        jobs.append(("efficientnet_b0", kw, dict(fusion=1, layout=1, squeeze_excite=2)))
    for name in configs.CONFIGS:
        for kw in (dict(), configs.SMALL[name]):
            full = int(not kw)          # the full-size fused plans are the ones bench.py tunes on the device
            for fusion in (1, 0):
                jobs.append((name, kw, dict(fusion=fusion, tune=int(fusion == 1) * full)))
                if fusion == 1 and name in ("transformer_encoder_layer", "gpt2_decoder"):
                    jobs.append((name, kw, dict(fusion=1, tune=full, attention=1)))
                    jobs.append((name, kw, dict(fusion=1, gemm_norm=2)))
                if name == "efficientnet_b0":     # the channels-last plans (data-format selection)
                    jobs.append((name, kw, dict(fusion=fusion, rewrite=bool(fusion), tune=int(fusion == 1) * full, layout=1)))
                    if fusion == 1:
                        jobs.append((name, kw, dict(fusion=1, tune=full, layout=1, broadcast_prologue=1)))
                        jobs.append((name, kw, dict(fusion=1, tune=full, layout=1, broadcast_prologue=1, squeeze_excite=2)))
                        jobs.append((name, kw, dict(fusion=1, layout=1, squeeze_excite=2)))
    return jobs


def _prewarm_one(job):
    sys.path.insert(0, ROOT)
    from paper_2108_13342_amd import api
    from workloads import configs

    name, kw, opts = job
    try:
        return api.precompile_spec(configs.CONFIGS[name](**kw), cache_dir=CACHE, **opts)
    except api.DnnfError as e:   # a family not built yet must not break the build
        return f"prewarm {name} {opts}: {e}"


def prewarm(verbose: bool = False, workers: int = 6) -> int:
    """Generate and compile the kernels of the benchmark graphs (fused and unfused plans) into kernel_cache/.
    Kernels are keyed by a hash of their source: code objects that are still current are kept, the ones earlier
    generator versions left behind are dropped at the end."""
    import multiprocessing as mp
    import time

    os.makedirs(CACHE, exist_ok=True)
    t0 = time.time() - 2.0
    os.environ["DNNF_CACHE_TOUCH"] = "1"
    try:
        jobs = _prewarm_jobs()
        # the largest plans first, so the pool's tail is short
        jobs.sort(key=lambda j: (not j[1], j[0] in ("gpt2_decoder", "efficientnet_b0")), reverse=True)
        with mp.get_context("spawn").Pool(min(workers, os.cpu_count() or 1)) as pool:
            results = pool.map(_prewarm_one, jobs, chunksize=1)
    finally:
        os.environ.pop("DNNF_CACHE_TOUCH", None)
    n = 0
    for r in results:
        if isinstance(r, str):
            if "hiprtc" in r:        # a generated kernel that does not compile is a broken build, not a missing feature
                raise RuntimeError(r[:4000])
            if verbose:
                print(r)
        else:
            n += r
    for f in glob.glob(os.path.join(CACHE, "*.hsaco")):
        if os.path.getmtime(f) < t0:
            os.remove(f)
    return n


if __name__ == "__main__":
    print(build_library(verbose=True))
    if "--prewarm" in sys.argv:
        print("kernels:", prewarm(verbose=True))
