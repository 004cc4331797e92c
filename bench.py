#!/usr/bin/env python3
"""Benchmark of the fused-block executor on one MI355X.

A step is one pass of the whole hot path (every block of the fusion plan) over
one batch of synthetic input that already sits in HBM.  The default workload is
the memory-bound chain (24 One-to-One layers + NCHW->NHWC + reshape + channel
shuffle on a 16x256x64x64 fp32 tensor).  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# Published MI355X peaks used for roofline fractions.
HBM_PEAK_GBS = 8000.0
# fp32 vector ALU issue rate: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3 T lane-operations/s, one fp32
# instruction per lane per cycle (the published 157.3 TFLOP/s counts a packed FMA as 4 flops per lane-cycle;
# packed fp32 forms are switched off in this build, and the chain's operators are not FMA-shaped anyway).
ALU_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12

# HBM traffic per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# (scaled by the same counters' reading for a plain copy); see profiles/.  None = not measured.
TRAFFIC_BYTES = {"memory_bound_chain": 134.32e6}   # profiles/memory_bound_chain_fused_ew_kernel.md

# ALU work of the chain per element, counted from its operators.  One round is Add, Mul, Clip, Exp, Sigmoid,
# Tanh, GELU(erf), Square, Abs, Add, Sqrt: 8 transcendental instructions (exp | exp, rcp | exp, rcp | rcp, exp |
# sqrt), each occupying 2 issue slots on this chip, and 24 full-rate fp32 instructions (1 + 1 + 1 for Add, Mul,
# Clip; 1 scaling per exp = 4; 2 adds and 1 fma closing sigmoid and tanh; 1/sqrt(2) scaling, 7 for the erf
# rational (fma, 4 fma + mul, fma) and x*x, then +1, *x, *0.5; square; +1).  3 rounds x (24 + 8 x 2) = 120
# lane-operations.  The 8 B of HBM traffic per element need 16.8 us at peak, this ALU work 51.2 us.
CHAIN_LANE_OPS_PER_ELEMENT = 3 * (24 + 8 * 2)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="memory_bound_chain")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-unfused", action="store_true")
    ap.add_argument("--no-attention", action="store_true", help="skip the extra timing with the streaming-softmax attention block")
    ap.add_argument("--layout", type=int, default=1, help="1 = global data-format selection (channels-last between convolution blocks), 0 = declared order")
    ap.add_argument("--graphs", type=int, default=0, help="1 = the run loop is replayed as a HIP graph, 0 = kernel-by-kernel launches")
    ap.add_argument("--top-blocks", type=int, default=12, help="how many of the slowest blocks to list")
    ap.add_argument("--sets", type=int, default=4, help="distinct input/output buffer sets rotated through")
    return ap.parse_args()


def block_entry(us, d, dtype):
    """One fusion block of the metric table: latency, algorithmic GB/s and TFLOP/s, and the fraction of the roofline
    that bounds it (matrix cores if its arithmetic intensity lies above the ridge of its data type, HBM otherwise)."""
    mfma_peak = 157.3 if dtype == "f32" else 2500.0            # TFLOP/s, dense
    ridge = mfma_peak * 1e12 / (HBM_PEAK_GBS * 1e9)
    gbps, tf = d["bytes"] / us / 1e3, d["flops"] / us / 1e6
    mfma = d["family"] in (2, 3, 6) and d["flops"] / max(d["bytes"], 1) > ridge
    return {"kernel": d["kernel_name"], "ops": d["n_ops"], "us": us, "GBps": gbps, "TFLOPs": tf,
            "bound": "mfma" if mfma else "hbm", "frac": tf / mfma_peak if mfma else gbps / HBM_PEAK_GBS}


def cpu_baseline(spec_fn, name):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload."""
    import numpy as np

    from oracle.interp import run_graph

    # bounded samples: every workload is independent along its batch axis, so a batch sub-range is
    # timed and scaled to the full batch
    samples = {
        "memory_bound_chain": (dict(), 1.0, "whole workload, one pass"),
        "residual_block": (dict(), 1.0, "whole workload, one pass"),
        "transformer_encoder_layer": (dict(B=2), 4.0, "2 of 8 sequences, time scaled x4"),
        "efficientnet_b0": (dict(N=2), 16.0, "2 of 32 images, time scaled x16"),
        "gpt2_decoder": (dict(B=1, L=3), 16.0, "1 of 4 sequences and 3 of 12 layers, time scaled x16"),
    }
    sample_kw, scale, what = samples.get(name, (dict(), 1.0, "whole workload, one pass"))
    spec = spec_fn(**sample_kw)
    t0 = time.perf_counter()
    run_graph(spec)
    dt = time.perf_counter() - t0
    return {"value": dt * scale * 1e3, "unit": "ms", "cores": 1, "kind": "oracle", "sample": what,
            "sample_seconds": dt}


def main():
    a = parse()
    if a.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU; --gpus {a.gpus} is not supported (no collectives, no sharding).",
              file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2108_13342_amd import api
    from workloads import configs

    spec_fn = configs.copy_calibration if a.workload == "copy_calibration" else configs.CONFIGS[a.workload]
    spec = spec_fn()
    dev = torch.device("cuda:0")
    sess = api.Session(spec, fusion=1, profile=1, tune=1, layout=a.layout, graphs=a.graphs, n_buffer_sets=a.sets)
    blocks = [d for d in sess.plan.describe() if not d["prepare_only"] and d["family"] != 5]

    def timed(s, steps, warmup):
        for i in range(warmup):
            s.run(i % s.n_sets)
        torch.cuda.synchronize(dev)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(torch.cuda.current_stream(dev))
        for i in range(steps):
            s.run(i % s.n_sets)
        e1.record(torch.cuda.current_stream(dev))
        torch.cuda.synchronize(dev)
        wall = (time.perf_counter() - t0) * 1e3 / steps
        return wall, e0.elapsed_time(e1) / steps

    wall_ms, dev_ms = timed(sess, a.steps, a.warmup)

    # dominant kernel: the block with the longest device time, measured by HIP events on its stream
    per_block = []
    for b, d in enumerate(sess.plan.describe()):
        if d["prepare_only"] or d["family"] == 5:
            continue
        us = 0.0
        for s in range(sess.n_sets):
            us += sess.plan.time_block(b, sess.in_ptrs(s), sess.out_ptrs(s), sess.workspace.data_ptr(), sess.stream,
                                       warmup=2, iters=max(a.steps // sess.n_sets, 5))
        per_block.append((us / sess.n_sets, b, d))
    per_block.sort(key=lambda x: -x[0])
    dom_us, dom_b, dom = per_block[0]
    if dom["family"] in (2, 3, 6) and dom["flops"] / max(dom["bytes"], 1) > 310:
        roof = {"bound": "mfma", "achieved": dom["flops"] / dom_us / 1e6, "peak": 2500.0 if spec.dtype != "f32" else 157.3,
                "unit": "TFLOP/s"}
    else:
        roof = {"bound": "hbm", "achieved": dom["bytes"] / dom_us / 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    if a.workload == "memory_bound_chain":
        hbm = dict(roof, frac=roof["achieved"] / roof["peak"])
        lane_ops = CHAIN_LANE_OPS_PER_ELEMENT * spec.meta["elements"]
        roof = {"bound": "alu", "achieved": lane_ops / dom_us / 1e6, "peak": ALU_PEAK_TLANEOPS, "unit": "T lane-ops/s",
                "algorithmic_lane_ops": lane_ops, "hbm": hbm}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = TRAFFIC_BYTES.get(a.workload)
    roof["kernel"] = dom["kernel_name"]
    roof["us_per_launch"] = dom_us
    roof["algorithmic_bytes"] = dom["bytes"]

    out = {
        "metric": "fused-block latency (e2e ms per inference)", "value": dev_ms, "unit": "ms", "n_gpus": 1,
        "steps": a.steps, "warmup": a.warmup, "ms_per_step": wall_ms, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": spec.dtype, "data": "synthetic",
        "config": {"workload": a.workload, "ops": len(spec.ops), "blocks": len(blocks), "buffer_sets": a.sets,
                   "layout": "selected" if a.layout else "declared", "launch": "hip_graph" if a.graphs else "per_kernel"},
        "roofline": roof,
        "blocks": [block_entry(us, d, spec.dtype) for us, _, d in per_block[:a.top_blocks]],
        "irs_bytes_removed": sum(d["irs_bytes_removed"] for d in blocks),
    }
    if roof["bound"] == "alu":      # the chain kernel is priced against the vector ALUs, in the block table too
        out["blocks"][0].update(bound="alu", frac=roof["frac"])
    # the paper's rewriting ablation (its Sec. 5.3 reports fused layer counts with and without graph rewriting):
    # the same planner on the graph as given, host only, nothing timed
    g0, _ = api.graph_from_spec(spec)
    p0 = api.Plan(g0, [1] * len(sess.weights), fusion=1, profile=0, layout=a.layout)
    nb0 = len([d for d in p0.describe() if not d["prepare_only"] and d["family"] != 5])
    rs = sess.rewrite_stats
    out["rewriting"] = {"ops_before": rs["ops_before"], "ops_after": rs["ops_after"], "rules_fired": rs["rules_fired"],
                        "canonicalisations": rs["canonicalisations"], "blocks_with_rewriting": len(blocks), "blocks_without_rewriting": nb0}
    del p0, g0
    if not a.no_attention and a.workload in ("transformer_encoder_layer", "gpt2_decoder"):
        # extension beyond the paper's table (MatMul - Softmax - MatMul as one block): reported beside `value`
        at = api.Session(spec, fusion=1, profile=1, tune=1, attention=1, n_buffer_sets=a.sets)
        aw, ad = timed(at, a.steps, a.warmup)
        ablk = [(b, d) for b, d in enumerate(at.plan.describe()) if d["family"] == 6]
        aus = at.plan.time_block(ablk[0][0], at.in_ptrs(0), at.out_ptrs(0), at.workspace.data_ptr(), at.stream, warmup=2, iters=20)
        out["attention_block"] = {"ms": ad, "blocks": len([d for d in at.plan.describe() if not d["prepare_only"] and d["family"] != 5]),
                                  "attention_kernels": len(ablk), "kernel": ablk[0][1]["kernel_name"], "us_per_launch": aus,
                                  "TFLOPs": ablk[0][1]["flops"] / aus / 1e6, "speedup_vs_table_plan": dev_ms / ad}
        del at
    if not a.no_attention and a.workload == "efficientnet_b0" and a.layout:
        # second extension beyond the table (squeeze-excite scaling as a prologue of the projection convolution)
        bp = api.Session(spec, fusion=1, profile=1, tune=1, layout=a.layout, broadcast_prologue=1, n_buffer_sets=a.sets)
        bw, bd = timed(bp, a.steps, a.warmup)
        bdesc = [d for d in bp.plan.describe() if not d["prepare_only"] and d["family"] != 5]
        out["broadcast_prologue"] = {"ms": bd, "blocks": len(bdesc), "prologue_kernels": sum(d["kernel_name"].endswith("_pro") for d in bdesc),
                                     "speedup_vs_table_plan": dev_ms / bd}
        del bp
    if not a.no_unfused:
        del sess
        torch.cuda.empty_cache()
        un = api.Session(spec, fusion=0, rewrite=False, profile=0, n_buffer_sets=min(a.sets, 2))
        uw, ud = timed(un, max(a.steps // 10, 5), 3)
        out["unfused_ms"] = ud
        out["unfused_kernels"] = len([d for d in un.plan.describe() if d["family"] != 5 and not d["prepare_only"]])
        out["speedup_vs_unfused"] = ud / dev_ms
        del un
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(spec_fn, a.workload)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
