#!/usr/bin/env python3
"""Benchmark of the fused-block executor on one MI355X.

A step is one pass of the whole hot path (every block of the fusion plan) over one batch of synthetic input that
already sits in HBM.  The headline workload is the largest one that fits one GPU, the GPT-2-small-shaped decoder
stack (12 layers + vocabulary projection, bf16); the other four workloads are measured in the same run and reported
in the `configs` array of the same JSON line.  Prints ONE JSON line.

For every workload: the fused plan end to end (profiled, tuned, data-format selection on), each block on its own
with HIP events on the launch stream, the unfused executor (one kernel per operator) and the fp64 oracle on the
host's cores (a reported baseline, not a target).
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
MFMA_PEAK_TFLOPS = {"f32": 157.3, "f16": 2500.0, "bf16": 2500.0}      # dense
# fp32 vector ALU issue rate: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3 T lane-operations/s, one fp32
# instruction per lane per cycle (the published 157.3 TFLOP/s counts a packed FMA as 4 flops per lane-cycle;
# packed fp32 forms are switched off in this build, and the chain's operators are not FMA-shaped anyway).
ALU_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12

# HBM traffic per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# (scaled by the same counters' reading for a plain copy); see profiles/.  None = not measured.
# Keyed by the dominant kernel's template variant: a plan tuned to another tile on another box reports null.
TRAFFIC_BYTES = {"memory_bound_chain": {"tiled_64x64": 134.32e6},                       # profiles/memory_bound_chain_fused_ew_kernel.md
                 "gpt2_decoder": {"mfma_256x256x64_a0b0_w16_dma": 988.7e6, "mfma_256x256x64_a0b0_w16": 1079.8e6}}               # profiles/gpt2_decoder_gemm_kernels_counters.md

# ALU work of the chain per element, counted from its operators.  One round is Add, Mul, Clip, Exp, Sigmoid,
# Tanh, GELU(erf), Square, Abs, Add, Sqrt: 8 transcendental instructions (exp | exp, rcp | exp, rcp | rcp, exp |
# sqrt), each occupying 2 issue slots on this chip, and 24 full-rate fp32 instructions (1 + 1 + 1 for Add, Mul,
# Clip; 1 scaling per exp = 4; 2 adds and 1 fma closing sigmoid and tanh; 1/sqrt(2) scaling, 7 for the erf
# rational (fma, 4 fma + mul, fma) and x*x, then +1, *x, *0.5; square; +1).  3 rounds x (24 + 8 x 2) = 120
# lane-operations.  The 8 B of HBM traffic per element need 16.8 us at peak, this ALU work 51.2 us.
CHAIN_LANE_OPS_PER_ELEMENT = 3 * (24 + 8 * 2)

HEADLINE = "gpt2_decoder"
OTHERS = ["residual_block", "memory_bound_chain", "transformer_encoder_layer", "efficientnet_b0"]
CONTRACTION_FAMILIES = (2, 3, 6)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--no-configs", action="store_true", help="only the named workload, without the `configs` array of the others")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-unfused", action="store_true")
    ap.add_argument("--no-attention", action="store_true", help="skip the extra timing with the streaming-softmax attention block")
    ap.add_argument("--layout", type=int, default=1, help="1 = global data-format selection (channels-last between convolution blocks), 0 = declared order")
    ap.add_argument("--graphs", type=int, default=0, help="1 = the run loop is replayed as a HIP graph, 0 = kernel-by-kernel launches")
    ap.add_argument("--top-blocks", type=int, default=12, help="how many of the slowest blocks to list")
    ap.add_argument("--sets", type=int, default=4, help="distinct input/output buffer sets rotated through")
    return ap.parse_args()


def ridge(dtype):
    return MFMA_PEAK_TFLOPS[dtype] * 1e12 / (HBM_PEAK_GBS * 1e9)


def block_entry(us, d, dtype):
    """One fusion block of the metric table: latency, algorithmic GB/s and TFLOP/s, and the fraction of the roofline
    that bounds it (matrix cores if its arithmetic intensity lies above the ridge of its data type, HBM otherwise)."""
    gbps, tf = d["bytes"] / us / 1e3, d["flops"] / us / 1e6
    mfma = d["family"] in CONTRACTION_FAMILIES and d["flops"] / max(d["bytes"], 1) > ridge(dtype)
    return {"kernel": d["kernel_name"], "ops": d["n_ops"], "us": us, "GBps": gbps, "TFLOPs": tf,
            "bound": "mfma" if mfma else "hbm", "frac": tf / MFMA_PEAK_TFLOPS[dtype] if mfma else gbps / HBM_PEAK_GBS}


# bounded samples of the oracle: every workload is independent along its batch axis (and the decoder's layers all
# cost the same), so a sub-range is timed and scaled to the full workload
CPU_SAMPLES = {
    "unet_decoder": (dict(N=2), 4.0, "2 of 8 images, time scaled x4"),
    "memory_bound_chain": (dict(), 1.0, "whole workload, one pass"),
    "residual_block": (dict(), 1.0, "whole workload, one pass"),
    "transformer_encoder_layer": (dict(), 1.0, "whole workload, one pass"),
    "efficientnet_b0": (dict(N=8), 4.0, "8 of 32 images, time scaled x4"),
    "gpt2_decoder": (dict(B=2), 2.0, "2 of 4 sequences (all 12 layers and the vocabulary projection), time scaled x2"),
}


def cpu_baseline(spec_fn, name):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload.  `cores` is the number of threads
    it actually kept busy (process CPU time over wall time: numpy's own loops are single-threaded, its matrix
    products run on the BLAS thread pool); `host_cores` is what the box offers."""
    from oracle.interp import run_graph

    sample_kw, scale, what = CPU_SAMPLES.get(name, (dict(), 1.0, "whole workload, one pass"))
    spec = spec_fn(**sample_kw)
    c0, t0 = os.times(), time.perf_counter()
    run_graph(spec)
    dt = time.perf_counter() - t0
    c1 = os.times()
    cpu = (c1.user - c0.user) + (c1.system - c0.system)
    try:
        host = len(os.sched_getaffinity(0))
    except AttributeError:
        host = os.cpu_count()
    return {"value": dt * scale * 1e3, "unit": "ms", "cores": max(1, round(cpu / max(dt, 1e-9))), "kind": "oracle", "sample": what,
            "sample_seconds": dt, "host_cores": host, "omp_num_threads": os.environ.get("OMP_NUM_THREADS")}


_LAUNCH_FLOOR = []


def launch_floor_us():
    """Duration of back-to-back launches of a kernel that does next to nothing (a 64-element Relu block), measured
    with HIP events on the launch stream: what any one-kernel plan costs at least."""
    if not _LAUNCH_FLOOR:
        import numpy as np

        from paper_2108_13342_amd import api
        from workloads.graph import GraphBuilder

        b = GraphBuilder("launch_floor", "f32")
        x = b.input("x", (64,), np.zeros(64, dtype=np.float32))
        b.mark_output(b.op("Relu", [x], (64,)))
        s = api.Session(b.finish(), fusion=1)
        _LAUNCH_FLOOR.append(s.plan.time_block(0, s.in_ptrs(), s.out_ptrs(), s.workspace.data_ptr(), s.stream, warmup=20, iters=200))
    return _LAUNCH_FLOOR[0]


def measure(name, a, steps, warmup):
    """Everything bench.py reports for one workload, as a dict."""
    import torch

    from paper_2108_13342_amd import api
    from workloads import configs

    spec_fn = configs.copy_calibration if name == "copy_calibration" else configs.EXTRA[name] if name in configs.EXTRA else configs.CONFIGS[name]
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

    wall_ms, dev_ms = timed(sess, steps, warmup)

    # dominant kernel: the block with the longest device time, measured by HIP events on its stream
    per_block = []
    for b, d in enumerate(sess.plan.describe()):
        if d["prepare_only"] or d["family"] == 5:
            continue
        us = 0.0
        for s in range(sess.n_sets):
            us += sess.plan.time_block(b, sess.in_ptrs(s), sess.out_ptrs(s), sess.workspace.data_ptr(), sess.stream,
                                       warmup=2, iters=max(steps // sess.n_sets, 5))
        per_block.append((us / sess.n_sets, b, d))
    per_block.sort(key=lambda x: -x[0])
    dom_us, dom_b, dom = per_block[0]
    dom_ai = dom["flops"] / max(dom["bytes"], 1)
    hbm = {"bound": "hbm", "achieved": dom["bytes"] / dom_us / 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    hbm["frac"] = hbm["achieved"] / hbm["peak"]
    if dom["family"] in CONTRACTION_FAMILIES and dom_ai > ridge(spec.dtype):
        roof = {"bound": "mfma", "achieved": dom["flops"] / dom_us / 1e6, "peak": MFMA_PEAK_TFLOPS[spec.dtype], "unit": "TFLOP/s"}
        roof["frac"] = roof["achieved"] / roof["peak"]
        roof["hbm"] = hbm           # the same launch against the other roof
    else:
        roof = hbm
    if name == "memory_bound_chain":
        # 8 bytes and 120 vector-ALU issue slots per element: the ALU roof (51 us) lies above the HBM roof (17 us), so
        # the launch cannot reach the HBM bound; `frac` stays the HBM fraction and the ALU roof is reported beside it
        lane_ops = CHAIN_LANE_OPS_PER_ELEMENT * spec.meta["elements"]
        alu = {"bound": "alu", "achieved": lane_ops / dom_us / 1e6, "peak": ALU_PEAK_TLANEOPS, "unit": "T lane-ops/s",
               "algorithmic_lane_ops": lane_ops}
        alu["frac"] = alu["achieved"] / alu["peak"]
        roof = dict(roof, alu=alu)
    if name == "residual_block":
        # 0.23 GFLOP and 1.75 MB: either roof is under 2 us, the block is bound by launch and by one wavefront's chain
        # of dependent matrix instructions; reported against the launch floor measured in this run
        roof = dict(roof, launch_floor_us=launch_floor_us(), note="launch/latency-bound: both roofs lie below the launch floor")
    # the same kernel inside the network: the plan's blocks launched one by one in plan order, events around the dominant
    # one (behind its producer, with weights that were last read an inference ago)
    order = [b for b, d in enumerate(sess.plan.describe()) if not d["prepare_only"] and d["family"] != 5]
    if len(order) > 1:
        net_us, reps = 0.0, 6
        for it in range(reps + 1):
            st = it % sess.n_sets
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            for b in order:
                if b == dom_b:
                    e0.record(torch.cuda.current_stream(dev))
                sess.plan.run_block(b, sess.in_ptrs(st), sess.out_ptrs(st), sess.workspace.data_ptr(), sess.stream)
                if b == dom_b:
                    e1.record(torch.cuda.current_stream(dev))
            torch.cuda.synchronize(dev)
            if it:
                net_us += e0.elapsed_time(e1) * 1e3 / reps
        roof["us_per_launch_in_network"] = net_us
        roof["frac_in_network"] = roof["frac"] * dom_us / net_us
    roof["traffic"] = TRAFFIC_BYTES.get(name, {}).get(dom["kernel_name"].split(":")[-1])
    roof["kernel"] = dom["kernel_name"]
    roof["us_per_launch"] = dom_us
    roof["algorithmic_bytes"] = dom["bytes"]
    roof["algorithmic_flops"] = dom["flops"]

    out = {
        "metric": "fused-block latency (e2e ms per inference)", "value": dev_ms, "unit": "ms", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": wall_ms, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": spec.dtype, "data": "synthetic",
        "config": {"workload": name, "ops": len(spec.ops), "blocks": len(blocks), "buffer_sets": a.sets,
                   "layout": "selected" if a.layout else "declared", "launch": "hip_graph" if a.graphs else "per_kernel"},
        "roofline": roof,
        "blocks": [block_entry(us, d, spec.dtype) for us, _, d in per_block[:a.top_blocks]],
        "per_block_sum_ms": sum(us for us, _, _ in per_block) / 1e3,
        "irs_bytes_removed": sum(d["irs_bytes_removed"] for d in blocks),
    }
    # the paper's rewriting ablation (its Sec. 5.3 reports fused layer counts with and without graph rewriting):
    # the same planner on the graph as given, host only, nothing timed
    g0, _ = api.graph_from_spec(spec)
    p0 = api.Plan(g0, [1] * len(sess.weights), fusion=1, profile=0, layout=a.layout)
    nb0 = len([d for d in p0.describe() if not d["prepare_only"] and d["family"] != 5])
    rs = sess.rewrite_stats
    out["rewriting"] = {"ops_before": rs["ops_before"], "ops_after": rs["ops_after"], "rules_fired": rs["rules_fired"], "derived_rules_fired": rs["derived_rules_fired"],
                        "canonicalisations": rs["canonicalisations"], "blocks_with_rewriting": len(blocks), "blocks_without_rewriting": nb0}
    del p0, g0
    if not a.no_attention and name in ("transformer_encoder_layer", "gpt2_decoder"):
        # extension beyond the paper's table (MatMul - Softmax - MatMul as one block): reported beside `value`
        at = api.Session(spec, fusion=1, profile=1, tune=1, attention=1, n_buffer_sets=a.sets)
        aw, ad = timed(at, steps, warmup)
        ablk = [(b, d) for b, d in enumerate(at.plan.describe()) if d["family"] == 6]
        aus = at.plan.time_block(ablk[0][0], at.in_ptrs(0), at.out_ptrs(0), at.workspace.data_ptr(), at.stream, warmup=2, iters=20)
        out["attention_block"] = {"ms": ad, "blocks": len([d for d in at.plan.describe() if not d["prepare_only"] and d["family"] != 5]),
                                  "attention_kernels": len(ablk), "kernel": ablk[0][1]["kernel_name"], "us_per_launch": aus,
                                  "TFLOPs": ablk[0][1]["flops"] / aus / 1e6, "speedup_vs_table_plan": dev_ms / ad}
        del at
    if not a.no_attention and name in ("transformer_encoder_layer", "gpt2_decoder"):
        # third extension beyond the table (LayerNorm joined to the linear layer in front of it; row-owning GEMM tiles):
        # the plan with every such block taken, and how many of them the planner keeps when it decides by measurement
        gn = api.Session(spec, fusion=1, profile=1, tune=1, gemm_norm=2, n_buffer_sets=a.sets)
        gw, gd = timed(gn, steps, warmup)
        gblk = [(b, d) for b, d in enumerate(gn.plan.describe()) if d["kernel_name"].endswith("_rownorm")]
        gus = [gn.plan.time_block(b, gn.in_ptrs(0), gn.out_ptrs(0), gn.workspace.data_ptr(), gn.stream, warmup=2, iters=20) for b, _ in gblk[-2:]]
        del gn
        gm = api.Session(spec, fusion=1, profile=1, tune=1, gemm_norm=1, n_buffer_sets=1)
        kept = sum(d["kernel_name"].endswith("_rownorm") for d in gm.plan.describe())
        decisions = [l for l in gm.plan.dump_json()["log"] if l.startswith("MatMul + normalisation") and "fused" in l][:2]
        del gm
        out["gemm_layernorm"] = {"ms": gd, "fused_blocks": len(gblk), "us_per_launch_last_two": gus, "speedup_vs_table_plan": dev_ms / gd,
                                 "kept_when_measured": kept, "measured": decisions}
    if not a.no_attention and name == "efficientnet_b0" and a.layout:
        # second extension beyond the table (squeeze-excite scaling as a prologue of the projection convolution)
        bp = api.Session(spec, fusion=1, profile=1, tune=1, layout=a.layout, broadcast_prologue=1, n_buffer_sets=a.sets)
        bw, bd = timed(bp, steps, warmup)
        bdesc = [d for d in bp.plan.describe() if not d["prepare_only"] and d["family"] != 5]
        out["broadcast_prologue"] = {"ms": bd, "blocks": len(bdesc), "prologue_kernels": sum(d["kernel_name"].endswith("_pro") for d in bdesc),
                                     "speedup_vs_table_plan": dev_ms / bd}
        del bp
        # fourth extension (the squeeze-excite tail - pool, two layers - as one kernel per block), together with the
        # second; and how many of the tails the planner keeps when it decides each by measurement
        res = {}
        for mode, key in ((1, "measured"), (2, "all")):
            se = api.Session(spec, fusion=1, profile=1, tune=1, layout=a.layout, broadcast_prologue=1, squeeze_excite=mode, n_buffer_sets=a.sets)
            sw, sd = timed(se, steps, warmup)
            sdesc = [(b, d) for b, d in enumerate(se.plan.describe()) if not d["prepare_only"] and d["family"] != 5]
            sus = [se.plan.time_block(b, se.in_ptrs(0), se.out_ptrs(0), se.workspace.data_ptr(), se.stream, warmup=2, iters=20) for b, d in sdesc if d["family"] == 7]
            res[key] = {"ms": sd, "blocks": len(sdesc), "launches": sum(d["n_kernel_launches"] for _, d in sdesc), "tail_kernels": len(sus),
                        "tails_with_pool": sum(d["family"] == 7 and "GlobalAveragePool" in d["ops"] for _, d in sdesc),
                        "us_per_tail_min_max": [min(sus), max(sus)] if sus else None, "speedup_vs_table_plan": dev_ms / sd}
            del se
        out["squeeze_excite"] = res
    if not a.no_unfused:
        del sess
        torch.cuda.empty_cache()
        un = api.Session(spec, fusion=0, rewrite=False, profile=0, n_buffer_sets=min(a.sets, 2))
        uw, ud = timed(un, max(steps // 10, 5), 3)
        out["unfused_ms"] = ud
        out["unfused_kernels"] = len([d for d in un.plan.describe() if d["family"] != 5 and not d["prepare_only"]])
        out["speedup_vs_unfused"] = ud / dev_ms
        del un
    torch.cuda.empty_cache()
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(spec_fn, name)
    return out


def main():
    a = parse()
    if a.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU; --gpus {a.gpus} is not supported (no collectives, no sharding).",
              file=sys.stderr)
        sys.exit(2)
    out = measure(a.workload, a, a.steps, a.warmup)
    if a.workload == HEADLINE and not a.no_configs:
        # the other four workloads, same run, same measurements; the small ones take more steps for a steady clock
        out["configs"] = []
        for w in OTHERS:
            r = measure(w, a, max(a.steps, 100) if w in ("residual_block", "memory_bound_chain") else a.steps, a.warmup)
            keep = ("value", "unit", "ms_per_step", "dtype", "config", "roofline", "per_block_sum_ms", "unfused_ms", "unfused_kernels",
                    "speedup_vs_unfused", "cpu_baseline", "rewriting", "attention_block", "gemm_layernorm", "broadcast_prologue", "squeeze_excite", "irs_bytes_removed")
            e = {k: r[k] for k in keep if k in r}
            e["blocks"] = r["blocks"][:4]
            out["configs"].append(e)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
