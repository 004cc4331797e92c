"""Shared helpers of the GPU parity tests."""
import types

import numpy as np

TOL = {"f32": 1e-5, "f16": 2e-2, "bf16": 2e-2}
GUARD = 256        # bytes of a fixed pattern before and after every output buffer and the workspace; checked after each run

_LIST_ATTRS = {"perm", "axes", "shape", "pads", "strides", "starts", "ends", "steps", "split", "scales", "kernel_shape", "output_padding"}


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


def check_against_oracle(spec, fusion=1, rewrite=True, profile=0, tol=None, intra_block=1, floor="rms", **session_kw):
    from oracle.interp import run_graph
    from paper_2108_13342_amd import api

    want = run_graph(spec)
    session_kw.setdefault("guard_bytes", GUARD)
    s = api.Session(spec, fusion=fusion, rewrite=rewrite, profile=profile, intra_block=intra_block, **session_kw)
    s.run()
    got = s.result()
    assert s.guards_intact(), f"{spec.name}: a kernel wrote outside an output buffer or the workspace (fusion={fusion})"
    tol = tol if tol is not None else TOL[spec.dtype]
    errs = {}
    for name, w in want.items():
        assert np.all(np.isfinite(got[name])), f"{name}: non-finite values from the GPU"
        errs[name] = rel_err(got[name], w, floor)
        assert errs[name] <= tol, f"{spec.name} {name}: max rel err {errs[name]:.3e} > {tol} (fusion={fusion})"
    return s, errs


def spec_from_dump(dump, orig_spec):
    """The library's (rewritten) graph, as reported by dnnf_graph_dump_json, as an object the oracle
    interprets.  Weight values come from the original workload by name, compiler-made constants from
    the dump itself."""
    tensors, by_id = {}, {}
    for t in dump["tensors"]:
        data = None
        if t["kind"] in ("input", "weight"):
            if t["name"] in orig_spec.tensors:
                data = orig_spec.tensors[t["name"]].data
            elif "const" in t:
                data = np.asarray(t["const"], dtype=np.float64).reshape(t["shape"])
        ts = types.SimpleNamespace(name=t["name"], dtype=t["dtype"], shape=tuple(t["shape"]), kind=t["kind"], data=data,
                                   origin=t.get("origin", ""))
        tensors[t["name"]] = ts
        by_id[t["id"]] = ts
    ops = []
    for o in dump["ops"]:
        attrs = {}
        for k, v in o["attrs"].items():
            vals = [int(x) if float(x).is_integer() and k in _LIST_ATTRS | {"axis", "group", "keepdims", "transA", "transB"} else x for x in v]
            attrs[k] = vals if k in _LIST_ATTRS else vals[0]
        ops.append(types.SimpleNamespace(id=o["id"], kind=o["kind"], inputs=[by_id[i].name for i in o["in"]],
                                         outputs=[by_id[i].name for i in o["out"]], attrs=attrs))
    return types.SimpleNamespace(name=orig_spec.name, dtype=orig_spec.dtype, tensors=tensors, ops=ops), by_id


def check_blocks_against_oracle(spec, tol=None, profile=0, fusion=1, **session_kw):
    """Per-block parity.  The oracle evaluates the library's rewritten graph once in fp64; then, block
    by block, the block's inputs are set to the oracle's values rounded once to the storage type,
    the block's own operators are evaluated by the oracle in fp64 FROM THOSE ROUNDED INPUTS, and the
    GPU block, run alone on the same inputs, must match within the per-block tolerance.  Errors do
    not compound across blocks and input rounding is charged to neither side.
    Returns (blocks checked, blocks skipped, worst error)."""
    import torch

    from oracle.interp import eval_op, run_graph
    from paper_2108_13342_amd import api
    from workloads import rng

    session_kw.setdefault("guard_bytes", GUARD)
    s = api.Session(spec, fusion=fusion, profile=profile, **session_kw)
    s.run()
    torch.cuda.synchronize()
    rspec, by_id = spec_from_dump(s.graph.dump_json(), spec)
    env = run_graph(rspec, keep="all")
    plan = s.plan.dump_json()
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16, "i32": torch.int32, "i64": torch.int64, "bool": torch.bool}
    tol = tol if tol is not None else TOL[spec.dtype]
    ops_by_id = {o.id: o for o in rspec.ops}
    out_names = {t.name for t in spec.tensors.values() if t.kind == "output"}      # (other tensors may live inside an output)

    def view(t):
        """The tensor where the plan keeps it - the workspace, or (a tensor kept inside a stacked graph output) the
        caller's output buffer - indexed in its declared (logical) order whatever order it is stored in."""
        n = int(np.prod(t["shape"])) if t["shape"] else 1
        esz = torch.empty((), dtype=tdt[t["dtype"]]).element_size()
        if t["kind"] == "output":
            base, off = s.outputs[0][t["ext"]].view(-1).view(torch.uint8), t.get("alias_offset", 0)
        else:
            base, off = s.workspace, t["ws_offset"] + t.get("alias_offset", 0)
        flat = base[off:off + n * esz].view(tdt[t["dtype"]])
        perm = t.get("perm") or []
        if not perm:
            return flat.view(t["shape"])
        stored = flat.view([t["shape"][d] for d in perm])            # dimensions major to minor as stored
        inv = [perm.index(d) for d in range(len(perm))]
        return stored.permute(inv)

    checked = skipped = 0
    worst = 0.0
    for b, blk in enumerate(plan["blocks"]):
        if blk["prepare_only"] or blk["family"] == 5:
            continue
        local = {}
        for t in blk["inputs"]:
            name = t["name"]
            if name not in env:
                # a tensor the plan made for itself (a filter re-laid at prepare time): it keeps its prepared contents and
                # the oracle reads the tensor it was made from, which is what the graph's own operators name
                continue
            if t["dtype"] in ("i32", "i64", "bool"):
                local[name] = env[name]
                continue
            v = rng.round_to(env[name], t["dtype"]).astype(np.float64)
            local[name] = v
            if (t["kind"] == "intermediate" and t["ws_offset"] >= 0) or (t["kind"] == "output" and t["name"] not in out_names):
                view(t).copy_(torch.from_numpy(np.ascontiguousarray(v)).to(tdt[t["dtype"]]))
        if any(oid not in ops_by_id or any(i not in local and i not in env for i in ops_by_id[oid].inputs) for oid in blk["ops"]):
            skipped += 1
            continue
        for oid in blk["ops"]:
            o = ops_by_id[oid]
            # operands the kernel inlines (scalar constants) are not block inputs: exact values
            res = eval_op(o.kind, [local[i] if i in local else env[i] for i in o.inputs], o.attrs)
            res = res if isinstance(res, (list, tuple)) else [res]
            for nm, val in zip(o.outputs, res):
                local[nm] = np.asarray(val, dtype=np.float64)
        s.plan.run_block(b, s.in_ptrs(), s.out_ptrs(), s.workspace.data_ptr(), s.stream)
        torch.cuda.synchronize()
        for t in blk["outputs"]:
            want = local[t["name"]]
            got = view(t).to(torch.float64).cpu().numpy()
            e = rel_err(got, want)
            worst = max(worst, e)
            assert e <= tol, f"{spec.name} block {b} ({blk['variant']}) output {t['name']}: max rel err {e:.3e} > {tol}"
        checked += 1
    assert s.guards_intact(), f"{spec.name}: a kernel wrote outside an output buffer or the workspace"
    return checked, skipped, worst
