"""Host-side checks of global data-format selection (no GPU: plans are built for inspection only)."""
from paper_2108_13342_amd import api
from workloads import configs


def _plan(spec, **kw):
    g, _ = api.graph_from_spec(spec)
    g.rewrite()
    nw = len([t for t in spec.tensors.values() if t.kind == "weight"])
    return g, api.Plan(g, [1] * nw, fusion=1, profile=0, **kw)


def test_convolutional_graph_gets_channels_last_tensors_and_relaid_filters():
    spec = configs.CONFIGS["efficientnet_b0"](**configs.SMALL["efficientnet_b0"])
    g, p1 = _plan(spec, layout=1)
    _, p0 = _plan(spec, layout=0)
    assert p0.dump_json()["stats"]["relaid_tensors"] == 0
    assert p1.dump_json()["stats"]["relaid_tensors"] > 16
    d0, d1 = p0.describe(), p1.describe()
    run0 = [d for d in d0 if not d["prepare_only"]]
    run1 = [d for d in d1 if not d["prepare_only"]]
    # the same blocks run per inference: no reformatting kernel between blocks
    assert [d["ops"] for d in run0] == [d["ops"] for d in run1]
    # one weight-only Identity block per depthwise convolution re-lays its filter when the plan is prepared
    n_dw = sum(1 for op in spec.ops if op.kind == "Conv" and op.attrs.get("group", 1) > 1)
    extra = [d for d in d1 if d["prepare_only"] and d["ops"] == ["Identity"]]
    assert n_dw == 16 and len(extra) == n_dw
    assert len([d for d in d1 if d["prepare_only"]]) == len([d for d in d0 if d["prepare_only"]]) + n_dw
    # operators the pass appended are visible through the plan, beyond the graph's own slots
    n_slots = g.num_op_slots()
    assert p1.op_kind(n_slots) == "Identity"
    # kernels of the channels-last templates were chosen
    names = [d["kernel_name"] for d in run1]
    assert any(":dw_chan" in n for n in names) and any(":mean_chan" in n for n in names)


def test_graphs_without_convolution_chains_are_untouched():
    for name in ("transformer_encoder_layer", "gpt2_decoder", "memory_bound_chain", "residual_block"):
        spec = configs.CONFIGS[name](**configs.SMALL[name])
        _, p1 = _plan(spec, layout=1)
        _, p0 = _plan(spec, layout=0)
        if name != "residual_block":   # there the convolution's in-block successors are marked, but none is ever stored
            assert p1.dump_json()["stats"]["relaid_tensors"] == 0
        assert [d["kernel_name"] for d in p1.describe()] == [d["kernel_name"] for d in p0.describe()]


def test_broadcast_prologue_option_moves_the_squeeze_excite_scaling_into_the_projection():
    spec = configs.CONFIGS["efficientnet_b0"]()
    _, p1 = _plan(spec, layout=1, broadcast_prologue=1)
    _, p0 = _plan(spec, layout=1)
    run1 = [d for d in p1.describe() if not d["prepare_only"]]
    run0 = [d for d in p0.describe() if not d["prepare_only"]]
    pro = [d for d in run1 if d["kernel_name"].endswith("_pro")]
    assert len(pro) == 16 and all(d["ops"][:2] == ["Mul", "Conv"] for d in pro)
    assert len(run1) == len(run0) - 16
    assert not any(d["kernel_name"].endswith("_pro") for d in run0)
    # blocks with a residual keep their Add behind the convolution
    assert sum("Add" in d["ops"] for d in pro) == sum(d["ops"] == ["Conv", "Add"] for d in run0) == 9
    # in the declared order the operand is not K-contiguous: every candidate is refused and logged
    _, p2 = _plan(spec, layout=0, broadcast_prologue=1)
    assert not any(d["kernel_name"].endswith("_pro") for d in p2.describe())
    assert sum("broadcast prologue refused" in l for l in p2.dump_json()["log"]) == 16


def test_squeeze_excite_option_turns_every_tail_into_one_block():
    """Plan option squeeze_excite (beyond the table): layer + layer of every MBConv block as one block of family 7, the
    pool in front of them inside the depthwise convolution's kernel or inside the tail's; maps of more than 256
    positions keep their own pooling kernel.  Config 4 goes from 112 to 85 blocks, to 69 together
    with the broadcast prologue."""
    spec = configs.CONFIGS["efficientnet_b0"]()
    _, p0 = _plan(spec, layout=1)
    _, p1 = _plan(spec, layout=1, squeeze_excite=2)
    _, p2 = _plan(spec, layout=1, squeeze_excite=2, broadcast_prologue=1)
    def live(p):
        return [d for d in p.describe() if not d["prepare_only"] and d["family"] != 5]
    tails = [d for d in live(p1) if d["family"] == 7]
    assert len(live(p0)) == 112 and len(live(p1)) == 85 and len(live(p2)) == 69
    # of the 11 pools over maps of up to 256 positions, 10 ride on the depthwise convolution that produces the map (its
    # staged kernel takes a whole image plane per workgroup); the one behind the stride-2 convolution over a 28x28 map, whose
    # input window does not fit a workgroup's LDS share, stays inside its tail
    on_conv = [d for d in live(p1) if d["family"] == 4 and "GlobalAveragePool" in d["ops"]]
    assert len(tails) == 16 and sum("GlobalAveragePool" in d["ops"] for d in tails) == 1 and len(on_conv) == 10
    assert all(d["ops"][0] == "Conv" and d["kernel_name"].endswith("_pool") for d in on_conv)
    assert all(d["ops"][-3:] == ["Mul", "Conv", "Sigmoid"] for d in tails)
