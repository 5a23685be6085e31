"""The seeded input generator: formats, determinism and the routing statistics it is meant to imitate."""
import numpy as np
import pytest
import torch

from oracle import moespec_oracle as O
from paper_2602_16052_amd import workloads as wl


def test_bf16_rounding_matches_torch_and_roundtrips():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(4096).astype(np.float32) * 3.0,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.0e38, 1e-40], dtype=np.float32)])
    bits = wl.round_to_bf16_bits(x)
    want = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(bits, want.view(torch.int16).numpy().view(np.uint16))
    back = wl.bf16_bits_to_f32(bits)
    assert np.array_equal(back, want.float().numpy())
    assert np.array_equal(wl.round_to_bf16_bits(back), bits)


def test_generators_are_seeded_and_per_expert_streams_are_independent():
    cfg = wl.small_config(d=64, n_experts=6, d_ff=48, M=5)
    a = wl.layer_weights(cfg)
    b = wl.layer_weights(cfg, threads=1)
    for key in a:
        assert np.array_equal(a[key], b[key])
    part = wl.layer_weights(cfg, experts=(1, 4))
    for key in ("w_gate", "w_up", "w_down"):
        assert np.array_equal(part[key][[1, 4]], a[key][[1, 4]])
        assert not part[key][[0, 2, 3, 5]].any()
    c = wl.layer_weights(cfg, seed=1)
    assert not np.array_equal(a["w_gate"], c["w_gate"])
    assert not np.array_equal(a["w_gate"][0], a["w_up"][0])
    assert not np.array_equal(wl.layer_weights(cfg, layer=1)["b_router"], a["b_router"]) or cfg.n_experts < 3


def test_shapes_dtypes_and_distributions():
    cfg = wl.CONFIGS["tiny_f32"]
    W = wl.layer_weights(cfg)
    h = wl.hidden_states(cfg)
    assert h.shape == (15, 128) and h.dtype == np.float32
    assert W["w_gate"].shape == (8, 256, 128) and W["w_down"].shape == (8, 128, 256)
    assert abs(float(h.std()) - 1.0) < 0.05
    assert abs(float(W["w_gate"].std()) - 0.02) < 0.001
    b = np.sort(W["b_router"])[::-1]
    np.testing.assert_allclose(b, 1.5 * np.log(1.0 / np.arange(1, 9)), rtol=1e-6)
    cfg2 = wl.small_config(dtype="bf16", d=64, n_experts=4, d_ff=32)
    W2 = wl.layer_weights(cfg2)
    assert W2["w_gate"].dtype == np.uint16 and W2["b_router"].dtype == np.float32
    assert abs(float(wl.as_f32(W2["w_gate"]).std()) - 0.02) < 0.002


def test_config_table_matches_the_five_workloads():
    c = wl.CONFIGS
    assert [c[n].M for n in wl.CONFIG_ORDER] == [15, 63, 127, 127, 63]
    assert c["olmoe_m63"].expert_bytes == 12 * 2 ** 20
    assert c["fine_m127"].expert_bytes == 9 * 2 ** 20
    assert c["coarse_stack"].expert_bytes == 336 * 2 ** 20 and c["coarse_stack"].n_layers == 8
    assert c["tiny_f32"].expert_bytes == 393216


@pytest.mark.parametrize("name", ["olmoe_m63", "olmoe_m127"])
def test_router_bias_gives_heavy_tailed_routing(name):
    """The paper reports that the top 32 of 64 experts hold about 93% of a 63-token tree's routing
    mass (Figure 2c); the synthetic bias is meant to land near 90%."""
    cfg = wl.CONFIGS[name]
    h = wl.as_f32(wl.hidden_states(cfg))
    w_r = wl.as_f32(wl.store(np.zeros(1, np.float32), cfg.dtype))  # format check only
    assert w_r.shape == (1,)
    W = wl.layer_weights(cfg, experts=())
    g, ids, _ = O.route(h, wl.as_f32(W["w_router"]), W["b_router"], cfg.top_k, cfg.renorm)
    s = O.aggregate_scores(g)
    cov32 = O.coverage(s, O.shortlist(s, 32))
    assert 0.85 <= cov32 <= 0.97, cov32
    union = O.expert_union(ids)
    assert cfg.top_k < len(union) <= cfg.n_experts
    m = O.decision_margins(g, 32, cfg.top_k, O.shortlist(s, 32))
    # fp64 decisions: any gap far above 1e-12 cannot be flipped by summation order or exp rounding
    assert min(m.values()) > 1e-9, m


def test_stored_stack_scales_show_why_the_stack_scales_its_layer_inputs(golden_dir):
    """tests/golden/coarse_stack_literal_scales.json (written by make_stack_literal_scales.py from the oracle alone):
    under the recurrence as the workload words it the hidden scale squares from layer to layer, the router saturates
    to one-hot probabilities and the state leaves the bf16 range before the 8 layers are through; with unit-RMS layer
    inputs the MoE outputs stay at one scale."""
    import json
    import os
    data = json.load(open(os.path.join(golden_dir, "coarse_stack_literal_scales.json")))
    lit, pre = data["literal"], data["pre_norm"]
    rms = [r["input_rms"] for r in lit]
    assert all(b > 4.0 * a for a, b in zip(rms[1:], rms[2:])), rms            # faster than geometric growth
    assert rms[4] > 1e5 and any(r["max_routing_prob"] == 1.0 for r in lit)     # softmax saturated
    assert not lit[-1]["next_state_finite_in_bf16"] and len(lit) < 8           # overflow before the last layer
    assert len(pre) == 8 and all(r["next_state_finite_in_bf16"] for r in pre)
    outs = [r["moe_output_max_abs"] for r in pre]
    assert max(outs) / min(outs) < 1.5, outs


def test_tracked_counter_summaries_were_measured_on_the_current_kernel_sources():
    """bench.py reports `roofline.traffic` and the kernel-trace duration only from summaries whose build id equals
    the hash of the kernel sources; a summary left behind by a kernel change would silently drop them."""
    import glob
    import os
    import re
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    sys.path.insert(0, root)
    import bench
    current = bench.source_hash()
    files = sorted(glob.glob(os.path.join(root, "profiles", "*.md")))
    assert files
    for f in files:
        ids = re.findall(r"csrc_sha256_16:\s*([0-9a-f]{16})", open(f).read())
        assert ids and all(i == current for i in ids), (os.path.basename(f), ids, current)
    assert bench.stored_traffic()[0] > 0 and bench.stored_kernel_trace() > 0
