"""Decision-margin audit of the seeded workloads.

Routing ids, shortlists and permutations of the HIP path must equal the oracle's bit for bit, while the two
sum and exponentiate in different orders.  That is only a fair demand if no decision of a workload hangs on
the last bits: for every workload, every budget of its sweep and both coverage policies, the smallest gap at
every decision boundary - adjacent routing probabilities among a token's k+1 best (natural top-k, Section 2.1),
among its k+1 best inside the shortlist (Eq. (8)), and adjacent aggregate scores among the B+1 best (Eq. (5),
Section 3.2) - must lie far above the rounding noise of fp64 arithmetic (about 1e-15 here)."""
import numpy as np
import pytest

from oracle import moespec_oracle as O
from paper_2602_16052_amd import workloads as wl

NOISE_FLOOR = 1e-9     # six orders above fp64 summation / exp rounding on probabilities <= 1 and scores <= M


def margins_of(cfg, h_f32, layer, B):
    W = wl.layer_weights(cfg, layer=layer, experts=())
    g, _, _ = O.route(h_f32, wl.as_f32(W["w_router"]), W["b_router"], cfg.top_k, cfg.renorm, cfg.gate)
    s = O.aggregate_scores(g)
    return O.decision_margins(g, B, cfg.top_k, O.shortlist(s, B))


@pytest.mark.parametrize("name", ["tiny_f32", "olmoe_m63", "olmoe_m127", "fine_m127", "olmoe_m255", "olmoe_m511"])
def test_every_budget_of_a_single_layer_workload_has_safe_margins(name):
    cfg = wl.CONFIGS[name]
    h = wl.as_f32(wl.hidden_states(cfg))
    for B in sorted(set(cfg.budgets) | {cfg.n_experts}):
        m = margins_of(cfg, h, 0, B)
        # "topk" guards truncation and the natural routing, "sub" substitution, "score" the shortlist of both
        assert m["topk"] > NOISE_FLOOR and m["score"] > NOISE_FLOOR, (name, B, m)
        if B >= cfg.top_k:
            assert m["sub"] > NOISE_FLOOR, (name, B, m)


@pytest.mark.parametrize("layer", range(wl.CONFIGS["coarse_stack"].n_layers))
def test_every_router_of_the_layer_stack_has_safe_margins(layer):
    """The routers of the 8 stacked layers (each with its own seeded bias), audited on unit-scale hidden rows of
    the workload's distribution: layer 0 on its actual input, the later ones on rows drawn from a seed of their
    own (their actual inputs depend on the layers before; the GPU stack test audits those)."""
    cfg = wl.CONFIGS["coarse_stack"]
    h = wl.as_f32(wl.hidden_states(cfg, seed=cfg.seed + 1000 * layer))
    for B in cfg.budgets:
        m = margins_of(cfg, h, layer, B)
        assert m["topk"] > NOISE_FLOOR and m["score"] > NOISE_FLOOR, (layer, B, m)
        if B >= cfg.top_k:
            assert m["sub"] > NOISE_FLOOR, (layer, B, m)


def test_margin_audit_sees_a_planted_tie():
    """Two identical router rows produce a zero gap: the audit must report it (so it cannot pass vacuously)."""
    cfg = wl.small_config(d=64, n_experts=6, top_k=2, d_ff=32, M=4, bias_alpha=0.0)
    W = wl.layer_weights(cfg, experts=())
    w_r = wl.as_f32(W["w_router"]).copy()
    w_r[3] = w_r[1]
    g, _, _ = O.route(wl.as_f32(wl.hidden_states(cfg)), w_r, None, cfg.top_k, cfg.renorm)
    m = O.decision_margins(g, 6, cfg.top_k, list(range(6)))
    assert m["score"] == 0.0
