"""GPU parity at the full sizes of the five workloads, in the launch configuration the benchmark times.

Routing (shortlist, per-token ids, segments, permutation) is compared with the oracle for every
token, bit-exact.  Layer outputs are compared with the oracle's Eq. (2)/(7)/(8) combine for EVERY token, at
every budget of the workload and under both policies (a few seconds of fp64 host work per case).  The trees
of 255 and 511 tokens, whose oracle needs 10-30 s per case, compare every token at one budget per policy and
a spread sample of tokens at the others."""
import dataclasses
import time

import numpy as np
import pytest
import torch

from oracle import moespec_oracle as O
from paper_2602_16052_amd import binding as mb
from paper_2602_16052_amd import workloads as wl

from gpu_common import (assert_out_close, assert_routing_equal, desc_of, oracle_weights, out_to_numpy, to_device,
                        upload_weights)

pytestmark = pytest.mark.gpu


def routing_reference(cfg, h_o, W_o, B, policy):
    g, ids, w = O.route(h_o, W_o["w_router"], W_o["b_router"], cfg.top_k, cfg.renorm, cfg.gate)
    r = O.budget(g, ids, w, B, policy, cfg.top_k, cfg.renorm)
    r.update(probs=g, loaded=sorted({int(e) for e in r["tok_ids"].ravel() if e >= 0}), union=O.expert_union(ids))
    return r


# a second routing scheme at full size: the OLMoE-shaped layer with a sigmoid gate per expert; and the benchmark
# workload drawn from other seeds (different expert popularity order, hidden rows and weights)
FULL = dict(wl.CONFIGS)
for _seed in (1, 2, 3, 4):
    FULL[f"olmoe_m63_seed{_seed}"] = dataclasses.replace(wl.CONFIGS["olmoe_m63"], name=f"olmoe_m63_seed{_seed}",
                                                         seed=_seed, budgets=(32, 64))
FULL["olmoe_m63_sigmoid"] = dataclasses.replace(wl.CONFIGS["olmoe_m63"], name="olmoe_m63_sigmoid", gate="sigmoid",
                                                budgets=(16, 32, 64))


# trees above this many tokens compare every token at ALL_TOKEN_BUDGET only and SAMPLED tokens at the other budgets
ALL_TOKEN_MAX_M, ALL_TOKEN_BUDGET, SAMPLED = 127, 32, 12


@pytest.fixture(scope="module", params=["olmoe_m63", "olmoe_m127", "fine_m127", "olmoe_m63_sigmoid", "olmoe_m255",
                                        "olmoe_m511", "olmoe_m63_seed1", "olmoe_m63_seed2", "olmoe_m63_seed3", "olmoe_m63_seed4"])
def full_case(request):
    cfg = FULL[request.param]
    t0 = time.time()
    W = wl.layer_weights(cfg, threads=16)
    h = wl.hidden_states(cfg)
    print(f"[{cfg.name}] generated weights in {time.time() - t0:.1f}s", flush=True)
    desc = desc_of(cfg)
    case = dict(cfg=cfg, W=W, desc=desc, h_d=to_device(h), W_d=upload_weights(W), h_o=wl.as_f32(h),
                W_o=dict(w_router=wl.as_f32(W["w_router"]), b_router=W["b_router"]),
                ws=mb.alloc_workspace(desc, cfg.M), widened={})
    yield case
    del case


@pytest.mark.parametrize("policy", [mb.TRUNCATE, mb.SUBSTITUTE])
def test_full_size_routing_and_outputs(full_case, policy):
    c = full_case
    cfg = c["cfg"]

    def widened(e):
        """float32 copies of expert e's stored matrices (exact), kept for the other budgets of the workload"""
        if e not in c["widened"]:
            c["widened"][e] = {key: wl.as_f32(c["W"][key][e]) for key in ("w_gate", "w_up", "w_down")}
        return c["widened"][e]

    for B in cfg.budgets:
        every = cfg.M <= ALL_TOKEN_MAX_M or B == ALL_TOKEN_BUDGET
        sample = list(range(cfg.M)) if every else sorted({int(t) for t in np.linspace(0, cfg.M - 1, SAMPLED)})
        print(f"[{cfg.name}] B={B} policy={policy} outputs compared on {len(sample)} of {cfg.M} tokens", flush=True)
        out, taps = mb.moespec_layer_forward(c["desc"], c["W_d"], c["h_d"], B, policy, c["ws"], taps=True)
        torch.cuda.synchronize()
        ref = routing_reference(cfg, c["h_o"], c["W_o"], B, policy)
        assert_routing_equal(taps, ref, B)
        got = out_to_numpy(out)
        assert np.all(np.isfinite(got))
        need = sorted({int(e) for t in sample for e in ref["tok_ids"][t] if e >= 0})
        Wexp = {key: {e: widened(e)[key] for e in need} for key in ("w_gate", "w_up", "w_down")}
        t0 = time.time()
        want = O.combine(c["h_o"], ref["tok_ids"], ref["tok_w"], Wexp["w_gate"], Wexp["w_up"], Wexp["w_down"],
                         tokens=sample)
        err, scale = assert_out_close(got, want, cfg.dtype, rows=sample, what=f"{cfg.name} B={B} policy={policy}")
        print(f"[{cfg.name}] B={B} policy={policy}: max|diff| {err:.3e} at output scale {scale:.3f}, oracle "
              f"{time.time() - t0:.1f}s", flush=True)
        # the call the benchmark times: no taps, so the budget stage skips the grouping of the pairs
        out_plain = torch.full_like(out, float("nan"))
        mb.LayerForwardCall(c["desc"], c["W_d"], c["h_d"], B, policy, c["ws"], out_plain)()
        torch.cuda.synchronize()
        assert torch.equal(out_plain, out), "layer output differs between the call with and without taps"
        if policy == mb.TRUNCATE:
            dropped = [t for t in range(cfg.M) if np.all(ref["tok_ids"][t] < 0)]
            if dropped:
                assert torch.all(out[dropped] == 0)
        if B == cfg.n_experts:
            # unbudgeted run: the loaded set is the expert union of Eq. (3)
            assert int(taps["n_loaded"][0]) == len(ref["union"])


def test_twenty_runs_are_bit_identical_at_full_size(full_case):
    """Same inputs, same bits: outputs and every integer intermediate of 20 consecutive calls."""
    c = full_case
    cfg = c["cfg"]
    B = 32 if 32 in cfg.budgets else cfg.budgets[0]
    first = None
    for _ in range(20):
        out, taps = mb.moespec_layer_forward(c["desc"], c["W_d"], c["h_d"], B, mb.SUBSTITUTE, c["ws"], taps=True)
        torch.cuda.synchronize()
        snap = [out.clone()] + [taps[key].clone() for key in sorted(taps)]
        if first is None:
            first = snap
        else:
            assert all(torch.equal(a, b) for a, b in zip(first, snap))


def test_budget_invariants_at_full_size(full_case):
    """Properties that hold at any size: at most B experts loaded, every surviving id inside the shortlist,
    exactly k experts per token under substitution, perm a permutation of the surviving pairs."""
    c = full_case
    cfg = c["cfg"]
    k = cfg.top_k
    for B in cfg.budgets:
        for policy in (mb.TRUNCATE, mb.SUBSTITUTE):
            _, taps = mb.moespec_layer_forward(c["desc"], c["W_d"], c["h_d"], B, policy, c["ws"], taps=True)
            torch.cuda.synchronize()
            S = set(taps["budget_ids"].cpu().numpy()[:B].tolist())
            ids = taps["tok_ids"].cpu().numpy()
            assert len(S) == B and set(ids[ids >= 0].tolist()) <= S
            assert int(taps["n_loaded"][0]) <= B
            P = int(taps["seg_off"][B])
            perm = taps["perm"].cpu().numpy()
            assert sorted(perm[:P].tolist()) == [i for i in range(cfg.M * k) if ids.ravel()[i] >= 0]
            if policy == mb.SUBSTITUTE:
                assert P == cfg.M * k and np.all(ids >= 0)
                assert all(len(set(row.tolist())) == k for row in ids)


# ---------------------------------------------------------------------------------------------- layer stack
STACK = wl.CONFIGS["coarse_stack"]


@pytest.fixture(scope="module")
def stack_state():
    """Hidden state carried from layer to layer by the GPU path (teacher forcing for the oracle)."""
    h = wl.hidden_states(STACK)
    return dict(h_d=to_device(h), layer=0, desc=desc_of(STACK), ws=mb.alloc_workspace(desc_of(STACK), STACK.M))


@pytest.mark.parametrize("layer", range(STACK.n_layers))
def test_coarse_stack_layer(stack_state, layer):
    """Layer `layer` of the 8-layer stack h <- h + MoE_S(x), x = h / rms(h), B=4, substitution, fed with the
    hidden state the GPU path itself produced for the previous layers (teacher forcing: the oracle gets the
    same bf16 input bits).  Routing of every budget and both policies is checked against the oracle on that
    input; outputs on sampled tokens.

    The unit-RMS scaling of the MoE input is scaffolding of this stack driver, not a step of the method: with
    N(0, 0.02) weights at d=4096, F=14336 the plain recurrence h <- h + MoE(h) squares the hidden scale every
    layer (measured output scales 8.5, 52, 1817, then overflow; routing probabilities underflow to 0/0)."""
    cfg, st = STACK, stack_state
    assert st["layer"] == layer, "stack layers must run in order"
    B_run, sample = 4, [0, cfg.M - 1]
    res_d = st["h_d"]
    hf = res_d.float()
    h_d = (hf / hf.pow(2).mean(dim=1, keepdim=True).sqrt()).to(torch.bfloat16)
    h_o = h_d.float().cpu().numpy()
    router = wl.layer_weights(cfg, layer=layer, experts=())
    W_o = dict(w_router=wl.as_f32(router["w_router"]), b_router=router["b_router"])
    ref = routing_reference(cfg, h_o, W_o, B_run, mb.SUBSTITUTE)
    t0 = time.time()
    W = wl.layer_weights(cfg, layer=layer, experts=tuple(int(e) for e in sorted(ref["S"])), threads=16)
    print(f"[stack layer {layer}] generated {B_run} experts in {time.time() - t0:.1f}s", flush=True)
    W_d = upload_weights(W)
    # routing for every budget / policy needs no expert weights beyond the router
    for B in cfg.budgets:
        for policy in (mb.TRUNCATE, mb.SUBSTITUTE):
            r = mb.moespec_route(st["desc"], W_d, h_d, st["ws"])
            b = mb.moespec_budget(st["desc"], r["probs"], B, policy, st["ws"])
            torch.cuda.synchronize()
            rr = routing_reference(cfg, h_o, W_o, B, policy)
            assert np.array_equal(b["budget_ids"].cpu().numpy()[:B], rr["S"])
            assert np.array_equal(b["tok_ids"].cpu().numpy(), rr["tok_ids"])
            assert np.array_equal(b["seg_off"].cpu().numpy()[:B + 1], rr["seg_off"])
            assert np.array_equal(b["perm"].cpu().numpy()[:int(rr["seg_off"][-1])], rr["perm"])
    moe, taps = mb.moespec_layer_forward(st["desc"], W_d, h_d, B_run, mb.SUBSTITUTE, st["ws"], taps=True)
    nxt = mb.moespec_layer_forward(st["desc"], W_d, h_d, B_run, mb.SUBSTITUTE, st["ws"], residual=res_d)
    torch.cuda.synchronize()
    assert_routing_equal(taps, ref, B_run)
    need = sorted({int(e) for t in sample for e in ref["tok_ids"][t]})
    Wexp = {key: {e: wl.as_f32(W[key][e]) for e in need} for key in ("w_gate", "w_up", "w_down")}
    want = O.combine(h_o, ref["tok_ids"], ref["tok_w"], Wexp["w_gate"], Wexp["w_up"], Wexp["w_down"], tokens=sample)
    err, scale = assert_out_close(out_to_numpy(moe), want, cfg.dtype, rows=sample, scale_aware=True,
                                  what=f"stack layer {layer} MoE output")
    print(f"[stack layer {layer}] max|diff| {err:.3e} at output scale {scale:.2f}", flush=True)
    # residual stream: h + MoE(h), stored in bf16 (half an ulp of the stored value on top of the MoE tolerance)
    got_h = out_to_numpy(nxt)[sample]
    want_h = res_d.float().cpu().numpy()[sample].astype(np.float64) + want[sample]
    assert np.all(np.abs(got_h - want_h) <= 2e-2 * max(1.0, scale) + 2.0 ** -8 * np.abs(want_h))
    assert np.all(np.isfinite(out_to_numpy(nxt)))
    st["h_d"], st["layer"] = nxt, layer + 1
    del W_d, W
    torch.cuda.empty_cache()
