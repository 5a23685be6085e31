"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Integer outputs (shortlist, routing ids, segments, permutation) must be bit-exact;
layer outputs within max-abs 2e-2 (bf16) / 1e-5 (fp32), absolute and relative to max|oracle|."""
import numpy as np
import pytest
import torch

from oracle import moespec_oracle as O
from paper_2602_16052_amd import binding as mb
from paper_2602_16052_amd import workloads as wl

from gpu_common import (TOL, assert_out_close, assert_routing_equal, desc_of, oracle_weights, out_to_numpy,
                        to_device, upload_weights)

pytestmark = pytest.mark.gpu

SMALL = {
    # name: config  (shapes chosen to span several 16-token tiles, ragged tails and every K-unroll variant)
    "s_bf16_a": wl.small_config("s_bf16_a", "bf16", d=256, n_experts=16, top_k=4, d_ff=192, M=37, budgets=(4, 8, 16)),
    "s_bf16_k1": wl.small_config("s_bf16_k1", "bf16", d=96, n_experts=8, top_k=1, d_ff=160, M=21, budgets=(1, 3, 8),
                                 renorm=False),
    "s_bf16_big_seg": wl.small_config("s_bf16_big_seg", "bf16", d=128, n_experts=4, top_k=2, d_ff=64, M=300,
                                      budgets=(2, 4), bias_alpha=0.3),
    "s_bf16_m1": wl.small_config("s_bf16_m1", "bf16", d=64, n_experts=8, top_k=2, d_ff=32, M=1, budgets=(2, 8)),
    "s_bf16_n100": wl.small_config("s_bf16_n100", "bf16", d=320, n_experts=100, top_k=6, d_ff=96, M=70,
                                   budgets=(6, 40, 100), bias_alpha=1.0, renorm=False),
    # d and F multiples of 128: both expert passes on the LDS-tiled kernels, whose workgroups find their
    # own segments inside the fused call
    "s_bf16_self": wl.small_config("s_bf16_self", "bf16", d=256, n_experts=16, top_k=4, d_ff=384, M=45,
                                   budgets=(4, 9, 16), bias_alpha=0.8),
    "s_bf16_self_big": wl.small_config("s_bf16_self_big", "bf16", d=128, n_experts=4, top_k=2, d_ff=128, M=300,
                                       budgets=(2, 3, 4), bias_alpha=0.3),
    # long F with few row tiles: the down pass is cut along F into partial sums that the combine adds up
    "s_bf16_split": wl.small_config("s_bf16_split", "bf16", d=128, n_experts=4, top_k=2, d_ff=4096, M=20,
                                    budgets=(2, 4), bias_alpha=0.5),
    # a tree beyond every small-tree limit: segments read from perm, routing table not staged in LDS
    # (M k > 8192), many pieces of up to 128 pairs per segment
    "s_bf16_m5000": wl.small_config("s_bf16_m5000", "bf16", d=128, n_experts=6, top_k=2, d_ff=128, M=5000,
                                    budgets=(2, 4, 6), bias_alpha=0.4),
    # a very large tree: the aggregate scores are summed once instead of in every workgroup
    "s_bf16_m20000": wl.small_config("s_bf16_m20000", "bf16", d=64, n_experts=8, top_k=2, d_ff=64, M=20000,
                                     budgets=(3, 8), bias_alpha=0.4),
    # the largest expert count and top-k the descriptor check admits
    "s_bf16_n1024": wl.small_config("s_bf16_n1024", "bf16", d=64, n_experts=1024, top_k=64, d_ff=32, M=9,
                                    budgets=(64, 300, 1024), bias_alpha=0.7),
    # segments of exactly M pairs (two experts, k = 2: every token is routed to both) around the 128-pair limit of
    # one walk over an expert: one piece, two uneven pieces, two full pieces, three pieces
    **{f"s_bf16_piece{M}": wl.small_config(f"s_bf16_piece{M}", "bf16", d=128, n_experts=2, top_k=2, d_ff=128, M=M,
                                           budgets=(2,), bias_alpha=0.2) for M in (128, 129, 256, 257)},
    # the same above the limit of the trees whose expert passes derive their own work items
    "s_bf16_piece1100": wl.small_config("s_bf16_piece1100", "bf16", d=128, n_experts=2, top_k=2, d_ff=128, M=1100,
                                        budgets=(2,), bias_alpha=0.2),
    # sigmoid-gated routing (an independent gate per expert instead of the softmax of Eq. (1))
    "s_bf16_sigmoid": wl.small_config("s_bf16_sigmoid", "bf16", d=256, n_experts=16, top_k=4, d_ff=128, M=45,
                                      budgets=(4, 9, 16), bias_alpha=0.8, gate="sigmoid"),
    "s_f32_sigmoid": wl.small_config("s_f32_sigmoid", "f32", d=100, n_experts=12, top_k=3, d_ff=52, M=19,
                                     budgets=(3, 6, 12), renorm=False, gate="sigmoid"),
    "s_f32_a": wl.small_config("s_f32_a", "f32", d=100, n_experts=12, top_k=3, d_ff=52, M=19, budgets=(3, 6, 12)),
    "tiny_f32": wl.CONFIGS["tiny_f32"],
}


def make_case(cfg):
    h = wl.hidden_states(cfg)
    W = wl.layer_weights(cfg)
    return h, W


@pytest.fixture(scope="module")
def cases():
    cache = {}

    def get(name):
        if name not in cache:
            cfg = SMALL[name]
            h, W = make_case(cfg)
            desc = desc_of(cfg)
            cache[name] = dict(cfg=cfg, h=h, W=W, desc=desc, h_d=to_device(h), W_d=upload_weights(W),
                               h_o=wl.as_f32(h), W_o=oracle_weights(W), ws=mb.alloc_workspace(desc, cfg.M))
        return cache[name]
    return get


@pytest.mark.parametrize("name", list(SMALL))
def test_route_parity(cases, name):
    c = cases(name)
    cfg = c["cfg"]
    r = mb.moespec_route(c["desc"], c["W_d"], c["h_d"], c["ws"])
    torch.cuda.synchronize()
    g, ids, w = O.route(c["h_o"], c["W_o"]["w_router"], c["W_o"]["b_router"], cfg.top_k, cfg.renorm, cfg.gate)
    np.testing.assert_allclose(r["probs"].cpu().numpy(), g, rtol=1e-11, atol=1e-300)
    assert np.array_equal(r["topk_ids"].cpu().numpy(), ids)
    np.testing.assert_allclose(r["topk_w"].cpu().numpy(), w, rtol=1e-6)


@pytest.mark.parametrize("policy", [mb.TRUNCATE, mb.SUBSTITUTE])
@pytest.mark.parametrize("name", list(SMALL))
def test_layer_forward_parity_small(cases, name, policy):
    c = cases(name)
    cfg = c["cfg"]
    for B in cfg.budgets:
        if policy == mb.SUBSTITUTE and B < cfg.top_k:
            continue
        print(f"case {name} B={B} policy={policy}", flush=True)
        out, taps = mb.moespec_layer_forward(c["desc"], c["W_d"], c["h_d"], B, policy, c["ws"], taps=True)
        torch.cuda.synchronize()
        ref = O.layer_forward(c["h_o"], c["W_o"], cfg.top_k, cfg.renorm, B, policy, gate=cfg.gate)
        assert_routing_equal(taps, ref, B)
        assert_out_close(out_to_numpy(out), ref["out"], cfg.dtype)
        # without taps the budget stage may skip the grouping of the pairs: same output, bit for bit
        out_plain = mb.moespec_layer_forward(c["desc"], c["W_d"], c["h_d"], B, policy, c["ws"])
        torch.cuda.synchronize()
        assert torch.equal(out_plain, out)
        if policy == mb.TRUNCATE:
            dropped = [t for t in range(cfg.M) if np.all(ref["tok_ids"][t] < 0)]
            if dropped:
                assert torch.all(out[dropped] == 0), "tokens without a surviving expert must get exact zeros"


@pytest.mark.parametrize("name", ["s_bf16_a", "s_bf16_self", "s_bf16_self_big", "s_bf16_piece257", "s_f32_a"])
def test_stage_calls_compose_to_the_fused_call(cases, name):
    """route -> budget -> expert_ffn through their own entry points equals layer_forward bit for bit."""
    c = cases(name)
    cfg = c["cfg"]
    B = cfg.budgets[min(1, len(cfg.budgets) - 1)]
    for policy in (mb.TRUNCATE, mb.SUBSTITUTE):
        r = mb.moespec_route(c["desc"], c["W_d"], c["h_d"], c["ws"])
        b = mb.moespec_budget(c["desc"], r["probs"], B, policy, c["ws"])
        out = mb.moespec_expert_ffn(c["desc"], c["W_d"], c["h_d"], b["seg_expert"], b["seg_off"], b["perm"],
                                    b["tok_ids"], b["tok_w"], c["ws"])
        out2, taps = mb.moespec_layer_forward(c["desc"], c["W_d"], c["h_d"], B, policy, c["ws"], taps=True)
        torch.cuda.synchronize()
        assert torch.equal(out, out2)
        for key in ("tok_ids", "tok_w", "seg_expert", "seg_off", "perm", "budget_ids", "n_loaded"):
            assert torch.equal(b[key], taps[key]), key
        # the fused call adds the router projection and the scores in another order than the stage calls
        torch.testing.assert_close(b["scores"], taps["scores"], rtol=1e-12, atol=0)
        torch.testing.assert_close(r["probs"], taps["probs"], rtol=1e-11, atol=1e-300)
        if policy == mb.TRUNCATE:
            # Eq. (7): kept weights are the natural top-k weights, bit for bit.
            keep = b["tok_ids"] >= 0
            assert torch.equal(b["tok_ids"][keep], r["topk_ids"][keep])
            assert torch.equal(b["tok_w"][keep], r["topk_w"][keep])
            assert torch.all(b["tok_w"][~keep] == 0)


def test_full_budget_is_the_unbudgeted_layer(cases):
    """B = N: both policies reproduce the natural routing and Eq. (2); the loaded set is the union of Eq. (3)."""
    c = cases("s_bf16_a")
    cfg = c["cfg"]
    r = mb.moespec_route(c["desc"], c["W_d"], c["h_d"], c["ws"])
    outs = []
    for policy in (mb.TRUNCATE, mb.SUBSTITUTE):
        out, taps = mb.moespec_layer_forward(c["desc"], c["W_d"], c["h_d"], cfg.n_experts, policy, c["ws"], taps=True)
        torch.cuda.synchronize()
        assert torch.equal(taps["tok_ids"], r["topk_ids"])
        assert torch.equal(taps["tok_w"], r["topk_w"])
        union = O.expert_union(r["topk_ids"].cpu().numpy())
        assert int(taps["n_loaded"][0]) == len(union)
        outs.append(out)
    assert torch.equal(outs[0], outs[1])
    ref = O.unbudgeted_forward(c["h_o"], c["W_o"], cfg.top_k, cfg.renorm)
    assert_out_close(out_to_numpy(outs[0]), ref, cfg.dtype)


def test_external_shortlist_and_residual(cases):
    c = cases("s_bf16_a")
    cfg = c["cfg"]
    ext = [11, 2, 7, 5, 14, 0]
    ext_d = torch.tensor(ext, dtype=torch.int32, device="cuda")
    resid = torch.randn(cfg.M, cfg.d, generator=torch.Generator().manual_seed(1)).to(torch.bfloat16).cuda()
    for policy in (mb.TRUNCATE, mb.SUBSTITUTE):
        out, taps = mb.moespec_layer_forward(c["desc"], c["W_d"], c["h_d"], len(ext), policy, c["ws"],
                                             ext_shortlist=ext_d, residual=resid, taps=True)
        torch.cuda.synchronize()
        ref = O.layer_forward(c["h_o"], c["W_o"], cfg.top_k, cfg.renorm, len(ext), policy, ext_shortlist=ext)
        assert_routing_equal(taps, ref, len(ext))
        want = ref["out"] + resid.float().cpu().numpy().astype(np.float64)
        assert_out_close(out_to_numpy(out), want, cfg.dtype)


def test_repeated_calls_are_bit_identical(cases):
    c = cases("s_bf16_n100")
    cfg = c["cfg"]
    first = None
    for _ in range(5):
        out, taps = mb.moespec_layer_forward(c["desc"], c["W_d"], c["h_d"], 40, mb.SUBSTITUTE, c["ws"], taps=True)
        torch.cuda.synchronize()
        snap = [out.clone()] + [taps[k].clone() for k in sorted(taps)]
        if first is None:
            first = snap
        else:
            for a, b in zip(first, snap):
                assert torch.equal(a, b)


def test_ties_go_to_the_lowest_id_on_the_gpu():
    """Duplicated router rows give exactly equal probabilities: ranking must break ties by id."""
    cfg = wl.small_config("ties", "bf16", d=64, n_experts=8, top_k=3, d_ff=32, M=9, budgets=(4,))
    h, W = make_case(cfg)
    W["w_router"][2] = W["w_router"][0]
    W["w_router"][5] = W["w_router"][0]
    W["w_router"][4] = W["w_router"][1]
    W["b_router"][:] = 0
    desc = desc_of(cfg)
    ws = mb.alloc_workspace(desc, cfg.M)
    for policy in (mb.TRUNCATE, mb.SUBSTITUTE):
        out, taps = mb.moespec_layer_forward(desc, upload_weights(W), to_device(h), 4, policy, ws, taps=True)
        torch.cuda.synchronize()
        ref = O.layer_forward(wl.as_f32(h), oracle_weights(W), cfg.top_k, cfg.renorm, 4, policy)
        assert_routing_equal(taps, ref, 4)
        assert_out_close(out_to_numpy(out), ref["out"], cfg.dtype)


def test_shortlist_that_nobody_routes_to_gives_exact_zeros_or_the_residual(cases):
    """Eq. (7) with an empty intersection for every token: no expert is loaded, the MoE output is exactly zero and
    only the residual passes through."""
    c = cases("s_bf16_self")
    cfg = c["cfg"]
    _, ids, _ = O.route(c["h_o"], c["W_o"]["w_router"], c["W_o"]["b_router"], cfg.top_k, cfg.renorm)
    unused = sorted(set(range(cfg.n_experts)) - set(O.expert_union(ids)))
    assert len(unused) >= 2, "the case needs experts outside the union"
    ext = torch.tensor(unused[:2], dtype=torch.int32, device="cuda")
    resid = torch.randn(cfg.M, cfg.d, generator=torch.Generator().manual_seed(3)).to(torch.bfloat16).cuda()
    out, taps = mb.moespec_layer_forward(c["desc"], c["W_d"], c["h_d"], 2, mb.TRUNCATE, c["ws"], ext_shortlist=ext,
                                         taps=True)
    plain = mb.moespec_layer_forward(c["desc"], c["W_d"], c["h_d"], 2, mb.TRUNCATE, c["ws"], ext_shortlist=ext)
    with_res = mb.moespec_layer_forward(c["desc"], c["W_d"], c["h_d"], 2, mb.TRUNCATE, c["ws"], ext_shortlist=ext,
                                        residual=resid)
    torch.cuda.synchronize()
    assert int(taps["n_loaded"][0]) == 0 and torch.all(taps["tok_ids"] == -1) and torch.all(taps["tok_w"] == 0)
    assert torch.all(taps["seg_off"][:3] == 0) and torch.all(taps["perm"] == -1)
    assert torch.all(out == 0) and torch.all(plain == 0) and torch.equal(with_res, resid)


def test_external_shortlist_with_repeated_and_invalid_ids(cases):
    """An external shortlist may repeat an expert or name ids outside [0, N): those entries are ignored, the rest
    behaves like the clean list (truncation keeps T_k intersected with the set, whatever B says)."""
    c = cases("s_bf16_a")
    cfg = c["cfg"]
    messy = [3, 3, 7, 99, -5, 1]
    clean = [3, 7, 1]
    out, taps = mb.moespec_layer_forward(c["desc"], c["W_d"], c["h_d"], len(messy), mb.TRUNCATE, c["ws"],
                                         ext_shortlist=torch.tensor(messy, dtype=torch.int32, device="cuda"), taps=True)
    torch.cuda.synchronize()
    ref = O.layer_forward(c["h_o"], c["W_o"], cfg.top_k, cfg.renorm, len(clean), O.TRUNCATE, ext_shortlist=clean)
    assert np.array_equal(taps["tok_ids"].cpu().numpy(), ref["tok_ids"])
    np.testing.assert_allclose(taps["tok_w"].cpu().numpy(), ref["tok_w"], rtol=1e-6, atol=1e-12)
    assert taps["seg_expert"].cpu().tolist() == sorted(clean) + [-1] * (len(messy) - len(clean))
    assert taps["seg_off"].cpu().numpy()[:len(clean) + 1].tolist() == ref["seg_off"].tolist()
    assert int(taps["n_loaded"][0]) == len(ref["loaded"])
    assert_out_close(out_to_numpy(out), ref["out"], cfg.dtype)


@pytest.mark.parametrize("name", ["s_bf16_a", "s_bf16_self", "s_f32_a"])
def test_non_finite_hidden_rows_leave_every_index_in_range(cases, name):
    """A NaN hidden row makes every routing score NaN, so no ranking comparison holds and selections cannot fill
    their slots.  The paper defines nothing for such input; the path must still finish normally, mark the
    unfilled slots as dropped (-1, weight 0) and hand the expert passes only ids inside [0, N)."""
    c = cases(name)
    cfg = c["cfg"]
    h_bad = c["h_d"].clone()
    h_bad[min(3, cfg.M - 1), 5] = float("nan")
    for policy in (mb.TRUNCATE, mb.SUBSTITUTE):
        for B in cfg.budgets:
            if policy == mb.SUBSTITUTE and B < cfg.top_k:
                continue
            for taps_on in (True, False):
                res = mb.moespec_layer_forward(c["desc"], c["W_d"], h_bad, B, policy, c["ws"], taps=taps_on)
                torch.cuda.synchronize()
                if taps_on:
                    taps = res[1]
                    ids, S, perm = taps["tok_ids"].cpu().numpy(), taps["budget_ids"].cpu().numpy(), taps["perm"].cpu().numpy()
                    assert np.all((ids >= -1) & (ids < cfg.n_experts)) and np.all((S >= -1) & (S < cfg.n_experts))
                    assert np.all((perm >= -1) & (perm < cfg.M * cfg.top_k))
                    assert np.all(taps["tok_w"].cpu().numpy()[ids < 0] == 0)
    # the same workspace serves a clean call afterwards
    out, taps = mb.moespec_layer_forward(c["desc"], c["W_d"], c["h_d"], cfg.budgets[-1], mb.TRUNCATE, c["ws"], taps=True)
    torch.cuda.synchronize()
    ref = O.layer_forward(c["h_o"], c["W_o"], cfg.top_k, cfg.renorm, cfg.budgets[-1], O.TRUNCATE, gate=cfg.gate)
    assert_routing_equal(taps, ref, cfg.budgets[-1])
    assert_out_close(out_to_numpy(out), ref["out"], cfg.dtype)
