"""GPU parity of the steps around the hot path: static ranking (Eq. (4)) feeding the layer as an external
shortlist, the coverage curve (Section 4.6) and the reconstruction error (Section 4.5)."""
import numpy as np
import pytest
import torch

from oracle import moespec_oracle as O
from paper_2602_16052_amd import binding as mb
from paper_2602_16052_amd import workloads as wl

from gpu_common import (assert_out_close, assert_routing_equal, desc_of, oracle_weights, out_to_numpy, to_device,
                        upload_weights)

pytestmark = pytest.mark.gpu

CASES = {
    "an_bf16": wl.small_config("an_bf16", "bf16", d=256, n_experts=24, top_k=4, d_ff=128, M=41, budgets=(6, 12, 24),
                               bias_alpha=1.0),
    "an_f32": wl.small_config("an_f32", "f32", d=64, n_experts=10, top_k=2, d_ff=40, M=17, budgets=(2, 5, 10),
                              bias_alpha=0.3),
}


@pytest.fixture(scope="module", params=list(CASES))
def case(request):
    cfg = CASES[request.param]
    h, W = wl.hidden_states(cfg), wl.layer_weights(cfg)
    desc = desc_of(cfg)
    return dict(cfg=cfg, desc=desc, W=W, W_d=upload_weights(W), W_o=oracle_weights(W), h_d=to_device(h),
                h_o=wl.as_f32(h), ws=mb.alloc_workspace(desc, 64))


def test_static_ranking_counts_shortlist_and_layer(case):
    """Calibration batches (different seeds, ragged sizes) -> c_i -> static shortlist -> budgeted layer."""
    c = case
    cfg, desc = c["cfg"], c["desc"]
    counts_d = torch.zeros(cfg.n_experts, dtype=torch.int64, device="cuda")
    counts_o = None
    for seed, M in ((11, 64), (12, 1), (13, 37)):
        hb = wl.hidden_states(cfg, M=M, seed=seed)
        r = mb.moespec_route(desc, c["W_d"], to_device(hb), c["ws"])
        mb.moespec_calibration_count(desc, r["topk_ids"], counts_d)
        _, ids, _ = O.route(wl.as_f32(hb), c["W_o"]["w_router"], c["W_o"]["b_router"], cfg.top_k, cfg.renorm)
        counts_o = O.calibration_counts(ids, cfg.n_experts, counts_o)
    torch.cuda.synchronize()
    assert np.array_equal(counts_d.cpu().numpy(), counts_o)
    assert int(counts_o.sum()) == (64 + 1 + 37) * cfg.top_k
    for B in cfg.budgets:
        S_d = mb.moespec_static_shortlist(desc, counts_d, B)
        torch.cuda.synchronize()
        S_o = O.static_shortlist(counts_o, B)
        assert S_d.cpu().tolist() == S_o
        for policy in (mb.TRUNCATE, mb.SUBSTITUTE):
            if policy == mb.SUBSTITUTE and B < cfg.top_k:
                continue
            out, taps = mb.moespec_layer_forward(desc, c["W_d"], c["h_d"], B, policy, c["ws"], ext_shortlist=S_d,
                                                 taps=True)
            torch.cuda.synchronize()
            ref = O.layer_forward(c["h_o"], c["W_o"], cfg.top_k, cfg.renorm, B, policy, ext_shortlist=S_o)
            assert_routing_equal(taps, ref, B)
            assert_out_close(out_to_numpy(out), ref["out"], cfg.dtype)


def test_static_shortlist_ties_and_out_of_range_ids(case):
    desc, N = case["desc"], case["cfg"].n_experts
    counts = torch.tensor([7 if i % 3 == 0 else 2 for i in range(N)], dtype=torch.int64, device="cuda")
    for B in (1, 4, N):
        got = mb.moespec_static_shortlist(desc, counts, B).cpu().tolist()
        assert got == O.static_shortlist(counts.cpu().numpy(), B)
    # ids outside [0, N) (dropped slots of a restricted table) are not counted
    ids = torch.tensor([[0, -1], [N, 3], [3, 3]], dtype=torch.int32, device="cuda")
    d2 = mb.LayerDesc(desc.d, desc.n_experts, 2, desc.d_ff, desc.dtype, desc.renorm)
    c = mb.moespec_calibration_count(d2, ids, torch.zeros(N, dtype=torch.int64, device="cuda"))
    want = np.zeros(N, dtype=np.int64)
    want[0], want[3] = 1, 3
    assert np.array_equal(c.cpu().numpy(), want)


def test_coverage_curve_and_reconstruction_error(case):
    c = case
    cfg, desc = c["cfg"], c["desc"]
    full, taps = mb.moespec_layer_forward(desc, c["W_d"], c["h_d"], cfg.n_experts, mb.SUBSTITUTE, c["ws"], taps=True)
    curve = mb.moespec_coverage_curve(desc, taps["scores"])
    torch.cuda.synchronize()
    ref = O.layer_forward(c["h_o"], c["W_o"], cfg.top_k, cfg.renorm, cfg.n_experts, O.SUBSTITUTE)
    np.testing.assert_allclose(curve.cpu().numpy(), O.coverage_curve(ref["scores"]), rtol=1e-12)
    # same input bits on both sides: the diagnostic itself is compared to 1e-12
    np.testing.assert_allclose(curve.cpu().numpy(), O.coverage_curve(taps["scores"].cpu().numpy()), rtol=1e-14)
    full_np = out_to_numpy(full)
    errs = []
    for B in cfg.budgets:
        for policy in (mb.TRUNCATE, mb.SUBSTITUTE):
            if policy == mb.SUBSTITUTE and B < cfg.top_k:
                continue
            out = mb.moespec_layer_forward(desc, c["W_d"], c["h_d"], B, policy, c["ws"])
            err = mb.moespec_reconstruction_error(desc, out, full, c["ws"])
            torch.cuda.synchronize()
            e = err.cpu().numpy()
            want = O.reconstruction_error(out_to_numpy(out), full_np)
            assert e[0] == pytest.approx(want, rel=1e-12, abs=1e-300)
            assert e[0] == pytest.approx(e[1] / e[2], rel=1e-15, abs=1e-300)
            if B == cfg.n_experts:
                assert e[0] == 0.0
            # against the oracle's own layer outputs the error agrees to the output tolerance
            ref_b = O.layer_forward(c["h_o"], c["W_o"], cfg.top_k, cfg.renorm, B, policy)
            want_o = O.reconstruction_error(ref_b["out"], ref["out"])
            assert abs(e[0] - want_o) <= 0.05 * max(want_o, 1e-3)
            errs.append(e[0])
    assert max(errs) > 0


def test_oracle_ranking_matches_the_cpu_greedy(case):
    """Eq. (6).  fp32 layers: same ordering and error curve.  bf16 layers (expert outputs carry ~1e-3 of bf16
    rounding): every pick must be a minimiser of the oracle's own error up to that rounding, and the error
    curve must agree."""
    c = case
    cfg, desc = c["cfg"], c["desc"]
    N = cfg.n_experts
    ranking, err = mb.moespec_oracle_ranking(desc, c["W_d"], c["h_d"], N, c["ws"])
    torch.cuda.synchronize()
    ranking, err = ranking.cpu().tolist(), err.cpu().numpy()
    _, ids, w = O.route(c["h_o"], c["W_o"]["w_router"], c["W_o"]["b_router"], cfg.top_k, cfg.renorm)
    C = O.expert_contributions(c["h_o"], ids, w, c["W_o"]["w_gate"], c["W_o"]["w_up"], c["W_o"]["w_down"], N)
    S, errs = O.oracle_ranking(C, N)
    assert sorted(ranking) == list(range(N))
    union = O.expert_union(ids)
    tol = 1e-5 if cfg.dtype == "f32" else 2e-2
    np.testing.assert_allclose(err, errs, atol=tol * 0.1, rtol=tol)
    assert err[len(union) - 1] <= tol * 0.1 and set(ranking[:len(union)]) == set(union)
    assert ranking[len(union):] == sorted(set(range(N)) - set(union))      # unused experts last, in id order
    if cfg.dtype == "f32":
        assert ranking == S
    # each GPU pick, judged by the oracle's arithmetic on the oracle's contributions
    gold = C.sum(axis=0)
    denom = float(np.sum(gold * gold))
    partial = np.zeros_like(gold)
    for step in range(len(union)):
        cand = {i: float(np.sum((gold - partial - C[i]) ** 2)) / denom for i in range(N) if i not in ranking[:step]}
        assert cand[ranking[step]] <= min(cand.values()) + tol * 0.1
        partial = partial + C[ranking[step]]
    # the ordering is usable as an external shortlist
    B = cfg.budgets[0]
    out = mb.moespec_layer_forward(desc, c["W_d"], c["h_d"], B, mb.TRUNCATE, c["ws"],
                                   ext_shortlist=torch.tensor(ranking[:B], dtype=torch.int32, device="cuda"))
    full = mb.moespec_layer_forward(desc, c["W_d"], c["h_d"], N, mb.TRUNCATE, c["ws"])
    e = mb.moespec_reconstruction_error(desc, out, full, c["ws"])
    torch.cuda.synchronize()
    assert float(e[0]) == pytest.approx(float(err[B - 1]), abs=3 * tol, rel=0.2)


@pytest.mark.parametrize("nbytes", [16, 4096, 1 << 20, (1 << 20) + 48, 24 << 20])
def test_stream_read_checksum(nbytes):
    """The streaming-read measurement kernel touches every byte once: its checksum is the sum of all 32-bit words."""
    g = torch.Generator(device="cuda").manual_seed(nbytes)
    buf = torch.randint(-2**31, 2**31 - 1, (nbytes // 4,), dtype=torch.int32, device="cuda", generator=g)
    got = mb.moespec_stream_read(buf)
    got = mb.moespec_stream_read(buf, got)          # a second call adds to the same words
    torch.cuda.synchronize()
    want = (2 * int(buf.cpu().numpy().astype(np.int64).sum())) % (1 << 32)
    assert int(got.cpu().numpy().astype(np.int64).sum()) % (1 << 32) == want
