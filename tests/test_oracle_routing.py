"""Pins for the oracle's routing, ranking and restriction steps (CPU only).

Each test checks the oracle against something other than itself: a hand-derived
worked example, brute-force enumeration, invariants the paper states, or a
library routine (torch CPU).
"""
import itertools
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import moespec_oracle as O


def frac(x):
    return float(Fraction(x))


def best_subset(values, size, candidates=None):
    """All `size`-subsets enumerated: the one with the largest value sum."""
    idx = list(range(len(values))) if candidates is None else sorted(candidates)
    best, best_sum = None, -math.inf
    for sub in itertools.combinations(idx, size):
        tot = math.fsum(float(values[i]) for i in sub)
        if tot > best_sum:
            best, best_sum = sub, tot
    return set(best)


@pytest.fixture(scope="module")
def worked(golden_dir):
    with open(os.path.join(golden_dir, "worked_example.json")) as f:
        ex = json.load(f)
    N, d, M, F = ex["N"], ex["d"], ex["M"], ex["F"]
    P = np.array(ex["P"], dtype=np.float64)            # P[t][i]
    w_router = np.log(P).T.copy()                       # w_i[t] = ln P[t][i]
    h = np.eye(M, d)
    ln3 = math.log(3.0)
    w_gate = np.zeros((N, F, d))
    w_gate[:, 0, :] = ln3
    w_gate[:, 1, :] = -ln3
    w_up = np.zeros((N, F, d))
    w_down = np.zeros((N, d, F))
    for i in range(N):
        for f in range(F):
            for t in range(d):
                w_up[i, f, t] = i + 2 * t + 3 * f + 1
        for j in range(d):
            w_down[i, j, 0] = j + 1
            w_down[i, j, 1] = i - j
    weights = dict(w_router=w_router, b_router=None, w_gate=w_gate, w_up=w_up, w_down=w_down)
    return ex, h, weights


# ------------------------------------------------------------------ worked example (Eq. 1, 3, 5, 7, 8)
def test_worked_example_routing(worked):
    ex, h, W = worked
    g, ids, w = O.route(h, W["w_router"], None, ex["k"], True)
    np.testing.assert_allclose(g, np.array(ex["P"]) / 10.0, rtol=0, atol=1e-15)
    assert ids.tolist() == ex["topk_ids"]
    np.testing.assert_allclose(w, [[frac(x) for x in r] for r in ex["topk_w"]], rtol=1e-14)
    assert O.expert_union(ids) == ex["union"]
    s = O.aggregate_scores(g)
    np.testing.assert_allclose(s, [frac(x) for x in ex["scores"]], rtol=1e-14)
    assert O.shortlist(s, ex["B"]) == ex["shortlist"]


@pytest.mark.parametrize("policy,key", [(O.TRUNCATE, "trunc"), (O.SUBSTITUTE, "sub")])
def test_worked_example_layer(worked, policy, key):
    ex, h, W = worked
    r = O.layer_forward(h, W, ex["k"], True, ex["B"], policy)
    assert r["S"].tolist() == ex["shortlist"]
    assert r["tok_ids"].tolist() == ex[key + "_ids"]
    np.testing.assert_allclose(r["tok_w"], [[frac(x) for x in row] for row in ex[key + "_w"]], rtol=1e-14)
    assert r["seg_expert"].tolist() == ex[key + "_seg_expert"]
    assert r["seg_off"].tolist() == ex[key + "_seg_off"]
    assert r["perm"].tolist() == ex[key + "_perm"]
    want = math.log(3.0) * np.array([[frac(x) for x in row] for row in ex[key + "_out_over_ln3"]])
    np.testing.assert_allclose(r["out"], want, rtol=1e-13, atol=1e-13)
    if policy == O.TRUNCATE:
        # Eq. (7): an empty intersection gives an exactly-zero MoE output.
        assert np.all(r["out"][2] == 0.0)


def test_raw_mixing_weights(worked):
    """Without renormalisation the mixing weights are the raw probabilities g_i."""
    ex, h, W = worked
    g, ids, w = O.route(h, W["w_router"], None, ex["k"], False)
    for t in range(ex["M"]):
        for j in range(ex["k"]):
            assert w[t, j] == pytest.approx(ex["P"][t][ids[t, j]] / 10.0, rel=1e-14)
    ids_s, w_s = O.restrict_substitution(g, ex["shortlist"], ex["k"], False)
    assert ids_s.tolist() == ex["sub_ids"]
    for t in range(ex["M"]):
        for j in range(ex["k"]):
            assert w_s[t, j] == pytest.approx(ex["P"][t][ids_s[t, j]] / 10.0, rel=1e-14)


# ------------------------------------------------------------------ Eq. (1) softmax against a library
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_softmax_matches_torch_and_sums(seed):
    rng = np.random.default_rng(seed)
    M, N, d = 9, 13, 32
    h = rng.standard_normal((M, d))
    w = rng.standard_normal((N, d)) * 0.3
    b = rng.standard_normal(N)
    logits = O.router_logits(h, w, b)
    want_logits = np.array([[sum(w[i, j] * h[t, j] for j in range(d)) + b[i] for i in range(N)] for t in range(M)])
    np.testing.assert_allclose(logits, want_logits, rtol=1e-12, atol=1e-12)
    g = O.routing_probs(logits)
    np.testing.assert_allclose(g.sum(axis=1), 1.0, atol=1e-14)
    want = torch.softmax(torch.from_numpy(logits), dim=1).numpy()
    np.testing.assert_allclose(g, want, rtol=1e-13, atol=1e-16)
    # Eq. (5): the scores of a tree of M tokens sum to M.
    assert O.aggregate_scores(g).sum() == pytest.approx(M, rel=1e-13)
    np.testing.assert_allclose(O.aggregate_scores(g), want.sum(axis=0), rtol=1e-13)


def test_softmax_is_shift_invariant_and_stable():
    logits = np.array([[1000.0, 999.0, 998.0], [-1000.0, -1001.0, -1002.0]])
    g = O.routing_probs(logits)
    e = np.exp([0.0, -1.0, -2.0])
    np.testing.assert_allclose(g, np.stack([e / e.sum()] * 2), rtol=1e-14)


def test_no_bias_is_plain_projection():
    rng = np.random.default_rng(5)
    h, w = rng.standard_normal((3, 8)), rng.standard_normal((5, 8))
    np.testing.assert_array_equal(O.router_logits(h, w, None), O.router_logits(h, w, np.zeros(5)))


# ------------------------------------------------------------------ top-k (Section 2.1)
@pytest.mark.parametrize("N,k", [(6, 2), (8, 3), (10, 4)])
def test_topk_brute_force_and_torch(N, k):
    rng = np.random.default_rng(N * 100 + k)
    for _ in range(20):
        g = O.routing_probs(rng.standard_normal((1, N)) * 2.0)[0]
        sel = O.top_k(g, k)
        assert set(sel) == best_subset(g, k)
        assert sel == torch.topk(torch.from_numpy(g), k).indices.tolist()
        assert all(g[a] >= g[b] for a, b in zip(sel, sel[1:]))


def test_ties_go_to_lowest_id_everywhere():
    # Duplicated router rows give exactly equal probabilities.
    rng = np.random.default_rng(3)
    d = 16
    base = rng.standard_normal((3, d))
    w = np.stack([base[0], base[1], base[0], base[2], base[1], base[0]])   # experts 0=2=5, 1=4
    h = rng.standard_normal((7, d))
    g, ids, _ = O.route(h, w, None, 3, True)
    assert np.array_equal(g[:, 0], g[:, 2]) and np.array_equal(g[:, 0], g[:, 5]) and np.array_equal(g[:, 1], g[:, 4])
    for t in range(7):
        sel = ids[t].tolist()
        for grp in ([0, 2, 5], [1, 4]):
            got = [e for e in sel if e in grp]
            assert got == grp[:len(got)]            # lowest ids first, and in ascending order
    s = O.aggregate_scores(g)
    for B in range(1, 7):
        S = O.shortlist(s, B)
        for grp in ([0, 2, 5], [1, 4]):
            got = [e for e in S if e in grp]
            assert got == grp[:len(got)]
    # exact tie on scores: two experts, constant probabilities
    assert O.shortlist([0.5, 0.5, 0.7, 0.5], 2) == [2, 0]
    assert O.rank_desc([0.1, 0.3, 0.3, 0.1], candidates=[3, 2, 1, 0]) == [1, 2, 0, 3]


# ------------------------------------------------------------------ top-B (Eq. 5 + shortlist)
@pytest.mark.parametrize("seed", range(4))
def test_shortlist_is_top_B_by_aggregate_probability(seed):
    rng = np.random.default_rng(seed)
    N, M = 11, 9
    g = O.routing_probs(rng.standard_normal((M, N)) * 1.5)
    s = O.aggregate_scores(g)
    prev, prev_cov = [], 0.0
    for B in range(1, N + 1):
        S = O.shortlist(s, B)
        assert len(S) == B and len(set(S)) == B
        assert set(S) == best_subset(s, B)                  # maximises the captured mass
        assert S[:len(prev)] == prev                        # nesting S_B subset of S_{B+1}
        cov = O.coverage(s, S)
        assert cov >= prev_cov - 1e-15
        prev, prev_cov = S, cov
    assert prev_cov == pytest.approx(1.0, rel=1e-14)


# ------------------------------------------------------------------ truncation (Eq. 7)
@pytest.mark.parametrize("renorm", [True, False])
def test_truncation_properties(renorm):
    rng = np.random.default_rng(11)
    N, M, k, d = 12, 17, 3, 24
    h, w = rng.standard_normal((M, d)), rng.standard_normal((N, d)) * 0.4
    g, ids, tw = O.route(h, w, None, k, renorm)
    s = O.aggregate_scores(g)
    seen_empty = False
    for B in range(1, N + 1):
        S = O.shortlist(s, B)
        tid, w_t = O.restrict_truncation(ids, tw, S)
        for t in range(M):
            for j in range(k):
                if ids[t, j] in S:
                    assert tid[t, j] == ids[t, j]
                    assert w_t[t, j] == tw[t, j]          # bitwise: not recomputed for the reduced set
                else:
                    assert tid[t, j] == -1 and w_t[t, j] == 0.0
            kept = [e for e in tid[t] if e >= 0]
            assert set(kept) == set(ids[t].tolist()) & set(S)
            seen_empty |= (len(kept) == 0)
    assert seen_empty, "test should exercise an empty intersection"


# ------------------------------------------------------------------ substitution (Eq. 8)
@pytest.mark.parametrize("renorm", [True, False])
def test_substitution_properties_and_brute_force(renorm):
    rng = np.random.default_rng(12)
    N, M, k, d = 10, 13, 3, 24
    h, w = rng.standard_normal((M, d)), rng.standard_normal((N, d)) * 0.4
    g, ids, tw = O.route(h, w, None, k, renorm)
    s = O.aggregate_scores(g)
    for B in range(k, N + 1):
        S = O.shortlist(s, B)
        sid, sw = O.restrict_substitution(g, S, k, renorm)
        for t in range(M):
            sel = sid[t].tolist()
            assert len(set(sel)) == k and set(sel) <= set(S)            # exactly k experts, all in S
            assert set(sel) >= set(ids[t].tolist()) & set(S)            # natural picks inside S survive
            assert set(sel) == best_subset(g[t], k, candidates=S)       # enumeration of k-subsets of S
            assert all(g[t, a] >= g[t, b] for a, b in zip(sel, sel[1:]))
            if set(ids[t].tolist()) <= set(S):
                assert sel == ids[t].tolist()
                np.testing.assert_allclose(sw[t], tw[t], rtol=1e-15)
            if renorm:
                assert sw[t].sum() == pytest.approx(1.0, rel=1e-14)
                np.testing.assert_allclose(sw[t], g[t, sel] / g[t, sel].sum(), rtol=1e-14)
            else:
                np.testing.assert_array_equal(sw[t], g[t, sel])
    with pytest.raises(ValueError):
        O.restrict_substitution(g, O.shortlist(s, k - 1), k, renorm)


# ------------------------------------------------------------------ B = N and union-covered budgets
@pytest.mark.parametrize("renorm", [True, False])
def test_full_budget_reproduces_unbudgeted_routing(renorm):
    rng = np.random.default_rng(21)
    N, M, k, d = 9, 11, 3, 16
    h, w = rng.standard_normal((M, d)), rng.standard_normal((N, d)) * 0.5
    g, ids, tw = O.route(h, w, None, k, renorm)
    for policy in (O.TRUNCATE, O.SUBSTITUTE):
        r = O.budget(g, ids, tw, N, policy, k, renorm)
        assert np.array_equal(r["tok_ids"], ids)
        np.testing.assert_array_equal(r["tok_w"], tw)


def test_budget_covering_union_reproduces_unbudgeted_routing():
    """If the shortlist contains the union of Eq. (3), both policies equal the natural routing."""
    rng = np.random.default_rng(22)
    N, M, k, d = 16, 12, 2, 16
    h, w = rng.standard_normal((M, d)), rng.standard_normal((N, d)) * 0.5
    b = 3.0 * np.log(1.0 / np.arange(1, N + 1))
    g, ids, tw = O.route(h, w, b, k, True)
    union = O.expert_union(ids)
    s = O.aggregate_scores(g)
    hits = 0
    for B in range(len(union), N + 1):
        S = O.shortlist(s, B)
        if not set(union) <= set(S):
            continue
        hits += 1
        for policy in (O.TRUNCATE, O.SUBSTITUTE):
            r = O.budget(g, ids, tw, B, policy, k, True)
            assert np.array_equal(r["tok_ids"], ids)
            np.testing.assert_allclose(r["tok_w"], tw, rtol=1e-15)
    assert hits >= 1


def test_union_sized_budget_can_miss_a_union_member():
    """B >= |union| alone does not guarantee S contains the union: Eq. (5) sums the full softmax,
    so an expert that is runner-up for every token can outscore one that is top-1 for a single token."""
    # 3 tokens, 4 experts, k=1.  Expert 3 is second for all tokens; expert 2 wins only token 2.
    g = np.array([[0.60, 0.02, 0.03, 0.35],
                  [0.02, 0.60, 0.03, 0.35],
                  [0.05, 0.05, 0.46, 0.44]])
    ids = np.array([[O.top_k(g[t], 1)[0]] for t in range(3)])
    assert O.expert_union(ids) == [0, 1, 2]
    s = O.aggregate_scores(g)
    S = O.shortlist(s, 3)
    assert set(S) == {3, 0, 1} and 2 not in S
    tid, _ = O.restrict_truncation(ids, np.ones((3, 1)), S)
    assert tid[:, 0].tolist() == [0, 1, -1]
    sid, _ = O.restrict_substitution(g, S, 1, True)
    assert sid[:, 0].tolist() == [0, 1, 3]


def test_expert_relabelling_equivariance():
    rng = np.random.default_rng(31)
    N, M, k, d, B = 10, 9, 3, 16, 5
    h, w = rng.standard_normal((M, d)), rng.standard_normal((N, d)) * 0.5
    p = rng.permutation(N)                       # new id p[i] for old expert i
    w2 = np.empty_like(w)
    w2[p] = w
    g, ids, tw = O.route(h, w, None, k, True)
    g2, ids2, tw2 = O.route(h, w2, None, k, True)
    assert np.array_equal(p[ids], ids2)
    for policy in (O.TRUNCATE, O.SUBSTITUTE):
        r = O.budget(g, ids, tw, B, policy, k, True)
        r2 = O.budget(g2, ids2, tw2, B, policy, k, True)
        assert np.array_equal(p[r["S"]], r2["S"])
        a = np.where(r["tok_ids"] >= 0, p[np.maximum(r["tok_ids"], 0)], -1)
        assert np.array_equal(a, r2["tok_ids"])
        np.testing.assert_allclose(r["tok_w"], r2["tok_w"], rtol=1e-13)


# ------------------------------------------------------------------ segments / permutation
@pytest.mark.parametrize("policy", [O.TRUNCATE, O.SUBSTITUTE])
def test_segments_are_a_stable_grouping(policy):
    rng = np.random.default_rng(41)
    N, M, k, d, B = 12, 19, 3, 16, 6
    h, w = rng.standard_normal((M, d)), rng.standard_normal((N, d)) * 0.5
    g, ids, tw = O.route(h, w, None, k, True)
    r = O.budget(g, ids, tw, B, policy, k, True)
    tok_ids, perm, seg_off, seg_expert = r["tok_ids"], r["perm"], r["seg_off"], r["seg_expert"]
    surviving = [i for i in range(M * k) if tok_ids.ravel()[i] >= 0]
    assert sorted(perm.tolist()) == surviving                       # a permutation of the surviving pairs
    assert seg_expert.tolist() == sorted(r["S"].tolist())
    assert seg_off[0] == 0 and seg_off[-1] == len(surviving)
    hist = np.bincount(tok_ids.ravel()[tok_ids.ravel() >= 0], minlength=N)
    for i, e in enumerate(seg_expert):
        seg = perm[seg_off[i]:seg_off[i + 1]]
        assert len(seg) == hist[e]
        assert all(tok_ids.ravel()[p] == e for p in seg)
        toks = [p // k for p in seg]
        assert toks == sorted(toks) and len(set(toks)) == len(toks)
    if policy == O.SUBSTITUTE:
        assert len(surviving) == M * k


def test_external_shortlist_is_used_verbatim():
    rng = np.random.default_rng(51)
    N, M, k, d = 8, 6, 2, 16
    h, w = rng.standard_normal((M, d)), rng.standard_normal((N, d)) * 0.5
    g, ids, tw = O.route(h, w, None, k, True)
    ext = [7, 1, 4]
    r = O.budget(g, ids, tw, 3, O.SUBSTITUTE, k, True, ext_shortlist=ext)
    assert r["S"].tolist() == ext and set(r["tok_ids"].ravel().tolist()) <= set(ext)
    assert r["seg_expert"].tolist() == [1, 4, 7]


def test_decision_margins_small_case():
    g = np.array([[0.5, 0.3, 0.15, 0.05], [0.1, 0.2, 0.3, 0.4]])
    m = O.decision_margins(g, B=2, k=2, S=[0, 1, 3])
    assert m["topk"] == pytest.approx(0.1)          # token 1: 0.4, 0.3, 0.2
    assert m["score"] == pytest.approx(0.05)        # scores .6 .5 .45 .45 -> top3 gaps .1, .05
    assert m["sub"] == pytest.approx(0.1)           # token 1 within S: .4 .2 .1 -> .2, .1 ; token 0: .5 .3 .05 -> .2, .25


# ------------------------------------------------------------------------------------- sigmoid gate
def test_sigmoid_gate_matches_library_sigmoid_and_keeps_the_selection():
    import torch
    rng = np.random.default_rng(12)
    logits = rng.standard_normal((9, 7)) * 3.0
    g = O.routing_probs(logits, O.SIGMOID)
    np.testing.assert_allclose(g, torch.sigmoid(torch.from_numpy(logits)).numpy(), rtol=1e-14)
    assert np.all((g > 0) & (g < 1)) and not np.allclose(g.sum(axis=1), 1.0)     # no normalisation across experts
    # both gates are increasing in the logit: the natural top-k sets and their order are the same
    gs = O.routing_probs(logits, O.SOFTMAX)
    for t in range(9):
        assert O.top_k(g[t], 3) == O.top_k(gs[t], 3) == list(np.argsort(-logits[t], kind="stable")[:3])
    # renormalised mixing weights: sigmoid scores over their sum
    sel = O.top_k(g[0], 3)
    w = O.mixing_weights(g[0], sel, True)
    np.testing.assert_allclose(w, g[0][sel] / g[0][sel].sum(), rtol=1e-15)
    with pytest.raises(ValueError):
        O.routing_probs(logits, "tanh")


def test_sigmoid_gate_changes_the_aggregate_ranking_but_not_the_full_budget_layer():
    rng = np.random.default_rng(13)
    M, d, N, k, F = 14, 8, 6, 2, 4
    W = dict(w_router=rng.standard_normal((N, d)), b_router=None, w_gate=rng.standard_normal((N, F, d)) * 0.3,
             w_up=rng.standard_normal((N, F, d)) * 0.3, w_down=rng.standard_normal((N, d, F)) * 0.3)
    h = rng.standard_normal((M, d))
    full = O.unbudgeted_forward(h, W, k, True, gate=O.SIGMOID)
    r = O.layer_forward(h, W, k, True, N, O.SUBSTITUTE, gate=O.SIGMOID)
    np.testing.assert_allclose(r["out"], full, rtol=1e-13, atol=1e-15)
    # Eq. (5) on sigmoid scores: the column sums of the gate values
    np.testing.assert_allclose(r["scores"], O.routing_probs(O.router_logits(h, W["w_router"]), O.SIGMOID).sum(axis=0),
                               rtol=1e-13)
    # one hot logit far above the rest: softmax gives it all the mass, sigmoid leaves the others near 1/2
    z = np.array([[20.0, 0.1, 0.0, -0.1]])
    assert O.routing_probs(z, O.SOFTMAX)[0, 1] < 1e-8 and abs(O.routing_probs(z, O.SIGMOID)[0, 1] - 0.525) < 1e-3


# ------------------------------------------------------------------------- softmax underflow, zero mass
def test_logits_hundreds_apart_underflow_to_exact_zeros_and_zero_mass_renormalises_to_nan():
    """Max-subtracted fp64 softmax: experts more than 745 below the row maximum get probability exactly 0, ties
    among them go to the lowest id, and a substitution set that holds only such experts has renormalised
    weights 0/0 = NaN (raw weights are 0)."""
    logits = np.array([[0.0, -10.0, -800.0, -900.0, -1000.0],
                       [-2000.0, 3.0, 1.0, -3000.0, 2.0]])
    g = O.routing_probs(logits, O.SOFTMAX)
    assert g[0, 2] == g[0, 3] == g[0, 4] == 0.0 and g[0, 0] > 0.9999 and 0 < g[0, 1] < 1e-4
    assert g[1, 0] == g[1, 3] == 0.0
    np.testing.assert_allclose(g.sum(axis=1), 1.0, rtol=1e-15)
    assert O.top_k(g[0], 4) == [0, 1, 2, 3]                     # zeros tie: lowest ids first
    S = [2, 3, 4]                                              # a shortlist without token 0's own experts
    ids, w = O.restrict_substitution(g, S, 2, True)
    assert list(ids[0]) == [2, 3] and np.all(np.isnan(w[0]))    # zero mass: 0/0
    assert list(ids[1]) == [4, 2] and np.all(np.isfinite(w[1]))     # descending probability
    np.testing.assert_allclose(w[1], g[1][[4, 2]] / (g[1, 2] + g[1, 4]), rtol=1e-15)
    ids_raw, w_raw = O.restrict_substitution(g, S, 2, False)
    assert list(ids_raw[0]) == [2, 3] and np.all(w_raw[0] == 0.0)
    # truncation never meets zero mass: its weights are those of the natural top-k, which holds the row maximum
    nat = O.top_k(g[0], 2)
    assert np.all(np.isfinite(O.mixing_weights(g[0], nat, True)))
