"""Pins of the oracle's analysis functions: static ranking (Eq. (4)), the coverage curve (Section 4.6)
and the reconstruction error (Section 4.5), against library routines, closed forms and brute force."""
import itertools

import numpy as np
import pytest

from oracle import moespec_oracle as O


def test_calibration_counts_match_a_histogram_and_accumulate_over_batches():
    rng = np.random.default_rng(3)
    N, k = 11, 3
    batches = [np.stack([rng.permutation(N)[:k] for _ in range(m)]).astype(np.int32) for m in (7, 1, 19)]
    c = None
    for b in batches:
        c = O.calibration_counts(b, N, c)
    want = np.bincount(np.concatenate([b.ravel() for b in batches]), minlength=N)
    assert c.dtype == np.int64 and np.array_equal(c, want)
    assert int(c.sum()) == sum(b.shape[0] for b in batches) * k      # every token selects exactly k experts
    # one token: the count vector is the indicator of its top-k set (Eq. (4) with a single h)
    one = O.calibration_counts(np.array([[4, 0, 9]]), N)
    assert one.tolist() == [1, 0, 0, 0, 1, 0, 0, 0, 0, 1, 0]


def test_calibration_counts_use_the_natural_top_k_of_the_router():
    """Eq. (4) counts membership in T_k(h): feed the oracle's own routing and compare with a brute-force count."""
    rng = np.random.default_rng(5)
    M, d, N, k = 23, 8, 6, 2
    h, w = rng.standard_normal((M, d)), rng.standard_normal((N, d))
    g, ids, _ = O.route(h, w, None, k, True)
    c = O.calibration_counts(ids, N)
    brute = [sum(1 for t in range(M) if i in set(np.argsort(-g[t], kind="stable")[:k].tolist())) for i in range(N)]
    assert c.tolist() == brute


def test_static_shortlist_is_the_brute_force_best_subset_with_ties_to_the_lowest_id():
    counts = [5, 9, 5, 0, 9, 2, 5]
    assert O.static_shortlist(counts, 3) == [1, 4, 0]
    assert O.static_shortlist(counts, 7) == [1, 4, 0, 2, 6, 5, 3]
    for B in range(1, len(counts) + 1):
        S = O.static_shortlist(counts, B)
        best = max(sum(counts[i] for i in sub) for sub in itertools.combinations(range(len(counts)), B))
        assert sum(counts[i] for i in S) == best and len(set(S)) == B
    # equal counts everywhere: the first B ids
    assert O.static_shortlist([3] * 6, 4) == [0, 1, 2, 3]


def test_coverage_curve_closed_forms():
    # geometric scores: closed-form partial sums
    s = np.array([2.0 ** -(i + 1) for i in range(10)])
    curve = O.coverage_curve(s)
    want = np.array([(1 - 2.0 ** -(B)) / (1 - 2.0 ** -10) for B in range(1, 11)])
    np.testing.assert_allclose(curve, want, rtol=1e-15)
    # permuting the experts does not change the curve; it is monotone and ends at 1
    perm = np.random.default_rng(0).permutation(10)
    np.testing.assert_allclose(O.coverage_curve(s[perm]), curve, rtol=1e-15)
    assert np.all(np.diff(curve) > 0) and curve[-1] == pytest.approx(1.0, abs=1e-15)
    # uniform scores: B / N
    np.testing.assert_allclose(O.coverage_curve(np.full(8, 0.7)), np.arange(1, 9) / 8, rtol=1e-15)


def test_coverage_curve_agrees_with_coverage_of_the_shortlist():
    rng = np.random.default_rng(9)
    g = rng.dirichlet(np.ones(12) * 0.3, size=31)
    s = O.aggregate_scores(g)
    curve = O.coverage_curve(s)
    for B in (1, 5, 12):
        assert curve[B - 1] == pytest.approx(O.coverage(s, O.shortlist(s, B)), rel=1e-14)
        # rows of g sum to one, so the total mass is M and the share is the mean shortlisted probability
        assert curve[B - 1] == pytest.approx(np.mean(g[:, O.shortlist(s, B)].sum(axis=1)), rel=1e-12)


def test_reconstruction_error_special_cases():
    rng = np.random.default_rng(1)
    full = rng.standard_normal((9, 16))
    assert O.reconstruction_error(full, full) == 0.0
    assert O.reconstruction_error(np.zeros_like(full), full) == pytest.approx(1.0, rel=1e-15)
    assert O.reconstruction_error(-full, full) == pytest.approx(4.0, rel=1e-15)
    assert O.reconstruction_error(1.5 * full, full) == pytest.approx(0.25, rel=1e-14)
    other = rng.standard_normal((9, 16))
    want = np.linalg.norm(other - full) ** 2 / np.linalg.norm(full) ** 2
    assert O.reconstruction_error(other, full) == pytest.approx(want, rel=1e-13)
    # not symmetric: the denominator is the full output
    assert O.reconstruction_error(full, other) == pytest.approx(np.linalg.norm(other - full) ** 2 /
                                                                np.linalg.norm(other) ** 2, rel=1e-13)


def test_reconstruction_error_of_the_budgeted_layer_falls_to_zero_at_full_budget():
    rng = np.random.default_rng(2)
    M, d, N, k, F = 12, 8, 6, 2, 4
    W = dict(w_router=rng.standard_normal((N, d)), b_router=None, w_gate=rng.standard_normal((N, F, d)) * 0.3,
             w_up=rng.standard_normal((N, F, d)) * 0.3, w_down=rng.standard_normal((N, d, F)) * 0.3)
    h = rng.standard_normal((M, d))
    full = O.unbudgeted_forward(h, W, k, True)
    errs = [O.reconstruction_error(O.layer_forward(h, W, k, True, B, O.SUBSTITUTE)["out"], full) for B in (2, 4, 6)]
    assert errs[-1] == 0.0 and errs[0] > 0.0


# ------------------------------------------------------------------------------------- Eq. (6)
def _random_contributions(rng, N, M, d, k):
    """Contributions with the structure of a routed layer: every token has exactly k non-zero experts."""
    C = np.zeros((N, M, d))
    for t in range(M):
        for i in rng.permutation(N)[:k]:
            C[i, t] = rng.standard_normal(d) * rng.uniform(0.1, 2.0)
    return C


def test_oracle_ranking_orthogonal_contributions_are_picked_by_energy():
    """Experts that write to disjoint coordinates: adding expert i lowers the error by ||C_i||^2 exactly,
    so the greedy order is descending energy and the error curve is the closed form."""
    rng = np.random.default_rng(0)
    N, M = 5, 7
    C = np.zeros((N, M, N * 3))
    for i in range(N):
        C[i, :, 3 * i:3 * i + 3] = rng.standard_normal((M, 3)) * (i + 1) * (1 if i != 2 else 3.5)
    energy = np.array([np.sum(C[i] ** 2) for i in range(N)])
    S, errs = O.oracle_ranking(C, N)
    assert S == list(np.argsort(-energy, kind="stable"))
    want = 1.0 - np.cumsum(energy[S]) / energy.sum()
    np.testing.assert_allclose(errs, want, atol=1e-14)


def test_oracle_ranking_each_step_is_the_brute_force_minimiser():
    rng = np.random.default_rng(4)
    N, M, d, k = 7, 9, 6, 3
    C = _random_contributions(rng, N, M, d, k)
    gold = C.sum(axis=0)
    S, errs = O.oracle_ranking(C, N)
    assert sorted(S) == list(range(N)) and errs[-1] == pytest.approx(0.0, abs=1e-28)
    assert np.all(np.diff(errs) <= 1e-15)          # adding the best expert never increases the error
    for step in range(N):
        chosen = S[:step]
        cand = {i: np.sum((gold - C[chosen + [i]].sum(axis=0)) ** 2) for i in range(N) if i not in chosen}
        best = min(cand, key=lambda i: (cand[i], i))
        assert best == S[step]
        assert errs[step] == pytest.approx(cand[best] / np.sum(gold ** 2), rel=1e-12)


def test_oracle_ranking_prefers_complementary_over_correlated_experts():
    """Two experts with the same large contribution direction: after taking one, the other's marginal gain
    collapses and a smaller but independent expert is taken first (Section 4.5's explanation of the gap)."""
    u, v = np.array([1.0, 0.0, 0.0]), np.array([0.0, 1.0, 0.0])
    C = np.zeros((3, 1, 3))
    C[0, 0], C[1, 0], C[2, 0] = 3.0 * u, 2.9 * u - 0.0 * v, 1.0 * v
    # gold = 5.9 u + v; single-expert errors: e0 = 2.9^2 + 1, e1 = 3^2 + 1, e2 = 5.9^2  -> pick 0
    # then: {0,1}: 1 ; {0,2}: 2.9^2 -> pick 1 (here the correlated expert still helps: same sign)
    S, errs = O.oracle_ranking(C, 3)
    assert S == [0, 1, 2]
    C[1, 0] = -2.9 * u          # now expert 1 cancels expert 0: gold = 0.1 u + v
    S, errs = O.oracle_ranking(C, 3)
    # single: e0 = 2.9^2 + 1, e1 = 3^2 + 1, e2 = 0.01 -> 2 ; then {2,0}: 2.9^2, {2,1}: 3^2 -> 0 ; then 1
    assert S == [2, 0, 1]
    np.testing.assert_allclose(errs, np.array([0.01, 2.9 ** 2, 0.0]) / 1.01, atol=1e-15)


def test_oracle_ranking_ties_and_unused_experts_go_in_id_order():
    rng = np.random.default_rng(8)
    C = np.zeros((6, 4, 5))
    C[4], C[1] = rng.standard_normal((4, 5)), rng.standard_normal((4, 5)) * 0.2
    S, errs = O.oracle_ranking(C, 6)
    assert S[:2] == [4, 1] and S[2:] == [0, 2, 3, 5]     # experts that no token uses change nothing: lowest id first
    assert errs[1] == pytest.approx(0.0, abs=1e-28) and np.all(errs[2:] == errs[1])


def test_expert_contributions_sum_to_the_unbudgeted_output_and_feed_the_ranking():
    rng = np.random.default_rng(6)
    M, d, N, k, F = 10, 8, 6, 2, 4
    W = dict(w_router=rng.standard_normal((N, d)), b_router=None, w_gate=rng.standard_normal((N, F, d)) * 0.3,
             w_up=rng.standard_normal((N, F, d)) * 0.3, w_down=rng.standard_normal((N, d, F)) * 0.3)
    h = rng.standard_normal((M, d))
    _, ids, w = O.route(h, W["w_router"], None, k, True)
    C = O.expert_contributions(h, ids, w, W["w_gate"], W["w_up"], W["w_down"], N)
    np.testing.assert_allclose(C.sum(axis=0), O.unbudgeted_forward(h, W, k, True), rtol=1e-13, atol=1e-15)
    for i in range(N):
        used = {t for t in range(M) if i in ids[t]}
        assert all((np.any(C[i, t] != 0)) == (t in used) for t in range(M))
    S, errs = O.oracle_ranking(C, N)
    # the oracle's error after B picks is never above the truncation error of the router-based shortlist of size B
    g = O.routing_probs(O.router_logits(h, W["w_router"]))
    for B in range(1, N + 1):
        Sr = O.shortlist(O.aggregate_scores(g), B)
        trunc = O.layer_forward(h, W, k, True, B, O.TRUNCATE)["out"]
        if B == 1:
            assert errs[0] <= O.reconstruction_error(trunc, C.sum(axis=0)) + 1e-12
    assert errs[-1] == pytest.approx(0.0, abs=1e-25)
