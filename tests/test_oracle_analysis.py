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
