"""Pins for the oracle's expert maths and the end-to-end layer (CPU only)."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import moespec_oracle as O


def rand_layer(seed, N, d, Fdim, M, scale=0.3):
    rng = np.random.default_rng(seed)
    W = dict(w_router=rng.standard_normal((N, d)) * scale, b_router=rng.standard_normal(N) * 0.5,
             w_gate=rng.standard_normal((N, Fdim, d)) * scale, w_up=rng.standard_normal((N, Fdim, d)) * scale,
             w_down=rng.standard_normal((N, d, Fdim)) * scale)
    return rng.standard_normal((M, d)), W


def test_silu_closed_forms():
    assert O.silu(0.0) == 0.0
    assert O.silu(math.log(3.0)) == pytest.approx(0.75 * math.log(3.0), rel=1e-15)
    assert O.silu(-math.log(3.0)) == pytest.approx(-0.25 * math.log(3.0), rel=1e-15)
    z = np.linspace(-6, 6, 25)
    np.testing.assert_allclose(O.silu(z), F.silu(torch.from_numpy(z)).numpy(), rtol=1e-14, atol=1e-16)


def test_single_expert_is_a_dense_swiglu_mlp():
    """N = k = B = 1: the layer is one dense MLP; compare with torch's own ops."""
    h, W = rand_layer(0, 1, 24, 40, 7)
    for policy in (O.TRUNCATE, O.SUBSTITUTE):
        r = O.layer_forward(h, W, 1, True, 1, policy)
        x = torch.from_numpy(h)
        want = (F.silu(x @ torch.from_numpy(W["w_gate"][0]).T) * (x @ torch.from_numpy(W["w_up"][0]).T)) \
            @ torch.from_numpy(W["w_down"][0]).T
        np.testing.assert_allclose(r["out"], want.numpy(), rtol=1e-12, atol=1e-13)
        np.testing.assert_array_equal(r["tok_w"], 1.0)


def test_all_experts_raw_weights_is_the_dense_mixture():
    """N = k = B without renormalisation: out_t = sum_i g_i(h_t) E_i(h_t), with plain matmuls."""
    N, d, Fdim, M = 5, 16, 24, 6
    h, W = rand_layer(1, N, d, Fdim, M)
    r = O.layer_forward(h, W, N, False, N, O.SUBSTITUTE)
    x = torch.from_numpy(h)
    g = torch.softmax(x @ torch.from_numpy(W["w_router"]).T + torch.from_numpy(W["b_router"]), dim=1)
    gate = torch.einsum("td,nfd->tnf", x, torch.from_numpy(W["w_gate"]))
    up = torch.einsum("td,nfd->tnf", x, torch.from_numpy(W["w_up"]))
    y = torch.einsum("tnf,ndf->tnd", F.silu(gate) * up, torch.from_numpy(W["w_down"]))
    want = torch.einsum("tn,tnd->td", g, y)
    np.testing.assert_allclose(r["out"], want.numpy(), rtol=1e-11, atol=1e-13)
    # Truncation with the full budget is the same thing (Eq. 2).
    r2 = O.layer_forward(h, W, N, False, N, O.TRUNCATE)
    np.testing.assert_allclose(r2["out"], r["out"], rtol=1e-13, atol=1e-15)


@pytest.mark.parametrize("policy", [O.TRUNCATE, O.SUBSTITUTE])
@pytest.mark.parametrize("renorm", [True, False])
def test_layer_against_masked_dense_mixture(policy, renorm):
    """out_t = sum_i c[t,i] E_i(h_t) where c scatters the restricted weights; E_i by torch einsum."""
    N, d, Fdim, M, k, B = 8, 16, 24, 9, 3, 4
    h, W = rand_layer(2, N, d, Fdim, M)
    r = O.layer_forward(h, W, k, renorm, B, policy)
    c = np.zeros((M, N))
    for t in range(M):
        for j in range(k):
            if r["tok_ids"][t, j] >= 0:
                c[t, r["tok_ids"][t, j]] += r["tok_w"][t, j]
    x = torch.from_numpy(h)
    gate = torch.einsum("td,nfd->tnf", x, torch.from_numpy(W["w_gate"]))
    up = torch.einsum("td,nfd->tnf", x, torch.from_numpy(W["w_up"]))
    y = torch.einsum("tnf,ndf->tnd", F.silu(gate) * up, torch.from_numpy(W["w_down"]))
    want = torch.einsum("tn,tnd->td", torch.from_numpy(c), y)
    np.testing.assert_allclose(r["out"], want.numpy(), rtol=1e-11, atol=1e-13)
    assert set(r["loaded"]) <= set(r["S"].tolist()) and len(r["loaded"]) <= B


def test_full_budget_equals_standard_moe_output():
    """B = N: both policies give Eq. (2) bit for bit."""
    N, d, Fdim, M, k = 7, 16, 24, 8, 2
    h, W = rand_layer(3, N, d, Fdim, M)
    ref = O.unbudgeted_forward(h, W, k, True)
    for policy in (O.TRUNCATE, O.SUBSTITUTE):
        r = O.layer_forward(h, W, k, True, N, policy)
        np.testing.assert_array_equal(r["out"], ref)


def test_output_is_linear_in_mixing_weights_and_zero_for_dropped_tokens():
    N, d, Fdim, M, k = 6, 16, 24, 5, 2
    h, W = rand_layer(4, N, d, Fdim, M)
    ids = np.array([[0, 1], [2, -1], [-1, -1], [3, 4], [-1, 5]])
    w = np.random.default_rng(0).random((M, k))
    out1 = O.combine(h, ids, w, W["w_gate"], W["w_up"], W["w_down"])
    out2 = O.combine(h, ids, 2.5 * w, W["w_gate"], W["w_up"], W["w_down"])
    np.testing.assert_allclose(out2, 2.5 * out1, rtol=1e-14)
    assert np.all(out1[2] == 0.0)
    e5 = O.expert(h[4], W["w_gate"][5], W["w_up"][5], W["w_down"][5])
    np.testing.assert_allclose(out1[4], w[4, 1] * e5, rtol=1e-14)
    # sampled evaluation leaves the other rows untouched and agrees on the sampled ones
    part = O.combine(h, ids, w, W["w_gate"], W["w_up"], W["w_down"], tokens=[0, 3])
    np.testing.assert_array_equal(part[[0, 3]], out1[[0, 3]])
    assert np.all(part[[1, 2, 4]] == 0.0)


def test_expert_operand_orientation():
    """A rectangular expert (d != F) with one-hot weights: catches a transposed operand."""
    d, Fdim = 3, 2
    wg = np.zeros((Fdim, d)); wu = np.zeros((Fdim, d)); wd = np.zeros((d, Fdim))
    wg[1, 2] = math.log(3.0)      # gate_1 = ln3 * x_2
    wu[1, 0] = 2.0                # up_1   = 2 x_0
    wd[1, 1] = 5.0                # y_1    = 5 a_1
    x = np.array([7.0, 11.0, 1.0])
    y = O.expert(x, wg, wu, wd)
    np.testing.assert_allclose(y, [0.0, 5.0 * (0.75 * math.log(3.0)) * 14.0, 0.0], rtol=1e-15)


def test_layer_stack_adds_the_residual():
    N, d, Fdim, M, k, B = 4, 16, 24, 5, 2, 3
    h, W0 = rand_layer(5, N, d, Fdim, M)
    _, W1 = rand_layer(6, N, d, Fdim, M)
    hL, res = O.layer_stack(h, [W0, W1], k, True, B, O.SUBSTITUTE)
    h1 = h + O.layer_forward(h, W0, k, True, B, O.SUBSTITUTE)["out"]
    h2 = h1 + O.layer_forward(h1, W1, k, True, B, O.SUBSTITUTE)["out"]
    np.testing.assert_array_equal(hL, h2)
    assert len(res) == 2


def test_rms_scale_gives_unit_rms_rows_and_matches_torch():
    rng = np.random.default_rng(3)
    h = rng.standard_normal((7, 48)) * np.array([[0.01], [1.0], [30.0], [2.0], [5.0], [0.3], [1e3]])
    x = O.rms_scale(h)
    np.testing.assert_allclose(np.sqrt(np.mean(x * x, axis=1)), 1.0, rtol=1e-14)
    ht = torch.from_numpy(h)
    np.testing.assert_allclose(x, (ht / ht.pow(2).mean(dim=1, keepdim=True).sqrt()).numpy(), rtol=1e-14)
    # scale invariance: a row and its multiple normalise to the same vector
    np.testing.assert_allclose(O.rms_scale(h[1:2] * 37.5), x[1:2], rtol=1e-14)


def test_layer_stack_with_pre_norm_feeds_scaled_rows_and_keeps_the_residual_unscaled():
    N, d, Fdim, M, k, B = 4, 16, 24, 5, 2, 3
    h, W0 = rand_layer(7, N, d, Fdim, M)
    _, W1 = rand_layer(8, N, d, Fdim, M)
    h = h * 3.0
    hL, res = O.layer_stack(h, [W0, W1], k, True, B, O.TRUNCATE, pre_norm=True)
    x0 = O.rms_scale(h)
    h1 = h + O.layer_forward(x0, W0, k, True, B, O.TRUNCATE)["out"]
    x1 = O.rms_scale(h1)
    h2 = h1 + O.layer_forward(x1, W1, k, True, B, O.TRUNCATE)["out"]
    np.testing.assert_array_equal(hL, h2)
    np.testing.assert_array_equal(res[0]["x"], x0)
    np.testing.assert_array_equal(res[1]["x"], x1)
    # the storage hook is applied to the MoE input and to the running state
    rounded = lambda a: np.round(a * 64.0) / 64.0
    hS, resS = O.layer_stack(h, [W0], k, True, B, O.TRUNCATE, store_fn=rounded, pre_norm=True)
    np.testing.assert_array_equal(resS[0]["x"], rounded(x0))
    np.testing.assert_array_equal(hS, rounded(h + O.layer_forward(rounded(x0), W0, k, True, B, O.TRUNCATE)["out"]))
