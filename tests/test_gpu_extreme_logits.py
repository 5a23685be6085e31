"""GPU parity when the router logits span hundreds to thousands: hidden rows scaled by up to 3000, so that
most routing probabilities underflow to exact zeros or denormals in the fp64 softmax (Eq. 1).  Routing must
stay bit-exact (zeros tie to the lowest id), outputs within tolerance relative to their scale, and a substitution
set of zero probability mass for a token must give NaN weights and a NaN output row on both sides."""
import numpy as np
import pytest
import torch

from oracle import moespec_oracle as O
from paper_2602_16052_amd import binding as mb
from paper_2602_16052_amd import workloads as wl

from gpu_common import TOL, assert_routing_equal, desc_of, oracle_weights, out_to_numpy, to_device, upload_weights

pytestmark = pytest.mark.gpu

CASES = [("bf16", 256, 64, 8, 128, 48, "softmax"),     # fused prologue, every workgroup rebuilds the table
         ("bf16", 128, 130, 4, 128, 200, "softmax"),   # fused prologue, row-wise gate kernel, ragged expert count
         ("f32", 64, 16, 2, 32, 20, "softmax"),        # staged fp32 path
         ("bf16", 256, 40, 6, 256, 130, "sigmoid"),
         ("bf16", 128, 64, 8, 128, 600, "softmax")]    # table beyond the LDS: staged budget kernel


@pytest.mark.parametrize("dtype,d,N,k,F,M,gate", CASES)
def test_underflowing_softmax_keeps_parity(dtype, d, N, k, F, M, gate):
    cfg = wl.small_config("extreme", dtype, d=d, n_experts=N, top_k=k, d_ff=F, M=M, budgets=(k, N // 2, N), seed=7,
                          gate=gate)
    scale = np.array([0.01, 1.0, 30.0, 100.0, 300.0, 1e3, 3e3], dtype=np.float32)[np.arange(M) % 7][:, None]
    h = wl.store(wl.as_f32(wl.hidden_states(cfg)) * scale, dtype)
    W = wl.layer_weights(cfg)
    desc = desc_of(cfg)
    h_d, W_d, ws = to_device(h), upload_weights(W), mb.alloc_workspace(desc, M)
    h_o, W_o = wl.as_f32(h), oracle_weights(W)
    seen_zero, seen_nan = False, False
    for B in cfg.budgets:
        for policy in (mb.TRUNCATE, mb.SUBSTITUTE):
            if policy == mb.SUBSTITUTE and B < k:
                continue
            print(f"  B={B} policy={policy}", flush=True)
            out, taps = mb.moespec_layer_forward(desc, W_d, h_d, B, policy, ws, taps=True)
            torch.cuda.synchronize()
            with np.errstate(over="ignore", invalid="ignore"):
                ref = O.layer_forward(h_o, W_o, k, cfg.renorm, B, policy, gate=gate)
            seen_zero |= bool((ref["probs"] == 0).any())
            assert_routing_equal(taps, ref, B)          # NaN weights compare equal position by position
            got, want = out_to_numpy(out), ref["out"]
            nan_rows = np.isnan(want).any(axis=1)
            assert np.array_equal(np.isnan(got).any(axis=1), nan_rows), "NaN rows differ"
            assert np.array_equal(nan_rows, np.isnan(ref["tok_w"]).any(axis=1))
            seen_nan |= bool(nan_rows.any())
            ok = ~nan_rows
            assert np.all(np.isfinite(got[ok]))
            if ok.any():
                # rows differ in scale by 3e5: each row against its own magnitude
                row_scale = np.maximum(np.max(np.abs(want[ok]), axis=1, keepdims=True), 1.0)
                assert np.max(np.abs(got[ok] - want[ok]) / row_scale) <= TOL[dtype]
    if gate == "softmax":
        assert seen_zero, "the case was meant to underflow"
    if gate == "softmax" and cfg.renorm:
        assert seen_nan, "the case was meant to reach a zero-mass substitution set"
