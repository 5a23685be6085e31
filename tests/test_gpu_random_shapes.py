"""GPU parity on seeded random layer shapes: every combination of kernel variant (LDS-tiled or direct passes,
self-derived or grouped segments, K-split down pass, pieces of long segments), dtype, gate, policy and budget
that a fixed seed reaches, each compared with the CPU oracle like the hand-picked cases."""
import numpy as np
import pytest
import torch

from oracle import moespec_oracle as O
from paper_2602_16052_amd import binding as mb
from paper_2602_16052_amd import workloads as wl

from gpu_common import (assert_out_close, assert_routing_equal, desc_of, oracle_weights, out_to_numpy, to_device,
                        upload_weights)

pytestmark = pytest.mark.gpu

N_CASES = 28


def random_case(i: int):
    """Shape i of the family: sizes small enough for the oracle, spread over the limits that select code paths."""
    r = np.random.default_rng(1000 + i)
    dtype = "bf16" if r.random() < 0.8 else "f32"
    mult = 32 if dtype == "bf16" else 4
    pick = lambda choices: int(choices[r.integers(len(choices))])
    if dtype == "bf16":
        d = pick([32, 64, 96, 128, 128, 256, 256, 384, 160])
        F = pick([32, 64, 128, 128, 256, 384, 192, 1024, 4096 if d <= 128 else 128])
    else:
        d, F = mult * int(r.integers(1, 30)), mult * int(r.integers(1, 30))
    N = pick([1, 2, 3, 5, 8, 16, 17, 40, 64, 130, 300])
    k = int(min(N, pick([1, 1, 2, 2, 3, 4, 6, 8, 17])))
    M = pick([1, 2, 15, 16, 17, 31, 64, 65, 127, 128, 129, 200, 260, 700, 1100])
    if M * k * max(d, F) > 6e7:       # keep the oracle and the buffers small
        M = max(1, int(6e7 // (k * max(d, F))))
    alpha = float(r.choice([0.0, 0.3, 1.0, 2.0]))
    renorm = bool(r.integers(2))
    gate = "sigmoid" if r.random() < 0.25 else "softmax"
    budgets = sorted({int(b) for b in (k, N, max(k, N // 2), int(r.integers(1, N + 1)))})
    return wl.small_config(f"rand{i}", dtype, d=d, n_experts=N, top_k=k, d_ff=F, M=M, budgets=tuple(budgets),
                           bias_alpha=alpha, renorm=renorm, seed=50 + i, gate=gate)


@pytest.mark.parametrize("i", range(N_CASES))
def test_random_shape_parity(i):
    cfg = random_case(i)
    print(f"case {i}: dtype={cfg.dtype} d={cfg.d} N={cfg.n_experts} k={cfg.top_k} F={cfg.d_ff} M={cfg.M} "
          f"budgets={cfg.budgets} renorm={cfg.renorm} gate={cfg.gate}", flush=True)
    h, W = wl.hidden_states(cfg), wl.layer_weights(cfg)
    desc = desc_of(cfg)
    h_d, W_d, ws = to_device(h), upload_weights(W), mb.alloc_workspace(desc, cfg.M)
    h_o, W_o = wl.as_f32(h), oracle_weights(W)
    for B in cfg.budgets:
        for policy in (mb.TRUNCATE, mb.SUBSTITUTE):
            if policy == mb.SUBSTITUTE and B < cfg.top_k:
                continue
            print(f"  B={B} policy={policy}", flush=True)
            out, taps = mb.moespec_layer_forward(desc, W_d, h_d, B, policy, ws, taps=True)
            torch.cuda.synchronize()
            ref = O.layer_forward(h_o, W_o, cfg.top_k, cfg.renorm, B, policy, gate=cfg.gate)
            assert_routing_equal(taps, ref, B)
            assert_out_close(out_to_numpy(out), ref["out"], cfg.dtype)
            out_plain = mb.moespec_layer_forward(desc, W_d, h_d, B, policy, ws)
            torch.cuda.synchronize()
            assert torch.equal(out_plain, out)
