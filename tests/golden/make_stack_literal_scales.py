#!/usr/bin/env python3
"""Writes tests/golden/coarse_stack_literal_scales.json: how the hidden scale of the 8-layer coarse-expert stack
evolves under the recurrence exactly as the workload words it (h <- h + MoE_S(h), no scaling of the layer input),
next to the same stack with every layer input scaled to unit root-mean-square.

Everything here comes from the CPU oracle and the seeded input generator; nothing from the HIP path.  A SwiGLU expert
with N(0, 0.02) weights at d = 4096, F = 14336 is quadratic in the scale of its input (gate and up projection both
grow with it), so the literal recurrence squares the hidden scale from layer to layer until fp64 softmax saturates
and the values overflow; the numbers stored here are the evidence for that statement.

Usage: python tests/golden/make_stack_literal_scales.py   (a few minutes on 8 cores; 4 of the 63 tree tokens)."""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import moespec_oracle as O                      # noqa: E402
from paper_2602_16052_amd import workloads as wl           # noqa: E402

TOKENS, BUDGET = 4, 4


class LazyF64:
    """Per-expert fp64 view of a stacked bf16 weight tensor, widened on first use (memory only)."""

    def __init__(self, stacked):
        self._w, self._cache = stacked, {}

    def __getitem__(self, e):
        if e not in self._cache:
            self._cache[e] = wl.as_f32(self._w[e]).astype(np.float64)
        return self._cache[e]


def bf16_round(a):
    with np.errstate(over="ignore", invalid="ignore"):
        return wl.as_f32(wl.round_to_bf16_bits(np.asarray(a, dtype=np.float32)))


def run(pre_norm: bool):
    cfg = wl.CONFIGS["coarse_stack"]
    h = wl.as_f32(wl.hidden_states(cfg))[:TOKENS].astype(np.float64)
    rows = []
    for layer in range(cfg.n_layers):
        W = wl.layer_weights(cfg, layer=layer, threads=8)
        weights = dict(w_router=wl.as_f32(W["w_router"]), b_router=W["b_router"],
                       **{key: LazyF64(W[key]) for key in ("w_gate", "w_up", "w_down")})
        with np.errstate(all="ignore"):
            h_next, res = O.layer_stack(h, [weights], cfg.top_k, cfg.renorm, BUDGET, O.SUBSTITUTE,
                                        store_fn=bf16_round, pre_norm=pre_norm)
        out = res[0]["out"]
        row = dict(layer=layer, input_rms=float(np.sqrt(np.mean(h * h))),
                   moe_output_max_abs=float(np.max(np.abs(out))) if np.all(np.isfinite(out)) else None,
                   probs_finite=bool(np.all(np.isfinite(res[0]["probs"]))),
                   max_routing_prob=float(np.nanmax(res[0]["probs"])),
                   output_finite=bool(np.all(np.isfinite(out))), next_state_finite_in_bf16=bool(np.all(np.isfinite(h_next))))
        rows.append(row)
        print(("pre_norm " if pre_norm else "literal  ") + json.dumps(row), flush=True)
        if not row["next_state_finite_in_bf16"]:
            break
        h = h_next
    return rows


if __name__ == "__main__":
    data = dict(workload="coarse_stack (d=4096, N=8, k=2, F=14336), first %d tree tokens, B=%d, substitution, hidden "
                         "state stored in bf16 between layers" % (TOKENS, BUDGET),
                literal=run(False), pre_norm=run(True))
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "coarse_stack_literal_scales.json")
    with open(path, "w") as f:
        json.dump(data, f, indent=1)
    print("wrote", path)
