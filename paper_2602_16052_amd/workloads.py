"""Seeded synthetic workloads for the budgeted MoE-layer forward.

This module only *draws inputs*: layer shapes, random tensors, the heavy-tailed
router bias and the storage rounding of those inputs.  It contains none of the
method's arithmetic (no routing, no budget, no expert math), so that the CPU
oracle and the HIP path can both be fed from it without sharing any code of
the method itself.

The five layer shapes follow the models the paper evaluates (Section 4.1 and
the model-configuration table of Appendix A: 64 experts / k=8, 128 experts /
k=8, 8 experts / k=2) and its draft-tree sizes (63 by default, 3-511 in the
sweep).  The paper's prompts and trained weights are not available; the
heavy-tailed aggregate routing it reports (Figure 2c: a few experts hold most
of the routing mass of a tree) is imitated with a per-expert router bias
``b_e = alpha * log(1 / rank_e)`` where ``rank`` is a seeded permutation of
``1..N``.

Storage formats
---------------
``"f32"`` tensors are numpy float32.  ``"bf16"`` tensors are numpy uint16
holding bfloat16 bit patterns (numpy has no bfloat16): values are drawn in
float32 and rounded once, to nearest-even; every consumer reads those bits.
``as_f32`` widens either form to float32 exactly.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, Optional, Tuple

import numpy as np

# Tensor identifiers mixed into the generator key so that every tensor has an
# independent stream for a given seed.
_TID_H, _TID_ROUTER, _TID_RANK, _TID_GATE, _TID_UP, _TID_DOWN = 1, 2, 3, 4, 5, 6


@dataclasses.dataclass(frozen=True)
class LayerConfig:
    """Shape and distribution of one synthetic MoE layer workload."""

    name: str
    dtype: str            # "f32" or "bf16": storage of h, weights and out
    d: int                # hidden size
    n_experts: int        # N
    top_k: int            # k
    d_ff: int             # expert intermediate size F
    M: int                # draft-tree tokens
    budgets: Tuple[int, ...]
    bias_alpha: float     # alpha of the Zipf-style router bias
    renorm: bool          # mixing weights renormalised over the selected set
    n_layers: int = 1
    seed: int = 0
    sigma_w: float = 0.02
    gate: str = "softmax"  # "softmax" (Eq. (1)) or "sigmoid" (independent gate per expert)

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def expert_bytes(self) -> int:
        """Bytes of one expert's three weight matrices."""
        return 3 * self.d * self.d_ff * self.elem_bytes


CONFIGS: Dict[str, LayerConfig] = {
    "tiny_f32": LayerConfig("tiny_f32", "f32", 128, 8, 2, 256, 15, (4,), 1.5, True),
    "olmoe_m63": LayerConfig("olmoe_m63", "bf16", 2048, 64, 8, 1024, 63,
                             (16, 24, 32, 48, 64), 1.5, True),
    "olmoe_m127": LayerConfig("olmoe_m127", "bf16", 2048, 64, 8, 1024, 127,
                              (16, 32, 48, 64), 1.5, True),
    "fine_m127": LayerConfig("fine_m127", "bf16", 2048, 128, 8, 768, 127,
                             (32, 48, 64, 96, 128), 1.2, False),
    "coarse_stack": LayerConfig("coarse_stack", "bf16", 4096, 8, 2, 14336, 63,
                                (2, 4, 6, 8), 1.5, True, n_layers=8),
    # larger draft trees of the paper's tree-size sweep (up to 511 nodes) on the OLMoE shape: segments of more
    # than 128 pairs, which the expert passes cut into pieces
    "olmoe_m255": LayerConfig("olmoe_m255", "bf16", 2048, 64, 8, 1024, 255, (16, 32, 64), 1.5, True),
    "olmoe_m511": LayerConfig("olmoe_m511", "bf16", 2048, 64, 8, 1024, 511, (16, 32, 64), 1.5, True),
}
CONFIG_ORDER = ("tiny_f32", "olmoe_m63", "olmoe_m127", "fine_m127", "coarse_stack")


def _rng(seed: int, tensor_id: int, layer: int = 0, part: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(seed << 20) ^ (layer << 8) ^ tensor_id, part]))


def round_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float32, exact."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def as_f32(x: np.ndarray) -> np.ndarray:
    """Widen a stored tensor (float32, or uint16 bfloat16 bits) to float32."""
    if x.dtype == np.uint16:
        return bf16_bits_to_f32(x)
    return np.asarray(x, dtype=np.float32)


def store(x_f32: np.ndarray, dtype: str) -> np.ndarray:
    """Round float32 values into the storage format ``dtype``."""
    if dtype == "bf16":
        return round_to_bf16_bits(x_f32)
    if dtype == "f32":
        return np.ascontiguousarray(x_f32, dtype=np.float32)
    raise ValueError(f"unknown dtype {dtype!r}")


def _normal(shape, sigma: float, dtype: str, seed: int, tid: int, layer: int, part: int) -> np.ndarray:
    g = _rng(seed, tid, layer, part)
    x = g.standard_normal(size=shape, dtype=np.float32)
    if sigma != 1.0:
        x *= np.float32(sigma)
    return store(x, dtype)


def hidden_states(cfg: LayerConfig, M: Optional[int] = None, seed: Optional[int] = None) -> np.ndarray:
    """Draft-tree hidden rows ``h[M, d] ~ N(0, 1)`` in the config's storage."""
    M = cfg.M if M is None else M
    seed = cfg.seed if seed is None else seed
    return _normal((M, cfg.d), 1.0, cfg.dtype, seed, _TID_H, 0, 0)


def router_bias(cfg: LayerConfig, layer: int = 0, seed: Optional[int] = None) -> np.ndarray:
    """``b_e = alpha * log(1 / rank_e)`` (float32), rank = seeded permutation of 1..N."""
    seed = cfg.seed if seed is None else seed
    rank = _rng(seed, _TID_RANK, layer, 0).permutation(cfg.n_experts) + 1
    return (cfg.bias_alpha * np.log(1.0 / rank.astype(np.float64))).astype(np.float32)


def layer_weights(cfg: LayerConfig, layer: int = 0, seed: Optional[int] = None,
                  experts: Optional[Tuple[int, ...]] = None, threads: int = 8) -> Dict[str, np.ndarray]:
    """All weights of one layer, in the config's storage format.

    Returns ``w_router[N, d]``, ``b_router[N]`` (float32), ``w_gate[N, F, d]``,
    ``w_up[N, F, d]`` and ``w_down[N, d, F]``.  Every expert matrix has a
    generator stream of its own, so ``experts=(...)`` draws only those experts
    (the other rows of the stacked arrays stay zero) with identical values.
    """
    seed = cfg.seed if seed is None else seed
    N, d, F = cfg.n_experts, cfg.d, cfg.d_ff
    np_dtype = np.uint16 if cfg.dtype == "bf16" else np.float32
    out = {
        "w_router": _normal((N, d), cfg.sigma_w, cfg.dtype, seed, _TID_ROUTER, layer, 0),
        "b_router": router_bias(cfg, layer, seed),
        "w_gate": np.zeros((N, F, d), dtype=np_dtype),
        "w_up": np.zeros((N, F, d), dtype=np_dtype),
        "w_down": np.zeros((N, d, F), dtype=np_dtype),
    }
    todo = range(N) if experts is None else experts

    def fill(job):
        e, key, tid, shape = job
        out[key][e] = _normal(shape, cfg.sigma_w, cfg.dtype, seed, tid, layer, e + 1)

    jobs = []
    for e in todo:
        jobs += [(e, "w_gate", _TID_GATE, (F, d)), (e, "w_up", _TID_UP, (F, d)),
                 (e, "w_down", _TID_DOWN, (d, F))]
    if threads > 1 and len(jobs) > 1:
        with ThreadPoolExecutor(max_workers=threads) as pool:
            list(pool.map(fill, jobs))
    else:
        for j in jobs:
            fill(j)
    return out


def small_config(name: str = "small", dtype: str = "bf16", d: int = 256, n_experts: int = 16, top_k: int = 4,
                 d_ff: int = 192, M: int = 37, budgets: Tuple[int, ...] = (8,), bias_alpha: float = 1.5,
                 renorm: bool = True, seed: int = 0, n_layers: int = 1, gate: str = "softmax") -> LayerConfig:
    """A free-form config for randomised parity cases (ragged sizes, edge shapes)."""
    return LayerConfig(name, dtype, d, n_experts, top_k, d_ff, M, tuple(budgets), bias_alpha, renorm,
                       n_layers=n_layers, seed=seed, gate=gate)
