"""Helpers shared by the GPU parity tests: upload seeded workloads, call the HIP path through the
C-ABI binding, and compare with the CPU oracle."""
import numpy as np
import torch

from oracle import moespec_oracle as O
from paper_2602_16052_amd import binding as mb
from paper_2602_16052_amd import workloads as wl

TOL = {"bf16": 2e-2, "f32": 1e-5}


def desc_of(cfg) -> mb.LayerDesc:
    return mb.LayerDesc(cfg.d, cfg.n_experts, cfg.top_k, cfg.d_ff, mb.BF16 if cfg.dtype == "bf16" else mb.F32,
                        cfg.renorm, mb.GATE_SIGMOID if cfg.gate == "sigmoid" else mb.GATE_SOFTMAX)


def to_device(x: np.ndarray) -> torch.Tensor:
    """Stored tensor (float32, or uint16 bfloat16 bits) -> GPU tensor of the matching torch dtype."""
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(x).cuda()


def upload_weights(W):
    return {key: to_device(val) for key, val in W.items() if val is not None}


def oracle_weights(W):
    """float32 views of the stored weights for the oracle (bf16 bits widened exactly)."""
    return {key: (wl.as_f32(val) if val is not None else None) for key, val in W.items()}


def out_to_numpy(out: torch.Tensor) -> np.ndarray:
    return out.float().cpu().numpy().astype(np.float64)


def assert_out_close(got: np.ndarray, want: np.ndarray, dtype: str, rows=None, what="out", scale_aware=False):
    """max|got - want| <= tol, absolutely and relative to max|want|.

    ``scale_aware`` (layers whose outputs are several units large, where bf16 cannot represent a value
    to 2e-2: half an ulp is 0.0156 in [4, 8)) widens the absolute bound to tol * max(1, max|want|)."""
    if rows is not None:
        got, want = got[rows], want[rows]
    tol = TOL[dtype]
    err = float(np.max(np.abs(got - want))) if got.size else 0.0
    scale = float(np.max(np.abs(want))) if want.size else 0.0
    assert np.all(np.isfinite(got)), f"{what}: non-finite values"
    abs_tol = tol * max(1.0, scale) if scale_aware else tol
    assert err <= abs_tol, f"{what}: max|diff| {err:.3e} > {abs_tol}"
    if scale > 0:
        assert err / scale <= tol, f"{what}: max|diff|/max|oracle| {err / scale:.3e} > {tol} (scale {scale:.3e})"
    return err, scale


def assert_routing_equal(taps, ref, B):
    """Integer outputs bit-exact; float side outputs to 1e-6 relative."""
    g = lambda key: taps[key].cpu().numpy()
    assert np.array_equal(g("budget_ids")[:B], ref["S"]), "shortlist differs"
    assert np.array_equal(g("tok_ids"), ref["tok_ids"]), "restricted routing ids differ"
    assert np.array_equal(g("seg_expert")[:B], ref["seg_expert"]), "seg_expert differs"
    assert np.array_equal(g("seg_off")[:B + 1], ref["seg_off"]), "seg_off differs"
    P = int(ref["seg_off"][-1])
    assert np.array_equal(g("perm")[:P], ref["perm"]), "perm differs"
    assert np.all(g("perm")[P:] == -1)
    assert int(g("n_loaded")[0]) == len(ref["loaded"])
    np.testing.assert_allclose(g("tok_w"), ref["tok_w"], rtol=1e-6, atol=1e-12)
    np.testing.assert_allclose(g("scores"), ref["scores"], rtol=1e-12)
    np.testing.assert_allclose(g("probs"), ref["probs"], rtol=1e-11, atol=1e-300)
