"""moespec_layer_forward_static - the fused layer call on the library's own fixed scratch array, for callers that
cannot allocate - against moespec_layer_forward with a caller-owned workspace: same kernels, so the outputs must be
equal bit for bit (which also puts them within the parity tolerance of the oracle that the workspace call is
tested against).  Two calls in a row on the shared array, the second on a smaller tree, then a different layer
shape: nothing a call leaves behind in the array may leak into the next one.  The static call itself must not
allocate device memory."""
import numpy as np
import pytest
import torch

from oracle import moespec_oracle as O
from paper_2602_16052_amd import binding as mb
from paper_2602_16052_amd import workloads as wl

from gpu_common import assert_out_close, desc_of, oracle_weights, out_to_numpy, to_device, upload_weights

pytestmark = pytest.mark.gpu


def run_pair(cfg, B, policy, M=None, residual=False):
    """The same layer through both entry points on the first M tokens of the workload."""
    h, W = wl.hidden_states(cfg), wl.layer_weights(cfg)
    M = cfg.M if M is None else M
    desc = desc_of(cfg)
    h_d, W_d = to_device(h[:M].copy()), upload_weights(W)
    res = torch.randn(M, cfg.d, generator=torch.Generator().manual_seed(7)).to(h_d.dtype).cuda() if residual else None
    want = mb.moespec_layer_forward(desc, W_d, h_d, B, policy, mb.alloc_workspace(desc, M), residual=res)
    out = torch.full_like(want, float("nan"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    mb.moespec_layer_forward_static(desc, W_d, h_d, B, policy, out, residual=res)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before, "the static-scratch call must not allocate through torch"
    assert torch.equal(out, want), f"{cfg.name} M={M} B={B} policy={policy}: static-scratch output differs"
    return h[:M], W, out


def test_two_calls_in_a_row_second_one_smaller_match_the_workspace_call():
    big = wl.small_config("na_big", "bf16", d=256, n_experts=16, top_k=4, d_ff=384, M=150, budgets=(9,), bias_alpha=0.8)
    h, W, out = run_pair(big, 9, mb.SUBSTITUTE)
    ref = O.layer_forward(wl.as_f32(h), oracle_weights(W), big.top_k, big.renorm, 9, O.SUBSTITUTE)
    assert_out_close(out_to_numpy(out), ref["out"], big.dtype)
    # second call: smaller tree on the same array, which still holds the first call's tables and counters
    h, W, out = run_pair(big, 5, mb.TRUNCATE, M=37)
    ref = O.layer_forward(wl.as_f32(h), oracle_weights(W), big.top_k, big.renorm, 5, O.TRUNCATE)
    assert_out_close(out_to_numpy(out), ref["out"], big.dtype)
    # and other shapes / dtypes / the residual afterwards
    run_pair(wl.small_config("na_odd", "bf16", d=96, n_experts=8, top_k=1, d_ff=160, M=21, renorm=False), 3, mb.TRUNCATE)
    run_pair(wl.CONFIGS["tiny_f32"], 4, mb.SUBSTITUTE, residual=True)
    run_pair(big, 16, mb.SUBSTITUTE, M=1)


def test_benchmark_shape_fits_and_matches():
    cfg = wl.CONFIGS["olmoe_m63"]
    run_pair(cfg, 32, mb.SUBSTITUTE)
    run_pair(cfg, 16, mb.TRUNCATE, M=20)


def test_oversized_layer_is_rejected_with_a_clear_error():
    cfg = wl.CONFIGS["olmoe_m511"]
    desc = desc_of(cfg)
    assert mb.workspace_bytes(desc, cfg.M) > mb.STATIC_SCRATCH_BYTES
    z = torch.zeros(8, dtype=torch.bfloat16, device="cuda")   # never dereferenced: the size check comes first
    fake = dict(w_router=torch.zeros(cfg.n_experts * cfg.d, dtype=torch.bfloat16, device="cuda"))
    cd = desc.c()
    w = mb.Weights(fake["w_router"].data_ptr(), None, z.data_ptr(), z.data_ptr(), z.data_ptr())
    import ctypes
    st = mb.load_library().moespec_layer_forward_static(ctypes.byref(cd), ctypes.byref(w), z.data_ptr(), cfg.M, 32,
                                                        mb.SUBSTITUTE, None, None, z.data_ptr(), None)
    assert st == mb.ERR_WORKSPACE_TOO_SMALL and "workspace" in mb.status_string(st)
