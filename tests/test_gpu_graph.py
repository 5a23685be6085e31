"""The fused call under HIP graph capture: it allocates nothing, clears its counters with kernels (no memset
nodes) and takes the capturing stream, so a captured layer must replay to the eager result every time."""
import pytest
import torch

from paper_2602_16052_amd import binding as mb
from paper_2602_16052_amd import workloads as wl

from gpu_common import desc_of, to_device, upload_weights

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("policy", [mb.TRUNCATE, mb.SUBSTITUTE])
def test_captured_layer_replays_to_the_eager_result(policy):
    cfg = wl.small_config("graph_bf16", "bf16", d=256, n_experts=16, top_k=4, d_ff=256, M=33, budgets=(8,),
                          bias_alpha=0.8)
    desc = desc_of(cfg)
    W_d = upload_weights(wl.layer_weights(cfg))
    ws = mb.alloc_workspace(desc, cfg.M)
    inputs = [to_device(wl.hidden_states(cfg, seed=s)) for s in (0, 1, 2)]
    eager = []
    for h in inputs:
        eager.append(mb.moespec_layer_forward(desc, W_d, h, 8, policy, ws).clone())
    torch.cuda.synchronize()

    h_static = inputs[0].clone()
    out_static = torch.empty_like(eager[0])
    call = mb.LayerForwardCall
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):     # warm-up on the side stream, as graph capture requires
        call(desc, W_d, h_static, 8, policy, ws, out_static, stream=side)()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        # the call is marshalled inside the capture so that it picks up the capturing stream
        call(desc, W_d, h_static, 8, policy, ws, out_static)()
    for rep in range(3):
        for h, want in zip(inputs, eager):
            h_static.copy_(h)
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(out_static, want), f"replay {rep} differs from the eager call"
            # eager work on the same workspace between replays
            again = mb.moespec_layer_forward(desc, W_d, h, 8, policy, ws)
            torch.cuda.synchronize()
            assert torch.equal(again, want)
