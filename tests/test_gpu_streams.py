"""Calls on different HIP streams with workspaces of their own may overlap: the library keeps no state between calls
(the one exception, moespec_layer_forward_static, says so in the header).  Two streams run different layers at the
same time, many times over, and every result must equal the one from a serial run, bit for bit."""
import pytest
import torch

from paper_2602_16052_amd import binding as mb
from paper_2602_16052_amd import workloads as wl

from gpu_common import desc_of, to_device, upload_weights

pytestmark = pytest.mark.gpu


def _case(name, seed, **kw):
    cfg = wl.small_config(name, "bf16", seed=seed, **kw)
    desc = desc_of(cfg)
    return dict(cfg=cfg, desc=desc, h=to_device(wl.hidden_states(cfg)), W=upload_weights(wl.layer_weights(cfg)),
                ws=mb.alloc_workspace(desc, cfg.M))


def test_overlapping_calls_on_two_streams_match_serial_runs():
    a = _case("stream_a", 3, d=256, n_experts=64, top_k=8, d_ff=256, M=63, budgets=(32,))
    b = _case("stream_b", 4, d=128, n_experts=130, top_k=4, d_ff=384, M=200, budgets=(40,))   # dynamic LDS above 64 KB
    ref = {}
    for tag, c, B, pol in (("a", a, 32, mb.SUBSTITUTE), ("b", b, 40, mb.TRUNCATE)):
        ref[tag] = mb.moespec_layer_forward(c["desc"], c["W"], c["h"], B, pol, c["ws"]).clone()
    torch.cuda.synchronize()
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    outs_a = [torch.empty_like(ref["a"]) for _ in range(40)]
    outs_b = [torch.empty_like(ref["b"]) for _ in range(40)]
    for i in range(40):
        mb.LayerForwardCall(a["desc"], a["W"], a["h"], 32, mb.SUBSTITUTE, a["ws"], outs_a[i], stream=sa)()
        mb.LayerForwardCall(b["desc"], b["W"], b["h"], 40, mb.TRUNCATE, b["ws"], outs_b[i], stream=sb)()
    torch.cuda.synchronize()
    for i in range(40):
        assert torch.equal(outs_a[i], ref["a"]), f"stream a, call {i}"
        assert torch.equal(outs_b[i], ref["b"]), f"stream b, call {i}"
