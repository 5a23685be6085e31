"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2602_16052_amd import binding as mb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(mb.LIB_PATH):
        from paper_2602_16052_amd import build
        build.build_library()
    return mb.load_library()


def header_functions():
    text = open(os.path.join(ROOT, "include", "moespec.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moespec_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = header_functions()
    assert set(names) == set(mb.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_status_strings(lib):
    assert mb.abi_version() == 5
    assert mb.status_string(mb.OK) == "ok"
    assert "workspace" in mb.status_string(mb.ERR_WORKSPACE_TOO_SMALL)
    assert mb.status_string(99) == "unknown status"


def D(**kw):
    base = dict(d=256, n_experts=16, top_k=4, d_ff=192 + 64, dtype=mb.BF16, renorm=True)
    base.update(kw)
    return mb.LayerDesc(**base)


def test_check_desc_and_workspace(lib):
    assert mb.check_desc(D()) == mb.OK
    assert mb.check_desc(D(dtype=7)) == mb.ERR_INVALID_ARG
    assert mb.check_desc(D(gate=mb.GATE_SIGMOID)) == mb.OK
    assert mb.check_desc(D(gate=2)) == mb.ERR_INVALID_ARG
    assert mb.check_desc(D(top_k=0)) == mb.ERR_INVALID_ARG
    assert mb.check_desc(D(top_k=17)) == mb.ERR_INVALID_ARG
    assert mb.check_desc(D(d=0)) == mb.ERR_INVALID_ARG
    assert mb.check_desc(D(d=250)) == mb.ERR_UNSUPPORTED_SHAPE
    assert mb.check_desc(D(d_ff=100)) == mb.ERR_UNSUPPORTED_SHAPE
    assert mb.check_desc(D(d_ff=100, d=132, dtype=mb.F32)) == mb.OK
    assert mb.check_desc(D(n_experts=2048)) == mb.ERR_UNSUPPORTED_SHAPE
    assert mb.check_desc(D(d=16384)) == mb.ERR_UNSUPPORTED_SHAPE
    assert lib.moespec_check_desc(None) == mb.ERR_INVALID_ARG
    w63, w127 = mb.workspace_bytes(D(), 63), mb.workspace_bytes(D(), 127)
    assert 0 < w63 < w127
    # at least the activations [M*k, F] bf16 and the expert outputs [M*k, d] f32
    assert w63 >= 63 * 4 * (256 * 2 + 256 * 4)
    assert mb.workspace_bytes(D(), 0) == 0
    assert mb.workspace_bytes(D(dtype=9), 63) == 0


def _call_layer(lib, desc, M=8, B=8, policy=mb.SUBSTITUTE, ws=0x10000, ws_bytes=None, h=0x20000, out=0x30000,
                wptr=0x40000, residual=None):
    cd = desc.c()
    w = mb.Weights(wptr, None, wptr, wptr, wptr)
    if ws_bytes is None:
        ws_bytes = max(mb.workspace_bytes(desc, max(M, 1)), 1)
    return lib.moespec_layer_forward(ctypes.byref(cd), ctypes.byref(w), h, M, B, policy, None, residual, out, None,
                                     ws, ws_bytes, None)


def test_layer_forward_rejects_bad_arguments_before_any_launch(lib):
    """All pointers here are fake: every case must fail validation on the host."""
    d = D()
    assert _call_layer(lib, d, M=0) == mb.ERR_INVALID_ARG
    assert _call_layer(lib, d, M=70000) == mb.ERR_INVALID_ARG
    assert _call_layer(lib, d, B=0) == mb.ERR_INVALID_ARG
    assert _call_layer(lib, d, B=17) == mb.ERR_INVALID_ARG
    assert _call_layer(lib, d, B=3, policy=mb.SUBSTITUTE) == mb.ERR_INVALID_ARG      # B < k
    assert _call_layer(lib, d, policy=5) == mb.ERR_INVALID_ARG
    assert _call_layer(lib, d, h=None) == mb.ERR_INVALID_ARG
    assert _call_layer(lib, d, out=None) == mb.ERR_INVALID_ARG
    assert _call_layer(lib, d, h=0x20004) == mb.ERR_INVALID_ARG                      # misaligned
    assert _call_layer(lib, d, residual=0x30008) == mb.ERR_INVALID_ARG
    assert _call_layer(lib, d, ws=None) == mb.ERR_INVALID_ARG
    assert _call_layer(lib, d, ws=0x10010) == mb.ERR_INVALID_ARG                     # not 256-byte aligned
    assert _call_layer(lib, d, wptr=None) == mb.ERR_INVALID_ARG
    assert _call_layer(lib, d, ws_bytes=mb.workspace_bytes(d, 8) - 1) == mb.ERR_WORKSPACE_TOO_SMALL
    assert _call_layer(lib, D(d=250)) == mb.ERR_UNSUPPORTED_SHAPE
    assert _call_layer(lib, D(dtype=3)) == mb.ERR_INVALID_ARG


def test_static_scratch_call_rejects_bad_arguments_and_oversized_layers_before_any_launch(lib):
    """moespec_layer_forward_static validates on the host before it touches the GPU: argument errors as in the
    workspace call, and a layer whose scratch need exceeds the fixed array is a workspace error."""
    def call(desc, M=8, B=8, policy=mb.SUBSTITUTE, h=0x20000, out=0x30000, wptr=0x40000, residual=None):
        cd = desc.c()
        w = mb.Weights(wptr, None, wptr, wptr, wptr)
        return lib.moespec_layer_forward_static(ctypes.byref(cd), ctypes.byref(w), h, M, B, policy, None, residual,
                                                out, None)
    d = D()
    assert call(d, M=0) == mb.ERR_INVALID_ARG
    assert call(d, B=17) == mb.ERR_INVALID_ARG
    assert call(d, B=3) == mb.ERR_INVALID_ARG                                        # B < k under substitution
    assert call(d, h=None) == mb.ERR_INVALID_ARG
    assert call(d, out=0x30004) == mb.ERR_INVALID_ARG
    assert call(d, wptr=None) == mb.ERR_INVALID_ARG
    assert call(D(d=250)) == mb.ERR_UNSUPPORTED_SHAPE
    olmoe = mb.LayerDesc(2048, 64, 8, 1024, mb.BF16, True)
    assert mb.workspace_bytes(olmoe, 127) <= mb.STATIC_SCRATCH_BYTES < mb.workspace_bytes(olmoe, 511)
    assert call(olmoe, M=511, B=32) == mb.ERR_WORKSPACE_TOO_SMALL
    header = open(os.path.join(ROOT, "include", "moespec.h")).read()
    assert re.search(r"#define MOESPEC_STATIC_SCRATCH_BYTES \(48u << 20\)", header) and mb.STATIC_SCRATCH_BYTES == 48 << 20


def test_stage_calls_reject_bad_arguments(lib):
    d = D()
    cd = d.c()
    w = mb.Weights(0x40000, None, 0x40000, 0x40000, 0x40000)
    wsb = mb.workspace_bytes(d, 8)
    P = 0x50000
    assert lib.moespec_route(ctypes.byref(cd), ctypes.byref(w), P, 8, None, None, None, 0x10000, wsb,
                             None) == mb.ERR_INVALID_ARG                             # probs missing
    assert lib.moespec_route(ctypes.byref(cd), None, P, 8, P, None, None, 0x10000, wsb, None) == mb.ERR_INVALID_ARG
    assert lib.moespec_route(ctypes.byref(cd), ctypes.byref(w), P, 8, P, None, None, 0x10000, 16,
                             None) == mb.ERR_WORKSPACE_TOO_SMALL
    args = [P] * 8
    assert lib.moespec_budget(ctypes.byref(cd), P, 8, 2, mb.SUBSTITUTE, None, *args, 0x10000, wsb,
                              None) == mb.ERR_INVALID_ARG                            # B < k
    assert lib.moespec_budget(ctypes.byref(cd), None, 8, 8, mb.TRUNCATE, None, *args, 0x10000, wsb,
                              None) == mb.ERR_INVALID_ARG
    assert lib.moespec_budget(ctypes.byref(cd), P, 8, 8, mb.TRUNCATE, None, P, P, None, P, P, P, P, P, 0x10000, wsb,
                              None) == mb.ERR_INVALID_ARG                            # tok_ids missing
    assert lib.moespec_expert_ffn(ctypes.byref(cd), ctypes.byref(w), P, 8, 0, P, P, P, P, P, None, P, 0x10000, wsb,
                                  None) == mb.ERR_INVALID_ARG                        # n_seg < 1
    assert lib.moespec_expert_ffn(ctypes.byref(cd), ctypes.byref(w), P, 8, 17, P, P, P, P, P, None, P, 0x10000, wsb,
                                  None) == mb.ERR_INVALID_ARG                        # n_seg > N
    assert lib.moespec_expert_ffn(ctypes.byref(cd), ctypes.byref(w), P, 8, 4, P, None, P, P, P, None, P, 0x10000,
                                  wsb, None) == mb.ERR_INVALID_ARG


def test_analysis_calls_reject_bad_arguments(lib):
    d = D()
    cd = d.c()
    wsb = mb.workspace_bytes(d, 8)
    P = 0x50000
    assert lib.moespec_calibration_count(ctypes.byref(cd), None, 8, P, None) == mb.ERR_INVALID_ARG
    assert lib.moespec_calibration_count(ctypes.byref(cd), P, 0, P, None) == mb.ERR_INVALID_ARG
    assert lib.moespec_calibration_count(ctypes.byref(cd), P, 8, None, None) == mb.ERR_INVALID_ARG
    assert lib.moespec_static_shortlist(ctypes.byref(cd), P, 0, P, None) == mb.ERR_INVALID_ARG
    assert lib.moespec_static_shortlist(ctypes.byref(cd), P, d.n_experts + 1, P, None) == mb.ERR_INVALID_ARG
    assert lib.moespec_static_shortlist(ctypes.byref(cd), None, 4, P, None) == mb.ERR_INVALID_ARG
    assert lib.moespec_coverage_curve(ctypes.byref(cd), None, P, None) == mb.ERR_INVALID_ARG
    assert lib.moespec_coverage_curve(ctypes.byref(cd), P, None, None) == mb.ERR_INVALID_ARG
    assert lib.moespec_reconstruction_error(ctypes.byref(cd), P, None, 8, P, 0x10000, wsb, None) == mb.ERR_INVALID_ARG
    assert lib.moespec_reconstruction_error(ctypes.byref(cd), P, P, 8, P, 0x10000, 16,
                                            None) == mb.ERR_WORKSPACE_TOO_SMALL
    assert lib.moespec_reconstruction_error(ctypes.byref(cd), P, P, 8, None, 0x10000, wsb, None) == mb.ERR_INVALID_ARG


def test_oracle_ranking_rejects_bad_arguments(lib):
    d = D()
    cd = d.c()
    w = mb.Weights(0x40000, None, 0x40000, 0x40000, 0x40000)
    wsb = mb.workspace_bytes(d, 8)
    P = 0x50000
    f = lib.moespec_oracle_ranking
    assert f(ctypes.byref(cd), ctypes.byref(w), P, 8, 0, P, P, 0x10000, wsb, None) == mb.ERR_INVALID_ARG
    assert f(ctypes.byref(cd), ctypes.byref(w), P, 8, d.n_experts + 1, P, P, 0x10000, wsb, None) == mb.ERR_INVALID_ARG
    assert f(ctypes.byref(cd), ctypes.byref(w), P, 8, 4, None, P, 0x10000, wsb, None) == mb.ERR_INVALID_ARG
    assert f(ctypes.byref(cd), ctypes.byref(w), P, 8, 4, P, P, 0x10000, 64, None) == mb.ERR_WORKSPACE_TOO_SMALL
    assert f(ctypes.byref(cd), None, P, 8, 4, P, P, 0x10000, wsb, None) == mb.ERR_INVALID_ARG


def test_stream_read_rejects_bad_arguments(lib):
    f = lib.moespec_stream_read
    P, C = 0x50000, 0x60000
    assert f(None, 1024, C, None) == mb.ERR_INVALID_ARG
    assert f(P, 1024, None, None) == mb.ERR_INVALID_ARG
    assert f(P + 8, 1024, C, None) == mb.ERR_INVALID_ARG       # buffer not 16-byte aligned
    assert f(P, 1024, C + 2, None) == mb.ERR_INVALID_ARG       # checksum word not 4-byte aligned
    assert f(P, 0, C, None) == mb.ERR_INVALID_ARG
    assert f(P, 1000, C, None) == mb.ERR_INVALID_ARG           # not a multiple of 16
    assert f(P, 1 << 40, C, None) == mb.ERR_INVALID_ARG


def test_binding_refuses_cpu_tensors(lib):
    import torch
    d = D()
    with pytest.raises(ValueError):
        mb.moespec_route(d, dict(w_router=torch.zeros(16, 256, dtype=torch.bfloat16)),
                         torch.zeros(8, 256, dtype=torch.bfloat16), torch.zeros(1 << 20, dtype=torch.uint8))


def test_missing_library_fails_loudly(tmp_path):
    with pytest.raises(FileNotFoundError):
        mb.load_library(str(tmp_path / "nope.so"))


def test_stack_calls_reject_bad_arguments(lib):
    d = D()
    cd = d.c()
    wsb = mb.workspace_bytes(d, 8)
    P = 0x50000
    two = (mb.Weights * 2)(mb.Weights(P, None, P, P, P), mb.Weights(P, None, P, P, P))
    f = lib.moespec_stack_forward
    assert f(ctypes.byref(cd), two, 0, P, 8, 8, mb.SUBSTITUTE, 1, None, None, 0x10000, wsb, None) == mb.ERR_INVALID_ARG
    assert f(ctypes.byref(cd), None, 2, P, 8, 8, mb.SUBSTITUTE, 1, None, None, 0x10000, wsb, None) == mb.ERR_INVALID_ARG
    assert f(ctypes.byref(cd), two, 2, None, 8, 8, mb.SUBSTITUTE, 1, None, None, 0x10000, wsb, None) == mb.ERR_INVALID_ARG
    assert f(ctypes.byref(cd), two, 2, P, 8, 8, mb.SUBSTITUTE, 2, None, None, 0x10000, wsb, None) == mb.ERR_INVALID_ARG
    assert f(ctypes.byref(cd), two, 2, P, 8, 3, mb.SUBSTITUTE, 1, None, None, 0x10000, wsb, None) == mb.ERR_INVALID_ARG
    assert f(ctypes.byref(cd), two, 2, P, 8, 8, mb.SUBSTITUTE, 1, None, None, 0x10000, 64,
             None) == mb.ERR_WORKSPACE_TOO_SMALL
    bad = (mb.Weights * 2)(mb.Weights(P, None, P, P, P), mb.Weights(P, None, None, P, P))   # second layer incomplete
    assert f(ctypes.byref(cd), bad, 2, P, 8, 8, mb.SUBSTITUTE, 1, None, None, 0x10000, wsb, None) == mb.ERR_INVALID_ARG
    g = lib.moespec_rms_scale
    assert g(ctypes.byref(cd), None, 8, P, None) == mb.ERR_INVALID_ARG
    assert g(ctypes.byref(cd), P, 0, P, None) == mb.ERR_INVALID_ARG
    assert g(ctypes.byref(cd), P, 8, P + 4, None) == mb.ERR_INVALID_ARG
