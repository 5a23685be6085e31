"""ctypes binding of libmoespec.so: argument marshalling only.

Every function takes torch tensors living on the GPU (device memory and streams are PyTorch's
job here), checks dtype / shape / contiguity, passes raw pointers and sizes through the C ABI and
raises ``MoeSpecError`` on a non-zero status.  No step of the method is computed in Python.
The library must have been built (``python -m paper_2602_16052_amd.build``); there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, c_char_p, c_int32, c_size_t, c_void_p
from dataclasses import dataclass
from typing import Dict, Optional

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libmoespec.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED_SHAPE, ERR_WORKSPACE_TOO_SMALL, ERR_HIP = range(5)
F32, BF16 = 0, 1
TRUNCATE, SUBSTITUTE = 0, 1
GATE_SOFTMAX, GATE_SIGMOID = 0, 1

EXPORTS = ("moespec_abi_version", "moespec_status_string", "moespec_check_desc", "moespec_workspace_bytes",
           "moespec_route", "moespec_budget", "moespec_expert_ffn", "moespec_layer_forward",
           "moespec_layer_forward_traced", "moespec_layer_forward_static", "moespec_stack_forward", "moespec_rms_scale",
           "moespec_calibration_count", "moespec_static_shortlist", "moespec_coverage_curve",
           "moespec_reconstruction_error", "moespec_oracle_ranking", "moespec_stream_read")


class MoeSpecError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class Desc(Structure):
    _fields_ = [("d", c_int32), ("n_experts", c_int32), ("top_k", c_int32), ("d_ff", c_int32),
                ("dtype", c_int32), ("renorm", c_int32), ("gate", c_int32)]


class Weights(Structure):
    _fields_ = [("w_router", c_void_p), ("b_router", c_void_p), ("w_gate", c_void_p), ("w_up", c_void_p),
                ("w_down", c_void_p)]


class Taps(Structure):
    _fields_ = [("probs", c_void_p), ("scores", c_void_p), ("budget_ids", c_void_p), ("tok_ids", c_void_p),
                ("tok_w", c_void_p), ("seg_expert", c_void_p), ("seg_off", c_void_p), ("perm", c_void_p),
                ("n_loaded", c_void_p)]


TRACE_POINTS = 5
TRACE_STAGES = ("prologue", "gate_up", "down", "combine")   # intervals between consecutive trace points


_lib = None


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """dlopen the library and declare its signatures.  Raises if it has not been built."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise FileNotFoundError(f"{p} is missing: build it with `python -m paper_2602_16052_amd.build` "
                                "(there is no non-HIP fallback)")
    lib = ctypes.CDLL(p)
    lib.moespec_abi_version.restype = c_int32
    lib.moespec_abi_version.argtypes = []
    lib.moespec_status_string.restype = c_char_p
    lib.moespec_status_string.argtypes = [c_int32]
    lib.moespec_check_desc.restype = c_int32
    lib.moespec_check_desc.argtypes = [POINTER(Desc)]
    lib.moespec_workspace_bytes.restype = c_size_t
    lib.moespec_workspace_bytes.argtypes = [POINTER(Desc), c_int32]
    lib.moespec_route.restype = c_int32
    lib.moespec_route.argtypes = [POINTER(Desc), POINTER(Weights), c_void_p, c_int32, c_void_p, c_void_p, c_void_p,
                                  c_void_p, c_size_t, c_void_p]
    lib.moespec_budget.restype = c_int32
    lib.moespec_budget.argtypes = [POINTER(Desc), c_void_p, c_int32, c_int32, c_int32, c_void_p, c_void_p, c_void_p,
                                   c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t,
                                   c_void_p]
    lib.moespec_expert_ffn.restype = c_int32
    lib.moespec_expert_ffn.argtypes = [POINTER(Desc), POINTER(Weights), c_void_p, c_int32, c_int32, c_void_p,
                                       c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                       c_size_t, c_void_p]
    lib.moespec_layer_forward.restype = c_int32
    lib.moespec_layer_forward.argtypes = [POINTER(Desc), POINTER(Weights), c_void_p, c_int32, c_int32, c_int32,
                                          c_void_p, c_void_p, c_void_p, POINTER(Taps), c_void_p, c_size_t, c_void_p]
    lib.moespec_layer_forward_traced.restype = c_int32
    lib.moespec_layer_forward_traced.argtypes = [POINTER(Desc), POINTER(Weights), c_void_p, c_int32, c_int32, c_int32,
                                                 c_void_p, c_void_p, c_void_p, c_void_p, POINTER(c_void_p), c_void_p,
                                                 c_size_t, c_void_p]
    lib.moespec_layer_forward_static.restype = c_int32
    lib.moespec_layer_forward_static.argtypes = [POINTER(Desc), POINTER(Weights), c_void_p, c_int32, c_int32, c_int32,
                                                 c_void_p, c_void_p, c_void_p, c_void_p]
    lib.moespec_stack_forward.restype = c_int32
    lib.moespec_stack_forward.argtypes = [POINTER(Desc), POINTER(Weights), c_int32, c_void_p, c_int32, c_int32, c_int32,
                                          c_int32, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.moespec_rms_scale.restype = c_int32
    lib.moespec_rms_scale.argtypes = [POINTER(Desc), c_void_p, c_int32, c_void_p, c_void_p]
    lib.moespec_calibration_count.restype = c_int32
    lib.moespec_calibration_count.argtypes = [POINTER(Desc), c_void_p, c_int32, c_void_p, c_void_p]
    lib.moespec_static_shortlist.restype = c_int32
    lib.moespec_static_shortlist.argtypes = [POINTER(Desc), c_void_p, c_int32, c_void_p, c_void_p]
    lib.moespec_coverage_curve.restype = c_int32
    lib.moespec_coverage_curve.argtypes = [POINTER(Desc), c_void_p, c_void_p, c_void_p]
    lib.moespec_reconstruction_error.restype = c_int32
    lib.moespec_reconstruction_error.argtypes = [POINTER(Desc), c_void_p, c_void_p, c_int32, c_void_p, c_void_p,
                                                 c_size_t, c_void_p]
    lib.moespec_oracle_ranking.restype = c_int32
    lib.moespec_oracle_ranking.argtypes = [POINTER(Desc), POINTER(Weights), c_void_p, c_int32, c_int32, c_void_p,
                                           c_void_p, c_void_p, c_size_t, c_void_p]
    lib.moespec_stream_read.restype = c_int32
    lib.moespec_stream_read.argtypes = [c_void_p, c_size_t, c_void_p, c_void_p]
    if path is None:
        _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().moespec_status_string(int(status)).decode()


def abi_version() -> int:
    return int(load_library().moespec_abi_version())


@dataclass
class LayerDesc:
    d: int
    n_experts: int
    top_k: int
    d_ff: int
    dtype: int          # F32 or BF16
    renorm: bool
    gate: int = 0       # GATE_SOFTMAX or GATE_SIGMOID

    def c(self) -> Desc:
        return Desc(self.d, self.n_experts, self.top_k, self.d_ff, self.dtype, int(self.renorm), int(self.gate))

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.bfloat16 if self.dtype == BF16 else torch.float32


def check_desc(desc: LayerDesc) -> int:
    c = desc.c()
    return int(load_library().moespec_check_desc(ctypes.byref(c)))


def workspace_bytes(desc: LayerDesc, M_max: int) -> int:
    c = desc.c()
    return int(load_library().moespec_workspace_bytes(ctypes.byref(c), int(M_max)))


def alloc_workspace(desc: LayerDesc, M_max: int, device="cuda") -> torch.Tensor:
    n = workspace_bytes(desc, M_max)
    if n == 0:
        raise MoeSpecError(ERR_INVALID_ARG, "moespec_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def _ptr(t: Optional[torch.Tensor], dtype: Optional[torch.dtype] = None, numel: Optional[int] = None,
         name: str = "tensor") -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must be a GPU tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if numel is not None and t.numel() < numel:
        raise ValueError(f"{name} needs at least {numel} elements, got {t.numel()}")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


def _weights(desc: LayerDesc, w: Dict[str, torch.Tensor], router: bool, experts: bool) -> Weights:
    N, d, F, dt = desc.n_experts, desc.d, desc.d_ff, desc.torch_dtype
    cw = Weights()
    if router:
        cw.w_router = _ptr(w["w_router"], dt, N * d, "w_router")
        cw.b_router = _ptr(w.get("b_router"), torch.float32, N, "b_router")
    if experts:
        cw.w_gate = _ptr(w["w_gate"], dt, N * F * d, "w_gate")
        cw.w_up = _ptr(w["w_up"], dt, N * F * d, "w_up")
        cw.w_down = _ptr(w["w_down"], dt, N * d * F, "w_down")
    return cw


def _check(status: int, where: str):
    if status != OK:
        raise MoeSpecError(int(status), where)


def moespec_route(desc: LayerDesc, weights: Dict[str, torch.Tensor], h: torch.Tensor, ws: torch.Tensor,
                  stream=None, want_topk: bool = True):
    """Eq. (1) + Section 2.1.  Returns dict(probs[M,N] f64, topk_ids[M,k] i32, topk_w[M,k] f32)."""
    M, N, k = h.shape[0], desc.n_experts, desc.top_k
    dev = h.device
    probs = torch.empty((M, N), dtype=torch.float64, device=dev)
    ids = torch.empty((M, k), dtype=torch.int32, device=dev) if want_topk else None
    tw = torch.empty((M, k), dtype=torch.float32, device=dev) if want_topk else None
    cd, cw = desc.c(), _weights(desc, weights, True, False)
    st = load_library().moespec_route(ctypes.byref(cd), ctypes.byref(cw), _ptr(h, desc.torch_dtype, M * desc.d, "h"),
                                      M, _ptr(probs), _ptr(ids), _ptr(tw), _ptr(ws), ws.numel(), _stream(stream))
    _check(st, "moespec_route")
    return dict(probs=probs, topk_ids=ids, topk_w=tw)


def moespec_budget(desc: LayerDesc, probs: torch.Tensor, B: int, policy: int, ws: torch.Tensor,
                   ext_shortlist: Optional[torch.Tensor] = None, stream=None):
    """Eq. (5), shortlist, Eq. (7)/(8), segments.  Returns a dict of the documented outputs."""
    M, N, k = probs.shape[0], desc.n_experts, desc.top_k
    dev = probs.device
    i32 = dict(dtype=torch.int32, device=dev)
    out = dict(scores=torch.empty(N, dtype=torch.float64, device=dev), budget_ids=torch.empty(max(B, 1), **i32),
               tok_ids=torch.empty((M, k), **i32), tok_w=torch.empty((M, k), dtype=torch.float32, device=dev),
               seg_expert=torch.empty(max(B, 1), **i32), seg_off=torch.empty(max(B, 1) + 1, **i32),
               perm=torch.empty(M * k, **i32), n_loaded=torch.empty(1, **i32))
    cd = desc.c()
    st = load_library().moespec_budget(
        ctypes.byref(cd), _ptr(probs, torch.float64, M * N, "probs"), M, int(B), int(policy),
        _ptr(ext_shortlist, torch.int32, max(B, 0), "ext_shortlist"), _ptr(out["scores"]), _ptr(out["budget_ids"]),
        _ptr(out["tok_ids"]), _ptr(out["tok_w"]), _ptr(out["seg_expert"]), _ptr(out["seg_off"]), _ptr(out["perm"]),
        _ptr(out["n_loaded"]), _ptr(ws), ws.numel(), _stream(stream))
    _check(st, "moespec_budget")
    return out


def moespec_expert_ffn(desc: LayerDesc, weights: Dict[str, torch.Tensor], h: torch.Tensor, seg_expert: torch.Tensor,
                       seg_off: torch.Tensor, perm: torch.Tensor, tok_ids: torch.Tensor, tok_w: torch.Tensor,
                       ws: torch.Tensor, residual: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                       stream=None) -> torch.Tensor:
    """Experts over the loaded set + weighted combine.  Returns out[M, d] in the layer dtype."""
    M, k, dt = h.shape[0], desc.top_k, desc.torch_dtype
    n_seg = seg_expert.numel()
    if out is None:
        out = torch.empty((M, desc.d), dtype=dt, device=h.device)
    cd, cw = desc.c(), _weights(desc, weights, False, True)
    st = load_library().moespec_expert_ffn(
        ctypes.byref(cd), ctypes.byref(cw), _ptr(h, dt, M * desc.d, "h"), M, n_seg,
        _ptr(seg_expert, torch.int32, n_seg, "seg_expert"), _ptr(seg_off, torch.int32, n_seg + 1, "seg_off"),
        _ptr(perm, torch.int32, M * k, "perm"), _ptr(tok_ids, torch.int32, M * k, "tok_ids"),
        _ptr(tok_w, torch.float32, M * k, "tok_w"), _ptr(residual, dt, M * desc.d, "residual"),
        _ptr(out, dt, M * desc.d, "out"), _ptr(ws), ws.numel(), _stream(stream))
    _check(st, "moespec_expert_ffn")
    return out


class HipEvents:
    """A fixed set of timing-enabled hipEvent_t handles (created through libamdhip64 directly, so that
    their raw handles can cross the C ABI).  Used for the library's optional trace hook."""

    def __init__(self, n: int):
        self._hip = ctypes.CDLL("libamdhip64.so")
        self._hip.hipEventCreate.argtypes = [POINTER(c_void_p)]
        self._hip.hipEventElapsedTime.argtypes = [POINTER(ctypes.c_float), c_void_p, c_void_p]
        self._hip.hipEventSynchronize.argtypes = [c_void_p]
        self._hip.hipEventDestroy.argtypes = [c_void_p]
        self._hip.hipEventRecord.argtypes = [c_void_p, c_void_p]
        self.handles = (c_void_p * n)()
        for i in range(n):
            ev = c_void_p()
            if self._hip.hipEventCreate(ctypes.byref(ev)) != 0:
                raise MoeSpecError(ERR_HIP, "hipEventCreate")
            self.handles[i] = ev

    def record(self, i: int, stream=None):
        if self._hip.hipEventRecord(self.handles[i], _stream(stream)) != 0:
            raise MoeSpecError(ERR_HIP, "hipEventRecord")

    def synchronize(self, i: int):
        if self._hip.hipEventSynchronize(self.handles[i]) != 0:
            raise MoeSpecError(ERR_HIP, "hipEventSynchronize")

    def elapsed_ms(self, i: int, j: int) -> float:
        ms = ctypes.c_float()
        if self._hip.hipEventElapsedTime(ctypes.byref(ms), self.handles[i], self.handles[j]) != 0:
            raise MoeSpecError(ERR_HIP, "hipEventElapsedTime")
        return float(ms.value)

    def __del__(self):
        try:
            for ev in self.handles:
                if ev:
                    self._hip.hipEventDestroy(ev)
        except Exception:
            pass


class LayerForwardCall:
    """moespec_layer_forward with its arguments marshalled once: calling the object only crosses the
    C ABI (for tight loops, where per-call marshalling would cost more than the kernels).  With ``trace`` the call
    goes through moespec_layer_forward_traced, which records the events at the stage boundaries."""

    def __init__(self, desc: LayerDesc, weights: Dict[str, torch.Tensor], h: torch.Tensor, B: int, policy: int,
                 ws: torch.Tensor, out: torch.Tensor, ext_shortlist: Optional[torch.Tensor] = None,
                 residual: Optional[torch.Tensor] = None, trace: Optional[HipEvents] = None,
                 n_loaded: Optional[torch.Tensor] = None, stream=None):
        M, dt = h.shape[0], desc.torch_dtype
        self._keep = (weights, h, ws, out, ext_shortlist, residual, trace, n_loaded)
        lib = load_library()
        self._cd, self._cw = desc.c(), _weights(desc, weights, True, True)
        head = (ctypes.byref(self._cd), ctypes.byref(self._cw), _ptr(h, dt, M * desc.d, "h"), M, int(B),
                int(policy), _ptr(ext_shortlist, torch.int32, max(int(B), 0), "ext_shortlist"),
                _ptr(residual, dt, M * desc.d, "residual"), _ptr(out, dt, M * desc.d, "out"))
        tail = (_ptr(ws), ws.numel(), _stream(stream))
        if trace is not None:
            if len(trace.handles) < TRACE_POINTS:
                raise ValueError(f"trace needs {TRACE_POINTS} events")
            self._fn, self._name = lib.moespec_layer_forward_traced, "moespec_layer_forward_traced"
            self._args = head + (_ptr(n_loaded, torch.int32, 1, "n_loaded"),
                                 ctypes.cast(trace.handles, POINTER(c_void_p))) + tail
        else:
            self._fn, self._name = lib.moespec_layer_forward, "moespec_layer_forward"
            self._taps = None
            if n_loaded is not None:
                self._taps = Taps()
                self._taps.n_loaded = _ptr(n_loaded, torch.int32, 1, "n_loaded")
            self._args = head + (ctypes.byref(self._taps) if self._taps is not None else None,) + tail

    def __call__(self):
        st = self._fn(*self._args)
        if st != OK:
            raise MoeSpecError(int(st), self._name)


def moespec_layer_forward(desc: LayerDesc, weights: Dict[str, torch.Tensor], h: torch.Tensor, B: int, policy: int,
                          ws: torch.Tensor, ext_shortlist: Optional[torch.Tensor] = None,
                          residual: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                          taps: bool = False, stream=None):
    """Algorithm 1 in one call.  Returns ``out`` or, with ``taps=True``, ``(out, dict of intermediates)``."""
    M, N, k, dt = h.shape[0], desc.n_experts, desc.top_k, desc.torch_dtype
    dev = h.device
    if out is None:
        out = torch.empty((M, desc.d), dtype=dt, device=dev)
    tap_t = None
    ctaps = None
    if taps:
        i32 = dict(dtype=torch.int32, device=dev)
        nb = max(int(B), 1)
        tap_t = dict(probs=torch.empty((M, N), dtype=torch.float64, device=dev),
                     scores=torch.empty(N, dtype=torch.float64, device=dev), budget_ids=torch.empty(nb, **i32),
                     tok_ids=torch.empty((M, k), **i32), tok_w=torch.empty((M, k), dtype=torch.float32, device=dev),
                     seg_expert=torch.empty(nb, **i32), seg_off=torch.empty(nb + 1, **i32),
                     perm=torch.empty(M * k, **i32), n_loaded=torch.empty(1, **i32))
        ctaps = Taps(**{key: _ptr(val) for key, val in tap_t.items()})
    cd, cw = desc.c(), _weights(desc, weights, True, True)
    st = load_library().moespec_layer_forward(
        ctypes.byref(cd), ctypes.byref(cw), _ptr(h, dt, M * desc.d, "h"), M, int(B), int(policy),
        _ptr(ext_shortlist, torch.int32, max(int(B), 0), "ext_shortlist"), _ptr(residual, dt, M * desc.d, "residual"),
        _ptr(out, dt, M * desc.d, "out"), ctypes.byref(ctaps) if ctaps is not None else None, _ptr(ws), ws.numel(),
        _stream(stream))
    _check(st, "moespec_layer_forward")
    return (out, tap_t) if taps else out


def moespec_rms_scale(desc: LayerDesc, h: torch.Tensor, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """x[t] = h[t] / rms(h[t]) (the input scaling of the layer stack).  Returns x[M, d] in the layer dtype."""
    M, dt = h.shape[0], desc.torch_dtype
    if out is None:
        out = torch.empty_like(h)
    cd = desc.c()
    st = load_library().moespec_rms_scale(ctypes.byref(cd), _ptr(h, dt, M * desc.d, "h"), M,
                                          _ptr(out, dt, M * desc.d, "x"), _stream(stream))
    _check(st, "moespec_rms_scale")
    return out


class StackForwardCall:
    """moespec_stack_forward with its arguments marshalled once (h is updated in place on every call)."""

    def __init__(self, desc: LayerDesc, layers, h: torch.Tensor, B: int, policy: int, ws: torch.Tensor,
                 pre_norm: bool = True, budget_ids: Optional[torch.Tensor] = None,
                 tok_ids: Optional[torch.Tensor] = None, stream=None):
        M, dt, L = h.shape[0], desc.torch_dtype, len(layers)
        self._keep = (layers, h, ws, budget_ids, tok_ids)
        self._fn = load_library().moespec_stack_forward
        self._cd = desc.c()
        self._cw = (Weights * L)(*[_weights(desc, w, True, True) for w in layers])
        self._args = (ctypes.byref(self._cd), self._cw, L, _ptr(h, dt, M * desc.d, "h"), M, int(B), int(policy),
                      int(bool(pre_norm)), _ptr(budget_ids, torch.int32, L * max(int(B), 1), "budget_ids"),
                      _ptr(tok_ids, torch.int32, L * M * desc.top_k, "tok_ids"), _ptr(ws), ws.numel(), _stream(stream))

    def __call__(self):
        st = self._fn(*self._args)
        if st != OK:
            raise MoeSpecError(int(st), "moespec_stack_forward")


def moespec_stack_forward(desc: LayerDesc, layers, h: torch.Tensor, B: int, policy: int, ws: torch.Tensor,
                          pre_norm: bool = True, taps: bool = False, stream=None):
    """The layer stack h <- h + MoE_S(x) over ``layers`` (a list of weight dicts), in place on ``h``.
    Returns ``h`` or, with ``taps=True``, ``(h, dict(budget_ids[L, B], tok_ids[L, M, k]))``."""
    L, M = len(layers), h.shape[0]
    tap = None
    if taps:
        i32 = dict(dtype=torch.int32, device=h.device)
        tap = dict(budget_ids=torch.empty((L, max(int(B), 1)), **i32), tok_ids=torch.empty((L, M, desc.top_k), **i32))
    StackForwardCall(desc, layers, h, B, policy, ws, pre_norm, tap["budget_ids"] if tap else None,
                     tap["tok_ids"] if tap else None, stream)()
    return (h, tap) if taps else h


STATIC_SCRATCH_BYTES = 48 << 20


def moespec_layer_forward_static(desc: LayerDesc, weights: Dict[str, torch.Tensor], h: torch.Tensor, B: int,
                                 policy: int, out: torch.Tensor, ext_shortlist: Optional[torch.Tensor] = None,
                                 residual: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Algorithm 1 in one call on the library's own fixed scratch array: no workspace argument, nothing allocated
    (``out`` is the caller's).  Returns ``out``."""
    M, dt = h.shape[0], desc.torch_dtype
    cd, cw = desc.c(), _weights(desc, weights, True, True)
    st = load_library().moespec_layer_forward_static(
        ctypes.byref(cd), ctypes.byref(cw), _ptr(h, dt, M * desc.d, "h"), M, int(B), int(policy),
        _ptr(ext_shortlist, torch.int32, max(int(B), 0), "ext_shortlist"), _ptr(residual, dt, M * desc.d, "residual"),
        _ptr(out, dt, M * desc.d, "out"), _stream(stream))
    _check(st, "moespec_layer_forward_static")
    return out


def moespec_calibration_count(desc: LayerDesc, topk_ids: torch.Tensor, counts: torch.Tensor, stream=None) -> torch.Tensor:
    """Eq. (4): counts[i] += number of rows of topk_ids [M, k] that contain expert i.  Returns counts."""
    M = topk_ids.shape[0]
    cd = desc.c()
    st = load_library().moespec_calibration_count(
        ctypes.byref(cd), _ptr(topk_ids, torch.int32, M * desc.top_k, "topk_ids"), M,
        _ptr(counts, torch.int64, desc.n_experts, "counts"), _stream(stream))
    _check(st, "moespec_calibration_count")
    return counts


def moespec_static_shortlist(desc: LayerDesc, counts: torch.Tensor, B: int, stream=None) -> torch.Tensor:
    """The B most frequently selected experts (Eq. (4)), most frequent first; int32 [B], usable as ext_shortlist."""
    out = torch.empty(max(int(B), 1), dtype=torch.int32, device=counts.device)
    cd = desc.c()
    st = load_library().moespec_static_shortlist(ctypes.byref(cd), _ptr(counts, torch.int64, desc.n_experts, "counts"),
                                                 int(B), _ptr(out), _stream(stream))
    _check(st, "moespec_static_shortlist")
    return out


def moespec_coverage_curve(desc: LayerDesc, scores: torch.Tensor, stream=None) -> torch.Tensor:
    """Section 4.6: share of the routing probability captured by the top-B experts, B = 1..N; float64 [N]."""
    out = torch.empty(desc.n_experts, dtype=torch.float64, device=scores.device)
    cd = desc.c()
    st = load_library().moespec_coverage_curve(ctypes.byref(cd), _ptr(scores, torch.float64, desc.n_experts, "scores"),
                                               _ptr(out), _stream(stream))
    _check(st, "moespec_coverage_curve")
    return out


def moespec_reconstruction_error(desc: LayerDesc, out_budgeted: torch.Tensor, out_full: torch.Tensor,
                                 ws: torch.Tensor, stream=None) -> torch.Tensor:
    """Section 4.5: float64 [3] = (||O_S - O*||^2 / ||O*||^2, numerator, denominator)."""
    M, dt = out_full.shape[0], desc.torch_dtype
    err = torch.empty(3, dtype=torch.float64, device=out_full.device)
    cd = desc.c()
    st = load_library().moespec_reconstruction_error(
        ctypes.byref(cd), _ptr(out_budgeted, dt, M * desc.d, "out_budgeted"), _ptr(out_full, dt, M * desc.d, "out_full"),
        M, _ptr(err), _ptr(ws), ws.numel(), _stream(stream))
    _check(st, "moespec_reconstruction_error")
    return err


def moespec_oracle_ranking(desc: LayerDesc, weights: Dict[str, torch.Tensor], h: torch.Tensor, B: int, ws: torch.Tensor,
                           stream=None):
    """Eq. (6): greedy oracle ordering.  Returns (ranking int32 [B], err float64 [B])."""
    M, dt = h.shape[0], desc.torch_dtype
    ranking = torch.empty(max(int(B), 1), dtype=torch.int32, device=h.device)
    err = torch.empty(max(int(B), 1), dtype=torch.float64, device=h.device)
    cd, cw = desc.c(), _weights(desc, weights, True, True)
    st = load_library().moespec_oracle_ranking(ctypes.byref(cd), ctypes.byref(cw), _ptr(h, dt, M * desc.d, "h"), M, int(B),
                                               _ptr(ranking), _ptr(err), _ptr(ws), ws.numel(), _stream(stream))
    _check(st, "moespec_oracle_ranking")
    return ranking, err


STREAM_READ_WORDS = 256


def moespec_stream_read(buf: torch.Tensor, checksum: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Measurement aid: stream `buf` (contiguous, a multiple of 16 bytes) once through a plain read kernel.
    Every workgroup adds the sum modulo 2^32 of the 32-bit words it read to its word of `checksum`
    (int32 [STREAM_READ_WORDS], zeroed here if not given); `checksum.sum()` modulo 2^32 is the buffer's checksum."""
    if not (buf.is_cuda and buf.is_contiguous()):
        raise ValueError("buf: expected a contiguous GPU tensor")
    if checksum is None:
        checksum = torch.zeros(STREAM_READ_WORDS, dtype=torch.int32, device=buf.device)
    st = load_library().moespec_stream_read(buf.data_ptr(), buf.numel() * buf.element_size(),
                                            _ptr(checksum, torch.int32, STREAM_READ_WORDS, "checksum"),
                                            _stream(stream))
    _check(st, "moespec_stream_read")
    return checksum
