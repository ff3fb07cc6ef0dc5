"""Thin ctypes binding of libmoesd (see include/moesd.h): argument marshalling
only.  Tensors are torch CUDA tensors used as plain device buffers; every step
of the path runs inside the library's HIP kernels.  There is no CPU fallback: if
the library is missing or no GPU is present the calls raise."""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmoesd.so")

OK, INVALID_ARG, UNSUPPORTED, WORKSPACE_TOO_SMALL, HIP_ERROR = 0, 1, 2, 3, 4
N_STAGE_EVENTS = 5
STATIC_SCRATCH_BYTES = 32 << 20

EXPORTS = ["moesd_expected_active_experts", "moesd_expected_active_experts_p",
           "moesd_expected_tokens_per_expert",
           "moesd_token_threshold", "moesd_workspace_bytes", "moesd_route", "moesd_permute",
           "moesd_moe_forward", "moesd_moe_forward_staged", "moesd_moe_forward_static",
           "moesd_status_string",
           "moesd_last_hip_error"]


class LayerDesc(C.Structure):
    _fields_ = [("d", C.c_int32), ("E", C.c_int32), ("top_k", C.c_int32), ("inter", C.c_int32),
                ("shared_inter", C.c_int32), ("score_func", C.c_int32), ("renormalize", C.c_int32),
                ("shared_gate", C.c_int32), ("routed_scale", C.c_float), ("n_group", C.c_int32),
                ("topk_group", C.c_int32), ("weight_format", C.c_int32)]


class Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("w_router", "router_bias", "w_gate", "w_up", "w_down",
                                          "ws_gate", "ws_up", "ws_down", "w_shared_gate",
                                          "w_gate_scale", "w_up_scale", "w_down_scale",
                                          "ws_gate_scale", "ws_up_scale", "ws_down_scale")]


class MoesdError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__(f"{what}: status {status} ({status_string(status)})")


_lib = None


def lib():
    """Load libmoesd.so (built by paper_2505_19645_amd.build); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} not built: run python -m paper_2505_19645_amd.build")
        # PyTorch ships its own HIP runtime; load it first so the library binds to
        # that one copy (two runtimes in a process would not share streams)
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        L.moesd_expected_active_experts.restype = C.c_double
        L.moesd_expected_active_experts.argtypes = [C.c_int32, C.c_int32, C.c_int64]
        L.moesd_expected_active_experts_p.restype = C.c_double
        L.moesd_expected_active_experts_p.argtypes = [C.POINTER(C.c_double), C.c_int32, C.c_int64]
        L.moesd_expected_tokens_per_expert.restype = C.c_double
        L.moesd_expected_tokens_per_expert.argtypes = [C.c_int32, C.c_int32, C.c_int64]
        L.moesd_token_threshold.restype = C.c_int64
        L.moesd_token_threshold.argtypes = [C.c_int32, C.c_int32, C.c_double]
        L.moesd_workspace_bytes.restype = C.c_size_t
        L.moesd_workspace_bytes.argtypes = [C.POINTER(LayerDesc), C.c_int32]
        L.moesd_route.restype = C.c_int32
        L.moesd_route.argtypes = [C.POINTER(LayerDesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                  C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.moesd_permute.restype = C.c_int32
        L.moesd_permute.argtypes = [C.c_int32, C.c_int32, C.c_int32] + [C.c_void_p] * 7
        fwd = [C.POINTER(LayerDesc), C.POINTER(Weights), C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
               C.c_void_p, C.c_size_t] + [C.c_void_p] * 7 + [C.c_void_p]
        L.moesd_moe_forward.restype = C.c_int32
        L.moesd_moe_forward.argtypes = fwd
        L.moesd_moe_forward_staged.restype = C.c_int32
        L.moesd_moe_forward_staged.argtypes = fwd + [C.POINTER(C.c_void_p)]
        L.moesd_moe_forward_static.restype = C.c_int32
        L.moesd_moe_forward_static.argtypes = [C.POINTER(LayerDesc), C.POINTER(Weights), C.c_void_p, C.c_int32,
                                               C.c_void_p, C.c_void_p] + [C.c_void_p] * 7 + [C.c_void_p]
        L.moesd_status_string.restype = C.c_char_p
        L.moesd_status_string.argtypes = [C.c_int32]
        L.moesd_last_hip_error.restype = C.c_int32
        L.moesd_last_hip_error.argtypes = []
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().moesd_status_string(status).decode()


def last_hip_error() -> int:
    return lib().moesd_last_hip_error()


def make_desc(shape) -> LayerDesc:
    """shape: object with d, E, top_k, inter, shared_inter, score_func, renormalize,
    shared_gate, routed_scale (e.g. synth.LayerShape)."""
    return LayerDesc(shape.d, shape.E, shape.top_k, shape.inter, shape.shared_inter,
                     shape.score_func, shape.renormalize, shape.shared_gate,
                     float(shape.routed_scale), int(getattr(shape, "n_group", 0)),
                     int(getattr(shape, "topk_group", 0)), int(getattr(shape, "weight_format", 0)))


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return C.c_void_p(t)
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return C.c_void_p(stream)
    return C.c_void_p(stream.cuda_stream)


def make_weights(w: dict) -> Weights:
    """w: dict of device tensors with the field names of moesd_weights."""
    out = Weights()
    for name, _ in Weights._fields_:
        t = w.get(name)
        setattr(out, name, None if t is None else t.data_ptr())
    return out


# ---- closed forms (host) ---------------------------------------------------

def moesd_expected_active_experts(E: int, K: int, t: int) -> float:
    return lib().moesd_expected_active_experts(E, K, t)


def moesd_expected_active_experts_p(p, t: int) -> float:
    """p: per-expert probabilities of being activated by one token (any sequence of floats)."""
    arr = (C.c_double * len(p))(*[float(v) for v in p])
    return lib().moesd_expected_active_experts_p(arr, len(p), t)


def moesd_expected_tokens_per_expert(E: int, K: int, t: int) -> float:
    return lib().moesd_expected_tokens_per_expert(E, K, t)


def moesd_token_threshold(E: int, K: int, tau: float = 0.95) -> int:
    return lib().moesd_token_threshold(E, K, tau)


def moesd_workspace_bytes(desc: LayerDesc, T_max: int) -> int:
    return lib().moesd_workspace_bytes(C.byref(desc), T_max)


# ---- hot path ----------------------------------------------------------------

def moesd_route(desc, x, w_router, router_bias, T, topk_ids, topk_w, workspace, workspace_bytes=None,
                stream=None, check=True):
    nbytes = workspace_bytes if workspace_bytes is not None else (
        0 if workspace is None else workspace.numel() * workspace.element_size())
    st = lib().moesd_route(C.byref(desc), _ptr(x), _ptr(w_router), _ptr(router_bias), T,
                           _ptr(topk_ids), _ptr(topk_w), _ptr(workspace), nbytes, _stream(stream))
    if check and st != OK:
        raise MoesdError(st, "moesd_route")
    return st


def moesd_permute(E, K, T, topk_ids, counts, offsets, perm, inv_perm, n_active, stream=None,
                  check=True):
    st = lib().moesd_permute(E, K, T, _ptr(topk_ids), _ptr(counts), _ptr(offsets), _ptr(perm),
                             _ptr(inv_perm), _ptr(n_active), _stream(stream))
    if check and st != OK:
        raise MoesdError(st, "moesd_permute")
    return st


def moesd_moe_forward(desc, weights, x, T, out, workspace, out_f32=None, workspace_bytes=None,
                      topk_ids=None, topk_w=None, counts=None, offsets=None, perm=None,
                      inv_perm=None, n_active=None, stream=None, events=None, check=True):
    """weights: a Weights struct (make_weights).  events: optional list of
    N_STAGE_EVENTS raw hipEvent_t handles (ints) -> the staged entry point."""
    nbytes = workspace_bytes if workspace_bytes is not None else (
        0 if workspace is None else workspace.numel() * workspace.element_size())
    args = [C.byref(desc), C.byref(weights) if weights is not None else None, _ptr(x), T, _ptr(out),
            _ptr(out_f32), _ptr(workspace), nbytes, _ptr(topk_ids), _ptr(topk_w), _ptr(counts),
            _ptr(offsets), _ptr(perm), _ptr(inv_perm), _ptr(n_active), _stream(stream)]
    if events is None:
        st = lib().moesd_moe_forward(*args)
    else:
        arr = (C.c_void_p * N_STAGE_EVENTS)(*[C.c_void_p(e) for e in events])
        st = lib().moesd_moe_forward_staged(*args, arr)
    if check and st != OK:
        raise MoesdError(st, "moesd_moe_forward")
    return st


def moesd_moe_forward_static(desc, weights, x, T, out, out_f32=None, topk_ids=None, topk_w=None, counts=None,
                             offsets=None, perm=None, inv_perm=None, n_active=None, stream=None, check=True):
    """moesd_moe_forward on the library's own static scratch array (no workspace argument)."""
    st = lib().moesd_moe_forward_static(C.byref(desc), C.byref(weights) if weights is not None else None, _ptr(x), T,
                                        _ptr(out), _ptr(out_f32), _ptr(topk_ids), _ptr(topk_w), _ptr(counts),
                                        _ptr(offsets), _ptr(perm), _ptr(inv_perm), _ptr(n_active), _stream(stream))
    if check and st != OK:
        raise MoesdError(st, "moesd_moe_forward_static")
    return st
