"""ctypes binding of the C oracle (oracle/moe_oracle.c).  Test infrastructure.

All tensors are numpy arrays: bf16 tensors are uint16 words, results are fp64.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build


class OracleDesc(C.Structure):
    _fields_ = [("d", C.c_int32), ("E", C.c_int32), ("top_k", C.c_int32), ("inter", C.c_int32),
                ("shared_inter", C.c_int32), ("score_func", C.c_int32),
                ("renormalize", C.c_int32), ("shared_gate", C.c_int32),
                ("routed_scale", C.c_double), ("n_group", C.c_int32), ("topk_group", C.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build()
        L = C.CDLL(path)
        L.oracle_expected_active_experts.restype = C.c_double
        L.oracle_expected_active_experts.argtypes = [C.c_int32, C.c_int32, C.c_int64]
        L.oracle_expected_tokens_per_expert.restype = C.c_double
        L.oracle_expected_tokens_per_expert.argtypes = [C.c_int32, C.c_int32, C.c_int64]
        L.oracle_expected_active_experts_p.restype = C.c_double
        L.oracle_token_threshold.restype = C.c_int64
        L.oracle_token_threshold.argtypes = [C.c_int32, C.c_int32, C.c_double]
        L.oracle_route.restype = C.c_int32
        L.oracle_permute.restype = C.c_int32
        L.oracle_moe_forward.restype = C.c_int32
        L.oracle_moe_forward_fp8.restype = C.c_int32
        L.oracle_fp8_e4m3_decode.restype = None
        L.oracle_ffn_row_f32.restype = C.c_int32
        L.oracle_ffn_row_f64.restype = C.c_int32
        L.oracle_round_bf16.restype = None
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _u8(a):
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint8, a.dtype
    return a


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, np.float32)


def fp8_decode(codes):
    """E4M3 codes (uint8, any shape) -> fp64 values (NaN for the two NaN codes)."""
    codes = _u8(codes)
    out = np.empty(codes.shape, np.float64)
    lib().oracle_fp8_e4m3_decode(_p(codes), C.c_int64(codes.size), _p(out))
    return out


def _u16(a):
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def desc_of(shape) -> OracleDesc:
    """shape: any object with d, E, top_k, inter, shared_inter, score_func,
    renormalize, shared_gate, routed_scale attributes."""
    return OracleDesc(shape.d, shape.E, shape.top_k, shape.inter, shape.shared_inter,
                      shape.score_func, shape.renormalize, shape.shared_gate,
                      float(shape.routed_scale), int(getattr(shape, "n_group", 0)),
                      int(getattr(shape, "topk_group", 0)))


def expected_active_experts(E, K, t):
    return lib().oracle_expected_active_experts(E, K, t)


def expected_active_experts_p(p, t):
    """N(t) for per-expert activation probabilities p (sums to K): sum_e 1 - (1 - p_e)^t."""
    p = np.ascontiguousarray(p, np.float64)
    return lib().oracle_expected_active_experts_p(_p(p), C.c_int32(p.size), C.c_int64(t))


def expected_tokens_per_expert(E, K, t):
    return lib().oracle_expected_tokens_per_expert(E, K, t)


def token_threshold(E, K, tau):
    return lib().oracle_token_threshold(E, K, tau)


def route(shape, x, w_router, router_bias=None):
    """-> (ids [T,K] int32, w [T,K] f64, logits [T,E] f64)"""
    x = _u16(x); w_router = _u16(w_router)
    T = x.shape[0]
    d = desc_of(shape)
    ids = np.empty((T, shape.top_k), np.int32)
    w = np.empty((T, shape.top_k), np.float64)
    logits = np.empty((T, shape.E), np.float64)
    b = None if router_bias is None else np.ascontiguousarray(router_bias, np.float32)
    rc = lib().oracle_route(C.byref(d), _p(x), _p(w_router), _p(b), C.c_int32(T), _p(logits),
                            _p(ids), _p(w))
    if rc:
        raise ValueError(f"oracle_route failed: {rc}")
    return ids, w, logits


def permute(E, K, ids):
    """ids [T,K] int32 -> dict(counts, offsets, perm, inv, n_active)"""
    ids = np.ascontiguousarray(ids, np.int32)
    T = ids.size // K
    n = T * K
    counts = np.empty(E, np.int32)
    offsets = np.empty(E + 1, np.int32)
    perm = np.empty(n, np.int32)
    inv = np.empty(n, np.int32)
    na = np.zeros(1, np.int32)
    rc = lib().oracle_permute(C.c_int32(E), C.c_int32(K), C.c_int32(T), _p(ids), _p(counts),
                              _p(offsets), _p(perm), _p(inv), _p(na))
    if rc:
        raise ValueError(f"oracle_permute failed: {rc}")
    return dict(counts=counts, offsets=offsets, perm=perm, inv=inv, n_active=int(na[0]))


def moe_forward(shape, weights: dict, x, tokens=None):
    """Full layer.  weights: dict with the keys of synth.make_layer.  tokens:
    optional list of token indices whose output rows are wanted.
    -> dict(out [n,d] f64, out_bf16 [n,d] u16, ids, w, counts, offsets, perm, inv,
            n_active, gate [T] f64)"""
    x = _u16(x)
    T = x.shape[0]
    K, E, dd = shape.top_k, shape.E, shape.d
    d = desc_of(shape)
    tl = None
    n_out = T
    if tokens is not None:
        tl = np.ascontiguousarray(tokens, np.int32)
        n_out = tl.size
    out = np.zeros((n_out, dd), np.float64)
    outb = np.zeros((n_out, dd), np.uint16)
    ids = np.empty((T, K), np.int32)
    w = np.empty((T, K), np.float64)
    counts = np.empty(E, np.int32)
    offsets = np.empty(E + 1, np.int32)
    perm = np.empty(T * K, np.int32)
    inv = np.empty(T * K, np.int32)
    na = np.zeros(1, np.int32)
    gate = np.ones(T, np.float64)
    b = weights.get("router_bias")
    b = None if b is None else np.ascontiguousarray(b, np.float32)
    mats = ("w_gate", "w_up", "w_down", "ws_gate", "ws_up", "ws_down")
    tail = (C.c_int32(T), _p(tl), C.c_int32(n_out if tl is not None else 0), _p(out), _p(outb), _p(ids), _p(w),
            _p(counts), _p(offsets), _p(perm), _p(inv), _p(na), _p(gate))
    wr, wsg = _u16(weights.get("w_router")), _u16(weights.get("w_shared_gate"))
    if weights.get("w_gate_scale") is not None:     # E4M3 codes + one fp32 scale per output row
        args = []
        for k in mats:
            args += [_p(_u8(weights.get(k))), _p(_f32(weights.get(k + "_scale")))]
        rc = lib().oracle_moe_forward_fp8(C.byref(d), _p(x), _p(wr), _p(b), *args, _p(wsg), *tail)
    else:
        wt = {k: _u16(weights.get(k)) for k in mats}
        rc = lib().oracle_moe_forward(C.byref(d), _p(x), _p(wr), _p(b), *[_p(wt[k]) for k in mats], _p(wsg), *tail)
    if rc:
        raise ValueError(f"oracle_moe_forward failed: {rc}")
    return dict(out=out, out_bf16=outb, ids=ids, w=w, counts=counts, offsets=offsets, perm=perm,
                inv=inv, n_active=int(na[0]), gate=gate)


def ffn_row(xrow, wg, wu, wd, f32=False):
    xrow = _u16(xrow); wg = _u16(wg); wu = _u16(wu); wd = _u16(wd)
    I, d = wg.shape
    if f32:
        y = np.empty(d, np.float32)
        lib().oracle_ffn_row_f32(_p(xrow), _p(wg), _p(wu), _p(wd), C.c_int32(d), C.c_int32(I), _p(y))
    else:
        y = np.empty(d, np.float64)
        lib().oracle_ffn_row_f64(_p(xrow), _p(wg), _p(wu), _p(wd), C.c_int32(d), C.c_int32(I), _p(y))
    return y


def round_bf16(v):
    v = np.ascontiguousarray(v, np.float64)
    out = np.empty(v.shape, np.uint16)
    lib().oracle_round_bf16(_p(v), C.c_int64(v.size), _p(out))
    return out
