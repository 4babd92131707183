"""ctypes front end of the C oracle (oracle/oea_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  Nothing in the product package imports it, and it imports nothing from the
product package.  All arrays are numpy, on the host.

dtype convention: a float32 array is taken as fp32 storage, a uint16 array as bf16 bit patterns.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None
F32, BF16 = 0, 1


def lib():
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        L.oracle_num_threads.restype = ctypes.c_int
        L.oracle_set_num_threads.argtypes = [ctypes.c_int]
        L.oracle_oea_route.restype = ctypes.c_int
        L.oracle_oea_route_general.restype = ctypes.c_int
        L.oracle_moe_decode.restype = ctypes.c_int
        _LIB = L
    return _LIB


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _dtype_of(a):
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError("oracle arrays must be float32 or uint16 (bf16 bits), got %s" % a.dtype)


def _c(a, dt=None):
    a = np.ascontiguousarray(a)
    if dt is not None and a.dtype != dt:
        a = a.astype(dt)
    return a


def num_threads():
    return int(lib().oracle_num_threads())


def set_num_threads(n):
    lib().oracle_set_num_threads(int(n))


def router_logits(x, w_router, bias=None):
    """fp32 router logits [B,N] (fp64 accumulate, one rounding)."""
    x, w_router = _c(x), _c(w_router)
    dt = _dtype_of(x)
    assert _dtype_of(w_router) == dt
    B, d = x.shape
    N = w_router.shape[0]
    assert w_router.shape == (N, d)
    bias = None if bias is None else _c(bias, np.float32)
    out = np.empty((B, N), np.float32)
    lib().oracle_router_logits(_p(x), _p(w_router), _p(bias), B, d, N, dt, _p(out))
    return out


def softmax(logits):
    logits = _c(logits, np.float32)
    B, N = logits.shape
    R = np.empty((B, N), np.float64)
    lib().oracle_softmax(_p(logits), B, N, _p(R))
    return R


def rank(logits):
    logits = _c(logits, np.float32)
    B, N = logits.shape
    r = np.empty((B, N), np.int32)
    lib().oracle_rank(_p(logits), B, N, _p(r))
    return r


def route(logits, k, k0, token_mask=None):
    """Simplified OEA (Algorithm 1).  Returns dict(expert_idx, gate_w, n_sel, active_list, n_active)."""
    logits = _c(logits, np.float32)
    B, N = logits.shape
    idx = np.empty((B, k), np.int32)
    gw = np.empty((B, k), np.float64)
    ns = np.empty((B,), np.int32)
    al = np.empty((N,), np.int32)
    T = ctypes.c_int32(0)
    tm = None if token_mask is None else _c(token_mask, np.uint8)
    rc = lib().oracle_oea_route(_p(logits), _p(tm), B, N, int(k), int(k0), _p(idx), _p(gw), _p(ns),
                                _p(al), ctypes.byref(T))
    if rc != 0:
        raise ValueError("oracle_oea_route: illegal parameters B=%d N=%d k=%d k0=%d" % (B, N, k, k0))
    return dict(expert_idx=idx, gate_w=gw, n_sel=ns, active_list=al, n_active=int(T.value))


def route_general(logits, k0, p, k_max, max_p, token_mask=None):
    """General OEA (Algorithm 2).  Output width is max(k0, k_max)."""
    logits = _c(logits, np.float32)
    B, N = logits.shape
    width = max(int(k0), int(k_max))
    idx = np.empty((B, width), np.int32)
    gw = np.empty((B, width), np.float64)
    ns = np.empty((B,), np.int32)
    nb = np.empty((B,), np.int32)
    al = np.empty((N,), np.int32)
    T = ctypes.c_int32(0)
    tm = None if token_mask is None else _c(token_mask, np.uint8)
    rc = lib().oracle_oea_route_general(_p(logits), _p(tm), B, N, int(k0), ctypes.c_double(p),
                                        int(k_max), int(max_p), _p(idx), _p(gw), _p(ns), _p(nb),
                                        _p(al), ctypes.byref(T))
    if rc != 0:
        raise ValueError("oracle_oea_route_general: illegal parameters")
    return dict(expert_idx=idx, gate_w=gw, n_sel=ns, n_base=nb, active_list=al, n_active=int(T.value))


def expert_ffn(x_row, w_gate, w_up, w_down):
    """One SwiGLU expert on one token: y [d] fp64."""
    x_row, w_gate, w_up, w_down = _c(x_row), _c(w_gate), _c(w_up), _c(w_down)
    dt = _dtype_of(x_row)
    I, d = w_gate.shape
    assert w_up.shape == (I, d) and w_down.shape == (d, I) and x_row.shape == (d,)
    h = np.empty((I,), np.float64)
    y = np.empty((d,), np.float64)
    lib().oracle_expert_ffn(_p(x_row), _p(w_gate), _p(w_up), _p(w_down), d, I, dt, _p(h), _p(y))
    return y


def moe_combine(x, w_gate, w_up, w_down, expert_idx, gate_w):
    """Eq. 1 over given expert sets and weights: out [B,d] fp64."""
    x, w_gate, w_up, w_down = _c(x), _c(w_gate), _c(w_up), _c(w_down)
    dt = _dtype_of(x)
    B, d = x.shape
    N, I, _ = w_gate.shape
    expert_idx = _c(expert_idx, np.int32)
    gate_w = _c(gate_w, np.float64)
    kk = expert_idx.shape[1]
    out = np.empty((B, d), np.float64)
    lib().oracle_moe_combine(_p(x), _p(w_gate), _p(w_up), _p(w_down), _p(expert_idx), _p(gate_w),
                             B, d, N, I, kk, dt, _p(out))
    return out


def moe_decode(x, w_router, w_gate, w_up, w_down, k, k0, router_bias=None, token_mask=None):
    """Whole layer.  Returns dict(out fp64 [B,d], logits, expert_idx, gate_w, n_sel, active_list, n_active)."""
    x, w_router, w_gate, w_up, w_down = _c(x), _c(w_router), _c(w_gate), _c(w_up), _c(w_down)
    dt = _dtype_of(x)
    for a in (w_router, w_gate, w_up, w_down):
        assert _dtype_of(a) == dt
    B, d = x.shape
    N, I, d2 = w_gate.shape
    assert d2 == d and w_router.shape == (N, d) and w_up.shape == (N, I, d) and w_down.shape == (N, d, I)
    out = np.empty((B, d), np.float64)
    logits = np.empty((B, N), np.float32)
    idx = np.empty((B, k), np.int32)
    gw = np.empty((B, k), np.float64)
    ns = np.empty((B,), np.int32)
    al = np.empty((N,), np.int32)
    T = ctypes.c_int32(0)
    bias = None if router_bias is None else _c(router_bias, np.float32)
    tm = None if token_mask is None else _c(token_mask, np.uint8)
    rc = lib().oracle_moe_decode(_p(x), _p(w_router), _p(w_gate), _p(w_up), _p(w_down), _p(bias),
                                 _p(tm), B, d, N, I, int(k), int(k0), dt, _p(out), _p(logits),
                                 _p(idx), _p(gw), _p(ns), _p(al), ctypes.byref(T))
    if rc != 0:
        raise ValueError("oracle_moe_decode: illegal parameters")
    return dict(out=out, logits=logits, expert_idx=idx, gate_w=gw, n_sel=ns, active_list=al,
                n_active=int(T.value))
