"""Thin ctypes binding over liboea.so: argument marshalling only.

Every step of the layer runs in the HIP kernels of the library; torch is used for device memory
and for the current stream handle, nothing else.  There is no CPU fallback: if the library is
missing or fails to load this module raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# OEA_LIB selects another build of the same library (bench.py --timeline loads the measurement variant)
LIB_PATH = os.environ.get("OEA_LIB") or os.path.join(_HERE, "liboea.so")

OEA_F32, OEA_BF16 = 0, 1
OEA_OK = 0
STATUS = {"OEA_ERR_NULL": -1, "OEA_ERR_SHAPE": -2, "OEA_ERR_K": -3, "OEA_ERR_ALIGN": -4,
          "OEA_ERR_WORKSPACE": -5, "OEA_ERR_DTYPE": -6, "OEA_ERR_HIP": -7, "OEA_ERR_TIMEOUT": -8,
          "OEA_ERR_LIMIT": -9, "OEA_ERR_WORKSPACE_STATE": -10}
EXPORTS = ("oea_status_string", "oea_workspace_bytes", "oea_workspace_bytes_deterministic", "oea_workspace_init", "oea_route", "oea_route_batched", "oea_route_general",
           "moe_decode", "moe_decode_ex", "moe_decode_static", "oea_workspace_check")
TEST_EXPORTS = ("moe_decode_test", "oea_read_probe")  # include/oea_testing.h


class OeaError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("liboea: %s (%d)" % (text, code))
        self.code = code


class DecodeEx(ctypes.Structure):
    _fields_ = [("router_bias", ctypes.c_void_p), ("token_mask", ctypes.c_void_p),
                ("logits_out", ctypes.c_void_p), ("expert_idx_out", ctypes.c_void_p),
                ("gate_w_out", ctypes.c_void_p), ("n_sel_out", ctypes.c_void_p),
                ("active_list_out", ctypes.c_void_p), ("n_active_out", ctypes.c_void_p),
                ("top_p", ctypes.c_double), ("max_p", ctypes.c_int32), ("deterministic", ctypes.c_int32),
                ("cooperative", ctypes.c_int32)]


class TestOpts(ctypes.Structure):  # oea_test_opts of include/oea_testing.h
    _fields_ = [("kernel_path", ctypes.c_int32), ("spin_limit", ctypes.c_uint32),
                ("h_kernel_events", ctypes.POINTER(ctypes.c_void_p))]


_lib = None


def lib():
    """Load liboea.so (built by `python -m paper_2511_02237_amd.build`).  Raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise OeaError(-100, "HIP library %s is not built; run python -m paper_2511_02237_amd.build" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        L.oea_status_string.restype = ctypes.c_char_p
        L.oea_status_string.argtypes = [ci]
        L.oea_workspace_bytes.restype = sz
        L.oea_workspace_bytes.argtypes = [ci] * 5
        L.oea_workspace_bytes_deterministic.restype = sz
        L.oea_workspace_bytes_deterministic.argtypes = [ci] * 5
        L.oea_workspace_init.restype = ci
        L.oea_workspace_init.argtypes = [vp, sz, vp]
        L.oea_route.restype = ci
        L.oea_route.argtypes = [vp, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp]
        L.oea_route_batched.restype = ci
        L.oea_route_batched.argtypes = [vp, vp, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp]
        L.oea_route_general.restype = ci
        L.oea_route_general.argtypes = [vp, vp, ci, ci, ci, ctypes.c_double, ci, ci, vp, vp, vp, vp, vp, vp, vp]
        L.oea_workspace_check.restype = ci
        L.oea_workspace_check.argtypes = [vp, sz, vp]
        L.oea_read_probe.restype = ci
        L.oea_read_probe.argtypes = [vp, sz, vp, vp]
        L.moe_decode.restype = ci
        L.moe_decode.argtypes = [vp] * 6 + [ci] * 7 + [vp, sz, vp]
        L.moe_decode_ex.restype = ci
        L.moe_decode_ex.argtypes = [vp] * 6 + [ci] * 7 + [vp, sz, vp, ctypes.POINTER(DecodeEx)]
        L.moe_decode_test.restype = ci
        L.moe_decode_test.argtypes = [vp] * 6 + [ci] * 7 + [vp, sz, vp, ctypes.POINTER(DecodeEx), ctypes.POINTER(TestOpts)]
        L.moe_decode_static.restype = ci
        L.moe_decode_static.argtypes = [vp] * 6 + [ci] * 7 + [vp, ctypes.POINTER(DecodeEx)]
        _lib = L
    return _lib


def status_string(code):
    return lib().oea_status_string(int(code)).decode()


def _check(code):
    if code != OEA_OK:
        raise OeaError(code, status_string(code))


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _dtype_code(t):
    if t.dtype == torch.float32:
        return OEA_F32
    if t.dtype == torch.bfloat16:
        return OEA_BF16
    raise TypeError("x and weights must be float32 or bfloat16, got %s" % t.dtype)


def workspace_bytes(B, d, N, I, k, deterministic=False):
    f = lib().oea_workspace_bytes_deterministic if deterministic else lib().oea_workspace_bytes
    return int(f(B, d, N, I, k))


def new_workspace(B, d, N, I, k, device="cuda", stream=None, deterministic=False):
    """Allocate (torch) and prepare (library) a workspace for moe_decode."""
    n = workspace_bytes(B, d, N, I, k, deterministic)
    if n == 0:
        raise OeaError(STATUS["OEA_ERR_SHAPE"], status_string(STATUS["OEA_ERR_SHAPE"]))
    ws = torch.empty(n, dtype=torch.uint8, device=device)
    workspace_init(ws, stream)
    return ws


def workspace_init(ws, stream=None):
    """Prepare (or prepare again) the control words of a workspace."""
    _check(lib().oea_workspace_init(_ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))


def oea_route(router_logits, k, k0, stream=None, out=None):
    """router_logits [B,N] float32 cuda -> dict(expert_idx, gate_w, n_sel, active_list, n_active) on device."""
    assert router_logits.is_cuda and router_logits.dtype == torch.float32 and router_logits.is_contiguous()
    B, N = router_logits.shape
    dev = router_logits.device
    if out is None:
        out = dict(expert_idx=torch.empty((B, k), dtype=torch.int32, device=dev),
                   gate_w=torch.empty((B, k), dtype=torch.float32, device=dev),
                   n_sel=torch.empty((B,), dtype=torch.int32, device=dev),
                   active_list=torch.empty((N,), dtype=torch.int32, device=dev),
                   n_active=torch.empty((1,), dtype=torch.int32, device=dev))
    _check(lib().oea_route(_ptr(router_logits), B, N, int(k), int(k0), _ptr(out["expert_idx"]),
                           _ptr(out["gate_w"]), _ptr(out["n_sel"]), _ptr(out["active_list"]),
                           _ptr(out["n_active"]), _stream(stream)))
    return out


def workspace_check(ws, stream=None):
    """Synchronise and raise OeaError (OEA_ERR_TIMEOUT) if a wait inside a kernel has given up on `ws`."""
    _check(lib().oea_workspace_check(_ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))


def read_probe(buf, stream=None):
    """Enqueue one streaming read of the tensor `buf` (measurement aid, see oea_read_probe)."""
    assert buf.is_cuda and buf.is_contiguous()
    _check(lib().oea_read_probe(_ptr(buf), buf.numel() * buf.element_size(), None, _stream(stream)))


def oea_route_batched(router_logits, k, k0, token_mask=None, stream=None):
    """router_logits [L,B,N] float32 cuda: L independent positions routed in one launch."""
    assert router_logits.is_cuda and router_logits.dtype == torch.float32 and router_logits.is_contiguous()
    L, B, N = router_logits.shape
    dev = router_logits.device
    if token_mask is not None:
        assert token_mask.is_cuda and token_mask.dtype == torch.uint8 and tuple(token_mask.shape) == (L, B)
        assert token_mask.is_contiguous()
    out = dict(expert_idx=torch.empty((L, B, k), dtype=torch.int32, device=dev),
               gate_w=torch.empty((L, B, k), dtype=torch.float32, device=dev),
               n_sel=torch.empty((L, B), dtype=torch.int32, device=dev),
               active_list=torch.empty((L, N), dtype=torch.int32, device=dev),
               n_active=torch.empty((L,), dtype=torch.int32, device=dev))
    _check(lib().oea_route_batched(_ptr(router_logits), _ptr(token_mask), L, B, N, int(k), int(k0),
                                   _ptr(out["expert_idx"]), _ptr(out["gate_w"]), _ptr(out["n_sel"]),
                                   _ptr(out["active_list"]), _ptr(out["n_active"]), _stream(stream)))
    return out


def oea_route_general(router_logits, k0, p, k_max, max_p, token_mask=None, stream=None, out=None):
    """General OEA routing (Algorithm 2).  Returns dict(expert_idx [B,kw], gate_w, n_sel, n_base,
    active_list, n_active) on device, kw = max(k0, k_max)."""
    assert router_logits.is_cuda and router_logits.dtype == torch.float32 and router_logits.is_contiguous()
    B, N = router_logits.shape
    dev = router_logits.device
    kw = max(int(k0), int(k_max))
    if token_mask is not None:
        assert token_mask.is_cuda and token_mask.dtype == torch.uint8 and token_mask.numel() == B
    if out is None:
        out = dict(expert_idx=torch.empty((B, kw), dtype=torch.int32, device=dev),
                   gate_w=torch.empty((B, kw), dtype=torch.float32, device=dev),
                   n_sel=torch.empty((B,), dtype=torch.int32, device=dev),
                   n_base=torch.empty((B,), dtype=torch.int32, device=dev),
                   active_list=torch.empty((N,), dtype=torch.int32, device=dev),
                   n_active=torch.empty((1,), dtype=torch.int32, device=dev))
    _check(lib().oea_route_general(_ptr(router_logits), _ptr(token_mask), B, N, int(k0), float(p), int(k_max),
                                   int(max_p), _ptr(out["expert_idx"]), _ptr(out["gate_w"]), _ptr(out["n_sel"]),
                                   _ptr(out["n_base"]), _ptr(out["active_list"]), _ptr(out["n_active"]),
                                   _stream(stream)))
    return out


def _layer_args(x, w_router, w_gate, w_up, w_down, k, k0, out):
    for t in (x, w_router, w_gate, w_up, w_down):
        assert t.is_cuda and t.is_contiguous()
    dt = _dtype_code(x)
    for t in (w_router, w_gate, w_up, w_down):
        assert _dtype_code(t) == dt
    B, d = x.shape
    N, I, d2 = w_gate.shape
    assert d2 == d and tuple(w_router.shape) == (N, d) and tuple(w_up.shape) == (N, I, d)
    assert tuple(w_down.shape) == (N, d, I)
    if out is None:
        out = torch.empty((B, d), dtype=torch.float32, device=x.device)
    args = [_ptr(x), _ptr(w_router), _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(out), B, d, N, I, int(k),
            int(k0), dt]
    return args, out, (B, d, N, I)


def _extras(shape, k, dev, router_bias, token_mask, taps, top_p, max_p, cooperative=False, deterministic=False):
    """The oea_decode_ex struct for the optional inputs and taps (None if none is asked for)."""
    B, d, N, I = shape
    if not taps and router_bias is None and token_mask is None and top_p is None and max_p is None \
            and not cooperative and not deterministic:
        return None, None
    ex = DecodeEx()
    tap = None
    ex.cooperative = 1 if cooperative else 0
    ex.deterministic = 1 if deterministic else 0
    if top_p is not None:
        ex.top_p = float(top_p)
    if max_p is not None:
        ex.max_p = int(max_p)
    if router_bias is not None:
        assert router_bias.is_cuda and router_bias.dtype == torch.float32 and router_bias.numel() == N
        ex.router_bias = router_bias.data_ptr()
    if token_mask is not None:
        assert token_mask.is_cuda and token_mask.dtype == torch.uint8 and token_mask.numel() == B
        ex.token_mask = token_mask.data_ptr()
    if taps:
        tap = dict(logits=torch.empty((B, N), dtype=torch.float32, device=dev),
                   expert_idx=torch.empty((B, k), dtype=torch.int32, device=dev),
                   gate_w=torch.empty((B, k), dtype=torch.float32, device=dev),
                   n_sel=torch.empty((B,), dtype=torch.int32, device=dev),
                   active_list=torch.empty((N,), dtype=torch.int32, device=dev),
                   n_active=torch.empty((1,), dtype=torch.int32, device=dev))
        ex.logits_out = tap["logits"].data_ptr()
        ex.expert_idx_out = tap["expert_idx"].data_ptr()
        ex.gate_w_out = tap["gate_w"].data_ptr()
        ex.n_sel_out = tap["n_sel"].data_ptr()
        ex.active_list_out = tap["active_list"].data_ptr()
        ex.n_active_out = tap["n_active"].data_ptr()
    return ex, tap


def test_opts(kernel_path=None, spin_limit=None, kernel_events=None):
    """oea_test_opts (include/oea_testing.h) or None if nothing is set.  kernel_events: ctypes array of
    6 hipEvent_t handles."""
    if kernel_path is None and spin_limit is None and kernel_events is None:
        return None
    o = TestOpts()
    o.kernel_path = int(kernel_path or 0)
    o.spin_limit = int(spin_limit or 0)
    if kernel_events is not None:
        o.h_kernel_events = ctypes.cast(kernel_events, ctypes.POINTER(ctypes.c_void_p))
    return o


def moe_decode(x, w_router, w_gate, w_up, w_down, k, k0, workspace, out=None, stream=None,
               router_bias=None, token_mask=None, taps=False, top_p=None, max_p=None, cooperative=False,
               deterministic=False, kernel_path=None, spin_limit=None, kernel_events=None):
    """One decode-time MoE layer with OEA routing.  Returns out [B,d] float32 (and a dict of routing
    taps when taps=True).  kernel_path, spin_limit and kernel_events are the test aids of
    moe_decode_test."""
    args, out, shape = _layer_args(x, w_router, w_gate, w_up, w_down, k, k0, out)
    args += [_ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)]
    ex, tap = _extras(shape, k, x.device, router_bias, token_mask, taps, top_p, max_p, cooperative, deterministic)
    opts = test_opts(kernel_path, spin_limit, kernel_events)
    if opts is not None:
        _check(lib().moe_decode_test(*args, None if ex is None else ctypes.byref(ex), ctypes.byref(opts)))
    elif ex is None:
        _check(lib().moe_decode(*args))
    else:
        _check(lib().moe_decode_ex(*args, ctypes.byref(ex)))
    return (out, tap) if taps else out


def moe_decode_static(x, w_router, w_gate, w_up, w_down, k, k0, out=None, stream=None, router_bias=None,
                      token_mask=None, taps=False, top_p=None, max_p=None, deterministic=False):
    """moe_decode on the scratch built into the library (no workspace argument, nothing allocated by
    the call; pass `out` to keep torch from allocating the result too)."""
    args, out, shape = _layer_args(x, w_router, w_gate, w_up, w_down, k, k0, out)
    ex, tap = _extras(shape, k, x.device, router_bias, token_mask, taps, top_p, max_p, False, deterministic)
    _check(lib().moe_decode_static(*args, _stream(stream), None if ex is None else ctypes.byref(ex)))
    return (out, tap) if taps else out


def to_device(a, device="cuda"):
    """numpy array from `workloads` (float32, or uint16 bf16 bits) -> torch tensor on the device."""
    import numpy as np

    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)
