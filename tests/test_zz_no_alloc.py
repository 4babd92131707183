"""moe_decode_static (the entry point that allocates nothing) against moe_decode_ex through the raw C ABI.

Two calls in a row on the library's built-in scratch, the second with a smaller input; each is
compared with the same layer run by moe_decode_ex on a caller-owned workspace: logits and routing
bit for bit, outputs to the tolerance of two runs of the same kernels (the down projection is
accumulated with fp32 atomics whose order is free), and the first also against the CPU oracle.
"""
import ctypes
import os
import sys

import numpy as np
import pytest

from paper_2511_02237_amd import workloads as W

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2511_02237_amd", "liboea.so")


class Ex(ctypes.Structure):  # oea_decode_ex of include/oea.h
    _fields_ = [("router_bias", ctypes.c_void_p), ("token_mask", ctypes.c_void_p),
                ("logits_out", ctypes.c_void_p), ("expert_idx_out", ctypes.c_void_p),
                ("gate_w_out", ctypes.c_void_p), ("n_sel_out", ctypes.c_void_p),
                ("active_list_out", ctypes.c_void_p), ("n_active_out", ctypes.c_void_p),
                ("top_p", ctypes.c_double), ("max_p", ctypes.c_int32), ("deterministic", ctypes.c_int32),
                ("cooperative", ctypes.c_int32)]


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def test_static_entry_point_matches_workspace_entry_point(oracle):
    import torch
    assert torch.cuda.is_available(), "no GPU visible"
    lib = ctypes.CDLL(LIB)
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.oea_workspace_bytes.restype = sz
    lib.oea_workspace_bytes.argtypes = [ci] * 5
    lib.oea_workspace_init.argtypes = [vp, sz, vp]
    lib.moe_decode_ex.argtypes = [vp] * 6 + [ci] * 7 + [vp, sz, vp, ctypes.POINTER(Ex)]
    lib.moe_decode_static.argtypes = [vp] * 6 + [ci] * 7 + [vp, ctypes.POINTER(Ex)]
    dev = torch.device("cuda:0")

    def up(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    def run(entry, L, k0, t):
        """One layer through `entry` ('static' or 'ex'); returns output and taps as numpy."""
        out = torch.full((L.B, L.d), 7.0, dtype=torch.float32, device=dev)
        tap = dict(logits=torch.empty((L.B, L.N), dtype=torch.float32, device=dev),
                   expert_idx=torch.empty((L.B, L.k), dtype=torch.int32, device=dev),
                   gate_w=torch.empty((L.B, L.k), dtype=torch.float32, device=dev),
                   n_sel=torch.empty((L.B,), dtype=torch.int32, device=dev),
                   active_list=torch.empty((L.N,), dtype=torch.int32, device=dev),
                   n_active=torch.empty((1,), dtype=torch.int32, device=dev))
        ex = Ex()
        ex.logits_out, ex.expert_idx_out = tap["logits"].data_ptr(), tap["expert_idx"].data_ptr()
        ex.gate_w_out, ex.n_sel_out = tap["gate_w"].data_ptr(), tap["n_sel"].data_ptr()
        ex.active_list_out, ex.n_active_out = tap["active_list"].data_ptr(), tap["n_active"].data_ptr()
        head = [t["x"].data_ptr(), t["w_router"].data_ptr(), t["w_gate"].data_ptr(), t["w_up"].data_ptr(),
                t["w_down"].data_ptr(), out.data_ptr(), L.B, L.d, L.N, L.I, L.k, k0, 1 if L.dtype == "bf16" else 0]
        if entry == "static":
            rc = lib.moe_decode_static(*head, None, ctypes.byref(ex))
        else:
            n = lib.oea_workspace_bytes(L.B, L.d, L.N, L.I, L.k)
            ws = torch.empty(n, dtype=torch.uint8, device=dev)
            assert lib.oea_workspace_init(ws.data_ptr(), n, None) == 0
            rc = lib.moe_decode_ex(*head, ws.data_ptr(), n, None, ctypes.byref(ex))
        assert rc == 0, (entry, rc)
        torch.cuda.synchronize()
        return out.cpu().numpy(), {n_: v.cpu().numpy() for n_, v in tap.items()}

    torch.cuda.set_device(dev)
    with torch.cuda.stream(torch.cuda.default_stream(dev)):  # stream argument NULL = the default stream
        # first the benchmark shape (single fused kernel), then smaller inputs on the same scratch: fewer
        # tokens of the same layer, and a small layer that runs as three kernels
        big = W.make_layer("qwen3_30b", 4100)
        tb = {f: up(getattr(big, f)) for f in ("x", "w_router", "w_gate", "w_up", "w_down")}
        small = W.Layer(**{**big.__dict__, "B": 5, "x": np.ascontiguousarray(big.x[:5])})
        ts = dict(tb, x=up(small.x))
        mid = W.make_layer("mid_bf16", 4101)
        tm = {f: up(getattr(mid, f)) for f in ("x", "w_router", "w_gate", "w_up", "w_down")}
        cases = [("30B shape B=16 k0=3", big, tb, 3), ("30B shape B=5 k0=2", small, ts, 2),
                 ("mid shape k0=3", mid, tm, 3), ("30B shape B=16 k0=8", big, tb, 8)]
        # all static calls first, back to back on the shared scratch; then the reference runs
        got = []
        for name, L, t, k0 in cases:
            say("static:", name)
            got.append(run("static", L, k0, t))
        for (name, L, t, k0), (o_s, tap_s) in zip(cases, got):
            say("workspace:", name)
            o_w, tap_w = run("ex", L, k0, t)
            assert np.array_equal(tap_s["logits"].view(np.uint32), tap_w["logits"].view(np.uint32)), name
            for f in ("expert_idx", "n_sel", "active_list", "n_active"):
                assert np.array_equal(tap_s[f], tap_w[f]), (name, f)
            assert np.array_equal(tap_s["gate_w"], tap_w["gate_w"]), name
            assert np.isfinite(o_s).all()
            drift = np.abs(o_s - o_w).max() / np.abs(o_w).max()
            assert drift <= 1e-5, "%s: static vs workspace entry point %.3e" % (name, drift)
            ref = oracle.moe_decode(L.x, L.w_router, L.w_gate, L.w_up, L.w_down, L.k, k0)
            assert np.array_equal(tap_s["expert_idx"], ref["expert_idx"]), name
            err = np.abs(o_s - ref["out"]).max() / np.abs(ref["out"]).max()
            assert err <= 5e-3, "%s: %.3e against the oracle" % (name, err)
            say("%s: T=%d, static vs workspace %.1e, vs oracle %.2e" % (name, int(tap_s["n_active"][0]), drift, err))
        # beyond the built-in scratch: refused before anything is enqueued
        rc = lib.moe_decode_static(tb["x"].data_ptr(), tb["w_router"].data_ptr(), tb["w_gate"].data_ptr(),
                                   tb["w_up"].data_ptr(), tb["w_down"].data_ptr(), tb["x"].data_ptr(), 1024, 4096,
                                   128, 1536, 8, 3, 1, None, None)
        assert rc == -9
