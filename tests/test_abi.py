"""The C-ABI library: loads, exports every declared symbol, host-side argument checks (no GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "oea.h")
TEST_HEADER = os.path.join(ROOT, "include", "oea_testing.h")
LIB = os.path.join(ROOT, "paper_2511_02237_amd", "liboea.so")


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(LIB):
        from paper_2511_02237_amd import build
        build.build(force=True)
    lib = ctypes.CDLL(LIB)
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.oea_status_string.restype = ctypes.c_char_p
    lib.oea_status_string.argtypes = [ci]
    lib.oea_workspace_bytes.restype = sz
    lib.oea_workspace_bytes.argtypes = [ci] * 5
    lib.oea_workspace_init.argtypes = [vp, sz, vp]
    lib.oea_read_probe.argtypes = [vp, sz, vp, vp]
    lib.oea_workspace_check.argtypes = [vp, sz, vp]
    lib.oea_route.argtypes = [vp, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp]
    lib.oea_route_batched.argtypes = [vp, vp, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp]
    lib.oea_route_general.argtypes = [vp, vp, ci, ci, ci, ctypes.c_double, ci, ci, vp, vp, vp, vp, vp, vp, vp]
    lib.moe_decode.argtypes = [vp] * 6 + [ci] * 7 + [vp, sz, vp]
    lib.moe_decode_ex.argtypes = [vp] * 6 + [ci] * 7 + [vp, sz, vp, vp]
    lib.moe_decode_static.argtypes = [vp] * 6 + [ci] * 7 + [vp, vp]
    lib.moe_decode_test.argtypes = [vp] * 6 + [ci] * 7 + [vp, sz, vp, vp, vp]
    return lib


def declared_functions(header=HEADER):
    text = open(header).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(\w+)\s*\([^;{}]*\)\s*;", text)))


def test_every_declared_symbol_is_exported(L):
    names = declared_functions()
    assert {"oea_route", "oea_route_general", "moe_decode", "moe_decode_ex", "oea_workspace_bytes", "oea_workspace_init",
            "oea_status_string"} <= set(names)
    for n in names + declared_functions(TEST_HEADER):
        assert hasattr(L, n), n
    # the product header carries no test or measurement aid
    assert not {"oea_set_kernel_path", "oea_read_probe", "moe_decode_test"} & set(names)
    assert "spin_limit" not in open(HEADER).read() and "h_kernel_events" not in open(HEADER).read()


def test_status_strings(L):
    seen = set()
    for code in range(0, -11, -1):
        s = L.oea_status_string(code).decode()
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 11
    assert L.oea_status_string(-99).decode() == "unknown status"


def test_workspace_bytes_is_pure_and_monotone(L):
    a = L.oea_workspace_bytes(16, 2048, 128, 768, 8)
    assert a == L.oea_workspace_bytes(16, 2048, 128, 768, 8)
    # the hidden buffer B*k*I in the wider type must fit
    assert a >= 16 * 8 * 768 * 4 + 16 * 128 * 4
    assert a < 2 * 1024 * 1024
    assert L.oea_workspace_bytes(32, 2048, 128, 768, 8) > a
    assert a % 256 == 0
    for bad in [(0, 2048, 128, 768, 8), (16, 2048, 0, 768, 8), (16, 2048, 128, 768, 0),
                (16, 2048, 513, 768, 8), (16, 9000, 128, 768, 8), (2000, 2048, 128, 768, 8)]:
        assert L.oea_workspace_bytes(*bad) == 0


P = 0x10000  # fake, 16-byte aligned, never dereferenced: every check below fails before any enqueue


def test_route_argument_checks(L):
    ok = [P, 16, 128, 8, 3, P, P, P, P, P, None]
    def call(**kw):
        a = list(ok)
        for i, v in kw.items():
            a[int(i[1:])] = v
        return L.oea_route(*a)
    assert call(a0=None) == -1 and call(a5=None) == -1 and call(a9=None) == -1
    assert call(a1=0) == -2 and call(a1=1025) == -2 and call(a2=0) == -2 and call(a2=513) == -2
    assert call(a4=0) == -3 and call(a4=9) == -3 and call(a3=129) == -3 and call(a3=33, a4=33) == -3


def test_route_batched_argument_checks(L):
    ok = [P, None, 4, 16, 128, 8, 3, P, P, P, P, P, None]
    assert L.oea_route_batched(*([None] + ok[1:])) == -1
    assert L.oea_route_batched(*(ok[:2] + [0] + ok[3:])) == -2
    assert L.oea_route_batched(*(ok[:2] + [70000] + ok[3:])) == -2
    assert L.oea_route_batched(*(ok[:6] + [9] + ok[7:])) == -3


def test_route_general_argument_checks(L):
    # logits, mask, B, N, k0, p, k_max, max_p, expert_idx, gate_w, n_sel, n_base, active_list, n_active, stream
    ok = [P, None, 16, 128, 3, 0.9, 8, 128, P, P, P, None, P, P, None]
    def call(**kw):
        a = list(ok)
        for i, v in kw.items():
            a[int(i[1:])] = v
        return L.oea_route_general(*a)
    assert call(a0=None) == -1 and call(a8=None) == -1 and call(a13=None) == -1
    assert call(a2=0) == -2 and call(a2=1025) == -2 and call(a3=0) == -2 and call(a3=513) == -2
    assert call(a4=0) == -3 and call(a4=129) == -3 and call(a6=0) == -3 and call(a6=33) == -3
    assert call(a7=0) == -3 and call(a7=129) == -3
    assert call(a5=0.0) == -3 and call(a5=1.5) == -3 and call(a5=float("nan")) == -3


def test_decode_argument_checks(L):
    big = 1 << 30
    ok = [P, P, P, P, P, P, 16, 2048, 128, 768, 8, 3, 1, P, big, None]
    def call(**kw):
        a = list(ok)
        for i, v in kw.items():
            a[int(i[1:])] = v
        return L.moe_decode(*a)
    for i in (0, 1, 2, 3, 4, 5, 13):
        assert call(**{"a%d" % i: None}) == -1
    assert call(a6=0) == -2 and call(a7=2052) == -2 and call(a9=4) == -2 and call(a7=16384) == -2
    assert call(a12=0, a7=8192) == -2  # fp32 rows: half the bf16 limit
    assert call(a10=200) == -3 and call(a11=0) == -3 and call(a11=9) == -3
    assert call(a12=7) == -6
    for i in (0, 1, 2, 3, 4, 5, 13):
        assert call(**{"a%d" % i: P + 2}) == -4
    assert call(a14=1024) == -5
    need = L.oea_workspace_bytes(16, 2048, 128, 768, 8)
    assert call(a14=need - 1) == -5
    # moe_decode_ex and moe_decode_test share the checks
    assert L.moe_decode_ex(*(ok[:14] + [16, None, None])) == -5
    assert L.moe_decode_test(*(ok[:14] + [16, None, None, None])) == -5
    assert L.moe_decode_test(*([None] + ok[1:] + [None, None])) == -1
    import ctypes as C

    class Opts(C.Structure):
        _fields_ = [("kernel_path", C.c_int32), ("spin_limit", C.c_uint32), ("h_kernel_events", C.c_void_p)]
    bad = Opts(kernel_path=5)
    assert L.moe_decode_test(*(ok + [None, C.addressof(bad)])) == -2  # refused before any enqueue

    # extras with a meaningless top_p / max_p are refused with the k-range error, before any enqueue
    class Ex(C.Structure):
        _fields_ = [(n, C.c_void_p) for n in ("router_bias", "token_mask", "logits_out", "expert_idx_out", "gate_w_out",
                                              "n_sel_out", "active_list_out", "n_active_out")] + \
                   [("top_p", C.c_double), ("max_p", C.c_int32), ("deterministic", C.c_int32), ("cooperative", C.c_int32)]
    for bad_ex in (Ex(top_p=-0.5), Ex(top_p=float("nan")), Ex(max_p=-1)):
        assert L.moe_decode_ex(*(ok + [C.addressof(bad_ex)])) == -3


def test_decode_static_argument_checks(L):
    """The allocation-free entry point: the same checks, and sizes beyond its built-in scratch are
    refused (all before any HIP call, so this runs without a GPU)."""
    ok = [P, P, P, P, P, P, 16, 2048, 128, 768, 8, 3, 1, None, None]
    def call(**kw):
        a = list(ok)
        for i, v in kw.items():
            a[int(i[1:])] = v
        return L.moe_decode_static(*a)
    for i in range(6):
        assert call(**{"a%d" % i: None}) == -1
        assert call(**{"a%d" % i: P + 2}) == -4
    assert call(a6=0) == -2 and call(a7=2052) == -2 and call(a11=9) == -3 and call(a12=7) == -6
    limit = 8 << 20
    assert L.oea_workspace_bytes(128, 4096, 128, 1536, 8) <= limit  # B <= 128 at both Qwen3 shapes fits
    assert L.oea_workspace_bytes(128, 2048, 128, 768, 8) <= limit
    assert L.oea_workspace_bytes(1024, 4096, 128, 1536, 8) > limit
    assert call(a6=1024, a7=4096, a9=1536) == -9
    assert call(a6=200, a7=4096, a9=1536, a10=16) == -9
    assert "scratch" in L.oea_status_string(-9).decode()


def test_workspace_init_argument_checks(L):
    assert L.oea_workspace_init(None, 1024, None) == -1
    assert L.oea_workspace_init(P + 4, 1024, None) == -4
    assert L.oea_workspace_init(P, 8, None) == -5


def test_workspace_check_argument_checks(L):
    assert L.oea_workspace_check(None, 1 << 20, None) == -1
    assert L.oea_workspace_check(P + 4, 1 << 20, None) == -4
    assert L.oea_workspace_check(P, 8, None) == -5


def test_read_probe_argument_checks(L):
    assert L.oea_read_probe(None, 1 << 20, None, None) == -1
    assert L.oea_read_probe(P + 4, 1 << 20, None, None) == -4
    assert L.oea_read_probe(P, (1 << 20) - 16, None, None) == -2


def test_binding_module_names_match_the_abi():
    from paper_2511_02237_amd import binding
    assert set(binding.EXPORTS) == set(declared_functions())
    assert set(binding.TEST_EXPORTS) == set(declared_functions(TEST_HEADER))
    for n in ("oea_route", "moe_decode", "workspace_bytes", "new_workspace", "status_string"):
        assert hasattr(binding, n)


def test_bench_refuses_more_than_one_gpu():
    """bench.py is a one-GPU measurement: --gpus N > 1 exits with a message before touching a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
