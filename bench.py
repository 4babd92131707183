#!/usr/bin/env python3
"""Benchmark of the OEA decode-time MoE layer on one MI355X.

A step is one moe_decode call (router GEMV -> OEA routing -> grouped SwiGLU FFN -> combine) on the
Qwen3-30B-A3B-shaped layer at B=16 (d=2048, N=128, I=768, k=8, bf16).  Expert weights rotate over
several independent sets, so every step streams cold HBM as consecutive layers of a model would and
nothing is served from the 256 MB infinity cache.  All inputs are in HBM before the timed region.

Prints ONE JSON line.  `value` is the layer latency with OEA at k0=3 (the setting the paper's
headline reduction is quoted at), timed over back-to-back calls in which the token batch changes
from call to call as well; the same line carries the latency and unique-expert count for
every k0 on each token batch by itself (k0=8 is the unmodified top-k router), the roofline of the dominant kernel (gate/up
mat-vec stage, or the single fused kernel) measured with HIP events, and the CPU oracle timed on the
host cores.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E peak


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="qwen3_30b", choices=["qwen3_30b", "qwen3_235b", "qwen3_30b_skew"])
    ap.add_argument("--batch", type=int, default=16)
    ap.add_argument("--k0", type=int, default=3, help="k0 of the headline value")
    ap.add_argument("--k0s", default="", help="comma list of k0 values to time (default: 1..k)")
    ap.add_argument("--trials", type=int, default=4, help="independent token batches per k0")
    ap.add_argument("--weight-sets", type=int, default=0, help="rotating expert-weight sets (0 = auto)")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="budget of the oracle timing")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--deterministic", action="store_true",
                    help="time the layer with oea_decode_ex.deterministic (slot-ordered combine in a last kernel)")
    ap.add_argument("--no-other", action="store_true",
                    help="skip the other_workloads block (235B shape, skewed routing, other batch sizes)")
    ap.add_argument("--kernel-path", type=int, default=0, help="oea_test_opts.kernel_path: 0 automatic, 1 generic, 2 streaming, 3 dot-product stage kernels, "
                                                                  "4 matrix-core stage kernels")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain device copy of known size (reference for rocprofv3 --pmc byte counters)")
    ap.add_argument("--sweep", default="", help="comma list of batch sizes: time each (k0 from --k0s, default 3,5,8) "
                                                "and fit latency = c + b*T + a*pairs instead of the one-line report")
    ap.add_argument("--launch", default="stream", choices=["stream", "graph"],
                    help="timed steps launched one by one, or captured into one HIP graph and replayed (measured: same latency)")
    ap.add_argument("--route-positions", type=int, default=0,
                    help="instead of the layer: time oea_route_batched over this many decode positions of the workload's "
                         "B, N, k at --k0 (the routing step alone, as a simulation over a trace would call it)")
    ap.add_argument("--route-general", action="store_true",
                    help="instead of the layer: time oea_route_general (Algorithm 2) at p in {0.5, 1} and maxP in {8, N} "
                         "beside oea_route (Algorithm 1) on the workload's B, N, k at --k0, one batch per launch")
    ap.add_argument("--timeline", type=int, default=0, metavar="CALLS",
                    help="instead of the report: per-workgroup phase stamps of the single-kernel layer, averaged over "
                         "this many calls; needs the measurement build of the library (python -m "
                         "paper_2511_02237_amd.build --timeline) selected with OEA_LIB=paper_2511_02237_amd/liboea_timeline.so")
    ap.add_argument("--verbose", action="store_true")
    return ap.parse_args()


class Hip:
    """The few HIP runtime calls the benchmark needs for event timing."""

    def __init__(self):
        self.rt = ctypes.CDLL("libamdhip64.so")
        self.rt.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.rt.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.rt.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.rt.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.rt.hipStreamBeginCapture.argtypes = [ctypes.c_void_p, ctypes.c_int]
        self.rt.hipStreamEndCapture.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p)]
        self.rt.hipGraphInstantiate.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_void_p, ctypes.c_void_p,
                                                ctypes.c_void_p, ctypes.c_size_t]
        self.rt.hipGraphLaunch.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.rt.hipGraphExecDestroy.argtypes = [ctypes.c_void_p]
        self.rt.hipGraphDestroy.argtypes = [ctypes.c_void_p]

    def capture(self, stream, enqueue):
        """Record what enqueue() puts on `stream` into a graph; returns the executable graph."""
        assert self.rt.hipStreamBeginCapture(stream, 1) == 0  # thread-local capture mode
        enqueue()
        graph, ex = ctypes.c_void_p(), ctypes.c_void_p()
        assert self.rt.hipStreamEndCapture(stream, ctypes.byref(graph)) == 0
        assert self.rt.hipGraphInstantiate(ctypes.byref(ex), graph, None, None, 0) == 0
        assert self.rt.hipGraphDestroy(graph) == 0
        return ex

    def launch_graph(self, ex, stream):
        assert self.rt.hipGraphLaunch(ex, stream) == 0

    def destroy_graph(self, ex):
        assert self.rt.hipGraphExecDestroy(ex) == 0

    def event(self):
        e = ctypes.c_void_p()
        assert self.rt.hipEventCreate(ctypes.byref(e)) == 0
        return e

    def record(self, e, stream):
        assert self.rt.hipEventRecord(e, stream) == 0

    def elapsed_ms(self, a, b):
        assert self.rt.hipEventSynchronize(b) == 0
        ms = ctypes.c_float()
        assert self.rt.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
        return float(ms.value)


def main():
    args = parse()
    if args.sweep:
        return sweep(args)
    if args.route_positions:
        return route_throughput(args)
    if args.timeline:
        return timeline(args)
    if args.route_general:
        return route_general_latency(args)
    print(json.dumps(run(args)))


def route_throughput(args):
    """Routing alone: L independent decode positions (Section 4 of the paper routes every position of
    a sequence separately) in one launch of oea_route_batched, on seeded Gaussian logits."""
    import torch

    from paper_2511_02237_amd import binding, workloads
    assert args.gpus == 1 and torch.cuda.is_available()
    cfg = workloads.CONFIGS[args.workload]
    N, k, B, L = cfg["N"], cfg["k"], args.batch, args.route_positions
    g = torch.Generator(device="cuda")
    g.manual_seed(777)
    lg = torch.randn((L, B, N), generator=g, device="cuda", dtype=torch.float32)
    for _ in range(args.warmup):
        res = binding.oea_route_batched(lg, k, args.k0)
    torch.cuda.synchronize()
    t_a = time.perf_counter()
    for _ in range(args.steps):
        binding.oea_route_batched(lg, k, args.k0)
    torch.cuda.synchronize()
    us = (time.perf_counter() - t_a) / args.steps * 1e6
    moved = L * (B * N * 4 + 2 * B * k * 4 + B * 4 + N * 4 + 4)  # logits in; indices, weights, counts, active list out
    print(json.dumps(dict(metric="OEA routing throughput (decode positions / s), B=%d N=%d k=%d k0=%d" % (B, N, k, args.k0),
                          value=round(L / us * 1e6, 1), unit="positions/s", n_gpus=1, steps=args.steps,
                          warmup=args.warmup, ms_per_step=round(us / 1e3, 6), higher_is_better=True, dtype="f32",
                          data="synthetic", config=dict(workload="%d positions of %s routing" % (L, args.workload)),
                          mean_unique_experts=round(float(res["n_active"].float().mean().item()), 2),
                          bytes_moved=moved, GBps=round(moved / us / 1e3, 1),
                          frac_of_hbm_peak=round(moved / us / 1e3 / HBM_PEAK_GBS, 4))))


TIMELINE_SLOTS = ["kernel entered", "logits stored, x staged", "grid barrier passed", "candidate keys in registers",
                  "Phase 1 done, union complete", "Phase 2 and gate weights done", "CSR offsets done",
                  "routing and row cuts done", "gate/up rows streamed, h written", "completion announced",
                  "first down tiles requested", "hidden vectors of own experts complete", "hidden vectors staged",
                  "down rows streamed, adds issued", "adds drained"]


def timeline(args):
    """Where the time goes inside the single-kernel layer: the 100 MHz wall clock of every workgroup at
    each phase boundary (measurement build of the library), relative to the first workgroup's entry,
    averaged over calls that rotate token batches and weight sets like the headline timing."""
    import numpy as np
    import torch

    from paper_2511_02237_amd import binding, workloads
    assert args.gpus == 1 and torch.cuda.is_available()
    lib = binding.lib()
    if not hasattr(lib, "oea_timeline_read"):
        print("bench.py --timeline: %s has no timeline stamps; build with `python -m paper_2511_02237_amd.build "
              "--timeline` and set OEA_LIB to the library it prints" % binding.LIB_PATH, file=sys.stderr)
        sys.exit(2)
    lib.oea_timeline_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t]
    cfg = workloads.CONFIGS[args.workload]
    d, N, I, k, B = cfg["d"], cfg["N"], cfg["I"], cfg["k"], args.batch
    dev = torch.device("cuda:0")
    base = workloads.make_layer(args.workload, 1000 * 2, B=B, I=8)  # x, router and bias; expert weights drawn on the device
    xs = [binding.to_device(base.x, dev)]
    if not cfg.get("skew"):
        xs += [binding.to_device(workloads.make_layer(args.workload, 1000 * 2 + t, B=B, N=1, I=8).x, dev)
               for t in range(1, args.trials)]
    w_router = binding.to_device(base.w_router, dev)
    bias = None if base.router_bias is None else torch.from_numpy(base.router_bias).to(dev)
    g = torch.Generator(device=dev)
    g.manual_seed(12345)
    R = args.weight_sets or 8
    sets = [tuple(torch.randn(sh, generator=g, device=dev, dtype=torch.float32).mul_(0.02).to(torch.bfloat16)
                  for sh in ((N, I, d), (N, I, d), (N, d, I))) for _ in range(R)]
    ws = binding.new_workspace(B, d, N, I, k, device=dev)
    out = torch.empty((B, d), dtype=torch.float32, device=dev)
    n_slots, n_wg = 24, 256
    buf = np.zeros(n_slots * n_wg, np.uint64)
    acc_med, acc_max, acc_min, Ts = 0.0, 0.0, 0.0, []
    step = 0
    for it in range(args.warmup + args.timeline):
        for _ in range(7):  # back-to-back calls before the sampled one, as in the timed loop
            binding.moe_decode(xs[step % len(xs)], w_router, *sets[step % R], k, args.k0, ws, out=out, router_bias=bias)
            step += 1
        _, tap = binding.moe_decode(xs[step % len(xs)], w_router, *sets[step % R], k, args.k0, ws, out=out,
                                    router_bias=bias, taps=True)
        step += 1
        assert lib.oea_timeline_read(buf.ctypes.data, buf.nbytes) == 0
        if it < args.warmup:
            continue
        t = buf.reshape(n_slots, n_wg).astype(np.int64)
        rel = (t[:len(TIMELINE_SLOTS)] - t[0].min()) / 100.0  # us
        rel[(t[:len(TIMELINE_SLOTS)] < t[0].min()).any(axis=1)] = np.nan  # not stamped by this kernel (an older launch's value)
        acc_med = acc_med + np.median(rel, axis=1)
        acc_max = acc_max + rel.max(axis=1)
        acc_min = acc_min + rel.min(axis=1)
        Ts.append(int(tap["n_active"].item()))
    n = args.timeline
    rows = [dict(slot=i, phase=TIMELINE_SLOTS[i], first_wg_us=round(float(acc_min[i] / n), 2),
                 median_wg_us=round(float(acc_med[i] / n), 2), slowest_wg_us=round(float(acc_max[i] / n), 2))
            for i in range(len(TIMELINE_SLOTS)) if np.isfinite(acc_med[i])]
    print(json.dumps(dict(workload="%s B=%d k0=%d" % (args.workload, B, args.k0), calls=n,
                          mean_unique_experts=round(float(np.mean(Ts)), 2), timeline=rows)))
    for r in rows:
        print("| %2d | %-42s | %7.2f | %7.2f | %7.2f |" % (r["slot"], r["phase"], r["first_wg_us"], r["median_wg_us"],
                                                       r["slowest_wg_us"]), file=sys.stderr)


def route_general_latency(args):
    """Routing alone, one decode batch per launch: Algorithm 1 (oea_route) and Algorithm 2
    (oea_route_general: top-p cut of the baseline, k^max, rank window maxP) on seeded Gaussian logits.
    Back-to-back launches on one stream; the figure is launch period, i.e. kernel plus dispatch gap."""
    import torch

    from paper_2511_02237_amd import binding, workloads
    assert args.gpus == 1 and torch.cuda.is_available()
    cfg = workloads.CONFIGS[args.workload]
    N, k, B = cfg["N"], cfg["k"], args.batch
    lg = torch.from_numpy(workloads.make_logits(B, N, 4242, "gaussian")).cuda()
    rows = []

    hip = Hip()
    e0, e1 = hip.event(), hip.event()
    sptr = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)

    def timed(name, fn):
        res = fn(None)  # the output tensors are allocated once and reused
        for _ in range(args.warmup):
            fn(res)
        torch.cuda.synchronize()
        hip.record(e0, sptr)
        for _ in range(args.steps):
            fn(res)
        hip.record(e1, sptr)
        torch.cuda.synchronize()
        us = hip.elapsed_ms(e0, e1) / args.steps * 1e3
        rows.append(dict(routing=name, us_per_call=round(us, 2), unique_experts=int(res["n_active"].item()),
                         mean_experts_per_token=round(float(res["n_sel"].float().mean().item()), 2)))

    timed("Algorithm 1: k0=%d, k=%d" % (args.k0, k), lambda o: binding.oea_route(lg, k, args.k0, out=o))
    for p_, maxp in ((1.0, N), (0.5, N), (1.0, 8), (0.5, 8)):
        timed("Algorithm 2: k0=%d, p=%g, k_max=%d, maxP=%d" % (args.k0, p_, k, maxp),
              lambda o, p_=p_, maxp=maxp: binding.oea_route_general(lg, args.k0, p_, k, maxp, out=o))
    # ---- the whole layer under the same routings (expert weights drawn on the device, rotating sets)
    d, I = cfg["d"], cfg["I"]
    base = workloads.make_layer(args.workload, 2000, B=B, I=8)  # x and router; their logits decide the routing
    x, wr = binding.to_device(base.x), binding.to_device(base.w_router)
    g = torch.Generator(device="cuda")
    g.manual_seed(12345)
    sets = [tuple(torch.randn(sh, generator=g, device="cuda", dtype=torch.float32).mul_(0.02).to(torch.bfloat16)
                  for sh in ((N, I, d), (N, I, d), (N, d, I))) for _ in range(8)]
    ws = binding.new_workspace(B, d, N, I, k)
    out = torch.empty((B, d), dtype=torch.float32, device="cuda")
    layer_rows = []

    def layer(name, **kw):
        _, tap = binding.moe_decode(x, wr, *sets[0], k, args.k0, ws, out=out, taps=True, **kw)
        for it in range(args.warmup):
            binding.moe_decode(x, wr, *sets[it % 8], k, args.k0, ws, out=out, **kw)
        torch.cuda.synchronize()
        hip.record(e0, sptr)
        for it in range(args.steps):
            binding.moe_decode(x, wr, *sets[it % 8], k, args.k0, ws, out=out, **kw)
        hip.record(e1, sptr)
        torch.cuda.synchronize()
        binding.workspace_check(ws)
        layer_rows.append(dict(routing=name, us_per_layer=round(hip.elapsed_ms(e0, e1) / args.steps * 1e3, 2),
                               unique_experts=int(tap["n_active"].item()),
                               mean_experts_per_token=round(float(tap["n_sel"].float().mean().item()), 2)))

    layer("Algorithm 1: k0=%d, k=%d" % (args.k0, k))
    layer("Algorithm 1, three kernels", kernel_path=2)
    for p_, maxp in ((0.1, None), (None, 8), (0.1, 24), (None, 32)):
        layer("Algorithm 2: k0=%d, p=%s, k_max=%d, maxP=%s" % (args.k0, p_ if p_ else 1, k, maxp if maxp else N),
              top_p=p_, max_p=maxp)
    print(json.dumps(dict(metric="OEA routing latency per decode batch (us), B=%d N=%d" % (B, N), unit="us", n_gpus=1,
                          steps=args.steps, warmup=args.warmup, dtype="f32", data="synthetic",
                          config=dict(workload="%s routing, one batch per launch" % args.workload), rows=rows,
                          layer_rows=layer_rows)))


def sweep(args):
    """Batch sweep on one workload: latency against unique experts T and (token, expert) pairs, fitted
    as latency = c + b*T + a*pairs (the two terms of the paper's latency model, Eq. 2)."""
    import numpy as np
    rows = []
    for B in [int(v) for v in args.sweep.split(",")]:
        a = argparse.Namespace(**vars(args))
        a.batch, a.trials, a.no_cpu, a.sweep = B, 1, True, ""
        a.k0s = args.k0s or "3,5,8"
        a.k0 = int(a.k0s.split(",")[0])
        r = run(a)
        for k0, v in r["per_k0"].items():
            rows.append(dict(B=B, k0=int(k0), T=v["unique_experts"], pairs=v["pairs"], latency_us=v["latency_us"],
                             frac_of_peak=v["frac_of_peak"]))
    A = np.array([[1.0, r_["T"], r_["pairs"]] for r_ in rows])
    y = np.array([r_["latency_us"] for r_ in rows])
    coef, *_ = np.linalg.lstsq(A, y, rcond=None)
    pred = A @ coef
    r2 = 1.0 - float(((pred - y) ** 2).sum() / ((y - y.mean()) ** 2).sum())
    print(json.dumps(dict(workload=args.workload, rows=rows,
                          fit=dict(intercept_us=round(float(coef[0]), 2), us_per_unique_expert=round(float(coef[1]), 4),
                                   us_per_pair=round(float(coef[2]), 4), r2=round(r2, 5)))))


def sources_digest():
    """sha256 over the kernel sources: the recorded PMC traffic is only quoted for the sources it was taken with."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2511_02237_amd", "csrc", "*"))):
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def other_workloads(args, hip, sptr, stream, sets_30b):
    """The configurations beside the headline one, timed like it (`warmup` untimed calls, then `steps`
    back-to-back calls between two events on the stream, weight sets rotating, inputs resident):
    the Qwen3-235B-A22B-shaped layer at B=16, the skewed-routing stress workload, other batch sizes of
    the 30B shape.  Token vectors, router and bias come from the seeded generators; expert weights
    are drawn on the device (they do not influence the routing).  No oracle here: parity of these
    shapes is the tests' part."""
    import numpy as np
    import torch

    from paper_2511_02237_amd import binding, workloads
    dev = torch.device("cuda:0")
    lib = binding.lib()
    e0, e1 = hip.event(), hip.event()
    rows = []

    def timed(tag, wl, B, k0s, sets, seed):
        cfg = workloads.CONFIGS[wl]
        d, N, I, k = cfg["d"], cfg["N"], cfg["I"], cfg["k"]
        base = workloads.make_layer(wl, seed, B=B, I=8)  # cheap: only x, the router and the bias are used
        x, w_router = binding.to_device(base.x, dev), binding.to_device(base.w_router, dev)
        bias = None if base.router_bias is None else torch.from_numpy(base.router_bias).to(dev)
        ws = binding.new_workspace(B, d, N, I, k, device=dev)
        out = torch.empty((B, d), dtype=torch.float32, device=dev)
        ex = binding.DecodeEx()
        if bias is not None:
            ex.router_bias = bias.data_ptr()
        for k0 in k0s:
            calls = []
            for wset in sets:
                a = [ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(w_router.data_ptr())] + \
                    [ctypes.c_void_p(w.data_ptr()) for w in wset] + \
                    [ctypes.c_void_p(out.data_ptr()), B, d, N, I, k, k0, binding.OEA_BF16,
                     ctypes.c_void_p(ws.data_ptr()), ws.numel(), sptr]
                calls.append((lambda a=a: lib.moe_decode_ex(*a, ctypes.byref(ex))) if bias is not None
                             else (lambda a=a: lib.moe_decode(*a)))
            _, tap = binding.moe_decode(x, w_router, *sets[0], k, k0, ws, out=out, router_bias=bias, taps=True)
            torch.cuda.synchronize()
            T, pairs = int(tap["n_active"].item()), int(tap["n_sel"].sum().item())
            for it in range(3 * args.warmup):  # also lets the workspace's speed weights settle
                assert calls[it % len(calls)]() == 0
            torch.cuda.synchronize()
            hip.record(e0, sptr)
            for it in range(args.steps):
                calls[it % len(calls)]()
            hip.record(e1, sptr)
            torch.cuda.synchronize()
            us = hip.elapsed_ms(e0, e1) / args.steps * 1e3
            nbytes = T * 3 * d * I * 2 + N * d * 2 + B * d * 2 + B * d * 4 + 2 * pairs * I * 2
            rows.append(dict(workload=tag, B=B, k0=k0, unique_experts=T, pairs=pairs, latency_us=round(us, 2),
                             layer_GBps=round(nbytes / us / 1e3, 1), frac_of_hbm_peak=round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4)))

    for B in (1, 32, 128, 512):  # 512: above the single kernel's range (router/routing kernels, matrix-core stages)
        timed("qwen3_30b", "qwen3_30b", B, (3,), sets_30b, 2100)
    timed("qwen3_30b_skew", "qwen3_30b_skew", 16, (2, 4), sets_30b, 2000)
    cfg = workloads.CONFIGS["qwen3_235b"]
    g = torch.Generator(device=dev)
    g.manual_seed(4242)
    sets_235 = [tuple(torch.randn(sh, generator=g, device=dev, dtype=torch.float32).mul_(0.02).to(torch.bfloat16)
                      for sh in ((cfg["N"], cfg["I"], cfg["d"]), (cfg["N"], cfg["I"], cfg["d"]), (cfg["N"], cfg["d"], cfg["I"])))
                for _ in range(2)]  # one call streams more than a gigabyte: two sets are cold enough
    timed("qwen3_235b", "qwen3_235b", 16, (3, 8), sets_235, 3000)
    del sets_235
    return rows


def run(args):
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path is a single-GPU kernel pipeline; no "
              "collectives are part of it). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2511_02237_amd import binding, workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    binding.lib()
    topts = binding.test_opts(kernel_path=args.kernel_path) if args.kernel_path else None  # test aid; default: product entry points
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    hip = Hip()
    stream = torch.cuda.Stream()  # a stream of its own (default priority): graph capture needs a non-null stream
    torch.cuda.set_stream(stream)
    sptr = ctypes.c_void_p(stream.cuda_stream)

    cfg = workloads.CONFIGS[args.workload]
    d, N, I, k = cfg["d"], cfg["N"], cfg["I"], cfg["k"]
    B = args.batch
    k0s = [int(v) for v in args.k0s.split(",")] if args.k0s else list(range(1, k + 1))
    for must in (args.k0, k):  # the headline k0 and plain top-k are always timed
        if must not in k0s:
            k0s.append(must)
    expert_bytes = 3 * d * I * 2
    # enough sets that a full rotation exceeds the infinity cache several times over
    R = args.weight_sets or max(8, int(np.ceil(4 * 256e6 / (N * expert_bytes))) + 1)

    # ---- inputs.  Set 0 comes from the seeded numpy generator (the oracle reads the same bits);
    # the other sets only have to be distinct cold memory of the same distribution.
    t0 = time.time()
    L = workloads.make_layer(args.workload, 1000 * 2 + 0, B=B)
    w_router = binding.to_device(L.w_router, dev)
    bias = None if L.router_bias is None else torch.from_numpy(L.router_bias).to(dev)
    sets = [tuple(binding.to_device(getattr(L, f), dev) for f in ("w_gate", "w_up", "w_down"))]
    g = torch.Generator(device=dev)
    g.manual_seed(12345)
    for _ in range(1, R):
        ws_ = []
        for shape in ((N, I, d), (N, I, d), (N, d, I)):
            w = torch.randn(shape, generator=g, device=dev, dtype=torch.float32).mul_(0.02).to(torch.bfloat16)
            ws_.append(w)
        sets.append(tuple(ws_))
    xs_np = [L.x]
    for t in range(1, args.trials):
        xs_np.append(workloads.make_layer(args.workload, 1000 * 2 + t, B=B, N=1, I=8).x)  # only x is used
    if cfg.get("skew"):
        xs_np = xs_np[:1]  # the skewed recipe ties x to the bias drawn with it
    xs = [binding.to_device(x, dev) for x in xs_np]
    ws = binding.new_workspace(B, d, N, I, k, device=dev, deterministic=args.deterministic)
    out = torch.empty((B, d), dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    if args.verbose:
        print("inputs ready in %.1fs, %d weight sets of %.2f GB" % (time.time() - t0, R, N * expert_bytes / 1e9),
              file=sys.stderr)

    lib = binding.lib()
    ws_bytes = ws.numel()

    def make_call(x, wset, k0, opts=None):
        a = [ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(w_router.data_ptr()),
             ctypes.c_void_p(wset[0].data_ptr()), ctypes.c_void_p(wset[1].data_ptr()),
             ctypes.c_void_p(wset[2].data_ptr()), ctypes.c_void_p(out.data_ptr()), B, d, N, I, k, k0,
             binding.OEA_BF16, ctypes.c_void_p(ws.data_ptr()), ws_bytes, sptr]
        opts = opts if opts is not None else topts
        if opts is None and bias is None and not args.deterministic:
            return lambda: lib.moe_decode(*a)
        exs = binding.DecodeEx()
        exs.deterministic = 1 if args.deterministic else 0
        if bias is not None:
            exs.router_bias = bias.data_ptr()
        ref = ctypes.byref(exs)
        if opts is None:
            return lambda: lib.moe_decode_ex(*a, ref)
        oref = ctypes.byref(opts)
        return lambda: lib.moe_decode_test(*a, ref, oref)

    # ---- routing statistics per (trial, k0): T and the number of (token, expert) pairs
    stats = {}
    for ti, x in enumerate(xs):
        for k0 in k0s:
            _, tap = binding.moe_decode(x, w_router, *sets[0], k, k0, ws, out=out, router_bias=bias, taps=True,
                                        kernel_path=args.kernel_path or None, deterministic=args.deterministic)
            torch.cuda.synchronize()
            stats[(ti, k0)] = (int(tap["n_active"].item()), int(tap["n_sel"].sum().item()))

    # ---- parity of the timed configuration against the oracle (trial 0, headline k0, weight set 0)
    parity = None
    if not args.no_cpu:
        import oracle
        ref = oracle.moe_decode(L.x, L.w_router, L.w_gate, L.w_up, L.w_down, k, args.k0, router_bias=L.router_bias)
        o, tap = binding.moe_decode(xs[0], w_router, *sets[0], k, args.k0, ws, router_bias=bias, taps=True,
                                    kernel_path=args.kernel_path or None, deterministic=args.deterministic)
        torch.cuda.synchronize()
        assert np.array_equal(tap["expert_idx"].cpu().numpy(), ref["expert_idx"]), "routing differs from the oracle"
        parity = float(np.abs(o.cpu().numpy() - ref["out"]).max() / np.abs(ref["out"]).max())
        assert parity <= 5e-3, parity

    if args.calib_copy:  # 256 MiB read + 256 MiB written per copy, by a plain elementwise copy kernel
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- the workspace is new: let the per-workgroup speed weights it carries from call to call settle
    # once (they move a quarter of the way per call), so that the first timed cell is not the odd one out
    settle = [make_call(xs[j % len(xs)], sets[j % R], k0s[0]) for j in range(R * len(xs))]
    for it in range(3 * args.warmup):
        assert settle[it % len(settle)]() == 0
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` calls per (trial, k0), synchronised on both sides
    e0, e1 = hip.event(), hip.event()
    lat_wall, lat_ev = {}, {}
    step = 0
    for ti, x in enumerate(xs):
        for k0 in k0s:
            calls = [make_call(x, sets[r], k0) for r in range(R)]
            for _ in range(args.warmup):
                rc = calls[step % R]()
                step += 1
                assert rc == 0, rc
            torch.cuda.synchronize()
            if args.launch == "graph":
                first = step

                def enqueue():
                    for j in range(args.steps):
                        assert calls[(first + j) % R]() == 0
                gexec = hip.capture(sptr, enqueue)
                step += args.steps
                torch.cuda.synchronize()
                t_a = time.perf_counter()
                hip.record(e0, sptr)
                hip.launch_graph(gexec, sptr)
                hip.record(e1, sptr)
                torch.cuda.synchronize()
                t_b = time.perf_counter()
                hip.destroy_graph(gexec)
            else:
                t_a = time.perf_counter()
                hip.record(e0, sptr)
                for _ in range(args.steps):
                    calls[step % R]()
                    step += 1
                hip.record(e1, sptr)
                torch.cuda.synchronize()
                t_b = time.perf_counter()
            lat_wall[(ti, k0)] = (t_b - t_a) / args.steps * 1e6
            lat_ev[(ti, k0)] = hip.elapsed_ms(e0, e1) / args.steps * 1e3

    # ---- per-kernel durations with HIP events recorded inside the library around each kernel
    kern = {}
    evs = (ctypes.c_void_p * 6)(*[hip.event() for _ in range(6)])
    for k0 in sorted({args.k0, k}):
        ev_opts = binding.test_opts(kernel_path=args.kernel_path, kernel_events=evs)
        calls = [make_call(xs[j % len(xs)], sets[j % R], k0, ev_opts) for j in range(R * len(xs))]  # rotating, as timed
        acc = np.zeros(3)
        n = min(args.steps, 100)
        for it in range(args.warmup + n):
            assert calls[it % len(calls)]() == 0
            if it >= args.warmup:
                acc += [hip.elapsed_ms(evs[0], evs[1]), hip.elapsed_ms(evs[2], evs[3]), hip.elapsed_ms(evs[4], evs[5])]
            torch.cuda.synchronize()
        kern[k0] = (acc / n * 1e3).tolist()  # us: router+route, gate/up, down

    # ---- spread of single calls and the cache-warm latency (token batch 0; outside the timed region):
    # an event pair around every call of a back-to-back run; then the same with ONE weight set, which
    # at small T is served from the 256 MB infinity cache instead of HBM (reported as such, never as value)
    def per_call(k0, n_sets):
        n = min(args.steps, 200)
        ev = [hip.event() for _ in range(n + 1)]
        calls = [make_call(xs[0], sets[r], k0) for r in range(n_sets)]
        for it in range(args.warmup):
            assert calls[it % n_sets]() == 0
        torch.cuda.synchronize()
        hip.record(ev[0], sptr)
        for it in range(n):
            calls[it % n_sets]()
            hip.record(ev[it + 1], sptr)
        torch.cuda.synchronize()
        us = np.array([hip.elapsed_ms(ev[i], ev[i + 1]) * 1e3 for i in range(n)])
        return dict(median=round(float(np.median(us)), 2), p10=round(float(np.percentile(us, 10)), 2),
                    p90=round(float(np.percentile(us, 90)), 2))
    per_call_us = {str(k0): per_call(k0, R) for k0 in sorted({args.k0, k})}
    cache_warm_us = {str(k0): per_call(k0, 1) for k0 in sorted({args.k0, k})}

    # ---- the other configurations (before the headline passes, which stay the last launches of the layer)
    others = None
    if args.workload == "qwen3_30b" and args.kernel_path == 0 and not args.no_other and not args.deterministic:
        others = other_workloads(args, hip, sptr, stream, sets)

    # ---- the headline timing: back-to-back calls in which the TOKEN BATCH changes from call to call as
    # well as the weight set (a server never sees the same batch twice, so the per-workgroup speed
    # weights cannot settle on one routing pattern).  `warmup` untimed calls, then exactly `steps`
    # calls between two synchronisations.
    def rotating(k0):
        calls = [make_call(xs[j % len(xs)], sets[j % R], k0) for j in range(R * len(xs))]
        for it in range(args.warmup):
            assert calls[it % len(calls)]() == 0
        torch.cuda.synchronize()
        t_a = time.perf_counter()
        hip.record(e0, sptr)
        for it in range(args.steps):
            calls[(args.warmup + it) % len(calls)]()
        hip.record(e1, sptr)
        torch.cuda.synchronize()
        rotating_ev[str(k0)] = hip.elapsed_ms(e0, e1) / args.steps * 1e3  # the same calls by HIP events on the stream
        return round((time.perf_counter() - t_a) / args.steps * 1e6, 2)
    rotating_ev = {}
    # (kept as the LAST passes that launch the layer: the profile summaries pick them out by position)
    rotating_us = {str(k0): rotating(k0) for k0 in sorted({args.k0, k})} if len(xs) > 1 else None

    # ---- the device's practical read ceiling (outside the timed region): the library's read probe
    # over every weight tensor in rotation, so that each pass reads memory no cache holds
    probe_bufs = [w for wset in sets for w in wset]
    probe_bytes = sum(w.numel() * w.element_size() for w in probe_bufs)
    for w in probe_bufs[:3]:
        binding.read_probe(w, stream)
    torch.cuda.synchronize()
    hip.record(e0, sptr)
    for w in probe_bufs:
        binding.read_probe(w, stream)
    hip.record(e1, sptr)
    torch.cuda.synchronize()
    read_ceiling = probe_bytes / (hip.elapsed_ms(e0, e1) * 1e-3) / 1e9

    # ---- report
    def mean_over_trials(dct, k0):
        return float(np.mean([dct[(ti, k0)] for ti in range(len(xs))]))

    def layer_bytes(T, pairs):
        # unique experts * 3*d*I*2  +  router, x, out, hidden (written + read, bf16)
        return T * expert_bytes + N * d * 2 + B * d * 2 + B * d * 4 + 2 * pairs * I * 2

    table = {}
    for k0 in sorted(k0s):
        T = float(np.mean([stats[(ti, k0)][0] for ti in range(len(xs))]))
        pairs = float(np.mean([stats[(ti, k0)][1] for ti in range(len(xs))]))
        lat = mean_over_trials(lat_wall, k0)
        gbs = float(np.mean([layer_bytes(*stats[(ti, k0)]) / lat_wall[(ti, k0)] for ti in range(len(xs))])) / 1e3
        table[str(k0)] = dict(unique_experts=round(T, 2), pairs=round(pairs, 1), latency_us=round(lat, 2),
                              latency_us_events=round(mean_over_trials(lat_ev, k0), 2),
                              layer_GBps=round(gbs, 1), frac_of_peak=round(gbs / HBM_PEAK_GBS, 4))
    Ts = np.array([stats[key][0] for key in lat_wall], dtype=np.float64)
    lats = np.array([lat_wall[key] for key in lat_wall], dtype=np.float64)
    # Eq. 2 of the paper: latency = b*T + a*B*k.  At a fixed batch size every token holds k experts in all
    # cells, so a*B*k is one constant: it is the intercept here, together with the fixed part of the kernel.
    # The line is descriptive: the streaming efficiency grows with T (the fixed part amortises), which the
    # slope absorbs, so the marginal rate it implies can exceed the HBM peak.  The two terms are separated
    # over several batch sizes in two_term_fit below.
    fit = None
    if len(set(Ts.tolist())) > 2:
        A = np.stack([Ts, np.ones_like(Ts)], axis=1)
        (slope, icpt), res, *_ = np.linalg.lstsq(A, lats, rcond=None)
        r2 = 1.0 - float(((A @ [slope, icpt] - lats) ** 2).sum() / ((lats - lats.mean()) ** 2).sum())
        fit = dict(form="latency = b*T + (a*B*k + fixed), B and k fixed", b_us_per_expert=round(float(slope), 4),
                   aBk_plus_fixed_us=round(float(icpt), 2), r2=round(r2, 5))

    # dominant kernel.  Automatic path: the whole layer is ONE fused kernel (events [0]..[5] bracket
    # it) and its algorithmic bytes are the layer's.  Three-kernel paths: the gate/up stage, which
    # streams 2/3 of the expert bytes.
    # (the launches behind kern[] rotate over the token batches: bytes are the mean over the batches)
    T0 = float(np.mean([stats[(ti, args.k0)][0] for ti in range(len(xs))]))
    pairs0 = float(np.mean([stats[(ti, args.k0)][1] for ti in range(len(xs))]))
    fused = args.kernel_path == 0 and kern[args.k0][1] < 0.25 * kern[args.k0][0]
    if fused:
        # one kernel per call: the timed region's own events (back-to-back launches, so a launch lasts from
        # the end of the previous one to its own end, as in a profiler's kernel trace); else one call at a
        # time between the events the library records around the kernel
        dom_us = rotating_ev[str(args.k0)] if rotating_us else kern[args.k0][0]
        dom_bytes = layer_bytes(T0, pairs0)
        dom_name = "moe_fused_kernel<bf16> (router + routing + gate/up + down)"
    else:
        dom_us = kern[args.k0][1]
        dom_bytes = T0 * 2 * d * I * 2 + pairs0 * d * 2 + pairs0 * I * 2  # weights + gathered x + hidden written
        # which gate/up kernel that is follows the library's choice (see include/oea_testing.h, kernel_path)
        dom_name = ("expert_dense_kernel<gate/up> (matrix cores)" if (args.kernel_path == 4 or (args.kernel_path == 0 and B > 128))
                    else "expert_stage_kernel<bf16, gate/up>" if args.kernel_path in (0, 3)
                    else "expert_stream_kernel<bf16, gate/up>" if args.kernel_path == 2 else "expert_kernel<bf16, gate/up>")
    achieved = dom_bytes / dom_us / 1e3
    # traffic: HBM bytes per launch from the rocprofv3 --pmc passes over this same command, RECORDED in
    # profiles/ (counters cannot be read from inside the run); quoted only if the kernel sources are the ones
    # the record was taken with, else null
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", "pmc_traffic_%s.txt" % args.workload)
    if os.path.exists(tpath):
        key = ("fused" if fused else "gate_up") + "_bytes_per_launch_k0_%d" % args.k0
        rec = dict(line.split("=", 1) for line in open(tpath) if "=" in line and not line.startswith("#"))
        rec = {a.strip(): b.strip() for a, b in rec.items()}
        if rec.get("kernel_sources_sha256_16") == sources_digest() and key in rec:
            traffic = float(rec[key])
            traffic_source = "recorded: profiles/pmc_traffic_%s.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes)" % args.workload
        elif rec.get("kernel_sources_sha256_16") != sources_digest():
            traffic_source = "none: the recorded counters in profiles/ belong to other kernel sources"
        else:
            traffic_source = "none: profiles/ holds no byte counters for this kernel and k0 (they cover the default command)"
    roofline = dict(bound="hbm", kernel=dom_name, achieved=round(achieved, 1),
                    peak=HBM_PEAK_GBS, unit="GB/s", frac=round(achieved / HBM_PEAK_GBS, 4), traffic=traffic,
                    traffic_source=traffic_source,
                    bytes_per_launch=int(dom_bytes), us_per_launch=round(dom_us, 2),
                    isolated_kernels_us={str(k0_): (dict(fused=round(v[0], 2)) if fused else
                                           dict(router_route=round(v[0], 2), gate_up=round(v[1], 2), down=round(v[2], 2)))
                                for k0_, v in kern.items()})

    cpu = None
    if not args.no_cpu:
        import oracle
        n_thr = oracle.num_threads()
        t_start = time.perf_counter()
        reps = 0
        while reps < 3 or time.perf_counter() - t_start < args.cpu_seconds:
            oracle.moe_decode(L.x, L.w_router, L.w_gate, L.w_up, L.w_down, k, args.k0, router_bias=L.router_bias)
            reps += 1
        cpu_us = (time.perf_counter() - t_start) / reps * 1e6
        cpu = dict(value=round(cpu_us, 1), unit="us", cores=n_thr, kind="oracle",
                   sample="%d whole-layer calls (fp64 C oracle, OpenMP over token-expert pairs) at k0=%d on "
                          "token batch 0 / weight set 0 of the timed workload" % (reps, args.k0))

    # ---- the other configurations, and the two-term fit over everything timed in this run
    fit2 = None
    if others is not None:
        cells = [(v["unique_experts"], v["pairs"], v["latency_us"]) for v in table.values()] + \
                [(r_["unique_experts"], r_["pairs"], r_["latency_us"]) for r_ in others if r_["workload"] == "qwen3_30b" and r_["B"] <= 128]  # the single kernel's range
        A2 = np.array([[1.0, c[0], c[1]] for c in cells])
        y2 = np.array([c[2] for c in cells])
        coef, *_ = np.linalg.lstsq(A2, y2, rcond=None)
        r2 = 1.0 - float(((A2 @ coef - y2) ** 2).sum() / ((y2 - y2.mean()) ** 2).sum())
        fit2 = dict(form="latency = fixed + b*T + a*pairs over B in {1,16,32,128} (30B shape; Eq. 2 with pairs = sum |S_i| <= B*k)",
                    fixed_us=round(float(coef[0]), 2), b_us_per_expert=round(float(coef[1]), 4),
                    a_us_per_pair=round(float(coef[2]), 4), r2=round(r2, 5), cells=len(cells))

    # headline: rotating token batches (several batches), else the single batch's figure
    value = rotating_us[str(args.k0)] if rotating_us else table[str(args.k0)]["latency_us"]
    topk_value = rotating_us[str(k)] if rotating_us else table[str(k)]["latency_us"]
    mean_bytes = float(np.mean([layer_bytes(*stats[(ti, args.k0)]) for ti in range(len(xs))]))
    line = dict(metric="MoE-layer decode latency (us) at B=%d, OEA k0=%d vs top-k" % (B, args.k0), value=value,
                unit="us", n_gpus=1, steps=args.steps, warmup=args.warmup, ms_per_step=round(value / 1e3, 6),
                higher_is_better=False, scaling="weak", vs_baseline=None, dtype="bf16", data="synthetic",
                config=dict(workload="%s B=%d d=%d N=%d I=%d k=%d, OEA k0=%d (k0=%d is plain top-k)"
                                     % (args.workload, B, d, N, I, k, args.k0, k),
                            trials=len(xs), weight_sets=R, k0=args.k0, launch=args.launch,
                            combine="deterministic (slot order, last kernel)" if args.deterministic else "fp32 atomics"),
                topk_latency_us=topk_value,
                latency_ratio_vs_topk=round(value / topk_value, 4),
                unique_expert_ratio_vs_topk=round(table[str(args.k0)]["unique_experts"] / table[str(k)]["unique_experts"], 4),
                layer_frac_of_hbm_peak=round(mean_bytes / value / 1e3 / HBM_PEAK_GBS, 4),
                timing="token batches and weight sets both rotate from call to call" if rotating_us else
                       "one token batch, weight sets rotate",
                fixed_batch_latency_us={str(k0_): table[str(k0_)]["latency_us"] for k0_ in sorted({args.k0, k})},
                per_k0=table, per_call_us=per_call_us,
                cache_warm_single_weight_set_us=cache_warm_us,
                latency_vs_unique_experts_fit=fit, two_term_fit=fit2, parity_max_rel_err=parity,
                read_ceiling=dict(measured_GBps=round(read_ceiling, 1), achieved_over_ceiling=round(achieved / read_ceiling, 4),
                                  note="the library's read-only probe kernel over the same weight sets; not a roofline"),
                other_workloads=others,
                roofline=roofline, cpu_baseline=cpu)
    return line


if __name__ == "__main__":
    main()
