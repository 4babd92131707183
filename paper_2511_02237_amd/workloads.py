"""Seeded synthetic inputs for the decode-time MoE layer (numpy only, host side).

This module holds NO arithmetic of the method: it only draws random numbers, rounds them once to
the storage type and packs them.  Both the HIP path and the CPU oracle are fed from here, so both
read identical bits.

Shapes and distributions follow the workloads the paper measures on (Section 4, "Hardware and
model": Qwen3-30B-A3B has N=128 experts, k=8, embedding 2048, expert hidden 768; Section 4.2:
Qwen3-235B-A22B doubles embedding and expert hidden size; decode batches bounded at 16).  The paper
runs real checkpoints on real benchmark traffic; neither is available, so Gaussian stand-ins with
the same shapes are drawn here.

bf16 arrays are carried as uint16 bit patterns (numpy has no bf16).
"""
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

# name -> (d, N, I, k, dtype, default B, k0 values exercised)
CONFIGS = {
    "toy": dict(d=64, N=16, I=32, k=4, dtype="f32", B=4, k0s=(1, 2, 4)),
    "qwen3_30b": dict(d=2048, N=128, I=768, k=8, dtype="bf16", B=16, k0s=tuple(range(1, 9))),
    "qwen3_235b": dict(d=4096, N=128, I=1536, k=8, dtype="bf16", B=16, k0s=tuple(range(1, 9))),
    # same layer as qwen3_30b; inputs are correlated and the router gets a Zipf popularity bias
    "qwen3_30b_skew": dict(d=2048, N=128, I=768, k=8, dtype="bf16", B=16, k0s=(2, 4), skew=True),
    # mid-size shapes the oracle finishes in seconds: several tiles, ragged tails
    "mid_bf16": dict(d=384, N=40, I=200, k=6, dtype="bf16", B=11, k0s=(1, 3, 6)),
    "mid_f32": dict(d=200, N=24, I=136, k=5, dtype="f32", B=7, k0s=(1, 2, 5)),
}


def bf16_round(a: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even.  Inputs are finite."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(u: np.ndarray) -> np.ndarray:
    return (u.astype(np.uint32) << np.uint32(16)).view(np.float32)


def widen(a: np.ndarray) -> np.ndarray:
    """Stored array (float32, or uint16 bf16 bits) -> float64 values, exactly."""
    if a.dtype == np.uint16:
        return bf16_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


@dataclass
class Layer:
    name: str
    B: int
    d: int
    N: int
    I: int
    k: int
    dtype: str  # "f32" | "bf16"
    x: np.ndarray  # [B,d]
    w_router: np.ndarray  # [N,d]
    w_gate: np.ndarray  # [N,I,d]
    w_up: np.ndarray  # [N,I,d]
    w_down: np.ndarray  # [N,d,I]
    router_bias: Optional[np.ndarray] = None  # [N] float32 (skewed workload only)
    k0s: tuple = field(default_factory=tuple)


def _store(a: np.ndarray, dtype: str) -> np.ndarray:
    return bf16_round(a) if dtype == "bf16" else np.ascontiguousarray(a, dtype=np.float32)


def zipf_bias(N: int, rng: np.random.Generator, s: float = 1.1) -> np.ndarray:
    """Per-expert bias 2*ln(popularity), popularity ~ rank^-s normalised, ranks given to experts by
    a seeded permutation.  A device of the synthetic workload, not of the method."""
    ranks = rng.permutation(N) + 1
    pop = ranks.astype(np.float64) ** (-s)
    pop /= pop.sum()
    return (2.0 * np.log(pop)).astype(np.float32)


def make_layer(name: str, seed: int, B: Optional[int] = None, **override) -> Layer:
    """Draw one layer + one decode batch.  x~N(0,1), W_router~N(0,1/d), experts~N(0,0.02^2)."""
    cfg = dict(CONFIGS[name])
    cfg.update(override)
    d, N, I, k, dtype = cfg["d"], cfg["N"], cfg["I"], cfg["k"], cfg["dtype"]
    B = int(B if B is not None else cfg["B"])
    rng = np.random.Generator(np.random.PCG64(seed))
    bias = None
    if cfg.get("skew"):
        shared = rng.standard_normal(d, dtype=np.float32)
        private = rng.standard_normal((B, d), dtype=np.float32)
        x = np.float32(0.7) * shared[None, :] + np.float32(0.3) * private
        bias = zipf_bias(N, rng)
    else:
        x = rng.standard_normal((B, d), dtype=np.float32)
    w_router = rng.standard_normal((N, d), dtype=np.float32) * np.float32(d ** -0.5)
    store_dt = np.uint16 if dtype == "bf16" else np.float32
    w_gate = np.empty((N, I, d), store_dt)
    w_up = np.empty((N, I, d), store_dt)
    w_down = np.empty((N, d, I), store_dt)
    std = np.float32(0.02)
    for e in range(N):  # per expert, to bound the float32 temporaries
        w_gate[e] = _store(rng.standard_normal((I, d), dtype=np.float32) * std, dtype)
        w_up[e] = _store(rng.standard_normal((I, d), dtype=np.float32) * std, dtype)
        w_down[e] = _store(rng.standard_normal((d, I), dtype=np.float32) * std, dtype)
    return Layer(name=name, B=B, d=d, N=N, I=I, k=k, dtype=dtype, x=_store(x, dtype),
                 w_router=_store(w_router, dtype), w_gate=w_gate, w_up=w_up, w_down=w_down,
                 router_bias=bias, k0s=tuple(cfg["k0s"]))


def make_logits(B: int, N: int, seed: int, kind: str = "gaussian") -> np.ndarray:
    """Router logits [B,N] float32 for routing-only tests.

    gaussian   : N(0,1), near-uniform expert popularity
    ties       : values on a grid of 5 levels -> many exact ties
    signed_zero: mixture of +0.0, -0.0 and a few non-zeros
    denormal   : tiny sub-normal magnitudes with both signs
    duplicate  : every token is a copy of token 0
    constant   : all logits equal
    skew       : gaussian + Zipf popularity bias
    wide       : gaussian * 30 (softmax saturates)
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    if kind == "gaussian":
        return rng.standard_normal((B, N), dtype=np.float32)
    if kind == "ties":
        return (rng.integers(-2, 3, size=(B, N)).astype(np.float32)) * np.float32(0.5)
    if kind == "signed_zero":
        z = np.zeros((B, N), np.float32)
        sel = rng.integers(0, 4, size=(B, N))
        z[sel == 1] = np.float32(-0.0)
        z[sel == 2] = np.float32(1.0)
        z[sel == 3] = np.float32(-1.0)
        return z
    if kind == "denormal":
        m = rng.integers(-3, 4, size=(B, N)).astype(np.int32)
        bits = (np.abs(m).astype(np.uint32)) | np.where(m < 0, np.uint32(0x80000000), np.uint32(0))
        return bits.astype(np.uint32).view(np.float32).reshape(B, N)
    if kind == "duplicate":
        row = rng.standard_normal((1, N), dtype=np.float32)
        return np.repeat(row, B, axis=0)
    if kind == "constant":
        return np.full((B, N), np.float32(0.25))
    if kind == "skew":
        return rng.standard_normal((B, N), dtype=np.float32) + zipf_bias(N, rng)[None, :]
    if kind == "wide":
        return rng.standard_normal((B, N), dtype=np.float32) * np.float32(30.0)
    raise ValueError(kind)


LOGIT_KINDS = ("gaussian", "ties", "signed_zero", "denormal", "duplicate", "constant", "skew", "wide")
