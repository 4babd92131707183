"""Pins for the oracle's router GEMV, expert FFN and whole-layer output (CPU only).

Reference values come from numpy fp64 library mat-muls written from the definitions (Eq. 1 and the
SwiGLU expert of Section 4), never from the oracle's own loops.
"""
import numpy as np
import pytest
from scipy.special import expit, softmax as sp_softmax

from paper_2511_02237_amd import workloads as W


def swiglu_np(xv, wg, wu, wd):
    g = wg @ xv
    u = wu @ xv
    return wd @ (g * expit(g) * u)  # silu(g) = g * sigmoid(g)


def layer_np(L, expert_idx, gate_w):
    """Eq. 1 evaluated with numpy fp64 mat-muls over given sets/weights."""
    x = W.widen(L.x)
    out = np.zeros((L.B, L.d))
    for i in range(L.B):
        for s in range(expert_idx.shape[1]):
            e = int(expert_idx[i, s])
            if e < 0:
                continue
            out[i] += gate_w[i, s] * swiglu_np(x[i], W.widen(L.w_gate[e]), W.widen(L.w_up[e]),
                                               W.widen(L.w_down[e]))
    return out


@pytest.mark.parametrize("name", ["toy", "mid_bf16", "mid_f32"])
def test_router_logits_match_numpy_fp64(oracle, name):
    L = W.make_layer(name, 3)
    bias = W.zipf_bias(L.N, np.random.default_rng(0))
    for b in (None, bias):
        got = oracle.router_logits(L.x, L.w_router, b)
        ref64 = W.widen(L.x) @ W.widen(L.w_router).T + (0.0 if b is None else b.astype(np.float64)[None, :])
        assert got.dtype == np.float32
        # one rounding of an fp64 sum: at most one fp32 ulp from the rounded library value,
        # and the value itself is within half an ulp of the fp64 result
        assert np.all(np.abs(got.astype(np.float64) - ref64) <= np.spacing(np.abs(ref64).astype(np.float32)) * 0.5000001)


def test_router_logits_transposed_operand_would_fail(oracle):
    # guards the index order x[i,c]*W[e,c]: a square W makes a transposed read type-check
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 8)).astype(np.float32)
    w = rng.standard_normal((8, 8)).astype(np.float32)
    got = oracle.router_logits(x, w)
    assert np.allclose(got, x.astype(np.float64) @ w.astype(np.float64).T, rtol=1e-6)
    assert not np.allclose(got, x.astype(np.float64) @ w.astype(np.float64), rtol=1e-3)


@pytest.mark.parametrize("name", ["toy", "mid_bf16", "mid_f32"])
def test_single_expert_is_dense_swiglu(oracle, name):
    # N = 1, k = k0 = 1: the layer is one dense SwiGLU MLP with weight 1 (Eq. 1 with |S| = 1)
    L = W.make_layer(name, 5, N=1, k=1)
    res = oracle.moe_decode(L.x, L.w_router, L.w_gate, L.w_up, L.w_down, 1, 1)
    x = W.widen(L.x)
    ref = np.stack([swiglu_np(x[i], W.widen(L.w_gate[0]), W.widen(L.w_up[0]), W.widen(L.w_down[0]))
                    for i in range(L.B)])
    assert np.all(res["gate_w"] == 1.0)
    assert np.allclose(res["out"], ref, rtol=1e-10, atol=1e-18)


def test_expert_ffn_rectangular_orientation(oracle):
    # d != I and asymmetric values: a transposed W_down or swapped gate/up changes the result
    rng = np.random.default_rng(2)
    d, I = 24, 40
    xv = rng.standard_normal(d).astype(np.float32)
    wg = rng.standard_normal((I, d)).astype(np.float32)
    wu = rng.standard_normal((I, d)).astype(np.float32)
    wd = rng.standard_normal((d, I)).astype(np.float32)
    y = oracle.expert_ffn(xv, wg, wu, wd)
    ref = swiglu_np(xv.astype(np.float64), wg.astype(np.float64), wu.astype(np.float64), wd.astype(np.float64))
    assert np.allclose(y, ref, rtol=1e-11)
    swapped = swiglu_np(xv.astype(np.float64), wu.astype(np.float64), wg.astype(np.float64), wd.astype(np.float64))
    assert not np.allclose(y, swapped, rtol=1e-3)


def test_silu_closed_values(oracle):
    # one-dimensional expert: y = w_d * silu(w_g x) * (w_u x); silu(0)=0, silu(z)->z for large z,
    # silu(-z) = -z*sigmoid(-z), silu(ln 3) = ln3 * 3/4
    one = np.ones((8, 8), np.float32)  # d = I = 8 (shape granularity), use only the first entry
    def run(xval, g, u, dn):
        xv = np.zeros(8, np.float32); xv[0] = xval
        wg = np.zeros((8, 8), np.float32); wg[0, 0] = g
        wu = np.zeros((8, 8), np.float32); wu[0, 0] = u
        wd = np.zeros((8, 8), np.float32); wd[0, 0] = dn
        return oracle.expert_ffn(xv, wg, wu, wd)[0]
    assert run(0.0, 1.0, 1.0, 1.0) == 0.0
    assert abs(run(1.0, 40.0, 1.0, 1.0) - 40.0) < 1e-12
    ln3 = float(np.float32(np.log(3.0)))
    assert abs(run(1.0, ln3, 2.0, 0.5) - (ln3 / (1 + np.exp(-ln3))) * 2.0 * 0.5) < 1e-15
    assert abs(run(1.0, np.float32(np.log(3.0)), 1.0, 1.0) - ln3 * 0.75) < 1e-6
    assert run(1.0, -2.0, 1.0, 1.0) == pytest.approx(-2.0 / (1 + np.exp(2.0)), rel=1e-14)
    del one


@pytest.mark.parametrize("name,seed", [("toy", 0), ("toy", 1), ("mid_bf16", 2), ("mid_f32", 3)])
def test_whole_layer_equals_eq1_in_numpy(oracle, name, seed):
    L = W.make_layer(name, seed)
    for k0 in L.k0s:
        res = oracle.moe_decode(L.x, L.w_router, L.w_gate, L.w_up, L.w_down, L.k, k0)
        # routing inside moe_decode == routing of its own logits
        again = oracle.route(res["logits"], L.k, k0)
        assert np.array_equal(again["expert_idx"], res["expert_idx"])
        # gate weights from the library softmax, output from numpy mat-muls
        R = sp_softmax(res["logits"].astype(np.float64), axis=1)
        gw = np.zeros_like(res["gate_w"])
        for i in range(L.B):
            n = res["n_sel"][i]
            sel = R[i, res["expert_idx"][i, :n]]
            gw[i, :n] = sel / sel.sum()
        ref = layer_np(L, res["expert_idx"], gw)
        scale = np.abs(ref).max()
        assert np.abs(res["out"] - ref).max() <= 1e-12 * scale


def test_zero_gate_matrix_gives_zero_and_linearity_in_w_down(oracle):
    L = W.make_layer("toy", 7)
    zero = np.zeros_like(L.w_gate)
    res = oracle.moe_decode(L.x, L.w_router, zero, L.w_up, L.w_down, L.k, 2)
    assert np.all(res["out"] == 0.0)
    base = oracle.moe_decode(L.x, L.w_router, L.w_gate, L.w_up, L.w_down, L.k, 2)["out"]
    doubled = oracle.moe_decode(L.x, L.w_router, L.w_gate, L.w_up, (L.w_down * np.float32(2)), L.k, 2)["out"]
    assert np.allclose(doubled, 2 * base, rtol=1e-13, atol=0)


def test_thread_count_does_not_change_result(oracle):
    L = W.make_layer("mid_bf16", 4)
    n = oracle.num_threads()
    oracle.set_num_threads(1)
    a = oracle.moe_decode(L.x, L.w_router, L.w_gate, L.w_up, L.w_down, L.k, 3)["out"]
    oracle.set_num_threads(max(2, n))
    b = oracle.moe_decode(L.x, L.w_router, L.w_gate, L.w_up, L.w_down, L.k, 3)["out"]
    oracle.set_num_threads(n)
    assert np.array_equal(a, b)


def test_skew_bias_enters_logits_and_padding_rows_are_zero(oracle):
    L = W.make_layer("mid_bf16", 9, skew=True)
    assert L.router_bias is not None
    mask = np.ones(L.B, np.uint8)
    mask[[2, 5]] = 0
    res = oracle.moe_decode(L.x, L.w_router, L.w_gate, L.w_up, L.w_down, L.k, 2,
                            router_bias=L.router_bias, token_mask=mask)
    ref_logits = W.widen(L.x) @ W.widen(L.w_router).T + L.router_bias.astype(np.float64)[None, :]
    assert np.allclose(res["logits"], ref_logits, rtol=1e-6, atol=1e-6)
    assert np.all(res["out"][[2, 5]] == 0.0) and np.all(res["n_sel"][[2, 5]] == 0)
    live = [i for i in range(L.B) if mask[i]]
    sub = oracle.moe_decode(L.x[live], L.w_router, L.w_gate, L.w_up, L.w_down, L.k, 2,
                            router_bias=L.router_bias)
    assert np.array_equal(res["expert_idx"][live], sub["expert_idx"])
    assert np.array_equal(res["out"][live], sub["out"])
