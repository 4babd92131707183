"""Pins for the oracle's general OEA routing (Algorithm 2), CPU only."""
import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

from paper_2511_02237_amd import workloads as W


def ranking(lg):
    return np.argsort(-lg.astype(np.float64), axis=1, kind="stable")


@pytest.mark.parametrize("kind", W.LOGIT_KINDS)
@pytest.mark.parametrize("k,k0", [(8, 3), (8, 8), (4, 1)])
def test_degenerate_settings_reproduce_alg1(oracle, kind, k, k0):
    # Section 4.1 (Simplifying OEA): p = 1, k^max = k, maxP = N leaves Algorithm 1
    lg = W.make_logits(16, 128, 3, kind)
    a = oracle.route(lg, k, k0)
    g = oracle.route_general(lg, k0, 1.0, k, 128)
    assert np.array_equal(a["expert_idx"], g["expert_idx"])
    assert np.array_equal(a["n_sel"], g["n_sel"])
    assert np.array_equal(a["active_list"], g["active_list"])
    assert np.array_equal(a["gate_w"], g["gate_w"])
    assert np.all(g["n_base"] == k0)


@pytest.mark.parametrize("p", [0.3, 0.5, 0.8, 0.95])
def test_top_p_baseline_size(oracle, p):
    # Algorithm 2, Phase 1: t_i = least t whose sorted cumulative mass reaches p; n_i = min(k0,t_i)
    lg = W.make_logits(16, 64, 8, "skew")
    k0 = 6
    res = oracle.route_general(lg, k0, p, 8, 64)
    R = sp_softmax(lg.astype(np.float64), axis=1)
    r = ranking(lg)
    cum = np.cumsum(np.take_along_axis(R, r, axis=1), axis=1)
    t = (cum >= p).argmax(axis=1) + 1
    margin = np.abs(np.take_along_axis(cum, (t - 1)[:, None], 1)[:, 0] - p)
    ok = margin > 1e-12  # ignore knife-edge rows (none expected)
    assert ok.all()
    assert np.array_equal(res["n_base"], np.minimum(k0, t))
    U = set()
    for i in range(16):
        U.update(r[i, :res["n_base"][i]].tolist())
    assert list(res["active_list"][:res["n_active"]]) == sorted(U)
    for i in range(16):
        n = res["n_sel"][i]
        S = res["expert_idx"][i, :n].tolist()
        assert S[:res["n_base"][i]] == r[i, :res["n_base"][i]].tolist()
        assert set(S) <= U and n <= 8
        # S_i = baseline + best-ranked union members, in rank order
        want = [e for e in r[i].tolist() if e in U][:min(8, len(U))]
        assert S == want


def test_maxp_equal_baseline_is_pruned_routing(oracle):
    # Phase 2 walks ranks n_i+1..maxP: with maxP = k0 there is nothing to walk -> Phase-1 only
    lg = W.make_logits(16, 128, 1, "gaussian")
    res = oracle.route_general(lg, 4, 1.0, 8, 4)
    assert np.all(res["n_sel"] == 4)
    assert np.array_equal(res["expert_idx"][:, :4], ranking(lg)[:, :4])


def test_maxp_limits_piggyback_rank(oracle):
    lg = W.make_logits(16, 128, 2, "gaussian")
    k0, kmax, maxp = 3, 8, 16
    res = oracle.route_general(lg, k0, 1.0, kmax, maxp)
    r = ranking(lg)
    U = set(r[:, :k0].ravel().tolist())
    for i in range(16):
        want = [e for e in r[i, :maxp].tolist() if e in U][:kmax]
        assert res["expert_idx"][i, :res["n_sel"][i]].tolist() == want


def test_kmax_above_and_below_k0(oracle):
    lg = W.make_logits(8, 32, 6, "gaussian")
    r = ranking(lg)
    # k^max larger than the model's k: more piggybacking allowed
    res = oracle.route_general(lg, 2, 1.0, 11, 32)
    U = set(r[:, :2].ravel().tolist())
    assert np.all(res["n_sel"] == min(11, len(U)))
    # baseline larger than k^max is kept whole (the listing initialises S_i with it)
    res = oracle.route_general(lg, 5, 1.0, 3, 32)
    assert np.all(res["n_sel"] == 5)
    assert np.array_equal(res["expert_idx"], r[:, :5])


def test_hand_example_alg2(oracle):
    # worked by hand from Algorithm 2.  Token 0 is confident (softmax mass of its best expert
    # > 0.6), token 1 is flat.  p = 0.6, k0 = 2, k^max = 3, maxP = 3, N = 4.
    lg = np.array([[4.0, 0.0, 0.0, 0.0],      # R = (.948,.017,.017,.017): t_0 = 1 -> n_0 = 1 -> {0}
                   [0.0, 0.3, 0.2, 0.1]],     # R = (.213,.288,.260,.236): .288+.260 < .6 -> t_1 = 3, n_1 = 2 -> {1,2}
                  np.float32)
    res = oracle.route_general(lg, 2, 0.6, 3, 3)
    assert res["n_base"].tolist() == [1, 2]
    assert res["active_list"][:res["n_active"]].tolist() == [0, 1, 2]
    # token 0 ranking 0,1,2,3: walks ranks 2..3 -> adds 1, 2 (cap 3 reached)
    # token 1 ranking 1,2,3,0: walks rank 3 only -> expert 3 not in union; rank 4 (expert 0) is beyond maxP
    assert res["expert_idx"].tolist() == [[0, 1, 2], [1, 2, -1]]
    assert res["n_sel"].tolist() == [3, 2]
