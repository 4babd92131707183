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


# ---- brute force on tiny inputs against a set-based statement of Algorithm 2

def alg2_by_sets(rank, mass, k0, p, k_max, max_p):
    """Algorithm 2 written as set algebra, with no loop over ranks that stops early.
    rank[i] = experts of token i from best to worst; mass[i][j] = softmax mass of the expert of rank j.
      t_i   = least t with mass[i][0] + ... + mass[i][t-1] >= p        (p = 1: no cut)
      n_i   = min(k0, t_i),  base_i = {rank[i][0..n_i-1]},  U = union of the base_i
      C_i   = members of U outside base_i whose rank index is below max_p
      S_i   = base_i + those members of C_i that have fewer than k_max - n_i members of C_i ranked above them
    """
    B, N = len(rank), len(rank[0])
    n = []
    for i in range(B):
        if p >= 1.0:
            t = N
        else:
            t = min(t for t in range(1, N + 1) if sum(mass[i][:t]) >= p)
        n.append(min(k0, t))
    base = [set(rank[i][:n[i]]) for i in range(B)]
    U = set().union(*base)
    S = []
    for i in range(B):
        pos = {e: j for j, e in enumerate(rank[i])}
        C = {e for e in U - base[i] if pos[e] < max_p}
        extra = {e for e in C if len({f for f in C if pos[f] < pos[e]}) < k_max - n[i]}
        S.append(sorted(base[i] | extra, key=lambda e: pos[e]))
    return n, sorted(U), S


@pytest.mark.parametrize("N,B", [(4, 2), (3, 2), (4, 1), (2, 2)])
def test_brute_force_all_rankings_alg2(oracle, N, B):
    import itertools
    # logits by rank; different spreads per token so that the top-p cut bites differently
    levels = [np.array([2.0, 1.1, 0.3, -0.6])[:N], np.array([0.9, 0.5, 0.2, -0.1])[:N]]
    masses = [np.exp(v) / np.exp(v).sum() for v in levels]
    # thresholds strictly between the cumulative masses of both tokens (never on a knife edge), and 1 (no cut)
    cums = sorted(set(np.round(np.concatenate([np.cumsum(m)[:-1] for m in masses]), 12).tolist()))
    ps = [cums[0] * 0.5] + [(a + b) / 2 for a, b in zip(cums[:-1], cums[1:])] + [(cums[-1] + 1.0) / 2, 1.0]
    for pv in ps[:-1]:
        assert min(abs(pv - c) for c in cums) > 1e-3
    perms = list(itertools.permutations(range(N)))
    n_cases = 0
    for ranks in itertools.product(perms, repeat=B):
        lg = np.zeros((B, N), np.float32)
        for i in range(B):
            for j, e in enumerate(ranks[i]):
                lg[i, e] = levels[i % 2][j]
        mass = [masses[i % 2].tolist() for i in range(B)]
        for k0 in range(1, N + 1):
            for k_max in range(1, N + 1):
                for max_p in range(1, N + 1):
                    for pv in ps:
                        res = oracle.route_general(lg, k0, pv, k_max, max_p)
                        n, U, S = alg2_by_sets(ranks, mass, k0, pv, k_max, max_p)
                        ctx = (ranks, k0, k_max, max_p, pv)
                        assert res["n_base"].tolist() == n, ctx
                        assert res["active_list"][:res["n_active"]].tolist() == U, ctx
                        kw = max(k0, k_max)
                        for i in range(B):
                            assert res["n_sel"][i] == len(S[i]), ctx
                            assert res["expert_idx"][i, :len(S[i])].tolist() == S[i], ctx
                            assert (res["expert_idx"][i, len(S[i]):kw] == -1).all(), ctx
                            w = np.array([mass[i][ranks[i].index(e)] for e in S[i]])
                            assert np.allclose(res["gate_w"][i, :len(S[i])], w / w.sum(), atol=1e-12), ctx
                        n_cases += 1
    assert n_cases == len(perms) ** B * N ** 3 * len(ps)
