"""Pins for the oracle's routing functions (CPU only).

Nothing here re-types the oracle's own loop: each test compares it with something the paper or
plain mathematics fixes - a library routine (numpy argsort / scipy softmax), an invariant stated in
the paper, a closed form, a hand-worked example, or a set-based brute-force definition.
"""
import itertools
import json
import os

import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

from paper_2511_02237_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def topk_stable(logits, k):
    """Library definition of the default router (Section 3.2: Top_k = first k of the ranking)."""
    order = np.argsort(-logits.astype(np.float64), axis=1, kind="stable")
    return order[:, :k].astype(np.int32)


def sets_of(res):
    return [set(int(e) for e in row[:n]) for row, n in zip(res["expert_idx"], res["n_sel"])]


CASES = [(B, N, k, k0, kind, seed)
         for (B, N, k) in [(4, 16, 4), (16, 128, 8), (3, 7, 5), (33, 64, 6), (1, 128, 8), (128, 128, 8)]
         for k0 in sorted({1, max(1, k // 2), k})
         for kind in W.LOGIT_KINDS
         for seed in (0, 1)]


# ---------------------------------------------------------------- ranking

@pytest.mark.parametrize("kind", W.LOGIT_KINDS)
def test_rank_is_stable_descending_sort(oracle, kind):
    # Section 3.2 (Notation): R_{e_{i,1}} >= R_{e_{i,2}} >= ...; ties -> lower id (stable argsort)
    lg = W.make_logits(9, 37, 5, kind)
    r = oracle.rank(lg)
    ref = np.argsort(-lg.astype(np.float64), axis=1, kind="stable")
    assert np.array_equal(r, ref)


def test_softmax_matches_library(oracle):
    lg = W.make_logits(6, 50, 3, "wide")
    assert np.allclose(oracle.softmax(lg), sp_softmax(lg.astype(np.float64), axis=1), rtol=1e-13, atol=0)


# ---------------------------------------------------------------- Algorithm 1 invariants

@pytest.mark.parametrize("B,N,k,k0,kind,seed", CASES)
def test_alg1_invariants(oracle, B, N, k, k0, kind, seed):
    lg = W.make_logits(B, N, seed, kind)
    res = oracle.route(lg, k, k0)
    S = sets_of(res)
    base = topk_stable(lg, k0)
    U = set(int(e) for e in base.ravel())
    T = res["n_active"]
    # the union is exactly the baseline union, listed ascending (Algorithm 1, Phase 2 first line)
    assert T == len(U)
    assert list(res["active_list"][:T]) == sorted(U)
    assert np.all(res["active_list"][T:] == -1)
    for i in range(B):
        # Phase 1 is batch independent: every token keeps its own top-k0 (Section 1, item 1)
        assert set(int(e) for e in base[i]) <= S[i]
        assert list(res["expert_idx"][i, :k0]) == list(base[i])
        # piggybacked experts only come from the union (Section 1, item 2)
        assert S[i] <= U
        # never more than k; exactly min(k,|U|) (Section 4.1, finding 2; reading R1/R5)
        assert res["n_sel"][i] == min(k, len(U)) == len(S[i])
        assert np.all(res["expert_idx"][i, res["n_sel"][i]:] == -1)
        assert np.all(res["gate_w"][i, res["n_sel"][i]:] == 0.0)
    # Phase 2 keeps the number of activated experts at |S^base| (Section 3.2, Phase 2)
    assert set().union(*S) == U
    # compute term of Eq. 2: total load never exceeds B*k
    assert int(res["n_sel"].sum()) <= B * k


@pytest.mark.parametrize("B,N,k,kind,seed",
                         [(B, N, k, kind, s) for (B, N, k) in [(4, 16, 4), (16, 128, 8), (5, 9, 9)]
                          for kind in W.LOGIT_KINDS for s in (0, 1, 2)])
def test_k0_equal_k_is_plain_topk(oracle, B, N, k, kind, seed):
    # Section 4.2: the base model is k0 = k
    lg = W.make_logits(B, N, seed, kind)
    res = oracle.route(lg, k, k)
    assert np.array_equal(res["expert_idx"], topk_stable(lg, k))
    assert np.all(res["n_sel"] == k)
    # Eq. 1 weights: softmax scores renormalised over the top-k
    R = sp_softmax(lg.astype(np.float64), axis=1)
    sel = np.take_along_axis(R, res["expert_idx"].astype(np.int64), axis=1)
    assert np.allclose(res["gate_w"], sel / sel.sum(1, keepdims=True), rtol=1e-12, atol=0)


@pytest.mark.parametrize("kind", W.LOGIT_KINDS)
def test_batch_of_one_has_no_piggybacking(oracle, kind):
    # Section 4.1 (Dataset): a batch size of 1 makes the piggybacking redundant
    lg = W.make_logits(1, 128, 11, kind)
    for k0 in (1, 3, 8):
        res = oracle.route(lg, 8, k0)
        assert res["n_sel"][0] == k0
        assert np.array_equal(res["expert_idx"][0, :k0], topk_stable(lg, k0)[0])


@pytest.mark.parametrize("kind", ["gaussian", "ties", "skew"])
def test_T_monotone_in_k0_and_bounded_by_topk(oracle, kind):
    lg = W.make_logits(16, 128, 21, kind)
    Ts = [oracle.route(lg, 8, k0)["n_active"] for k0 in range(1, 9)]
    assert all(a <= b for a, b in zip(Ts, Ts[1:]))
    assert Ts[-1] == len(set(topk_stable(lg, 8).ravel().tolist()))


# ---------------------------------------------------------------- closed form: masked top-k

def masked_topk(lg, k, k0):
    """Alg. 1 rewritten: S_i = best min(k,|U|) experts of token i among U = union of top-k0."""
    B, N = lg.shape
    base = topk_stable(lg, k0)
    mask = np.zeros(N, bool)
    mask[base.ravel()] = True
    out = np.full((B, k), -1, np.int32)
    key = np.where(mask[None, :], lg.astype(np.float64), -np.inf)
    order = np.argsort(-key, axis=1, kind="stable")
    n = min(k, int(mask.sum()))
    out[:, :n] = order[:, :n]
    return out, n


@pytest.mark.parametrize("B,N,k,k0,kind,seed", CASES)
def test_alg1_equals_masked_topk(oracle, B, N, k, k0, kind, seed):
    lg = W.make_logits(B, N, seed, kind)
    if not np.all(np.isfinite(lg)):
        pytest.skip("non-finite")
    res = oracle.route(lg, k, k0)
    ref, n = masked_topk(lg, k, k0)
    assert np.array_equal(res["expert_idx"], ref)
    assert np.all(res["n_sel"] == n)


# ---------------------------------------------------------------- exhaustive brute force

def brute_sets(ranks, k, k0):
    """Set-based definition on explicit rankings: U = union of first k0; S_i = the min(k,|U|)
    members of U that token i ranks best."""
    U = set()
    for r in ranks:
        U.update(r[:k0])
    n = min(k, len(U))
    out = []
    for r in ranks:
        pos = {e: j for j, e in enumerate(r)}
        out.append(sorted(U, key=lambda e: pos[e])[:n])
    return sorted(U), out


@pytest.mark.parametrize("N,B", [(3, 3), (4, 3), (5, 2)])
def test_exhaustive_rank_tuples(oracle, N, B):
    perms = list(itertools.permutations(range(N)))
    # logits realising a ranking: expert at rank j gets value N-j
    def logits_of(r):
        v = np.empty(N, np.float32)
        for j, e in enumerate(r):
            v[e] = N - j
        return v
    rows = {r: logits_of(r) for r in perms}
    n_checked = 0
    for ranks in itertools.product(perms, repeat=B):
        lg = np.stack([rows[r] for r in ranks])
        for k in range(1, N + 1):
            for k0 in range(1, k + 1):
                res = oracle.route(lg, k, k0)
                U, sets = brute_sets(ranks, k, k0)
                assert list(res["active_list"][:res["n_active"]]) == U
                for i in range(B):
                    assert list(res["expert_idx"][i, :res["n_sel"][i]]) == sets[i]
                n_checked += 1
    assert n_checked == len(perms) ** B * N * (N + 1) // 2


# ---------------------------------------------------------------- equivariance

def test_permutation_equivariance(oracle):
    rng = np.random.default_rng(4)
    lg = W.make_logits(12, 48, 9, "gaussian")
    k, k0 = 6, 2
    res = oracle.route(lg, k, k0)
    # reorder tokens
    tp = rng.permutation(12)
    res_t = oracle.route(lg[tp], k, k0)
    assert np.array_equal(res_t["expert_idx"], res["expert_idx"][tp])
    assert np.array_equal(res_t["active_list"], res["active_list"])
    # relabel experts (distinct logits, so no tie-break dependence on ids)
    ep = rng.permutation(48)  # new id ep[j] holds old expert j
    lg2 = np.empty_like(lg)
    lg2[:, ep] = lg
    res_e = oracle.route(lg2, k, k0)
    assert np.array_equal(res_e["expert_idx"], np.where(res["expert_idx"] >= 0, ep[res["expert_idx"]], -1))
    assert np.allclose(res_e["gate_w"], res["gate_w"], rtol=1e-12)


# ---------------------------------------------------------------- gate weights (Eq. 1)

@pytest.mark.parametrize("kind", ["gaussian", "skew", "wide", "ties"])
def test_gate_weights_renormalised_scores(oracle, kind):
    lg = W.make_logits(16, 128, 2, kind)
    res = oracle.route(lg, 8, 3)
    R = sp_softmax(lg.astype(np.float64), axis=1)
    for i in range(16):
        n = res["n_sel"][i]
        sel = R[i, res["expert_idx"][i, :n]]
        assert np.allclose(res["gate_w"][i, :n], sel / sel.sum(), rtol=1e-11, atol=1e-300)
        assert abs(res["gate_w"][i].sum() - 1.0) < 1e-12
    # adding a per-token constant to the logits changes nothing (softmax shift invariance);
    # power-of-two shifts of a 0.5-grid stay exact in fp32
    if kind == "ties":
        res2 = oracle.route(lg + np.float32(4.0), 8, 3)
        assert np.array_equal(res2["expert_idx"], res["expert_idx"])
        assert np.allclose(res2["gate_w"], res["gate_w"], rtol=1e-12)


# ---------------------------------------------------------------- hand-worked examples

def test_golden_hand_examples(oracle):
    with open(os.path.join(GOLDEN, "alg1_hand_examples.json")) as f:
        examples = json.load(f)["examples"]
    assert len(examples) >= 4
    for ex in examples:
        lg = np.array(ex["logits"], np.float32)
        res = oracle.route(lg, ex["k"], ex["k0"])
        assert list(res["active_list"][:res["n_active"]]) == ex["union"], ex["name"]
        got = [list(map(int, row[:n])) for row, n in zip(res["expert_idx"], res["n_sel"])]
        assert got == ex["sets"], ex["name"]


# ---------------------------------------------------------------- expected number of active experts

@pytest.mark.parametrize("B,N,k0s", [(16, 128, range(1, 9)), (4, 16, (1, 2, 4))])
def test_mean_T_matches_uniform_routing_formula(oracle, B, N, k0s):
    # Section 2, footnote: E[T] = N (1 - (1 - k/N)^B) under uniform routing (82 at N=128,k=8,B=16)
    seeds = 256
    logits = [W.make_logits(B, N, 7000 + s, "gaussian") for s in range(seeds)]
    for k0 in k0s:
        k = max(k0s)
        mean_T = np.mean([oracle.route(lg, k, k0)["n_active"] for lg in logits])
        expect = N * (1.0 - (1.0 - k0 / N) ** B)
        assert abs(mean_T - expect) <= 0.03 * expect, (k0, mean_T, expect)
    assert round(128 * (1 - (1 - 8 / 128) ** 16)) == 82


# ---------------------------------------------------------------- parameter checks / padding mask

def test_illegal_parameters_rejected(oracle):
    lg = W.make_logits(4, 16, 0)
    for k, k0 in [(4, 0), (4, 5), (17, 1), (0, 0)]:
        with pytest.raises(ValueError):
            oracle.route(lg, k, k0)


def test_token_mask_removes_padded_tokens(oracle):
    # Section 6 (A note on padding): padded tokens must not add experts
    lg = W.make_logits(10, 64, 5, "gaussian")
    live = oracle.route(lg[:6], 8, 3)
    mask = np.array([1] * 6 + [0] * 4, np.uint8)
    res = oracle.route(lg, 8, 3, token_mask=mask)
    assert res["n_active"] == live["n_active"]
    assert np.array_equal(res["active_list"], live["active_list"])
    assert np.array_equal(res["expert_idx"][:6], live["expert_idx"])
    assert np.all(res["n_sel"][6:] == 0) and np.all(res["expert_idx"][6:] == -1)
    assert np.all(res["gate_w"][6:] == 0.0)
