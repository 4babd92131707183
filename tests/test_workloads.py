"""The seeded input generators: determinism, storage rounding, recipe (CPU only)."""
import numpy as np
import pytest

from paper_2511_02237_amd import workloads as W


def test_bf16_round_matches_torch():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(0)
    a = np.concatenate([rng.standard_normal(20000).astype(np.float32) * np.float32(s)
                        for s in (1e-3, 0.02, 1.0, 300.0)])
    # exact ties and signed zeros
    a = np.concatenate([a, np.array([1.00390625, 1.01171875, -1.00390625, 0.0, -0.0], np.float32)])
    ours = W.bf16_round(a)
    ref = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)
    assert np.array_equal(W.bf16_to_f32(ours), torch.from_numpy(a).to(torch.bfloat16).float().numpy())


def test_layers_are_reproducible_and_shaped():
    a = W.make_layer("toy", 12)
    b = W.make_layer("toy", 12)
    c = W.make_layer("toy", 13)
    for f in ("x", "w_router", "w_gate", "w_up", "w_down"):
        assert np.array_equal(getattr(a, f), getattr(b, f))
        assert not np.array_equal(getattr(a, f), getattr(c, f))
    assert a.x.shape == (4, 64) and a.w_router.shape == (16, 64)
    assert a.w_gate.shape == (16, 32, 64) and a.w_up.shape == (16, 32, 64) and a.w_down.shape == (16, 64, 32)
    assert a.x.dtype == np.float32
    m = W.make_layer("mid_bf16", 1)
    assert m.x.dtype == np.uint16 and m.w_down.dtype == np.uint16


def test_distributions_follow_recipe():
    L = W.make_layer("mid_bf16", 2, B=64)
    x, wr, wg = W.widen(L.x), W.widen(L.w_router), W.widen(L.w_gate)
    assert abs(x.std() - 1.0) < 0.02 and abs(x.mean()) < 0.02
    assert abs(wr.std() - L.d ** -0.5) < 0.05 * L.d ** -0.5
    assert abs(wg.std() - 0.02) < 0.001
    # logits come out ~N(0,1): near-uniform expert popularity
    lg = x @ wr.T
    assert abs(lg.std() - 1.0) < 0.1


def test_skew_recipe():
    L = W.make_layer("mid_bf16", 3, skew=True, B=32)
    x = W.widen(L.x)
    # tokens share a common component: pairwise correlation ~ 0.49/(0.49+0.09)
    c = np.corrcoef(x)
    off = c[~np.eye(32, dtype=bool)].mean()
    assert 0.75 < off < 0.92
    b = L.router_bias.astype(np.float64)
    pop = np.exp(b / 2)
    assert abs(pop.sum() - 1.0) < 1e-5
    ranks = np.sort(pop)[::-1]
    assert np.allclose(ranks / ranks[0], np.arange(1, L.N + 1) ** -1.1, rtol=1e-4)


@pytest.mark.parametrize("kind", W.LOGIT_KINDS)
def test_logit_kinds(kind):
    a = W.make_logits(5, 33, 1, kind)
    assert a.shape == (5, 33) and a.dtype == np.float32
    assert np.array_equal(a.view(np.uint32), W.make_logits(5, 33, 1, kind).view(np.uint32))
    if kind == "signed_zero":
        assert (np.signbit(a) & (a == 0)).any() and ((~np.signbit(a)) & (a == 0)).any()
    if kind == "denormal":
        assert (np.abs(a[a != 0]) < np.finfo(np.float32).tiny).all()
