"""Pins of the oracle's non-gated ReLU FFN (OPT family) -- CPU only."""
import numpy as np
import pytest

import oracle


def _toy(seed, d, F, B):
    rng = np.random.default_rng(seed)
    wi = (rng.standard_normal((F, d)) * 0.3).astype(np.float32)
    wo = (rng.standard_normal((F, d)) * 0.3).astype(np.float32)
    bi = (rng.standard_normal(F) * 0.2).astype(np.float32)
    bo = (rng.standard_normal(d) * 0.2).astype(np.float32)
    x = rng.standard_normal((B, d)).astype(np.float32)
    return wi, bi, wo, bo, x


def test_hand_case():
    # x = (1, 2); neuron 0: 1*1 + 0*2 + 0.5 = 1.5 -> 1.5; neuron 1: -1 - 2 + 1 = -2 -> 0; neuron 2: 0.5*2 - 0.25 = 0.75
    wi = np.array([[1, 0], [-1, -1], [0, 0.5]], np.float32)
    bi = np.array([0.5, 1.0, -0.25], np.float32)
    wo = np.array([[1, 1], [5, 5], [2, -2]], np.float32)
    bo = np.array([0.125, -0.125], np.float32)
    x = np.array([[1, 2]], np.float32)
    r = oracle.relu_decode(wi, bi, wo, bo, x)
    assert r["act"][0].tolist() == [1.5, 0.0, 0.75]
    assert r["y"][0].tolist() == [1.5 + 1.5 + 0.125, 1.5 - 1.5 - 0.125]
    r = oracle.relu_decode(wi, bi, wo, bo, x, tau=[0.75])          # tie kept
    assert r["active_idx"].tolist() == [0, 2]
    r = oracle.relu_decode(wi, bi, wo, bo, x, tau=[0.7500001])
    assert r["active_idx"].tolist() == [0] and r["y"][0].tolist() == [1.5 + 0.125, 1.5 - 0.125]
    r = oracle.relu_decode(wi, bi, wo, bo, x, tau=[0.0])           # zero activations are kept at tau = 0
    assert r["active_idx"].tolist() == [0, 1, 2] and r["n_active"].tolist() == [3, 3]
    r = oracle.relu_decode(wi, bi, wo, bo, x, tau=[np.inf])
    assert r["active_idx"].tolist() == [] and r["y"][0].tolist() == [0.125, -0.125]


@pytest.mark.parametrize("seed", [0, 1])
def test_matches_numpy(seed):
    wi, bi, wo, bo, x = _toy(seed, 40, 96, 3)
    a = np.maximum(x.astype(np.float64) @ wi.astype(np.float64).T + bi, 0.0)
    r = oracle.relu_decode(wi, bi, wo, bo, x)
    np.testing.assert_allclose(r["act"], a, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(r["y"], a @ wo.astype(np.float64) + bo, rtol=1e-12, atol=1e-13)
    tau = np.array([0.1, 0.3, 0.0])
    keep = a >= tau[:, None]
    r = oracle.relu_decode(wi, bi, wo, bo, x, tau=tau)
    assert np.array_equal(r["mask"], keep)
    np.testing.assert_allclose(r["y"], (a * keep) @ wo.astype(np.float64) + bo, rtol=1e-12, atol=1e-13)
    assert r["n_active"].tolist() == [int(keep.any(0).sum())] + keep.sum(1).tolist()
    assert r["active_idx"].tolist() == np.flatnonzero(keep.any(0)).tolist()
    # a given mask reproduces the thresholded result; no biases = zero biases
    r2 = oracle.relu_decode(wi, bi, wo, bo, x, mask=keep)
    assert np.array_equal(r2["y"], r["y"])
    r3 = oracle.relu_decode(wi, None, wo, None, x)
    a0 = np.maximum(x.astype(np.float64) @ wi.astype(np.float64).T, 0.0)
    np.testing.assert_allclose(r3["y"], a0 @ wo.astype(np.float64), rtol=1e-12, atol=1e-13)


def test_tau_zero_is_dense_and_rows_are_independent():
    wi, bi, wo, bo, x = _toy(5, 24, 50, 4)
    dense = oracle.relu_decode(wi, bi, wo, bo, x)["y"]
    assert np.array_equal(oracle.relu_decode(wi, bi, wo, bo, x, tau=np.zeros(4))["y"], dense)
    for b in range(4):
        assert np.array_equal(oracle.relu_decode(wi, bi, wo, bo, x[b:b + 1])["y"][0], dense[b])


def test_prefix_stats_match_numpy_and_the_decode_function():
    wi, bi, wo, bo, x = _toy(9, 32, 70, 11)
    r = oracle.relu_prefix_stats(wi, bi, wo, bo, x)
    a = np.maximum(x.astype(np.float64) @ wi.astype(np.float64).T + bi, 0.0)
    np.testing.assert_allclose(r["abs_act_pool"], a, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(r["sum_abs_act"], a.sum(0), rtol=1e-12)
    np.testing.assert_allclose(r["sum_sq_act"], (a * a).sum(0), rtol=1e-12)
    np.testing.assert_allclose(r["sum_sq_h"], (a * a).sum(0), rtol=1e-12)
    np.testing.assert_allclose(r["max_abs_act"], a.max(0), rtol=1e-13)
    np.testing.assert_allclose(r["A"], np.sqrt((a * a).sum(0)) * np.linalg.norm(wo.astype(np.float64), axis=1), rtol=1e-12)
    # the prefill output is the dense decode of every prefix token
    np.testing.assert_allclose(r["y"], oracle.relu_decode(wi, bi, wo, bo, x)["y"], rtol=1e-12, atol=1e-13)


def test_cett_hand_case():
    """The hand case above: a = (1.5, 0, 0.75), rows (1,1), (5,5), (2,-2), b_out = (0.125, -0.125).
    MLP(x) = (1.5 + 1.5 + 0.125, 1.5 - 1.5 - 0.125) = (3.125, -0.125).  eps = 1: neurons 1 (a = 0) and 2 are
    cut, their contribution is 0.75 (2, -2) = (1.5, -1.5); eps = 0.75 cuts only the zero neuron (strict)."""
    wi = np.array([[1, 0], [-1, -1], [0, 0.5]], np.float32)
    bi = np.array([0.5, 1.0, -0.25], np.float32)
    wo = np.array([[1, 1], [5, 5], [2, -2]], np.float32)
    bo = np.array([0.125, -0.125], np.float32)
    x = np.array([[1, 2]], np.float32)
    den = np.hypot(3.125, 0.125)
    c, m = oracle.relu_cett(wi, bi, wo, bo, x, 1.0)
    assert c[0] == pytest.approx(np.hypot(1.5, 1.5) / den, rel=1e-15) and m == c[0]
    assert oracle.relu_cett(wi, bi, wo, bo, x, 0.75)[0][0] == 0.0
    assert oracle.relu_cett(wi, bi, wo, bo, x, 0.0)[0][0] == 0.0
    c, _ = oracle.relu_cett(wi, bi, wo, bo, x, np.inf)               # everything cut: the bias stays
    assert c[0] == pytest.approx(np.hypot(3.0, 0.0) / den, rel=1e-15)
    c, _ = oracle.relu_cett(wi, None, wo, None, x, np.inf)           # without biases: a = (1, 0, 1), all cut = the output
    assert c[0] == pytest.approx(1.0, rel=1e-15)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_cett_is_dense_minus_sparse_over_dense_and_search_is_brute_force(seed):
    wi, bi, wo, bo, x = _toy(seed, 24, 40, 6)
    act = oracle.relu_decode(wi, bi, wo, bo, x)["act"]
    dense = oracle.relu_decode(wi, bi, wo, bo, x)["y"]
    cands = np.unique(act)
    means = []
    for eps in list(cands) + [np.inf]:
        kept = oracle.relu_decode(wi, bi, wo, bo, x, tau=eps)["y"]                 # keeps a >= eps, adds b_out
        want = np.linalg.norm(dense - kept, axis=1) / np.linalg.norm(dense, axis=1)
        got, mean = oracle.relu_cett(wi, bi, wo, bo, x, eps)
        np.testing.assert_allclose(got, want, rtol=1e-9, atol=1e-12)
        assert mean == pytest.approx(want.mean(), rel=1e-9, abs=1e-12)
        means.append(want.mean())
    assert means[0] == 0.0                                                           # the smallest value cuts nothing
    for bound in (0.0, 0.05, 0.2, 0.5):
        feasible = [i for i in range(len(cands)) if means[i] <= bound * (1 + 1e-12)]
        tau, mean, rc = oracle.relu_cett_search(wi, bi, wo, bo, x, bound)
        assert rc == 0 and tau == cands[feasible[-1]] and mean == pytest.approx(means[feasible[-1]], rel=1e-9, abs=1e-12)
    tau, mean, rc = oracle.relu_cett_search(wi, None, wo, None, x, 0.999999)         # without a bias cutting all loses all: 1 > bound
    assert rc == 0 and np.isfinite(tau)


def test_cett_search_takes_the_last_feasible_value_not_the_first_crossing():
    """Constructed: a = (1, 2, 3), output rows (1,0), (-0.5,0), (0,1), so MLP(x) = (0, 3).  eps = 2 cuts the first
    neuron (CETT 1/3), eps = 3 cuts the first two, whose contributions cancel (CETT 0): with bound 0.2 the
    feasible values are 1 and 3, and the maximum is 3 although 2 already broke the bound."""
    wi = np.array([[1, 0], [2, 0], [0, 3]], np.float32)
    wo = np.array([[1, 0], [-0.5, 0], [0, 1]], np.float32)
    x = np.array([[1, 1]], np.float32)
    assert [oracle.relu_cett(wi, None, wo, None, x, e)[1] for e in (1, 2, 3)] == [0.0, pytest.approx(1 / 3), 0.0]
    tau, mean, rc = oracle.relu_cett_search(wi, None, wo, None, x, 0.2)
    assert (tau, mean, rc) == (3.0, 0.0, 0)
