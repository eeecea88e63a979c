"""Pins of the oracle's GELU-gated FFN (sigma = tanh-form GELU, the Gemma model of the paper's
experiments) -- CPU only.  Every gated oracle function takes sigma="gelu_tanh"."""

import numpy as np
import pytest
import torch

import oracle
from oracle import brute


def _toy(seed, d, F, B, scale=0.6):
    rng = np.random.default_rng(seed)
    w = [(rng.standard_normal((F, d)) * scale).astype(np.float32) for _ in range(3)]
    x = rng.standard_normal((B, d)).astype(np.float32)
    return w, x


def test_sigma_values_closed_forms():
    """gate_act on a 1 x 1 'layer' evaluates sigma itself: GELU(0) = 0, GELU(g) - GELU(-g) = g (tanh is
    odd), GELU(g) -> g for large g and -> -0 for very negative g, the minimum is about -0.17 near -0.75."""
    one = np.ones((1, 1), np.float32)
    def s(g):
        return float(oracle.gate_act(one, np.array([[g]], np.float32), sigma="gelu_tanh")[0, 0])
    assert s(0.0) == 0.0
    for g in (0.25, 1.0, 2.5, 7.0):
        assert s(g) - s(-g) == pytest.approx(g, rel=1e-14)
    assert s(12.0) == pytest.approx(12.0, rel=1e-12) and abs(s(-12.0)) < 1e-12
    grid = np.linspace(-3, 0, 3001)
    vals = np.array([s(g) for g in grid])
    assert vals.min() == pytest.approx(-0.17, abs=2e-3) and grid[vals.argmin()] == pytest.approx(-0.75, abs=0.01)
    # and it is not SiLU
    assert abs(s(1.0) - float(oracle.gate_act(one, np.array([[1.0]], np.float32))[0, 0])) > 0.1


@pytest.mark.parametrize("seed", [0, 1])
def test_matches_library_gelu(seed):
    """Against torch's own tanh-form GELU in fp64 (a library routine, not this formula retyped)."""
    w, x = _toy(seed, 24, 40, 3)
    g = torch.from_numpy(x.astype(np.float64)) @ torch.from_numpy(w[0].astype(np.float64)).T
    a = torch.nn.functional.gelu(g, approximate="tanh").numpy()
    np.testing.assert_allclose(oracle.gate_act(w[0], x, sigma="gelu_tanh"), a, rtol=1e-12, atol=1e-15)
    u = x.astype(np.float64) @ w[1].astype(np.float64).T
    y = (a * u) @ w[2].astype(np.float64)
    np.testing.assert_allclose(oracle.dense_decode(*w, x, sigma="gelu_tanh"), y, rtol=1e-11, atol=1e-13)
    tau = np.array([0.05, 0.15, 0.0])
    keep = np.abs(a) >= tau[:, None]
    r = oracle.sparse_decode(*w, x, tau, sigma="gelu_tanh")
    assert np.array_equal(r["mask"], keep)
    np.testing.assert_allclose(r["y"], (a * u * keep) @ w[2].astype(np.float64), rtol=1e-11, atol=1e-13)
    assert r["active_idx"].tolist() == np.flatnonzero(keep.any(0)).tolist()
    st = oracle.prefix_stats(*w, x, sigma="gelu_tanh")
    np.testing.assert_allclose(st["abs_act_pool"], np.abs(a), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(st["y"], y, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(st["A"], np.sqrt(((a * u) ** 2).sum(0)) * np.linalg.norm(w[2].astype(np.float64), axis=1),
                               rtol=1e-11)


def test_limits_and_brute_force_masks():
    """tau = 0 keeps everything (= dense), tau = inf keeps nothing; on an 8-neuron toy layer the kept set and
    the output agree with the pure-Python brute force."""
    w, x = _toy(5, 6, 8, 1)
    dense = oracle.dense_decode(*w, x, sigma="gelu_tanh")
    assert np.array_equal(oracle.sparse_decode(*w, x, [0.0], sigma="gelu_tanh")["y"], dense)
    r = oracle.sparse_decode(*w, x, [np.inf], sigma="gelu_tanh")
    assert r["n_active"].tolist() == [0, 0] and not r["y"].any()
    wl = [a.astype(np.float64).tolist() for a in w]
    xl = x[0].astype(np.float64).tolist()
    for tau in (0.02, 0.1, 0.3):
        kept = brute.kept_set(wl[0], xl, tau, sigma=brute.gelu_tanh)
        r = oracle.sparse_decode(*w, x, [tau], sigma="gelu_tanh")
        assert r["active_idx"].tolist() == kept
        yb = brute.ffn_for_subset(wl[0], wl[1], wl[2], xl, kept, sigma=brute.gelu_tanh)
        np.testing.assert_allclose(r["y"][0], yb, rtol=1e-12, atol=1e-14)
    assert 0 < len(brute.kept_set(wl[0], xl, 0.1, sigma=brute.gelu_tanh)) < 8


def test_cett_with_gelu_sigma():
    """CETT limits and its definition written out with the library GELU."""
    w, X = _toy(9, 12, 20, 5)
    per, mean = oracle.cett(*w, X, 0.0, sigma="gelu_tanh")
    assert not per.any() and mean == 0.0
    per, mean = oracle.cett(*w, X, np.inf, sigma="gelu_tanh")
    np.testing.assert_allclose(per, 1.0, rtol=1e-12)
    eps = 0.12
    g = torch.from_numpy(X.astype(np.float64)) @ torch.from_numpy(w[0].astype(np.float64)).T
    a = torch.nn.functional.gelu(g, approximate="tanh").numpy()
    h = a * (X.astype(np.float64) @ w[1].astype(np.float64).T)
    wd = w[2].astype(np.float64)
    ref = np.linalg.norm((h * (np.abs(a) < eps)) @ wd, axis=1) / np.linalg.norm(h @ wd, axis=1)
    per, mean = oracle.cett(*w, X, eps, sigma="gelu_tanh")
    np.testing.assert_allclose(per, ref, rtol=1e-10)
    assert mean == pytest.approx(ref.mean(), rel=1e-12)
    tau, m, rc = oracle.cett_search(*w, X, 0.2, sigma="gelu_tanh")
    assert rc == 0 and m <= 0.2 and oracle.cett(*w, X, np.nextafter(tau, np.inf), sigma="gelu_tanh")[1] > 0.2


def test_sigma_argument_does_not_leak_between_calls():
    w, x = _toy(2, 8, 8, 2)
    a = oracle.dense_decode(*w, x)
    b = oracle.dense_decode(*w, x, sigma="gelu_tanh")
    assert not np.allclose(a, b)
    assert np.array_equal(oracle.dense_decode(*w, x), a)
