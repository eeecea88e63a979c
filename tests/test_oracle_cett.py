"""Pins of the oracle's CETT evaluation and base-threshold search (section 3.2.2) -- CPU only.

The pins are independent of the code they check: a hand-worked example, a pure-Python brute force
over every candidate threshold, the already pinned sparse/dense decode functions (a different code
path), a closed form for orthogonal output rows, and a constructed case where the error is not
monotone in the threshold."""
import math
import os

import numpy as np
import pytest

import oracle
from oracle import brute

GOLD = os.path.join(os.path.dirname(__file__), "golden", "cett_worked_example.txt")


def _gold():
    out = {}
    for line in open(GOLD):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            out[k] = float(v)
    return out


def _toy(seed, d, F, T, scale=0.5):
    rng = np.random.default_rng(seed)
    w = [(rng.standard_normal((F, d)) * scale).astype(np.float32) for _ in range(3)]
    x = rng.standard_normal((T, d)).astype(np.float32)
    return w, x


def test_worked_example():
    g = _gold()
    ln3 = np.float32(g["ln3"])
    wg = np.array([[ln3, 0], [-ln3, 0], [0, 0]], np.float32)
    wu = np.array([[1, 0], [2, 0], [5, 0]], np.float32)
    wd = np.array([[1, 0], [0, 1], [1, 1]], np.float32)
    x = np.array([[1, 0]], np.float32)
    for eps, want in ((0.0, 0.0), (0.1, 0.0), (g["a1_abs"] * 0.999, 0.0), (0.3, g["cett_mid"]),
                      (g["a0"] * 0.999, g["cett_mid"]), (0.9, 1.0), (math.inf, 1.0)):
        c, m = oracle.cett(wg, wu, wd, x, eps)
        assert c[0] == pytest.approx(want, abs=1e-7) and m == pytest.approx(want, abs=1e-7)
    tau, mean, rc = oracle.cett_search(wg, wu, wd, x, 0.2)
    assert rc == 0 and tau == pytest.approx(g["tau_bound_0.2"], rel=1e-6) and mean == pytest.approx(0.0, abs=1e-12)
    tau, mean, rc = oracle.cett_search(wg, wu, wd, x, 0.6)
    assert rc == 0 and tau == pytest.approx(g["tau_bound_0.6"], rel=1e-6) and mean == pytest.approx(g["cett_mid"], abs=1e-7)
    tau, mean, rc = oracle.cett_search(wg, wu, wd, x, 1.0)
    assert rc == 3 and math.isinf(tau) and mean == pytest.approx(1.0, abs=1e-12)


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_against_pure_python_brute_force(seed):
    d, F, T = 6, 9, 4
    w, x = _toy(seed, d, F, T)
    wl = [a.astype(np.float64).tolist() for a in w]
    xl = x.astype(np.float64).tolist()
    mags = np.sort(np.abs(oracle.gate_act(w[0], x)).ravel())
    for eps in (0.0, float(mags[3]), float(mags[F * T // 2]) * 1.0000001, float(mags[-1]), float(mags[-1]) * 2):
        c, m = oracle.cett(*w, x, eps)
        want = [brute.cett_token(*wl, xt, eps) for xt in xl]
        np.testing.assert_allclose(c, want, rtol=1e-10, atol=1e-13)
        assert m == pytest.approx(sum(want) / T, rel=1e-12, abs=1e-15)
    for bound in (0.0, 0.05, 0.2, 0.5, 0.999, 1.0):
        tau, mean, rc = oracle.cett_search(*w, x, bound)
        want = brute.cett_argmax(*wl, xl, bound)
        if want is None:
            assert rc == 4
        elif math.isinf(want):
            assert rc == 3 and math.isinf(tau)
        else:
            assert rc == 0 and tau == pytest.approx(want, rel=1e-12)
            assert mean <= bound


def test_equals_dense_minus_sparse_decode():
    """The cut sum is the dense output minus the kept sum: ties CETT to the decode functions."""
    w, x = _toy(7, 48, 160, 6, scale=0.2)
    dense = oracle.dense_decode(*w, x)
    for eps in (0.02, 0.1, 0.4):
        sparse = oracle.sparse_decode(*w, x, np.full(len(x), eps))["y"]
        want = np.linalg.norm(dense - sparse, axis=1) / np.linalg.norm(dense, axis=1)
        c, m = oracle.cett(*w, x, eps)
        np.testing.assert_allclose(c, want, rtol=1e-9, atol=1e-12)
        assert m == pytest.approx(want.mean(), rel=1e-12)


def test_closed_form_for_orthogonal_output_rows():
    """W_down = diag(s): contributions are orthogonal, so CETT^2 = sum_cut (h s)^2 / sum_all (h s)^2."""
    rng = np.random.default_rng(11)
    n, T = 40, 5
    wg = (rng.standard_normal((n, n)) * 0.3).astype(np.float32)
    wu = (rng.standard_normal((n, n)) * 0.3).astype(np.float32)
    s = rng.uniform(0.5, 2.0, n).astype(np.float32)
    wd = np.diag(s).astype(np.float32)
    x = rng.standard_normal((T, n)).astype(np.float32)
    g = x.astype(np.float64) @ wg.astype(np.float64).T
    a = g / (1.0 + np.exp(-g))
    h = a * (x.astype(np.float64) @ wu.astype(np.float64).T)
    for eps in (0.05, 0.2, 0.6):
        e2 = (h * s) ** 2
        want = np.sqrt((e2 * (np.abs(a) < eps)).sum(1) / e2.sum(1))
        c, _ = oracle.cett(wg, wu, wd, x, eps)
        np.testing.assert_allclose(c, want, rtol=1e-10)


def test_limits_and_zero_output_token():
    w, x = _toy(3, 16, 32, 3)
    c, m = oracle.cett(*w, x, 0.0)
    assert np.all(c == 0.0) and m == 0.0                       # nothing is strictly below 0
    c, m = oracle.cett(*w, x, np.inf)
    np.testing.assert_allclose(c, 1.0, rtol=1e-12)             # everything cut: the whole output is lost
    x[1] = 0.0                                                 # a token with zero dense output
    c, _ = oracle.cett(*w, x, 0.3)
    assert c[1] == 0.0 and c[0] > 0.0


def test_search_takes_the_last_feasible_candidate_not_the_first_crossing():
    """Contributions (1,0), (-1,0), (0,2) at magnitudes m0 < m1 < m2: cutting {0} loses half the
    output norm, cutting {0,1} loses nothing.  The maximum of the feasible set is m2."""
    gs = np.array([0.2, 0.4, 1.0])
    a = gs / (1.0 + np.exp(-gs))
    wg = np.array([[gs[0], 0], [gs[1], 0], [gs[2], 0]], np.float32)
    wu = np.array([[1, 0], [1, 0], [1, 0]], np.float32)
    wd = np.array([[1 / a[0], 0], [-1 / a[1], 0], [0, 2 / a[2]]], np.float32)
    x = np.array([[1, 0]], np.float32)
    assert oracle.cett(wg, wu, wd, x, 0.5 * (a[0] + a[1]))[1] == pytest.approx(0.5, rel=1e-6)
    assert oracle.cett(wg, wu, wd, x, 0.5 * (a[1] + a[2]))[1] == pytest.approx(0.0, abs=1e-6)
    tau, mean, rc = oracle.cett_search(wg, wu, wd, x, 0.2)
    assert rc == 0 and tau == pytest.approx(a[2], rel=1e-6) and mean < 1e-6


@pytest.mark.parametrize("bound", [0.1, 0.2, 0.35])
def test_search_result_is_a_pooled_magnitude_and_the_boundary(bound):
    """tau is one of the pooled |a|; it is feasible; every larger pooled magnitude is infeasible
    (checked with the evaluation function, which shares no state with the search)."""
    w, x = _toy(21, 64, 256, 12, scale=0.15)
    tau, mean, rc = oracle.cett_search(*w, x, bound)
    assert rc == 0
    pool = np.sort(oracle.prefix_stats(*w, x, want_y=False)["abs_act_pool"].ravel())
    k = int(np.searchsorted(pool, tau))
    assert pool[k] == tau
    assert oracle.cett(*w, x, tau)[1] == pytest.approx(mean, rel=1e-10) and mean <= bound
    for kk in list(range(k + 1, min(k + 12, len(pool)))) + [min(len(pool) - 1, k + 200), len(pool) - 1]:
        if pool[kk] > tau:
            assert oracle.cett(*w, x, pool[kk])[1] > bound
