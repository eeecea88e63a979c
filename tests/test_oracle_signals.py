"""Pins for the oracle's signals, threshold and calibration functions."""
import math
import os

import numpy as np
import pytest
from scipy.special import log_softmax

import oracle
from oracle import brute

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_closed_form_fixture():
    for w, tok, s_ref, h_ref in _rows("signals_closed_forms.txt"):
        z = np.log(np.array([float(v) for v in w.split(",")]))
        # logits are stored as fp32: compare against the closed form at 1e-6
        s, h = oracle.signals(z[None, :], [int(tok)])
        assert s[0] == pytest.approx(float(s_ref), abs=2e-7)
        assert h[0] == pytest.approx(float(h_ref), abs=2e-7)


@pytest.mark.parametrize("V", [1000, 32000, 128256])
def test_uniform_is_log_v(V):
    for c in (0.0, -3.5, 40.0):
        s, h = oracle.signals(np.full((1, V), c, np.float32), [V // 3])
        assert h[0] == pytest.approx(math.log(V), abs=1e-9)   # plain ascending fp64 sum of V terms
        assert s[0] == pytest.approx(math.log(V), abs=1e-11)


def test_two_point_closed_form():
    for delta in (0.0, 0.5, 3.0, 20.0):
        z = np.array([[0.0, delta]], np.float32)
        p1 = 1.0 / (1.0 + math.exp(-float(np.float32(delta))))
        p0 = 1.0 - p1
        h_ref = -(p0 * math.log(p0) + p1 * math.log(p1)) if p0 > 0 else 0.0
        s, h = oracle.signals(z, [1])
        assert s[0] == pytest.approx(-math.log(p1), abs=1e-12)
        assert h[0] == pytest.approx(h_ref, abs=1e-12)


def test_matches_scipy_log_softmax_and_pure_python():
    r = np.random.default_rng(0)
    z = (r.standard_normal((4, 257)) * 3).astype(np.float32)
    tok = r.integers(0, 257, 4).astype(np.int32)
    s, h = oracle.signals(z, tok)
    lp = log_softmax(z.astype(np.float64), axis=-1)
    np.testing.assert_allclose(s, -lp[np.arange(4), tok], rtol=1e-12)
    np.testing.assert_allclose(h, -(np.exp(lp) * lp).sum(-1), rtol=1e-12)
    for b in range(4):
        sb, hb = brute.softmax_signals(z[b].astype(np.float64).tolist(), int(tok[b]))
        assert s[b] == pytest.approx(sb, rel=1e-12)
        assert h[b] == pytest.approx(hb, rel=1e-12)


def test_shift_invariance_bounds_and_one_hot_limit():
    r = np.random.default_rng(1)
    z = r.standard_normal((3, 500)).astype(np.float32)
    tok = [0, 10, 499]
    s0, h0 = oracle.signals(z, tok)
    s1, h1 = oracle.signals(z + np.float32(8.0), tok)      # +8 is exact in fp32 at this range? use tolerance
    np.testing.assert_allclose(s1, s0, atol=1e-5)
    np.testing.assert_allclose(h1, h0, atol=1e-5)
    assert (h0 >= 0).all() and (h0 <= math.log(500) + 1e-12).all() and (s0 >= 0).all()
    z = np.zeros((1, 100), np.float32)
    z[0, 7] = 80.0
    s, h = oracle.signals(z, [7])
    assert 0 <= s[0] < 1e-30 or s[0] == 0.0
    assert 0 <= h[0] < 1e-30


def test_expected_surprisal_is_entropy():
    # E_{w~p}[s(w)] = H exactly, by summing p_w * s(w) over the whole vocabulary
    r = np.random.default_rng(2)
    z = (r.standard_normal((1, 64)) * 2).astype(np.float32)
    s_all = np.array([oracle.signals(z, [w])[0][0] for w in range(64)])
    _, h = oracle.signals(z, [0])
    assert float((np.exp(-s_all) * s_all).sum()) == pytest.approx(h[0], rel=1e-12)


def test_minus_inf_nan_and_bad_token():
    z = np.array([[0.0, -np.inf, math.log(3.0)]], np.float32)   # p = 1/4, 0, 3/4
    s, h = oracle.signals(z, [2])
    assert s[0] == pytest.approx(math.log(4 / 3), abs=2e-7)
    assert h[0] == pytest.approx(math.log(4) - 0.75 * math.log(3), abs=2e-7)
    for bad in ([np.nan, 0.0, 1.0], [np.inf, 0.0, 1.0], [-np.inf] * 3):
        s, h = oracle.signals(np.array([bad], np.float32), [0])
        assert math.isnan(s[0]) and math.isnan(h[0])
    s, h = oracle.signals(np.zeros((2, 5), np.float32), [-1, 5])
    assert np.isnan(s).all() and np.allclose(h, math.log(5))


def test_threshold_truth_table_fixture():
    # indicators driven through s and H around tau_s = 2, tau_H = 3 (strict '>')
    for i_s, i_h, factor in _rows("threshold_factors.txt"):
        s = 2.5 if int(i_s) else 2.0          # s == tau_s must NOT fire
        h = 3.5 if int(i_h) else 3.0
        t = oracle.threshold([0.25, 2.0], [0.80, 0.80], [0.12, 0.12], [s], [h], 2.0, 3.0)
        assert t.shape == (2, 1)
        assert t[0, 0] == pytest.approx(0.25 * float(factor), rel=1e-15)
        assert t[1, 0] == pytest.approx(2.0 * float(factor), rel=1e-15)


def test_threshold_layout_signed_coefficients_and_ablation():
    tb, lam, gam = [1.0, 2.0, 4.0], [0.5, -0.8, 0.0], [0.25, -0.12, 0.0]
    s, h = [0.0, 9.0], [9.0, 9.0]
    t = oracle.threshold(tb, lam, gam, s, h, 1.0, 1.0)
    expect = [[1.25, 1.75], [2 * 0.88, 2 * 0.08], [4.0, 4.0]]     # [layer][token]
    np.testing.assert_allclose(t, expect, rtol=1e-15)
    # lambda = gamma = 0 is the "without semantic adaptation" ablation: tau_final = tau_base
    t0 = oracle.threshold(tb, [0, 0, 0], [0, 0, 0], s, h, -np.inf, -np.inf)
    np.testing.assert_array_equal(t0, np.repeat(np.array(tb)[:, None], 2, 1))
    # indicators off / always on
    np.testing.assert_array_equal(oracle.threshold(tb, lam, gam, s, h, np.inf, np.inf), t0)
    # NaN signals never fire an indicator
    tn = oracle.threshold(tb, lam, gam, [np.nan], [np.nan], 0.0, 0.0)
    np.testing.assert_array_equal(tn[:, 0], tb)


@pytest.mark.parametrize("n,q", [(10, 0.4), (1000, 0.45), (999, 0.3), (7, 0.0), (5, 0.999)])
def test_calibrate_is_nearest_rank_order_statistic(n, q):
    r = np.random.default_rng(n)
    pool = np.abs(r.standard_normal(n))
    k = max(1, math.ceil(float(np.float32(q)) * n))
    assert oracle.quantile_rank(n, q) == k
    tau = oracle.calibrate(pool, q)
    assert tau == np.partition(pool, k - 1)[k - 1]
    # achieved sparsity of the pool itself: exactly (k-1)/n lie strictly below
    assert (pool < tau).sum() == k - 1


def test_calibrate_monotone_in_q_and_ties():
    r = np.random.default_rng(5)
    pool = np.abs(r.standard_normal(501))
    taus = [oracle.calibrate(pool, q) for q in np.linspace(0, 0.99, 34)]
    assert all(a <= b for a, b in zip(taus, taus[1:]))
    assert oracle.calibrate([3.0, 1.0, 1.0, 1.0, 2.0], 0.5) == 1.0      # k = 3 -> third smallest
    assert oracle.calibrate([3.0, 1.0, 1.0, 1.0, 2.0], 0.7) == 2.0      # k = 4


def test_calibrated_threshold_hits_target_sparsity_on_fresh_tokens():
    """End-to-end sanity of the percentile reading: threshold from the pooled
    prefix magnitudes gives about the target sparsity on new iid tokens."""
    import synth
    cfg = synth.CONFIGS["c1"]
    w = synth.layer_weights(cfg, 0, 0, d=128, d_ff=344)
    X = synth.prefix_hidden(cfg, 0, 0, T=64, d=128)
    tau = oracle.calibrate(oracle.prefix_stats(*w, X, want_y=False)["abs_act_pool"], cfg.q)
    x = synth.decode_hidden(cfg, 0, 0, 0, B=16, d=128)
    r = oracle.sparse_decode(*w, x, [tau] * 16)
    rho = 1.0 - r["n_active"][1:].mean() / 344
    assert abs(rho - cfg.q) < 0.05
