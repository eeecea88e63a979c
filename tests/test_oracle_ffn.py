"""Pins for the oracle's FFN functions (prefill, sparse decode, dense twin).

The oracle is checked against things other than itself: numpy's fp64 matmul
(a library routine), scalar hand cases, a pure-Python brute force over all 2^8
masks of toy layers, and the invariants the definitions fix (tau=0 => dense,
tau=inf => 0, nested masks, y(tau) = y_dense - cut terms, row independence,
neuron permutation).  Shapes are non-square so a transposed operand fails.
"""
import math

import numpy as np
import pytest

import oracle
from oracle import brute


def _toy(seed, d=6, F=8, T=5, B=3, scale=0.7):
    r = np.random.default_rng(seed)
    wg = (r.standard_normal((F, d)) * scale).astype(np.float32)
    wu = (r.standard_normal((F, d)) * scale).astype(np.float32)
    wd = (r.standard_normal((F, d)) * scale).astype(np.float32)
    X = r.standard_normal((T, d)).astype(np.float32)
    x = r.standard_normal((B, d)).astype(np.float32)
    return wg, wu, wd, X, x


def _np_dense(wg, wu, wd, x):
    """Dense SwiGLU FFN with numpy's fp64 matmul."""
    wg, wu, wd, x = (a.astype(np.float64) for a in (wg, wu, wd, x))
    g = x @ wg.T
    a = g / (1.0 + np.exp(-g))
    h = a * (x @ wu.T)
    return h @ wd, a, h


def test_scalar_hand_case():
    # d = d_ff = 1: y = SiLU(wg x) * (wu x) * wd
    wg, wu, wd, x = 0.5, -1.25, 2.0, 1.5
    g = wg * x
    expect = g / (1 + math.exp(-g)) * (wu * x) * wd
    y = oracle.dense_decode([[wg]], [[wu]], [[wd]], [[x]])
    assert y.shape == (1, 1)
    assert y[0, 0] == pytest.approx(expect, rel=1e-15)
    r = oracle.sparse_decode([[wg]], [[wu]], [[wd]], [[x]], [0.0])
    assert r["y"][0, 0] == pytest.approx(expect, rel=1e-15)
    assert r["act"][0, 0] == pytest.approx(g / (1 + math.exp(-g)), rel=1e-15)


@pytest.mark.parametrize("seed,d,F,B", [(0, 6, 8, 3), (1, 40, 24, 2), (2, 17, 33, 5)])
def test_dense_matches_numpy_matmul(seed, d, F, B):
    wg, wu, wd, _, x = _toy(seed, d=d, F=F, B=B)
    y_np, _, _ = _np_dense(wg, wu, wd, x)
    y = oracle.dense_decode(wg, wu, wd, x)
    np.testing.assert_allclose(y, y_np, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("seed,d,F,T", [(3, 6, 8, 5), (4, 24, 40, 7), (5, 33, 17, 3)])
def test_prefix_matches_numpy(seed, d, F, T):
    wg, wu, wd, X, _ = _toy(seed, d=d, F=F, T=T)
    y_np, a, h = _np_dense(wg, wu, wd, X)
    r = oracle.prefix_stats(wg, wu, wd, X)
    np.testing.assert_allclose(r["y"], y_np, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(r["abs_act_pool"], np.abs(a), rtol=1e-13)
    np.testing.assert_allclose(r["sum_abs_act"], np.abs(a).sum(0), rtol=1e-13)
    np.testing.assert_allclose(r["sum_sq_act"], (a * a).sum(0), rtol=1e-13)
    np.testing.assert_allclose(r["max_abs_act"], np.abs(a).max(0), rtol=1e-13)
    np.testing.assert_allclose(r["sum_sq_h"], (h * h).sum(0), rtol=1e-13)
    wn = np.linalg.norm(wd.astype(np.float64), axis=1)
    np.testing.assert_allclose(r["A"], np.sqrt((h * h).sum(0)) * wn, rtol=1e-13)


def test_neuron_magnitude_is_frobenius_norm_of_rank_one_term():
    # A_j by its literal reading (norm of h_{:,j} W_down[j,:]) via pure-Python loops
    wg, wu, wd, X, _ = _toy(6, d=5, F=8, T=4)
    r = oracle.prefix_stats(wg, wu, wd, X)
    lists = [a.astype(np.float64).tolist() for a in (wg, wu, wd, X)]
    for j in range(8):
        assert r["A"][j] == pytest.approx(brute.neuron_magnitude(*lists, j), rel=1e-12)
    # T = 1: A_j = |h_j| * ||W_down[j]||
    r1 = oracle.prefix_stats(wg, wu, wd, X[:1])
    _, _, h = _np_dense(wg, wu, wd, X[:1])
    np.testing.assert_allclose(r1["A"], np.abs(h[0]) * np.linalg.norm(wd.astype(np.float64), axis=1),
                               rtol=1e-13)


def test_tau_zero_is_dense_bitwise_and_tau_inf_is_zero():
    wg, wu, wd, _, x = _toy(7, d=12, F=20, B=4)
    dense = oracle.dense_decode(wg, wu, wd, x)
    r0 = oracle.sparse_decode(wg, wu, wd, x, [0.0] * 4)
    assert np.array_equal(r0["y"], dense)
    assert r0["mask"].all() and list(r0["n_active"]) == [20] * 5
    assert np.array_equal(r0["active_idx"], np.arange(20))
    ri = oracle.sparse_decode(wg, wu, wd, x, [np.inf] * 4)
    assert np.array_equal(ri["y"], np.zeros_like(dense))
    assert not ri["mask"].any() and list(ri["n_active"]) == [0] * 5
    assert ri["active_idx"].size == 0


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_brute_force_all_masks_8_neuron_toy(seed):
    """Among all 2^8 masks the oracle picks exactly {j : |a_j| >= tau} and its
    output is that mask's sum, for thresholds at, between and outside the
    activation magnitudes."""
    wg, wu, wd, _, x = _toy(seed, d=5, F=8, B=1)
    L = [a.astype(np.float64).tolist() for a in (wg, wu, wd)]
    xl = x[0].astype(np.float64).tolist()
    table = brute.all_subset_outputs(*L, xl)
    mags = sorted(abs(t[0]) for t in brute.neuron_terms(L[0], L[1], xl))
    taus = [0.0, mags[0] * 0.5, mags[-1] * 2.0]
    taus += [(mags[i] + mags[i + 1]) / 2 for i in range(7)]      # between magnitudes
    taus += mags                                                  # ties: |a| == tau is kept
    for tau in taus:
        r = oracle.sparse_decode(wg, wu, wd, x, [tau])
        kept = brute.kept_set(L[0], xl, tau)
        bits = sum(1 << j for j in kept)
        assert list(r["active_idx"]) == kept
        assert [int(b) for b in r["mask"][0]] == [bits >> j & 1 for j in range(8)]
        np.testing.assert_allclose(r["y"][0], table[bits], rtol=1e-12, atol=1e-14)
        # every other mask gives a different output (so the choice is identified)
        others = [k for k, v in table.items()
                  if k != bits and np.allclose(v, r["y"][0], rtol=1e-9, atol=1e-12)]
        assert others == []


def test_tie_is_kept_and_strictly_below_is_cut():
    wg, wu, wd, _, x = _toy(21, d=7, F=9, B=1)
    a = np.abs(oracle.gate_act(wg, x)[0])
    j = int(np.argsort(a)[4])
    r_eq = oracle.sparse_decode(wg, wu, wd, x, [a[j]])
    assert r_eq["mask"][0, j]
    r_up = oracle.sparse_decode(wg, wu, wd, x, [np.nextafter(a[j], np.inf)])
    assert not r_up["mask"][0, j]
    assert r_up["n_active"][0] == r_eq["n_active"][0] - 1


def test_masks_nested_and_output_is_dense_minus_cut_terms():
    wg, wu, wd, _, x = _toy(22, d=10, F=30, B=1)
    y_dense, a, h = _np_dense(wg, wu, wd, x)
    prev = None
    for tau in [0.0, 0.05, 0.1, 0.2, 0.4, 0.8, 5.0]:
        r = oracle.sparse_decode(wg, wu, wd, x, [tau])
        m = r["mask"][0]
        assert np.array_equal(m, np.abs(a[0]) >= tau)
        if prev is not None:
            assert not (m & ~prev).any()           # mask(tau2) subset of mask(tau1)
        prev = m
        cut = (h[0][~m, None] * wd.astype(np.float64)[~m]).sum(0)
        np.testing.assert_allclose(r["y"][0], y_dense[0] - cut, rtol=1e-10, atol=1e-12)


def test_batch_rows_are_independent_and_union_list():
    wg, wu, wd, _, x = _toy(23, d=9, F=16, B=4)
    tau = [0.05, 0.3, 0.0, 1.5]
    r = oracle.sparse_decode(wg, wu, wd, x, tau)
    union = np.zeros(16, bool)
    for b in range(4):
        rb = oracle.sparse_decode(wg, wu, wd, x[b:b + 1], tau[b:b + 1])
        assert np.array_equal(rb["y"][0], r["y"][b])
        assert np.array_equal(rb["mask"][0], r["mask"][b])
        assert rb["n_active"][0] == r["n_active"][1 + b]
        union |= rb["mask"][0]
    assert np.array_equal(r["active_idx"], np.flatnonzero(union))
    assert r["n_active"][0] == union.sum()


def test_neuron_permutation_permutes_indices_only():
    wg, wu, wd, _, x = _toy(24, d=8, F=12, B=1)
    perm = np.random.default_rng(0).permutation(12)
    r = oracle.sparse_decode(wg, wu, wd, x, [0.2])
    rp = oracle.sparse_decode(wg[perm], wu[perm], wd[perm], x, [0.2])
    assert np.array_equal(rp["mask"][0], r["mask"][0][perm])
    np.testing.assert_allclose(rp["y"], r["y"], rtol=1e-12, atol=1e-14)


def test_decode_given_mask_matches_subset_sum():
    wg, wu, wd, _, x = _toy(25, d=5, F=8, B=2)
    mask = np.array([[1, 0, 1, 1, 0, 0, 1, 0], [0, 0, 0, 1, 1, 1, 1, 1]], np.uint8)
    y = oracle.decode_given_mask(wg, wu, wd, x, mask)
    L = [a.astype(np.float64).tolist() for a in (wg, wu, wd)]
    for b in range(2):
        ref = brute.ffn_for_subset(*L, x[b].astype(np.float64).tolist(),
                                   [j for j in range(8) if mask[b, j]])
        np.testing.assert_allclose(y[b], ref, rtol=1e-12, atol=1e-14)


def test_nan_activation_is_cut():
    wg, wu, wd, _, x = _toy(26, d=4, F=6, B=1)
    wg = wg.copy()
    wg[2, 0] = np.nan
    r = oracle.sparse_decode(wg, wu, wd, x, [0.0])
    assert not r["mask"][0, 2] and r["n_active"][0] == 5
    assert np.isfinite(r["y"]).all()


def test_thread_count_does_not_change_bits(monkeypatch):
    import subprocess
    import sys
    code = ("import numpy as np, oracle, synth;"
            "c=synth.CONFIGS['c1'];w=synth.layer_weights(c,0,0,d=64,d_ff=96);"
            "x=synth.decode_hidden(c,0,0,0,B=2,d=64);"
            "r=oracle.sparse_decode(*w,x,[0.1,0.2]);print(r['y'].tobytes().hex()[:4096])")
    outs = []
    for nt in ("1", "5"):
        env = dict(__import__("os").environ, OMP_NUM_THREADS=nt)
        outs.append(subprocess.run([sys.executable, "-c", code], env=env, capture_output=True,
                                   text=True, check=True, cwd=__import__("conftest").ROOT).stdout)
    assert outs[0] == outs[1] and len(outs[0]) > 100
