"""Pins of the oracle's prefix-static mask builders -- CPU only: hand cases, numpy order statistics,
pure-Python selection, and the tie / NaN / signed-zero rules."""
import numpy as np
import pytest

import oracle


def test_threshold_hand_case():
    A = [0.5, 0.2, 0.7, 0.2, float("nan"), 0.0]
    mask, idx = oracle.static_mask_threshold(A, 0.2)
    assert idx.tolist() == [0, 1, 2, 3] and mask.tolist() == [True, True, True, True, False, False]
    assert oracle.static_mask_threshold(A, 0.2000001)[1].tolist() == [0, 2]     # cut iff strictly below
    assert oracle.static_mask_threshold(A, 0.0)[1].tolist() == [0, 1, 2, 3, 5]  # NaN is cut even at 0
    assert oracle.static_mask_threshold(A, float("inf"))[1].tolist() == []


def test_threshold_matches_numpy():
    rng = np.random.default_rng(0)
    A = np.abs(rng.standard_normal(5000))
    for tau in (0.0, 0.3, 1.0, 5.0):
        mask, idx = oracle.static_mask_threshold(A, tau)
        assert np.array_equal(idx, np.flatnonzero(A >= tau)) and np.array_equal(mask, A >= tau)


def test_topk_hand_cases():
    s = [3.0, 1.0, 3.0, 2.0, 3.0, float("nan"), -1.0]
    assert oracle.static_mask_topk(s, 0)[1].tolist() == []
    assert oracle.static_mask_topk(s, 1)[1].tolist() == [0]                  # ties go to the lower index
    assert oracle.static_mask_topk(s, 2)[1].tolist() == [0, 2]
    assert oracle.static_mask_topk(s, 4)[1].tolist() == [0, 2, 3, 4]
    assert oracle.static_mask_topk(s, 6)[1].tolist() == [0, 1, 2, 3, 4, 6]   # -1 still ranks above NaN
    assert oracle.static_mask_topk(s, 7)[1].tolist() == [0, 1, 2, 3, 4, 5, 6]
    assert oracle.static_mask_topk([0.0, -0.0, 0.0], 2)[1].tolist() == [0, 1]  # signed zeros are equal


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_topk_matches_numpy_and_python(seed):
    rng = np.random.default_rng(seed)
    s = np.round(rng.standard_normal(3000), 1)            # many ties
    for k in (1, 17, 1500, 2999, 3000):
        mask, idx = oracle.static_mask_topk(s, k)
        order = np.lexsort((np.arange(s.size), -s))        # score descending, then index ascending
        assert np.array_equal(idx, np.sort(order[:k]))
        assert mask.sum() == k
        py = sorted(sorted(range(s.size), key=lambda j: (-s[j], j))[:k])
        assert idx.tolist() == py
        # the k-th largest value by numpy's partition bounds the kept scores from below
        kth = np.partition(s, s.size - k)[s.size - k]
        assert s[idx].min() == kth and (s[~mask] <= kth).all()
