"""Pins for the oracle's selection rule (Alg. 1 TopK, ties -> lower index)."""
import numpy as np
import pytest

from oracle import vitcop_oracle as O


def brute_smallest(s, keep):
    # independent formulation: lexicographic sort on (score, index)
    order = np.lexsort((np.arange(len(s)), s))
    return np.sort(order[:keep]).astype(np.int32)


def brute_largest(s, keep):
    order = np.lexsort((np.arange(len(s)), -np.asarray(s)))
    return np.sort(order[:keep]).astype(np.int32)


@pytest.mark.parametrize("seed", range(20))
def test_brute_force_with_ties(seed):
    g = np.random.default_rng(seed)
    n = int(g.integers(1, 65))
    # few distinct values -> many exact ties
    s = g.integers(0, 6, size=n).astype(np.float64) * 0.25
    for keep in {0, 1, n // 3, n // 2, n - 1, n} - {-1}:
        if 0 <= keep <= n:
            assert np.array_equal(O.topk_smallest(s, keep), brute_smallest(s, keep))
            assert np.array_equal(O.topk_largest(s, keep), brute_largest(s, keep))


@pytest.mark.parametrize("seed", range(5))
def test_brute_force_distinct(seed):
    g = np.random.default_rng(100 + seed)
    s = g.random(64)
    for keep in (1, 7, 32, 63):
        assert np.array_equal(O.topk_smallest(s, keep), brute_smallest(s, keep))
        assert np.array_equal(O.topk_largest(s, keep), brute_largest(s, keep))


def test_uniform_scores_keep_lowest_indices():
    s = np.full(50, 3.5)
    assert np.array_equal(O.topk_smallest(s, 13), np.arange(13))
    assert np.array_equal(O.topk_largest(s, 13), np.arange(13))


def test_hand_example():
    # scores:            0    1    2    3    4    5
    s = np.array([2.0, 1.0, 2.0, 0.5, 1.0, 3.0])
    assert O.topk_smallest(s, 2).tolist() == [1, 3]        # 0.5, then the first 1.0
    assert O.topk_smallest(s, 3).tolist() == [1, 3, 4]
    assert O.topk_smallest(s, 4).tolist() == [0, 1, 3, 4]  # first of the two 2.0
    assert O.topk_largest(s, 2).tolist() == [0, 5]         # 3.0, then the first 2.0
    assert O.topk_largest(s, 1).tolist() == [5]


def test_complement_rule():
    # kept smallest-k == complement of the (n-k) largest when the dropped side
    # breaks ties toward the HIGHER index
    g = np.random.default_rng(7)
    s = g.integers(0, 5, size=40).astype(np.float64)
    n = len(s)
    for keep in (0, 5, 17, 40):
        order = np.lexsort((-np.arange(n), -s))   # score desc, index desc
        dropped = set(order[:n - keep].tolist())
        kept = sorted(set(range(n)) - dropped)
        assert O.topk_smallest(s, keep).tolist() == kept


def test_keep_list_layout_and_count():
    g = np.random.default_rng(3)
    B, T, vs, nv, keep = 3, 40, 5, 24, 7
    norms = g.random((B, nv)) + 0.5
    idx = O.keep_list(norms, T, vs, keep)
    assert idx.shape == (B, T - nv + keep) and idx.dtype == np.int32
    for b in range(B):
        row = idx[b]
        assert np.all(np.diff(row) > 0)
        assert row[:vs].tolist() == list(range(vs))
        assert row[vs + keep:].tolist() == list(range(vs + nv, T))
        vis = row[vs:vs + keep] - vs
        assert np.array_equal(vis, brute_smallest(norms[b], keep))


def test_keep_all_and_keep_none():
    norms = np.random.default_rng(1).random((2, 10))
    assert np.array_equal(O.keep_list(norms, 16, 2, 10), np.tile(np.arange(16), (2, 1)))
    assert np.array_equal(O.keep_list(norms, 16, 2, 0),
                          np.tile(np.r_[0:2, 12:16], (2, 1)))


def test_tie_band():
    s = np.array([1.0, 1.0004, 0.5, 2.0, 0.9995, 1.5])
    band = O.tie_band(s, 2, largest=False)           # 2nd smallest is 0.9995
    assert band.tolist() == [True, True, False, False, True, False]
    band = O.tie_band(s, 1, largest=True)            # largest is 2.0
    assert band.tolist() == [False, False, False, True, False, False]
    assert not O.tie_band(s, 0, False).any() and not O.tie_band(s, 6, False).any()
