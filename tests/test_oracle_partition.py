"""Pins for the oracle's step-2 partition (ranking the blocks, threshold, pools)."""
import numpy as np
import pytest

from oracle import partition as PT


def brute(score, n_top, higher):
    """Rank by explicit pairwise counting: block i stays iff fewer than n_top blocks beat it strictly."""
    s = [float(v) for v in score]
    keep = []
    for v in s:
        better = sum(1 for u in s if (u > v if higher else u < v))
        keep.append(better < n_top)
    return np.array(keep)


@pytest.mark.parametrize("higher", [True, False])
def test_brute_force_on_small_inputs_with_ties(higher):
    rng = np.random.default_rng(5)
    for N in (1, 2, 7, 33):
        s = rng.integers(-3, 4, N).astype(np.float32) / np.float32(4.0)   # many equal scores
        for n_top in range(N + 1):
            tau, pool_b, n_a = PT.partition(s, n_top, higher)
            keep = brute(s, n_top, higher)
            assert np.array_equal(pool_b == 0, keep)
            assert n_a == keep.sum() and n_a >= n_top
            if n_top:
                # tau is the score of rank n_top in a full sort
                srt = np.sort(s)[::-1] if higher else np.sort(s)
                assert tau == srt[n_top - 1]


def test_distinct_scores_give_exactly_n_top_and_match_argsort():
    rng = np.random.default_rng(6)
    s = rng.permutation(1000).astype(np.float32) / np.float32(1000.0) * 2 - 1
    for n_top in (0, 1, 250, 999, 1000):
        tau, pool_b, n_a = PT.partition(s, n_top, True)
        assert n_a == n_top
        top = np.argsort(-s, kind="stable")[:n_top]
        assert set(np.flatnonzero(pool_b == 0)) == set(top)
        # numpy's selection routine gives the same threshold
        if n_top:
            assert tau == np.partition(s, s.size - n_top)[s.size - n_top]
    tau, pool_b, n_a = PT.partition(s, 0, True)
    assert np.isposinf(tau) and pool_b.all()
    tau, _, _ = PT.partition(s, 0, False)
    assert np.isneginf(tau)


def test_order_of_blocks_does_not_matter_and_zeros_tie():
    rng = np.random.default_rng(7)
    s = rng.standard_normal(500).astype(np.float32)
    s[:5] = 0.0
    s[5:9] = -0.0
    perm = rng.permutation(s.size)
    n_top = int((s > 0).sum()) + 2                    # the threshold falls among the zeros
    tau, pool_b, n_a = PT.partition(s, n_top, True)
    tau2, pool_b2, n_a2 = PT.partition(s[perm], n_top, True)
    assert tau == tau2 == 0.0 and n_a == n_a2 == (s >= 0).sum()
    assert np.array_equal(pool_b[perm], pool_b2)
    assert not pool_b[:9].any()                        # +0 and -0 both stay


def test_percentage_to_count():
    assert PT.top_count(0.0, 1000) == 0 and PT.top_count(100.0, 1000) == 1000
    assert PT.top_count(50.0, 7) == 4 and PT.top_count(87.5, 16) == 14     # 3.5 -> 4, 14.0
    assert PT.top_count(12.5, 4) == 1                                     # 0.5 -> 1
    with pytest.raises(ValueError):
        PT.top_count(101.0, 10)
    with pytest.raises(ValueError):
        PT.partition(np.array([np.nan], dtype=np.float32), 1)
