"""Pins of the Hits@K oracle: the rank formulation written out independently, hand cases, ties, degenerate sizes."""
import numpy as np
import pytest

from oracle import eval_oracle as E


def hits_by_rank(pos, neg, K):
    """A positive is a hit iff fewer than K negatives score at least as high (brute force, O(n_pos * n_neg))."""
    return sum(1 for p in pos if sum(1 for q in neg if q >= p) < K)


@pytest.mark.parametrize("seed", range(6))
def test_matches_the_rank_formulation_on_small_random_inputs(seed):
    rng = np.random.default_rng(seed)
    n_pos, n_neg = int(rng.integers(1, 40)), int(rng.integers(1, 60))
    # few distinct values: ties between positives and negatives are common
    pos = rng.integers(-5, 6, n_pos).astype(np.float32) / 4
    neg = rng.integers(-5, 6, n_neg).astype(np.float32) / 4
    for K in (1, 2, 5, n_neg, n_neg + 1):
        hits, thr = E.hits_at_k(pos, neg, K)
        if K > n_neg:
            assert hits == n_pos and thr == float("-inf")
        else:
            assert hits == hits_by_rank(pos, neg, K), (seed, K)
            assert (neg >= thr).sum() >= K and (neg > thr).sum() < K      # thr really is the K-th largest


def test_hand_cases():
    neg = [0.1, 0.9, 0.5, 0.7]
    assert E.hits_at_k([0.8, 0.6, 0.95], neg, 1) == (1, 0.9)              # only 0.95 beats the best negative
    assert E.hits_at_k([0.8, 0.6, 0.95], neg, 2) == (2, 0.7)
    assert E.hits_at_k([0.7], neg, 2) == (0, 0.7)                          # a tie with the threshold is not a hit
    assert E.hits_at_k([0.7], neg, 3) == (1, 0.5)
    assert E.hits_at_k([-3.0, 2.0], neg, 5) == (2, float("-inf"))          # fewer negatives than K
    assert E.hits_at_k([], neg, 1)[0] == 0 and E.hits_ratio([], neg, 1) == 0.0
    assert E.hits_ratio([1.0, 0.0], [0.5], 1) == 0.5


def test_monotone_in_k_and_invariant_under_order():
    rng = np.random.default_rng(9)
    pos, neg = rng.standard_normal(200), rng.standard_normal(500)
    prev = -1
    for K in (1, 3, 10, 100, 500):
        h = E.hits_at_k(pos, neg, K)[0]
        assert h >= prev
        prev = h
        assert E.hits_at_k(rng.permutation(pos), rng.permutation(neg), K)[0] == h
    with pytest.raises(ValueError):
        E.hits_at_k(pos, neg, 0)
