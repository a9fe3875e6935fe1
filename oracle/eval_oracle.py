"""CPU oracle for the accuracy metric of the paper's experiments.

TEST INFRASTRUCTURE ONLY: imported by tests; shares no code with the HIP path.

What the paper fixes ("Hyperparameters"): accuracy is Hits@100, the metric of the Open Graph Benchmark's link
prediction tasks.  Its published definition, restated: given the scores of the positive test edges and the scores of
a set of negative edges, take the K-th largest negative score as the threshold; Hits@K is the fraction of positive
edges whose score is strictly greater than the threshold.  With fewer than K negatives every positive counts as a
hit.  An empty positive set gives 0 by convention here (the published code would divide by zero).
"""
from __future__ import annotations

import numpy as np


def hits_at_k(pos_scores, neg_scores, K: int):
    """Returns (number of hits, threshold); the threshold is -inf when there are fewer than K negatives."""
    pos = np.asarray(pos_scores, np.float64)
    neg = np.asarray(neg_scores, np.float64)
    if K < 1:
        raise ValueError("K must be positive")
    if neg.size < K:
        return int(pos.size), float("-inf")
    thr = np.sort(neg)[neg.size - K]          # K-th largest
    return int((pos > thr).sum()), float(thr)


def hits_ratio(pos_scores, neg_scores, K: int) -> float:
    n = np.asarray(pos_scores).size
    return hits_at_k(pos_scores, neg_scores, K)[0] / n if n else 0.0
