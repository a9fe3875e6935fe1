"""CPU oracle for the degree-based graph sparsifier of the paper (Algorithm 1, "Graph Sparsification" part).

TEST INFRASTRUCTURE ONLY: imported by the tests, the smoke check and the benchmark's cpu_baseline leg; it shares
no code with the HIP path and never calls it.

What the paper fixes (Sec. IV-B, second paragraph, and Algorithm 1, the loop "for l = 1 to L^i"):
  * L draws, independent, with replacement, from the edge list of one partition;
  * edge (u, v) is drawn with probability p_(u,v) proportional to 1/d_u + 1/d_v (the degree bound on the
    effective resistance, Theorem 2), d being the node degrees in that partition's edge list;
  * a drawn edge enters the sparsified set with weight 1/(L p_(u,v)); drawing it again adds the same amount.
Hence the result is: the set of distinct drawn edges, and for each the weight c_e / (L p_e), c_e = times drawn.

What the paper leaves open, and the reading taken here so that the drawn edge indices are reproducible bit for bit:
  * probabilities are carried as integers, q_e = floor(2^32 / d_u) + floor(2^32 / d_v), p_e = q_e / Q, Q = sum q_e
    (each p_e is within d_max / 2^32 relative of the exact ratio; Q < 2^63 because sum_e (1/d_u + 1/d_v) equals
    the number of nodes that have an edge);
  * draw l takes the 64-bit number r = word0 * 2^32 + word1 of Philox4x32-10(counter = (l_lo, l_hi, 0, 0),
    key = (seed_lo, seed_hi)), maps it to t = floor(r * Q / 2^64) and selects the edge whose slice
    [cum_e, cum_e + q_e) of [0, Q) holds t, cum being the running sum of q in input order;
  * the output lists the distinct drawn edges in input order.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from oracle.lp_oracle import philox4x32_10

SCALE_BITS = 32


@dataclass
class Sparsified:
    kept_edge: np.ndarray     # int32 [n_kept]: indices into the input edge list, ascending
    count: np.ndarray         # int32 [n_kept]: how many of the L draws chose the edge
    weight: np.ndarray        # float64 [n_kept]: count / (L * p_e)
    q: np.ndarray             # uint64 [n_edges]: integer sampling weights
    total: int                # Q


def degrees(n_nodes: int, eu: np.ndarray, ev: np.ndarray) -> np.ndarray:
    """d_u = number of listed edges that touch u (Sec. IV-A: degree = row sum of the adjacency matrix)."""
    return np.bincount(np.asarray(eu, np.int64), minlength=n_nodes) + np.bincount(np.asarray(ev, np.int64), minlength=n_nodes)


def sampling_weights(n_nodes: int, eu: np.ndarray, ev: np.ndarray) -> np.ndarray:
    """q_e = floor(2^32/d_u) + floor(2^32/d_v): the degree bound 1/d_u + 1/d_v on the effective resistance
    (Theorem 2), in units of 2^-32."""
    d = degrees(n_nodes, eu, ev).astype(np.uint64)
    one = np.uint64(1) << np.uint64(SCALE_BITS)
    return one // d[np.asarray(eu, np.int64)] + one // d[np.asarray(ev, np.int64)]


def _mulhi64(a: np.ndarray, b: int) -> np.ndarray:
    """floor(a * b / 2^64) for uint64 arrays a and a Python int 0 <= b < 2^64, by 32-bit limbs."""
    m32 = np.uint64(0xFFFFFFFF)
    s32 = np.uint64(32)
    a_lo, a_hi = a & m32, a >> s32
    b_lo, b_hi = np.uint64(b & 0xFFFFFFFF), np.uint64(b >> 32)
    ll = a_lo * b_lo
    lh = a_lo * b_hi
    hl = a_hi * b_lo
    hh = a_hi * b_hi
    mid = (ll >> s32) + (lh & m32) + (hl & m32)
    return hh + (lh >> s32) + (hl >> s32) + (mid >> s32)


def draw_edges(q: np.ndarray, n_draws: int, seed: int) -> np.ndarray:
    """Edge index of each of the n_draws draws (int64 [n_draws])."""
    cum = np.concatenate([np.zeros(1, np.uint64), np.cumsum(q, dtype=np.uint64)])
    total = int(cum[-1])
    l = np.arange(n_draws, dtype=np.uint64)
    zero = np.zeros(n_draws, np.uint64)
    w = philox4x32_10(l & np.uint64(0xFFFFFFFF), l >> np.uint64(32), zero, zero, seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    r = (w[0] << np.uint64(32)) | w[1]
    t = _mulhi64(r, total)
    return np.searchsorted(cum, t, side="right").astype(np.int64) - 1


def sparsify(n_nodes: int, eu: np.ndarray, ev: np.ndarray, n_draws: int, seed: int) -> Sparsified:
    """The sparsified edge set of one partition and its weights (Algorithm 1, lines of the sparsification loop)."""
    m = int(np.asarray(eu).size)
    if m == 0 or n_draws <= 0:
        z = np.zeros(0, np.int32)
        return Sparsified(z, z.copy(), np.zeros(0), np.zeros(m, np.uint64), 0)
    q = sampling_weights(n_nodes, eu, ev)
    total = int(q.sum(dtype=np.uint64))
    e = draw_edges(q, n_draws, seed)
    counts = np.bincount(e, minlength=m)
    kept = np.flatnonzero(counts)
    p = q[kept].astype(np.float64) / float(total)
    weight = counts[kept].astype(np.float64) / (float(n_draws) * p)
    return Sparsified(kept.astype(np.int32), counts[kept].astype(np.int32), weight, q, total)
