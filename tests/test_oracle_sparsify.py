"""Pins for the sparsifier oracle (Algorithm 1, "Graph Sparsification"; Sec. IV-B second paragraph; Theorems 1-2).

None of these re-types the oracle's own formula: probabilities are checked against exact rational arithmetic and
closed forms on regular / star / path graphs, the draw map against a draw-by-draw walk with Python integers, the
weights against the unbiasedness that Theorem 1's estimator has by construction, the sparsified Laplacian against
the original one (Theorem 1), and the degree bound itself against exact effective resistances (Theorem 2).
"""
from fractions import Fraction

import numpy as np
import pytest

from oracle import lp_oracle as O
from oracle import sparsify_oracle as S


def random_simple_graph(rng, n, m):
    pairs = set()
    while len(pairs) < m:
        u, v = rng.integers(0, n, 2)
        if u != v:
            pairs.add((min(u, v), max(u, v)))
    e = np.array(sorted(pairs), np.int32)
    rng.shuffle(e)
    return e[:, 0].copy(), e[:, 1].copy()


def test_probabilities_match_exact_rationals():
    rng = np.random.default_rng(0)
    n = 40
    eu, ev = random_simple_graph(rng, n, 120)
    q = S.sampling_weights(n, eu, ev)
    deg = [0] * n
    for u, v in zip(eu.tolist(), ev.tolist()):
        deg[u] += 1
        deg[v] += 1
    exact = [Fraction(1, deg[u]) + Fraction(1, deg[v]) for u, v in zip(eu.tolist(), ev.tolist())]
    z = sum(exact)
    # sum over edges of 1/d_u + 1/d_v counts every node that has an edge exactly once
    assert z == sum(1 for d in deg if d > 0)
    total = int(q.sum())
    for qe, pe in zip(q.tolist(), exact):
        assert abs(Fraction(qe, total) - pe / z) < Fraction(1, 10 ** 8) * (pe / z)


def test_regular_star_and_path_graphs():
    # cycle: every degree 2 -> uniform
    n = 12
    eu = np.arange(n, dtype=np.int32)
    ev = ((np.arange(n) + 1) % n).astype(np.int32)
    q = S.sampling_weights(n, eu, ev)
    assert np.all(q == q[0]) and int(q[0]) == 2 ** 32
    # star: every edge joins the hub (degree n-1) and a leaf (degree 1) -> uniform
    eu = np.zeros(n - 1, np.int32)
    ev = np.arange(1, n, dtype=np.int32)
    q = S.sampling_weights(n, eu, ev)
    assert np.all(q == q[0]) and int(q[0]) == 2 ** 32 + 2 ** 32 // (n - 1)
    # path on 5 nodes: end edges 1 + 1/2, inner edges 1/2 + 1/2
    eu = np.array([0, 1, 2, 3], np.int32)
    ev = np.array([1, 2, 3, 4], np.int32)
    q = S.sampling_weights(5, eu, ev).astype(np.float64)
    np.testing.assert_allclose(q / q[1], [1.5, 1.0, 1.0, 1.5], rtol=1e-9)
    # orientation of a listed edge does not matter
    assert np.array_equal(S.sampling_weights(5, ev, eu), S.sampling_weights(5, eu, ev))


def scalar_draws(q, n_draws, seed):
    """Draw by draw with Python integers."""
    cum = [0]
    for x in q.tolist():
        cum.append(cum[-1] + x)
    total = cum[-1]
    out = []
    for l in range(n_draws):
        w = O.philox4x32_10(l & 0xFFFFFFFF, l >> 32, 0, 0, seed & 0xFFFFFFFF, seed >> 32)
        r = (w[0] << 32) | w[1]
        t = (r * total) >> 64
        assert 0 <= t < total
        e = max(i for i in range(len(q)) if cum[i] <= t)       # the slice [cum_e, cum_e + q_e) that holds t
        assert t < cum[e + 1]
        out.append(e)
    return np.array(out, np.int64)


@pytest.mark.parametrize("seed", [0, 1, 2 ** 40 + 17])
def test_draws_match_scalar_walkthrough(seed):
    rng = np.random.default_rng(3)
    eu, ev = random_simple_graph(rng, 30, 80)
    q = S.sampling_weights(30, eu, ev)
    assert np.array_equal(S.draw_edges(q, 500, seed), scalar_draws(q, 500, seed))


def test_mulhi_against_python_integers():
    rng = np.random.default_rng(4)
    a = rng.integers(0, 2 ** 64, 1000, dtype=np.uint64)
    a[:3] = [0, 2 ** 64 - 1, 2 ** 63]
    for b in (1, 2 ** 63 - 1, 2 ** 32 * 235000 + 12345, 3):
        got = S._mulhi64(a, b)
        assert [int(x) for x in got] == [(int(x) * b) >> 64 for x in a]


def test_draw_frequencies_follow_the_probabilities():
    rng = np.random.default_rng(5)
    eu, ev = random_simple_graph(rng, 25, 60)
    q = S.sampling_weights(25, eu, ev)
    L = 200000
    e = S.draw_edges(q, L, 99)
    obs = np.bincount(e, minlength=q.size).astype(np.float64)
    exp = L * q.astype(np.float64) / float(q.sum())
    chi2 = ((obs - exp) ** 2 / exp).sum()
    assert chi2 < 59 + 5 * np.sqrt(2 * 59)           # 59 degrees of freedom, five sigma


def test_result_structure_and_counts():
    rng = np.random.default_rng(6)
    n, m, L = 200, 900, 135                          # L = 0.15 |E|, the paper's default level
    eu, ev = random_simple_graph(rng, n, m)
    r = S.sparsify(n, eu, ev, L, 7)
    assert np.all(np.diff(r.kept_edge) > 0) and r.kept_edge.min() >= 0 and r.kept_edge.max() < m
    assert int(r.count.sum()) == L and np.all(r.count >= 1)
    assert r.kept_edge.size <= L                     # at least 85 % of the edges are gone at level 0.15
    p = r.q[r.kept_edge].astype(np.float64) / r.total
    np.testing.assert_allclose(r.weight, r.count / (L * p), rtol=1e-12)
    again = S.sparsify(n, eu, ev, L, 7)
    assert np.array_equal(again.kept_edge, r.kept_edge) and np.array_equal(again.count, r.count)
    other = S.sparsify(n, eu, ev, L, 8)
    assert not np.array_equal(other.kept_edge, r.kept_edge)
    empty = S.sparsify(n, eu[:0], ev[:0], 10, 1)
    assert empty.kept_edge.size == 0
    none = S.sparsify(n, eu, ev, 0, 1)
    assert none.kept_edge.size == 0


def test_weights_are_unbiased_estimates_of_the_unit_edge_weights():
    """E[w_e] = L p_e / (L p_e) = 1 for every edge: the mean over many independent seeds approaches 1."""
    rng = np.random.default_rng(8)
    n, m, L = 20, 40, 400
    eu, ev = random_simple_graph(rng, n, m)
    acc = np.zeros(m)
    trials = 300
    for s in range(trials):
        r = S.sparsify(n, eu, ev, L, 1000 + s)
        acc[r.kept_edge] += r.weight
    mean = acc / trials
    # Var[w_e] = (1 - p_e)/(L p_e) <= 1/(L p_min); p_min here is about 1/(3 m)
    sigma = np.sqrt(3.0 * m / L / trials)
    assert np.abs(mean - 1.0).max() < 6 * sigma


def laplacian(n, eu, ev, w):
    Lm = np.zeros((n, n))
    for u, v, x in zip(eu.tolist(), ev.tolist(), np.asarray(w, np.float64).tolist()):
        Lm[u, u] += x
        Lm[v, v] += x
        Lm[u, v] -= x
        Lm[v, u] -= x
    return Lm


def test_sparsified_laplacian_approximates_the_original_quadratic_form():
    """Theorem 1 with the degree bound of Theorem 2 as the sampling law: with many draws, x^T L~ x stays within
    a small factor of x^T L x."""
    rng = np.random.default_rng(9)
    n, m = 60, 900                                    # dense enough for a small spectral gap penalty
    eu, ev = random_simple_graph(rng, n, m)
    r = S.sparsify(n, eu, ev, 40 * m, 11)
    L0 = laplacian(n, eu, ev, np.ones(m))
    L1 = laplacian(n, eu[r.kept_edge], ev[r.kept_edge], r.weight)
    for _ in range(20):
        x = rng.standard_normal(n)
        a, b = x @ L0 @ x, x @ L1 @ x
        assert abs(b - a) < 0.1 * a


def test_degree_bound_brackets_the_exact_effective_resistance():
    """Theorem 2: (1/2)(1/d_u + 1/d_v) <= r_(u,v) <= (1/gamma)(1/d_u + 1/d_v), r from the pseudo-inverse (Eq. 3)."""
    rng = np.random.default_rng(10)
    n, m = 30, 140
    eu, ev = random_simple_graph(rng, n, m)
    d = S.degrees(n, eu, ev).astype(np.float64)
    assert d.min() > 0
    Lm = laplacian(n, eu, ev, np.ones(m))
    Lp = np.linalg.pinv(Lm)
    Dm = np.diag(d ** -0.5)
    gamma = np.sort(np.linalg.eigvalsh(Dm @ Lm @ Dm))[1]
    assert gamma > 1e-6                               # connected
    q = S.sampling_weights(n, eu, ev).astype(np.float64) / 2.0 ** 32
    for i, (u, v) in enumerate(zip(eu.tolist(), ev.tolist())):
        x = np.zeros(n)
        x[u], x[v] = 1.0, -1.0
        r = x @ Lp @ x
        assert 0.5 * q[i] * (1 - 1e-6) <= r <= q[i] / gamma * (1 + 1e-6)
