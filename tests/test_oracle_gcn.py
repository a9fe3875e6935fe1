"""Pins for the GCN oracle: the dense matrix form D^-1/2 (A + I) D^-1/2 of Kipf and Welling's propagation rule on
small graphs, its spectral properties, regular-graph closed forms, the adjoint identity, and central finite
differences for every gradient entry."""
import numpy as np
import pytest

from oracle import gcn_oracle as G
from oracle import lp_oracle as O


def dense_S(n, r, c, sym):
    A = np.zeros((n, n))
    A[r, c] = 1.0
    if sym:
        A[c, r] = 1.0
    A[np.arange(n), np.arange(n)] = 1.0                    # every self-pair present once
    d = A.sum(axis=1)
    return A / np.sqrt(np.outer(d, d)), A


def setup(seed, n=40, e=120, sym=True):
    rng = np.random.default_rng(seed)
    r = rng.integers(0, n, e).astype(np.int32)
    c = rng.integers(0, n, e).astype(np.int32)
    rl, cl = G.add_self_pairs(n, r, c)
    return rng, r, c, O.build_csr(n, rl, cl, sym)


@pytest.mark.parametrize("sym", [True, False])
def test_aggregate_equals_dense_symmetric_normalisation(sym):
    rng, r, c, csr = setup(0, sym=sym)
    n = csr.n_nodes
    S, A = dense_S(n, r, c, sym)
    assert np.array_equal(np.diff(csr.rowptr), A.sum(axis=1).astype(int))
    H = rng.standard_normal((n, 7))
    np.testing.assert_allclose(G.normalised_aggregate(csr, H), S @ H, rtol=1e-12, atol=1e-14)
    T = rng.standard_normal((n, 7))
    np.testing.assert_allclose(G.normalised_aggregate_adjoint(csr, T), S.T @ T, rtol=1e-12, atol=1e-14)
    assert abs((G.normalised_aggregate(csr, H) * T).sum() - (H * G.normalised_aggregate_adjoint(csr, T)).sum()) < 1e-10


def test_spectrum_and_regular_graph_closed_forms():
    rng, r, c, csr = setup(1, sym=True)
    n = csr.n_nodes
    S, A = dense_S(n, r, c, True)
    ev = np.linalg.eigvalsh(S)
    assert ev.max() < 1 + 1e-12 and ev.min() > -1 - 1e-12   # the normalised adjacency has its spectrum in [-1, 1]
    d = A.sum(axis=1)
    np.testing.assert_allclose(G.normalised_aggregate(csr, np.sqrt(d)[:, None]), np.sqrt(d)[:, None], rtol=1e-12)  # eigenvalue 1
    # cycle: every node has itself and two neighbours, so the layer is the plain three-point average
    m = 9
    rr = np.arange(m, dtype=np.int32)
    cc = ((rr + 1) % m).astype(np.int32)
    rl, cl = G.add_self_pairs(m, rr, cc)
    cyc = O.build_csr(m, rl, cl, True)
    x = rng.standard_normal((m, 3))
    np.testing.assert_allclose(G.normalised_aggregate(cyc, x), (x + np.roll(x, 1, 0) + np.roll(x, -1, 0)) / 3.0, rtol=1e-12)
    # a node without neighbours keeps its own feature (its only pair is the self-pair)
    rl, cl = G.add_self_pairs(3, np.array([0], np.int32), np.array([1], np.int32))
    iso = O.build_csr(3, rl, cl, True)
    x = rng.standard_normal((3, 2))
    a = G.normalised_aggregate(iso, x)
    np.testing.assert_allclose(a[2], x[2], rtol=1e-12)
    np.testing.assert_allclose(a[0], (x[0] + x[1]) / 2.0, rtol=1e-12)


def test_forward_is_the_textbook_recurrence():
    rng, r, c, csr = setup(2)
    n = csr.n_nodes
    S, _ = dense_S(n, r, c, True)
    dims = [5, 8, 6, 4]
    W = [rng.standard_normal((dims[k], dims[k + 1])) * 0.5 for k in range(3)]
    b = [rng.standard_normal(dims[k + 1]) * 0.1 for k in range(3)]
    X = rng.standard_normal((n, 5))
    H = X
    for k in range(3):
        Z = S @ H @ W[k] + b[k]
        H = np.maximum(Z, 0) if k < 2 else Z
    np.testing.assert_allclose(G.gcn_forward(csr, W, b, X).H[3], H, rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("dims", [[4, 6, 3], [5, 7, 6, 4]])
def test_gradients_match_central_finite_differences(dims):
    rng, r, c, csr = setup(3 + len(dims), n=30, e=80)
    K = len(dims) - 1
    W = [rng.standard_normal((dims[k], dims[k + 1])) * 0.5 for k in range(K)]
    b = [rng.standard_normal(dims[k + 1]) * 0.2 for k in range(K)]
    X = rng.standard_normal((csr.n_nodes, dims[0]))
    es, ed = rng.integers(0, 30, 14).astype(np.int32), rng.integers(0, 30, 14).astype(np.int32)

    def loss_of(W_, b_, X_):
        return O.score_loss(G.gcn_forward(csr, W_, b_, X_).H[K], es, ed, 6)[1]

    acts = G.gcn_forward(csr, W, b, X)
    _, _, ds = O.score_loss(acts.H[K], es, ed, 6)
    g = G.gcn_backward(csr, W, acts, es, ed, ds)
    h = 1e-6
    for arrs, grads in ((W, g.dW_neigh), (b, g.dbias), ([X], [g.dX])):
        for k in range(len(arrs)):
            it = np.nditer(arrs[k], flags=["multi_index"])
            for _ in it:
                idx = it.multi_index
                old = arrs[k][idx]
                arrs[k][idx] = old + h
                lp_ = loss_of(W, b, X)
                arrs[k][idx] = old - h
                lm_ = loss_of(W, b, X)
                arrs[k][idx] = old
                fd = (lp_ - lm_) / (2 * h)
                assert abs(fd - grads[k][idx]) < 1e-7 + 1e-5 * abs(fd), (k, idx, fd, grads[k][idx])
