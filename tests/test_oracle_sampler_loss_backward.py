"""Pins for the oracle's negative sampler, loss and backward pass.

Sampler: the generator core is pinned by published known-answer vectors; the
vectorised bookkeeping is pinned by a scalar walk through the same rule on
small graphs, by validity/uniformity properties, and by cases with a single
valid answer.  Loss: closed forms.  Gradients: central finite differences of
the oracle's own forward+loss, which involve none of the backward code.
"""
import math
import os

import numpy as np
import pytest

from oracle import lp_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def random_pairs(rng, n, e):
    return rng.integers(0, n, e).astype(np.int32), rng.integers(0, n, e).astype(np.int32)


# ---------------------------------------------------------------- Philox core
def _kat():
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if not line.startswith("#") and line.strip():
            w = [int(x, 16) for x in line.split()]
            yield w[:6], tuple(w[6:])


def test_philox_known_answers_scalar_and_array():
    n = 0
    for inp, out in _kat():
        assert O.philox4x32_10(*inp) == out
        arr = O.philox4x32_10(*[np.array([x, x], np.uint64) for x in inp[:4]], inp[4], inp[5])
        assert tuple(int(a[1]) for a in arr) == out
        n += 1
    assert n == 3


# ---------------------------------------------------------------- sampler bookkeeping
def scalar_sampler(n_nodes, rowptr, colidx, pos_src, k_neg, n_space, seed, step):
    """One sample at a time, with Python sets for adjacency."""
    nbrs = [set(colidx[rowptr[v]:rowptr[v + 1]].tolist()) for v in range(n_nodes)]
    out, failed = [], 0
    for i, u in enumerate(pos_src.tolist()):
        for j in range(k_neg):
            q = i * k_neg + j
            c = None
            for t in range(16):
                w = O.philox4x32_10(q, t // 4, step & 0xFFFFFFFF, step >> 32, seed & 0xFFFFFFFF, seed >> 32)
                c = (w[t % 4] * n_space) >> 32
                if c != u and c not in nbrs[u]:
                    break
            else:
                start = c
                for _ in range(n_space):
                    c = (c + 1) % n_space
                    if c != u and c not in nbrs[u]:
                        break
                else:
                    c = start
                    failed += 1
            out.append(c)
    return np.array(out, np.int32), failed


@pytest.mark.parametrize("seed", range(5))
def test_sampler_matches_scalar_walkthrough(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(3, 40))
    r, c = random_pairs(rng, n, int(rng.integers(0, n * n // 2 + 1)))     # dense enough to force retries
    g = O.build_csr(n, r, c, True)
    pos = rng.integers(0, n, 50).astype(np.int32)
    k_neg = int(rng.integers(1, 4))
    n_space = n if seed % 2 else n + 5                  # sample space may exceed the visible nodes
    s, st = int(rng.integers(0, 2 ** 63)), int(rng.integers(0, 2 ** 40))
    got, nf = O.sample_neg(g, pos, k_neg, n_space, s, st)
    exp, ef = scalar_sampler(n, g.rowptr, g.colidx, pos, k_neg, n_space, s, st)
    assert np.array_equal(got, exp) and nf == ef


def test_sampler_properties_and_determinism():
    rng = np.random.default_rng(7)
    n = 500
    r, c = random_pairs(rng, n, 3000)
    g = O.build_csr(n, r, c, True)
    pos = rng.integers(0, n, 2000).astype(np.int32)
    a, nf = O.sample_neg(g, pos, 3, n, 123, 4)
    assert nf == 0 and a.dtype == np.int32 and a.size == 6000
    u = np.repeat(pos, 3)
    assert np.all((a >= 0) & (a < n)) and np.all(a != u)
    nb = [set(g.colidx[g.rowptr[v]:g.rowptr[v + 1]].tolist()) for v in range(n)]
    assert not any(int(d) in nb[int(s)] for s, d in zip(u, a))
    b, _ = O.sample_neg(g, pos, 3, n, 123, 4)
    assert np.array_equal(a, b)
    assert not np.array_equal(a, O.sample_neg(g, pos, 3, n, 123, 5)[0])     # step changes the draw
    assert not np.array_equal(a, O.sample_neg(g, pos, 3, n, 124, 4)[0])     # seed changes the draw


def test_sampler_single_valid_destination_full_row_and_probe_path():
    # node 0 is joined to 1 and 2 in a 4-node graph: only node 3 is a valid destination
    g = O.build_csr(4, np.array([0, 0]), np.array([1, 2]), True)
    out, nf = O.sample_neg(g, np.zeros(64, np.int32), 2, 4, 99, 0)
    assert np.all(out == 3) and nf == 0
    # node 0 joined to everyone: nothing is valid, every sample is counted as failed
    g = O.build_csr(4, np.array([0, 0, 0]), np.array([1, 2, 3]), True)
    out, nf = O.sample_neg(g, np.zeros(5, np.int32), 1, 4, 99, 0)
    assert nf == 5 and np.all((out >= 0) & (out < 4))
    # 1 valid destination among 200: sixteen rejections in a row are common, so the probe path runs
    n = 200
    g = O.build_csr(n, np.zeros(n - 2, np.int64), np.arange(1, n - 1), True)
    out, nf = O.sample_neg(g, np.zeros(40, np.int32), 1, n, 5, 1)
    assert np.all(out == n - 1) and nf == 0


def test_sampler_destinations_are_uniform_over_valid_nodes():
    # source 0 with neighbours {1, 2}; valid destinations 3..12, ten equally likely cells
    n = 13
    g = O.build_csr(n, np.array([0, 0]), np.array([1, 2]), True)
    out, _ = O.sample_neg(g, np.zeros(20000, np.int32), 1, n, 2024, 0)
    counts = np.bincount(out, minlength=n)
    assert counts[:3].sum() == 0
    expected = 20000 / 10
    chi2 = ((counts[3:] - expected) ** 2 / expected).sum()
    assert chi2 < 27.9          # 99.9 % point of chi-square with 9 degrees of freedom


# ---------------------------------------------------------------- scores and loss
def test_zero_embeddings_give_ln2_and_half_gradients():
    H = np.zeros((6, 4))
    es, ed = np.array([0, 1, 2, 3]), np.array([1, 2, 3, 4])
    s, loss, ds = O.score_loss(H, es, ed, 1)
    assert np.all(s == 0) and loss == pytest.approx(math.log(2.0), rel=1e-15)
    np.testing.assert_allclose(ds, np.array([-0.5, 0.5, 0.5, 0.5]) / 4, rtol=1e-15)


def test_loss_hand_example_and_symmetries():
    H = np.array([[1.0, 2.0], [3.0, -1.0], [0.5, 0.5]])
    s, loss, ds = O.score_loss(H, np.array([0, 0]), np.array([1, 2]), 1)
    assert np.array_equal(s, np.array([1.0, 1.5]))
    sig = lambda x: 1.0 / (1.0 + math.exp(-x))
    expect = (-math.log(sig(1.0)) - math.log(1.0 - sig(1.5))) / 2
    assert loss == pytest.approx(expect, rel=1e-14)
    np.testing.assert_allclose(ds, [(sig(1.0) - 1) / 2, sig(1.5) / 2], rtol=1e-14)
    s2, loss2, _ = O.score_loss(H, np.array([1, 2]), np.array([0, 0]), 1)      # s(u,v) = s(v,u)
    assert np.array_equal(s, s2) and loss == loss2
    # l(s, 1) == l(-s, 0)
    Hp = np.array([[2.0], [3.0], [-3.0]])
    _, lpos, _ = O.score_loss(Hp, np.array([0]), np.array([1]), 1)
    _, lneg, _ = O.score_loss(Hp, np.array([0]), np.array([2]), 0)
    assert lpos == pytest.approx(lneg, rel=1e-15)


def test_loss_is_finite_for_huge_scores_and_dscore_is_its_derivative():
    H = np.array([[80.0], [1.0], [-1.0], [0.3]])
    es, ed = np.array([0, 0, 0, 3]), np.array([1, 2, 1, 3])
    s, loss, ds = O.score_loss(H * np.array([[12.0], [1], [1], [1]]), es, ed, 2)
    assert np.isfinite(loss) and np.all(np.isfinite(ds)) and abs(s[0]) == 960.0
    # derivative check through the score vector, at moderate scores
    rng = np.random.default_rng(0)
    Hm = rng.standard_normal((5, 3))
    es, ed = np.array([0, 1, 2, 3]), np.array([4, 3, 0, 1])
    s, loss, ds = O.score_loss(Hm, es, ed, 2)

    def loss_of_scores(sv):
        y = np.array([1, 1, 0, 0.0])
        p = 1 / (1 + np.exp(-sv))
        return float(-(y * np.log(p) + (1 - y) * np.log(1 - p)).mean())
    assert loss == pytest.approx(loss_of_scores(s), rel=1e-13)
    for e in range(4):
        d = np.zeros(4)
        d[e] = 1e-6
        fd = (loss_of_scores(s + d) - loss_of_scores(s - d)) / 2e-6
        assert ds[e] == pytest.approx(fd, rel=1e-7)


# ---------------------------------------------------------------- gradients
def _setup(rng, n, dims, n_edges, batch):
    r, c = random_pairs(rng, n, n_edges)
    g = O.build_csr(n, r, c, True)
    K = len(dims) - 1
    Ws = [rng.standard_normal((dims[k], dims[k + 1])) * 0.6 for k in range(K)]
    Wn = [rng.standard_normal((dims[k], dims[k + 1])) * 0.6 for k in range(K)]
    b = [rng.standard_normal(dims[k + 1]) * 0.3 for k in range(K)]
    X = rng.standard_normal((n, dims[0]))
    es = rng.integers(0, n, batch).astype(np.int32)
    ed = rng.integers(0, n, batch).astype(np.int32)      # may repeat nodes and contain u == v
    return g, Ws, Wn, b, X, es, ed


def _loss(g, Ws, Wn, b, X, es, ed, n_pos):
    return O.score_loss(O.sage_forward(g, Ws, Wn, b, X).H[-1], es, ed, n_pos)[1]


@pytest.mark.parametrize("dims", [[3, 4, 2], [2, 3, 3, 2], [4, 3]])
def test_gradients_match_central_finite_differences_on_every_entry(dims):
    rng = np.random.default_rng(len(dims) * 11 + dims[0])
    g, Ws, Wn, b, X, es, ed = _setup(rng, 9, dims, 14, 10)
    n_pos = 4
    acts = O.sage_forward(g, Ws, Wn, b, X)
    _, _, ds = O.score_loss(acts.H[-1], es, ed, n_pos)
    grads = O.backward(g, Ws, Wn, acts, es, ed, ds)
    h = 1e-6
    groups = [(Ws, grads.dW_self), (Wn, grads.dW_neigh), (b, grads.dbias), ([X], [grads.dX])]
    checked = 0
    for params, gr in groups:
        for P, Gd in zip(params, gr):
            assert P.shape == Gd.shape
            it = np.nditer(P, flags=["multi_index"])
            for _ in it:
                idx = it.multi_index
                old = P[idx]
                P[idx] = old + h
                lp = _loss(g, Ws, Wn, b, X, es, ed, n_pos)
                P[idx] = old - h
                lm = _loss(g, Ws, Wn, b, X, es, ed, n_pos)
                P[idx] = old
                fd = (lp - lm) / (2 * h)
                assert Gd[idx] == pytest.approx(fd, rel=2e-5, abs=2e-9), (idx, Gd[idx], fd)
                checked += 1
    assert checked == sum(p.size for ps, _ in groups for p in ps)


def test_adjoint_identity_and_mass_conservation():
    rng = np.random.default_rng(21)
    n, f = 50, 7
    r, c = random_pairs(rng, n, 120)
    g = O.build_csr(n, r, c, False)          # asymmetric on purpose
    Xm, Y = rng.standard_normal((n, f)), rng.standard_normal((n, f))
    lhs = (O.mean_aggregate(g, Xm) * Y).sum()
    rhs = (Xm * O.mean_aggregate_adjoint(g, Y)).sum()
    assert lhs == pytest.approx(rhs, rel=1e-12)
    has_nb = np.diff(g.rowptr) > 0
    np.testing.assert_allclose(O.mean_aggregate_adjoint(g, Y).sum(0), Y[has_nb].sum(0), rtol=1e-12)
    # the adjoint can be read off the transposed CSR as a gather: same numbers
    inv = np.where(has_nb, 1.0 / np.maximum(np.diff(g.rowptr), 1), 0.0)
    gathered = np.zeros_like(Y)
    for u in range(n):
        vs = g.t_colidx[g.t_rowptr[u]:g.t_rowptr[u + 1]]
        gathered[u] = (Y[vs] * inv[vs, None]).sum(0)
    np.testing.assert_allclose(O.mean_aggregate_adjoint(g, Y), gathered, rtol=1e-12, atol=1e-15)


def test_zero_weight_closed_form_and_untouched_far_node():
    # all weights and biases zero: H^K = 0, every score 0, g_e = (1/2 - y)/B, so dL/dH^K = 0 and all
    # weight gradients vanish
    rng = np.random.default_rng(8)
    g, Ws, Wn, b, X, es, ed = _setup(rng, 10, [3, 4, 2], 15, 8)
    z = lambda L: [np.zeros_like(a) for a in L]
    acts = O.sage_forward(g, z(Ws), z(Wn), z(b), X)
    s, loss, ds = O.score_loss(acts.H[-1], es, ed, 3)
    assert loss == pytest.approx(math.log(2))
    gr = O.backward(g, z(Ws), z(Wn), acts, es, ed, ds)
    assert all(np.all(a == 0) for a in gr.dW_self + gr.dW_neigh + gr.dbias)
    # last-layer bias gradient with constant embeddings: H^K = b for all nodes when the weights are zero
    bb = z(b)
    bb[-1] = np.array([0.5, -0.25])
    acts = O.sage_forward(g, z(Ws), z(Wn), bb, X)
    s, loss, ds = O.score_loss(acts.H[-1], es, ed, 3)
    gr = O.backward(g, z(Ws), z(Wn), acts, es, ed, ds)
    np.testing.assert_allclose(gr.dbias[-1], 2 * ds.sum() * bb[-1], rtol=1e-13)
    # path graph 0-1-2-3-4-5-6, one layer deep model of K=2: batch touches nodes 0 and 1 only; node 6
    # is more than K+1 hops away, so its features get zero gradient
    g = O.build_csr(7, np.arange(6), np.arange(1, 7), True)
    Ws = [rng.standard_normal((2, 3)), rng.standard_normal((3, 2))]
    Wn = [rng.standard_normal((2, 3)), rng.standard_normal((3, 2))]
    b = [rng.standard_normal(3), rng.standard_normal(2)]
    X = rng.standard_normal((7, 2))
    acts = O.sage_forward(g, Ws, Wn, b, X)
    es, ed = np.array([0], np.int32), np.array([1], np.int32)
    _, _, ds = O.score_loss(acts.H[-1], es, ed, 1)
    gr = O.backward(g, Ws, Wn, acts, es, ed, ds)
    assert np.all(gr.dX[4:] == 0) and np.any(gr.dX[3] != 0)


def test_the_step_reads_the_last_layer_only_at_the_end_points_of_the_batch():
    """Eq. (2) takes h^(K) of the two end points of each scored edge and nothing else, and dL/dh^(K) is zero at every
    other node: replacing the rows of A^K, Z^K and H^K of all nodes that are no end point by arbitrary finite values
    changes neither the scores, nor the loss, nor a single bit of any gradient.  (What licenses a training forward
    pass that evaluates its last layer only at those nodes.)"""
    rng = np.random.default_rng(26)
    g, Ws, Wn, b, X, es, ed = _setup(rng, 40, [3, 5, 4, 2], 70, 7)
    acts = O.sage_forward(g, Ws, Wn, b, X)
    s, loss, ds = O.score_loss(acts.H[-1], es, ed, 3)
    gr = O.backward(g, Ws, Wn, acts, es, ed, ds)
    rest = np.ones(40, bool)
    rest[np.concatenate([es, ed])] = False
    assert 20 <= rest.sum() < 40
    K = 3
    H, A, Z = list(acts.H), list(acts.A), list(acts.Z)
    H[K], A[K], Z[K] = H[K].copy(), A[K].copy(), Z[K].copy()
    for M in (H[K], A[K], Z[K]):
        M[rest] = rng.standard_normal((int(rest.sum()), M.shape[1])) * 1e6
    other = O.Activations(H, A, Z)
    s2, loss2, ds2 = O.score_loss(other.H[-1], es, ed, 3)
    gr2 = O.backward(g, Ws, Wn, other, es, ed, ds2)
    assert np.array_equal(s, s2) and loss == loss2 and np.array_equal(ds, ds2)
    for a, c in zip(gr.dW_self + gr.dW_neigh + gr.dbias + [gr.dX], gr2.dW_self + gr2.dW_neigh + gr2.dbias + [gr2.dX]):
        assert np.array_equal(a, c)
    # one layer down the gradient is no longer confined to the end points (it has spread to their neighbours): the
    # input rows of layer K-1 at the same nodes do enter its weight gradient
    H[K - 2] = H[K - 2].copy()
    H[K - 2][rest] += 1.0
    gr3 = O.backward(g, Ws, Wn, O.Activations(H, A, Z), es, ed, ds2)
    assert not np.allclose(gr3.dW_self[K - 2], gr.dW_self[K - 2])


def test_train_step_assembles_the_batch_in_the_documented_order():
    rng = np.random.default_rng(9)
    g, Ws, Wn, b, X, es, ed = _setup(rng, 30, [3, 4, 2], 40, 6)
    res = O.train_step(g, Ws, Wn, b, X, es, ed, 2, 30, 1, 2)
    assert np.array_equal(res.e_src, np.concatenate([es, np.repeat(es, 2)]))
    assert np.array_equal(res.e_dst[:6], ed) and np.array_equal(res.e_dst[6:], res.neg_dst)
    assert res.scores.size == 18


def test_bf16_storage_mode_is_the_same_mathematics_with_rounded_stores():
    # small integers keep every intermediate exactly representable in bfloat16: both storage modes must agree
    rng = np.random.default_rng(12)
    g = O.build_csr(6, np.array([0, 1, 2, 3]), np.array([1, 2, 3, 4]), True)     # degrees 1 and 2 only
    Ws = [rng.integers(-2, 3, (2, 2)).astype(np.float64) for _ in range(2)]
    Wn = [rng.integers(-2, 3, (2, 2)).astype(np.float64) * 2 for _ in range(2)]   # even: halves stay integers
    b = [rng.integers(-1, 2, 2).astype(np.float64) for _ in range(2)]
    X = rng.integers(-2, 3, (6, 2)).astype(np.float64) * 2
    a32 = O.sage_forward(g, Ws, Wn, b, X, storage="f32")
    a16 = O.sage_forward(g, Ws, Wn, b, X, storage="bf16")
    for k in (1, 2):
        assert np.array_equal(a32.H[k], a16.H[k]) and np.array_equal(a32.A[k], a16.A[k])
    # with generic inputs every stored activation of the bf16 mode lies on the bfloat16 grid
    X = rng.standard_normal((6, 2))
    a16 = O.sage_forward(g, Ws, Wn, b, X, storage="bf16")
    for k in (1, 2):
        assert np.array_equal(a16.H[k], O._round_bf16(a16.H[k])) and np.array_equal(a16.A[k], O._round_bf16(a16.A[k]))
    es, ed = np.array([0, 2], np.int32), np.array([1, 5], np.int32)
    _, _, ds = O.score_loss(a16.H[-1], es, ed, 1)
    g16 = O.backward(g, Ws, Wn, a16, es, ed, ds, storage="bf16")
    g32 = O.backward(g, Ws, Wn, a16, es, ed, ds, storage="f32")
    assert np.array_equal(g16.dX, O._round_bf16(g16.dX))
    for x, y in zip(g16.dW_self + g16.dW_neigh, g32.dW_self + g32.dW_neigh):
        assert np.abs(x - y).max() <= 0.02 * np.abs(y).max()          # bf16 rounding noise only (2^-8 per stored value)
