"""Pins for the sampled-neighbourhood oracle.

Main pin: with fan-outs at least as large as every degree the sampled computational graph is the exact K-hop
neighbourhood of the batch endpoints, so embeddings, loss and weight gradients must coincide with the (separately
pinned) full-graph oracle.  The sampler is pinned by structure (subset of the neighbours, right size, distinct,
all neighbours when the degree fits), uniformity, and a known-answer check of the shuffle on a tiny case; the
sampled backward pass by central finite differences of the sampled forward pass.
"""
import numpy as np
import pytest

from oracle import blocks_oracle as Bk
from oracle import lp_oracle as O


def graph(rng, n, e, hub=None):
    r = rng.integers(0, n, e).astype(np.int32)
    c = rng.integers(0, n, e).astype(np.int32)
    if hub:
        r = np.concatenate([r, np.full(hub, 1, np.int32)])
        c = np.concatenate([c, rng.choice(n, hub, replace=False).astype(np.int32)])
    return O.build_csr(n, r, c, True)


def model(rng, dims, scale=0.4):
    K = len(dims) - 1
    Ws = [rng.standard_normal((dims[k], dims[k + 1])) * scale for k in range(K)]
    Wn = [rng.standard_normal((dims[k], dims[k + 1])) * scale for k in range(K)]
    b = [rng.standard_normal(dims[k + 1]) * 0.2 for k in range(K)]
    return Ws, Wn, b


def test_unbounded_fanout_reproduces_the_full_graph_step():
    rng = np.random.default_rng(0)
    n, dims = 300, [6, 10, 8, 5]
    csr = graph(rng, n, 700, hub=60)
    Ws, Wn, b = model(rng, dims)
    X = rng.standard_normal((n, dims[0]))
    B = 40
    es, ed = rng.integers(0, n, B).astype(np.int32), rng.integers(0, n, B).astype(np.int32)
    big = int(np.diff(csr.rowptr).max())
    blocks = Bk.sample_blocks(csr, es, ed, [big, big + 3, big], seed=5, step=2)
    acts = Bk.forward_blocks(blocks, Ws, Wn, b, X)
    full = O.sage_forward(csr, Ws, Wn, b, X)
    seeds = blocks.nodes[:blocks.n[3]]
    assert np.array_equal(seeds, np.unique(np.concatenate([es, ed])))
    np.testing.assert_allclose(acts.H[3], full.H[3][seeds], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(acts.H[1], full.H[1][blocks.nodes[:blocks.n[1]]], rtol=1e-12, atol=1e-13)
    s, loss, ds = O.score_loss(acts.H[3], blocks.e_src_pos, blocks.e_dst_pos, 25)
    s_f, loss_f, ds_f = O.score_loss(full.H[3], es, ed, 25)
    np.testing.assert_allclose(s, s_f, rtol=1e-12, atol=1e-13)
    assert abs(loss - loss_f) < 1e-13
    g = Bk.backward_blocks(blocks, Ws, Wn, acts, ds)
    g_f = O.backward(csr, Ws, Wn, full, es, ed, ds_f)
    for k in range(3):
        np.testing.assert_allclose(g.dW_self[k], g_f.dW_self[k], rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(g.dW_neigh[k], g_f.dW_neigh[k], rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(g.dbias[k], g_f.dbias[k], rtol=1e-10, atol=1e-13)


def test_block_structure():
    rng = np.random.default_rng(1)
    n = 400
    csr = graph(rng, n, 1500, hub=150)
    es, ed = rng.integers(0, n, 30).astype(np.int32), rng.integers(0, n, 30).astype(np.int32)
    fan = [7, 4, 3]
    b = Bk.sample_blocks(csr, es, ed, fan, seed=9, step=1)
    K = 3
    assert np.all(np.diff(b.n) <= 0) and b.nodes.size == b.n[0] and np.unique(b.nodes).size == b.nodes.size
    assert np.array_equal(b.nodes[b.e_src_pos], es) and np.array_equal(b.nodes[b.e_dst_pos], ed)
    for hop in range(1, K + 1):
        k = K + 1 - hop
        ptr, col = b.ptr[k - 1], b.col[k - 1]
        assert ptr.size == b.n[k] + 1 and ptr[0] == 0 and ptr[-1] == col.size
        assert col.min() >= 0 and col.max() < b.n[k - 1]
        new = b.nodes[b.n[k]:b.n[k - 1]]
        assert np.all(np.diff(new) > 0)                                  # nodes that join the frontier: ascending
        seen = np.zeros(b.n[k - 1], bool)
        seen[col] = True
        assert np.all(seen[b.n[k]:])                                     # every new node was sampled by someone
        for i in range(b.n[k]):
            v = b.nodes[i]
            nb = csr.colidx[csr.rowptr[v]:csr.rowptr[v + 1]]
            row = b.nodes[col[ptr[i]:ptr[i + 1]]]
            assert row.size == min(nb.size, fan[hop - 1]) and np.unique(row).size == row.size
            assert np.all(np.isin(row, nb))
            if nb.size <= fan[hop - 1]:
                assert np.array_equal(row, nb)                           # everything, in list order
        # the transposed block holds the same entries grouped by source position
        tp, tc = b.t_ptr[k - 1], b.t_col[k - 1]
        assert tp.size == b.n[k - 1] + 1 and tp[-1] == col.size
        pairs = sorted((int(c), p, i) for i in range(b.n[k]) for p, c in enumerate(col[ptr[i]:ptr[i + 1]], start=int(ptr[i])))
        assert [x[2] for x in pairs] == tc.tolist()
        assert np.array_equal(np.bincount(col, minlength=b.n[k - 1]), np.diff(tp))
    again = Bk.sample_blocks(csr, es, ed, fan, seed=9, step=1)
    assert all(np.array_equal(x, y) for x, y in zip(again.col, b.col))
    other = Bk.sample_blocks(csr, es, ed, fan, seed=9, step=2)
    assert not all(np.array_equal(x, y) for x, y in zip(other.col, b.col))


def test_shuffle_known_answer_and_uniformity():
    # hand check of the swap rule with d = 5, f = 2 and fixed "random" words: swap 0 with 0 + floor(w0*5/2^32),
    # swap 1 with 1 + floor(w1*4/2^32)
    nb = np.array([10, 20, 30, 40, 50], np.int32)
    w = O.philox4x32_10(3, (1 << 16) + 0, 7, 0, 11, 0)
    r0 = (w[0] * 5) >> 32
    a = [0, 1, 2, 3, 4]
    a[0], a[r0] = a[r0], a[0]
    r1 = 1 + ((w[1] * 4) >> 32)
    a[1], a[r1] = a[r1], a[1]
    assert Bk.sample_row(nb, 2, v=3, hop=1, seed=11, step=7).tolist() == [nb[a[0]], nb[a[1]]]
    # every neighbour is equally likely to be in the sample: 12 neighbours, 5 drawn, 6000 different steps
    nb = np.arange(100, 112, dtype=np.int32)
    hits = np.zeros(12)
    trials = 6000
    for step in range(trials):
        row = Bk.sample_row(nb, 5, v=77, hop=2, seed=1, step=step)
        assert np.unique(row).size == 5
        hits[row - 100] += 1
    exp = trials * 5 / 12
    chi2 = ((hits - exp) ** 2 / (exp * (1 - 5 / 12))).sum()             # hypergeometric marginals
    assert chi2 < 11 + 5 * np.sqrt(22)
    # and the first drawn element is uniform too
    first = np.bincount([Bk.sample_row(nb, 5, 77, 2, 1, s)[0] - 100 for s in range(3000)], minlength=12)
    assert ((first - 250.0) ** 2 / 250.0).sum() < 11 + 5 * np.sqrt(22)


@pytest.mark.parametrize("dims", [[4, 6, 3], [5, 7, 6, 4]])
def test_sampled_gradients_match_central_finite_differences(dims):
    rng = np.random.default_rng(2 + len(dims))
    n = 60
    csr = graph(rng, n, 240, hub=25)
    K = len(dims) - 1
    Ws, Wn, b = model(rng, dims)
    X = rng.standard_normal((n, dims[0]))
    es, ed = rng.integers(0, n, 12).astype(np.int32), rng.integers(0, n, 12).astype(np.int32)
    blocks = Bk.sample_blocks(csr, es, ed, [4, 3, 2][:K], seed=3, step=4)
    assert any(np.diff(p).max() < np.diff(csr.rowptr).max() for p in blocks.ptr)      # sampling really truncates

    def loss_of(Ws_, Wn_, b_):
        a = Bk.forward_blocks(blocks, Ws_, Wn_, b_, X)
        return O.score_loss(a.H[K], blocks.e_src_pos, blocks.e_dst_pos, 7)[1]

    acts = Bk.forward_blocks(blocks, Ws, Wn, b, X)
    _, _, ds = O.score_loss(acts.H[K], blocks.e_src_pos, blocks.e_dst_pos, 7)
    g = Bk.backward_blocks(blocks, Ws, Wn, acts, ds)
    h = 1e-6
    for k in range(K):
        for name, arrs, grad in (("Ws", Ws, g.dW_self), ("Wn", Wn, g.dW_neigh), ("b", b, g.dbias)):
            it = np.nditer(arrs[k], flags=["multi_index"])
            for _ in it:
                idx = it.multi_index
                old = arrs[k][idx]
                arrs[k][idx] = old + h
                lp_ = loss_of(Ws, Wn, b)
                arrs[k][idx] = old - h
                lm_ = loss_of(Ws, Wn, b)
                arrs[k][idx] = old
                fd = (lp_ - lm_) / (2 * h)
                assert abs(fd - grad[k][idx]) < 1e-7 + 1e-5 * abs(fd), (name, k, idx, fd, grad[k][idx])


def test_sampled_gradients_with_mlp_scorer_match_central_finite_differences():
    """The seed_grad path: the MLP scorer's gradient on frontier K, pushed through the sampled blocks, against central
    differences of the loss of the whole chain (blocks forward -> MLP scores -> BCE mean)."""
    from oracle import mlp_oracle as M
    rng = np.random.default_rng(41)
    n, dims = 50, [4, 6, 5]
    csr = graph(rng, n, 200, hub=20)
    K = len(dims) - 1
    Ws, Wn, b = model(rng, dims)
    X = rng.standard_normal((n, dims[0]))
    es, ed = rng.integers(0, n, 10).astype(np.int32), rng.integers(0, n, 10).astype(np.int32)
    blocks = Bk.sample_blocks(csr, es, ed, [3, 2], seed=9, step=1)
    W = [rng.standard_normal((dims[-1], 4)) * 0.5, rng.standard_normal((4, 1)) * 0.5]
    c = [rng.standard_normal(4) * 0.2, rng.standard_normal(1) * 0.2]

    def loss_of(Ws_, Wn_, b_):
        a = Bk.forward_blocks(blocks, Ws_, Wn_, b_, X)
        s, _ = M.mlp_scores(a.H[K], blocks.e_src_pos, blocks.e_dst_pos, W, c)
        return M.bce_mean(s, 6)[0]

    acts = Bk.forward_blocks(blocks, Ws, Wn, b, X)
    s, macts = M.mlp_scores(acts.H[K], blocks.e_src_pos, blocks.e_dst_pos, W, c)
    _, ds = M.bce_mean(s, 6)
    _, _, _, G = M.mlp_backward(acts.H[K], blocks.e_src_pos, blocks.e_dst_pos, W, macts, ds)
    g = Bk.backward_blocks(blocks, Ws, Wn, acts, None, seed_grad=G)
    h = 1e-6
    for k in range(K):
        for name, arrs, grad in (("Ws", Ws, g.dW_self), ("Wn", Wn, g.dW_neigh), ("b", b, g.dbias)):
            it = np.nditer(arrs[k], flags=["multi_index"])
            for _ in it:
                idx = it.multi_index
                old = arrs[k][idx]
                arrs[k][idx] = old + h
                lp_ = loss_of(Ws, Wn, b)
                arrs[k][idx] = old - h
                lm_ = loss_of(Ws, Wn, b)
                arrs[k][idx] = old
                fd = (lp_ - lm_) / (2 * h)
                assert abs(fd - grad[k][idx]) < 1e-7 + 1e-5 * abs(fd), (name, k, idx, fd, grad[k][idx])


def gcn_setup(rng, n, e, dims, hub=None):
    from oracle import gcn_oracle as Gc
    r = rng.integers(0, n, e).astype(np.int32)
    c = rng.integers(0, n, e).astype(np.int32)
    if hub:
        r = np.concatenate([r, np.full(hub, 1, np.int32)])
        c = np.concatenate([c, rng.choice(n, hub, replace=False).astype(np.int32)])
    r2, c2 = Gc.add_self_pairs(n, r, c)
    csr = O.build_csr(n, r2, c2, True)
    K = len(dims) - 1
    W = [rng.standard_normal((dims[k], dims[k + 1])) * 0.4 for k in range(K)]
    b = [rng.standard_normal(dims[k + 1]) * 0.2 for k in range(K)]
    return csr, W, b


def test_full_neighbourhood_gcn_blocks_reproduce_the_full_graph_gcn():
    """Fan-out 0 = all neighbours: the GCN layers on the blocks must equal the (separately pinned) full-graph GCN on
    every node of the computational graph, and the weight gradients must coincide."""
    from oracle import gcn_oracle as Gc
    rng = np.random.default_rng(3)
    n, dims = 250, [5, 9, 7, 4]
    csr, W, b = gcn_setup(rng, n, 600, dims, hub=50)
    X = rng.standard_normal((n, dims[0]))
    es, ed = rng.integers(0, n, 30).astype(np.int32), rng.integers(0, n, 30).astype(np.int32)
    blocks = Bk.sample_blocks(csr, es, ed, [0, 0, 0], seed=1, step=1)
    for k in range(1, 4):       # every row of every block holds the node's whole list, in order
        for i in range(0, int(blocks.n[k]), 7):
            v = blocks.nodes[i]
            row = blocks.nodes[blocks.col[k - 1][blocks.ptr[k - 1][i]:blocks.ptr[k - 1][i + 1]]]
            assert np.array_equal(row, csr.colidx[csr.rowptr[v]:csr.rowptr[v + 1]])
    inv = O.inverse_degrees(csr)
    acts = Bk.forward_blocks_gcn(blocks, inv, W, b, X)
    full = Gc.gcn_forward(csr, W, b, X)
    for k in (1, 2, 3):
        np.testing.assert_allclose(acts.H[k], full.H[k][blocks.nodes[:blocks.n[k]]], rtol=1e-11, atol=1e-13)
    s, loss, ds = O.score_loss(acts.H[3], blocks.e_src_pos, blocks.e_dst_pos, 20)
    s_f, loss_f, ds_f = O.score_loss(full.H[3], es, ed, 20)
    np.testing.assert_allclose(s, s_f, rtol=1e-11, atol=1e-13)
    g = Bk.backward_blocks_gcn(blocks, inv, W, acts, ds)
    g_f = Gc.gcn_backward(csr, W, full, es, ed, ds_f)
    for k in range(3):
        np.testing.assert_allclose(g.dW_neigh[k], g_f.dW_neigh[k], rtol=1e-9, atol=1e-13)
        np.testing.assert_allclose(g.dbias[k], g_f.dbias[k], rtol=1e-9, atol=1e-13)
    # the same fan-out convention for the GraphSAGE layers: equal to the full-graph step as well
    Ws, Wn, bb = model(rng, dims)
    a2 = Bk.forward_blocks(blocks, Ws, Wn, bb, X)
    np.testing.assert_allclose(a2.H[3], O.sage_forward(csr, Ws, Wn, bb, X).H[3][blocks.nodes[:blocks.n[3]]], rtol=1e-11, atol=1e-13)


def test_sampled_gcn_is_unbiased_and_its_gradients_match_finite_differences():
    rng = np.random.default_rng(8)
    n, dims = 60, [4, 6, 3]
    csr, W, b = gcn_setup(rng, n, 260, dims, hub=25)
    K = 2
    X = rng.standard_normal((n, dims[0]))
    inv = O.inverse_degrees(csr)
    es, ed = rng.integers(0, n, 12).astype(np.int32), rng.integers(0, n, 12).astype(np.int32)
    # one layer, many independent draws: the mean of the sampled aggregate tends to the full aggregate
    from oracle import gcn_oracle as Gc
    exact = Gc.normalised_aggregate(csr, X)
    acc, reps = 0.0, 400
    for s in range(reps):
        blk = Bk.sample_blocks(csr, es[:4], ed[:4], [3], seed=100 + s, step=0)
        a = Bk.gcn_block_aggregate(blk.ptr[0], blk.col[0], inv[blk.nodes[:blk.n[0]]], X[blk.nodes[:blk.n[0]]])
        acc = acc + a
        seeds = blk.nodes[:blk.n[1]]
    err = np.abs(acc / reps - exact[seeds]).max()
    assert err < 0.25, err                                  # Monte-Carlo error ~ 1/sqrt(400) of an O(1) quantity
    blocks = Bk.sample_blocks(csr, es, ed, [4, 3], seed=3, step=4)
    assert any(np.diff(p).max() < np.diff(csr.rowptr).max() for p in blocks.ptr)

    def loss_of(W_, b_):
        a = Bk.forward_blocks_gcn(blocks, inv, W_, b_, X)
        return O.score_loss(a.H[K], blocks.e_src_pos, blocks.e_dst_pos, 7)[1]

    acts = Bk.forward_blocks_gcn(blocks, inv, W, b, X)
    _, _, ds = O.score_loss(acts.H[K], blocks.e_src_pos, blocks.e_dst_pos, 7)
    g = Bk.backward_blocks_gcn(blocks, inv, W, acts, ds)
    h = 1e-6
    for k in range(K):
        for name, arrs, grad in (("W", W, g.dW_neigh), ("b", b, g.dbias)):
            it = np.nditer(arrs[k], flags=["multi_index"])
            for _ in it:
                idx = it.multi_index
                old = arrs[k][idx]
                arrs[k][idx] = old + h
                lp_ = loss_of(W, b)
                arrs[k][idx] = old - h
                lm_ = loss_of(W, b)
                arrs[k][idx] = old
                fd = (lp_ - lm_) / (2 * h)
                assert abs(fd - grad[k][idx]) < 1e-7 + 1e-5 * abs(fd), (name, k, idx, fd, grad[k][idx])
