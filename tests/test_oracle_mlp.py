"""Pins for the MLP edge-predictor oracle: a one-layer all-ones predictor IS the dot product (ties it to the pinned
dot-product path), symmetry in the end points, a hand example, and central finite differences for every parameter
and for the embeddings."""
import numpy as np

from oracle import lp_oracle as O
from oracle import mlp_oracle as M


def test_single_layer_of_ones_is_the_dot_product_and_pair_symmetry():
    rng = np.random.default_rng(0)
    H = rng.standard_normal((30, 6))
    es, ed = rng.integers(0, 30, 20), rng.integers(0, 30, 20)
    s, _ = M.mlp_scores(H, es, ed, [np.ones((6, 1))], [np.zeros(1)])
    s_dot, loss_dot, ds_dot = O.score_loss(H, es, ed, 8)
    np.testing.assert_allclose(s, s_dot, rtol=1e-12)
    loss, ds = M.bce_mean(s, 8)
    assert abs(loss - loss_dot) < 1e-14
    np.testing.assert_allclose(ds, ds_dot, rtol=1e-12)
    # and its embedding gradient is the dot-product path's edge-gradient scatter
    _, _, eg, G = M.mlp_backward(H, es, ed, [np.ones((6, 1))], M.mlp_scores(H, es, ed, [np.ones((6, 1))], [np.zeros(1)])[1], ds)
    np.testing.assert_allclose(G, O.edge_grad_scatter(H, es, ed, ds_dot), rtol=1e-12, atol=1e-15)
    W = [rng.standard_normal((6, 5)), rng.standard_normal((5, 4)), rng.standard_normal((4, 1))]
    c = [rng.standard_normal(5), rng.standard_normal(4), rng.standard_normal(1)]
    a, _ = M.mlp_scores(H, es, ed, W, c)
    b, _ = M.mlp_scores(H, ed, es, W, c)
    np.testing.assert_allclose(a, b, rtol=1e-13)


def test_hand_example():
    H = np.array([[1.0, 2.0], [3.0, -1.0]])
    W = [np.array([[1.0, -1.0], [0.5, 2.0]]), np.array([[2.0], [1.0]])]
    c = [np.array([0.0, 1.0]), np.array([-0.5])]
    # x = (3, -2); z = (3 - 1, -3 - 4 + 1) = (2, -6); u = (2, 0); s = 4 - 0.5
    s, acts = M.mlp_scores(H, np.array([0]), np.array([1]), W, c)
    assert np.allclose(acts.X, [[3.0, -2.0]]) and np.allclose(acts.U[1], [[2.0, 0.0]]) and np.allclose(s, [3.5])


def test_gradients_match_central_finite_differences():
    rng = np.random.default_rng(1)
    N, F = 12, 5
    H = rng.standard_normal((N, F))
    es, ed = rng.integers(0, N, 15), rng.integers(0, N, 15)
    W = [rng.standard_normal((F, 6)) * 0.6, rng.standard_normal((6, 4)) * 0.6, rng.standard_normal((4, 1)) * 0.6]
    c = [rng.standard_normal(6) * 0.3, rng.standard_normal(4) * 0.3, rng.standard_normal(1)]

    def loss_of(H_, W_, c_):
        return M.bce_mean(M.mlp_scores(H_, es, ed, W_, c_)[0], 7)[0]

    s, acts = M.mlp_scores(H, es, ed, W, c)
    _, ds = M.bce_mean(s, 7)
    dW, dc, eg, G = M.mlp_backward(H, es, ed, W, acts, ds)
    h = 1e-6
    for arrs, grads in ((W, dW), (c, dc), ([H], [G])):
        for k in range(len(arrs)):
            it = np.nditer(arrs[k], flags=["multi_index"])
            for _ in it:
                idx = it.multi_index
                old = arrs[k][idx]
                arrs[k][idx] = old + h
                lp_ = loss_of(H, W, c)
                arrs[k][idx] = old - h
                lm_ = loss_of(H, W, c)
                arrs[k][idx] = old
                fd = (lp_ - lm_) / (2 * h)
                assert abs(fd - np.asarray(grads[k]).reshape(arrs[k].shape)[idx]) < 1e-8 + 1e-5 * abs(fd), (k, idx)
