"""GPU parity of the MLP edge predictor (lp_mlp_score_loss, lp_mlp_backward, lp_backward_edge_grads) with its
oracle: scores, loss, dscore within 1e-4; predictor and model gradients within 1e-3 (fp32 vs fp64)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2506_20818_amd as lp
from oracle import lp_oracle as O
from oracle import mlp_oracle as M
from gpu_util import assert_close, dev_f32, dev_i32, host, make_model
from test_gpu_parity import TOL_ACT, TOL_GRAD, graph_with_hub_and_empty_rows, toy_model


def say(msg):
    print("[case] " + msg, flush=True)


def mlp_weights(rng, widths, scale=0.3):
    dims = list(widths) + [1]
    W = [(rng.standard_normal((dims[j], dims[j + 1])) * scale).astype(np.float32) for j in range(len(dims) - 1)]
    c = [(rng.standard_normal(dims[j + 1]) * 0.2).astype(np.float32) for j in range(len(dims) - 1)]
    return W, c


@pytest.mark.parametrize("widths", [[8], [16, 12], [64, 256, 256], [36, 68, 32, 20]])
def test_mlp_predictor_alone(widths):
    rng = np.random.default_rng(sum(widths))
    n, B, n_pos = 500, 1333, 600
    H = rng.standard_normal((n, widths[0])).astype(np.float32)
    es, ed = rng.integers(0, n, B).astype(np.int32), rng.integers(0, n, B).astype(np.int32)
    W, c = mlp_weights(rng, widths)
    say("mlp widths=%s B=%d" % (widths, B))
    p = lp.Mlp([dev_f32(w) for w in W], [dev_f32(x) for x in c])
    s, loss, ds, acts = lp.lp_mlp_score_loss(dev_f32(H), dev_i32(es), dev_i32(ed), n_pos, p)
    s_ref, a_ref = M.mlp_scores(H, es, ed, W, c)
    loss_ref, ds_ref = M.bce_mean(s_ref, n_pos)
    assert_close(host(s), s_ref, TOL_ACT, "scores")
    assert abs(float(host(loss)[0]) - loss_ref) <= TOL_ACT * abs(loss_ref)
    assert_close(host(ds), ds_ref, TOL_ACT, "dscore")
    grads, eg = lp.lp_mlp_backward(p, acts, ds)
    dW, dc, eg_ref, G_ref = M.mlp_backward(H, es, ed, W, a_ref, ds_ref)
    for j in range(len(W)):
        assert_close(host(grads.dW[j]), dW[j], TOL_GRAD, "dW_%d" % (j + 1))
        assert_close(host(grads.dbias[j]), dc[j], TOL_GRAD, "dc_%d" % (j + 1))
    assert_close(host(eg)[:B], eg_ref, TOL_GRAD, "edge_grad")


def test_mlp_predictor_edge_cases():
    say("mlp: empty batch, id out of range")
    rng = np.random.default_rng(3)
    H = rng.standard_normal((20, 8)).astype(np.float32)
    W, c = mlp_weights(rng, [8, 12])
    p = lp.Mlp([dev_f32(w) for w in W], [dev_f32(x) for x in c])
    z = np.zeros(0, np.int32)
    s, loss, ds, acts = lp.lp_mlp_score_loss(dev_f32(H), dev_i32(z), dev_i32(z), 0, p)
    assert float(host(loss)[0]) == 0.0
    grads, eg = lp.lp_mlp_backward(p, acts, ds)
    assert all(np.all(host(t) == 0) for t in grads.dW + grads.dbias)
    es, ed = np.array([1, 25, 3], np.int32), np.array([2, 4, -1], np.int32)
    s, loss, ds, acts = lp.lp_mlp_score_loss(dev_f32(H), dev_i32(es), dev_i32(ed), 1, p)
    s_ref, _ = M.mlp_scores(H, es[:1], ed[:1], W, c)
    assert host(s)[1] == 0 and host(s)[2] == 0 and host(ds)[1] == 0 and host(ds)[2] == 0
    assert abs(host(s)[0] - s_ref[0]) < 1e-5


@pytest.mark.parametrize("dims", [[12, 20, 8], [128, 256, 256, 256]])
def test_whole_step_with_mlp_predictor(dims):
    rng = np.random.default_rng(900 + sum(dims))
    n = 1300
    r, c = graph_with_hub_and_empty_rows(rng, n, 3500, 600)
    ref = O.build_csr(n, r, c, True)
    g = lp.lp_build_csr(n, dev_i32(r), dev_i32(c), True)
    Ws, Wn, b = toy_model(rng, dims, scale=0.25)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    B, n_pos = 2500, 1000
    es, ed = rng.integers(0, n, B).astype(np.int32), rng.integers(0, n, B).astype(np.int32)
    es[:700] = 3                                     # the hub is scored 700 times (workgroup-per-row path of the scatter)
    W, cc = mlp_weights(rng, [dims[-1], 64, 32], scale=0.4)
    say("step with MLP predictor dims=%s" % dims)
    model = make_model(Ws, Wn, b)
    p = lp.Mlp([dev_f32(w) for w in W], [dev_f32(x) for x in cc])
    Xd = dev_f32(X)
    acts = lp.lp_sage_forward(g, model, Xd)
    s, loss, ds, macts = lp.lp_mlp_score_loss(acts.H[-1], dev_i32(es), dev_i32(ed), n_pos, p)
    mgrads, eg = lp.lp_mlp_backward(p, macts, ds)
    grads = lp.lp_backward_edge_grads(g, model, Xd, acts, dev_i32(es), dev_i32(ed), eg, want_dX=True)
    # the same step on the first 400 edges after the training forward (a batch small enough for its last layer to be
    # listed) and after the full forward pass: the predictor and the edge-gradient backward read only listed rows
    from gpu_util import nan_filled_acts
    e4, d4 = dev_i32(es[:400]), dev_i32(ed[:400])
    listed = nan_filled_acts(n, model, Xd)
    lp.lp_sage_forward_edges(g, model, Xd, e4, d4, listed)
    assert int(torch.isnan(listed.H[-1]).any(dim=1).sum()) == n - np.unique(np.concatenate([es[:400], ed[:400]])).size
    results = []
    for a in (listed, acts):
        s4, loss4, ds4, m4 = lp.lp_mlp_score_loss(a.H[-1], e4, d4, 150, p)
        mg4, eg4 = lp.lp_mlp_backward(p, m4, ds4)
        results.append((s4, mg4, lp.lp_backward_edge_grads(g, model, Xd, a, e4, d4, eg4, want_dX=True)))
    (sa, ma, ga), (sb, mb, gb) = results
    assert_close(host(sa), host(sb), 1e-6, "MLP scores after either forward pass")
    for k in range(len(dims) - 1):
        assert_close(host(ga.dW_self[k]), host(gb.dW_self[k]), 1e-5, "dW_self^%d after either forward pass" % (k + 1))
        assert_close(host(ga.dW_neigh[k]), host(gb.dW_neigh[k]), 1e-5, "dW_neigh^%d after either forward pass" % (k + 1))
    for j in range(len(W)):
        assert_close(host(ma.dW[j]), host(mb.dW[j]), 1e-5, "predictor dW^%d after either forward pass" % (j + 1))
    a_ref = O.sage_forward(ref, Ws, Wn, b, X)
    s_ref, ma_ref = M.mlp_scores(a_ref.H[-1], es, ed, W, cc)
    loss_ref, ds_ref = M.bce_mean(s_ref, n_pos)
    assert_close(host(s), s_ref, TOL_ACT, "scores")
    dW, dc, eg_ref, G_ref = M.mlp_backward(a_ref.H[-1], es, ed, W, ma_ref, ds_ref)
    out = {"ref": O.backward(ref, Ws, Wn, a_ref, es, ed, None, seed_grad=G_ref)}
    K = len(dims) - 1
    for k in range(K):
        assert_close(host(grads.dW_self[k]), out["ref"].dW_self[k], TOL_GRAD, "dW_self^%d" % (k + 1))
        assert_close(host(grads.dW_neigh[k]), out["ref"].dW_neigh[k], TOL_GRAD, "dW_neigh^%d" % (k + 1))
        assert_close(host(grads.dbias[k]), out["ref"].dbias[k], TOL_GRAD, "dbias^%d" % (k + 1))
    assert_close(host(grads.dX), out["ref"].dX, TOL_GRAD, "dX")


def test_mlp_predictor_bf16_storage():
    """bfloat16 storage of the embeddings, the products, the hidden layers and the predictor's weights (fp32
    accumulation); bars as for the other bf16 paths: 2^-7 on scores, 2e-2 on gradients."""
    from lp_workloads import to_bf16_grid
    rng = np.random.default_rng(55)
    n, B, n_pos, widths = 600, 2000, 900, [64, 256, 128]
    say("mlp bf16 widths=%s" % widths)
    H = to_bf16_grid((rng.standard_normal((n, widths[0])) * 0.7).astype(np.float32))
    es, ed = rng.integers(0, n, B).astype(np.int32), rng.integers(0, n, B).astype(np.int32)
    W, c = mlp_weights(rng, widths, scale=0.15)
    W = [to_bf16_grid(w) for w in W]
    bf = lambda a: dev_f32(a).to(torch.bfloat16)
    p = lp.Mlp([bf(w) for w in W], [dev_f32(x) for x in c])
    s, loss, ds, acts = lp.lp_mlp_score_loss(bf(H), dev_i32(es), dev_i32(ed), n_pos, p)
    s_ref, a_ref = M.mlp_scores(H, es, ed, W, c, storage="bf16")
    loss_ref, ds_ref = M.bce_mean(s_ref, n_pos)
    assert_close(host(s), s_ref, 2.0 ** -7, "scores")
    assert abs(float(host(loss)[0]) - loss_ref) <= 2.0 ** -7 * abs(loss_ref)
    grads, eg = lp.lp_mlp_backward(p, acts, ds)
    dW, dc, eg_ref, _ = M.mlp_backward(H, es, ed, W, a_ref, ds_ref, storage="bf16")
    for j in range(len(W)):
        assert_close(host(grads.dW[j]), dW[j], 2e-2, "dW_%d" % (j + 1))
        assert_close(host(grads.dbias[j]), dc[j], 2e-2, "dc_%d" % (j + 1))
    assert_close(host(eg.float())[:B], eg_ref, 2e-2, "edge_grad")
