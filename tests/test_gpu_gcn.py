"""GPU parity of the GCN layer type (lp_sage_forward / lp_backward with LP_LAYER_GCN) with the GCN oracle."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2506_20818_amd as lp
from lp_workloads import make_workload
from oracle import gcn_oracle as G
from oracle import lp_oracle as O
from gpu_util import assert_close, dev_f32, dev_i32, host
from test_gpu_parity import TOL_ACT, TOL_GRAD, graph_with_hub_and_empty_rows


def say(msg):
    print("[case] " + msg, flush=True)


def gcn_model(W, b, bf16=False):
    cast = (lambda a: dev_f32(a).to(torch.bfloat16)) if bf16 else dev_f32
    return lp.Model(None, [cast(w) for w in W], [dev_f32(x) for x in b], layer_type=lp.LP_LAYER_GCN)


def toy_weights(rng, dims, scale=0.3):
    K = len(dims) - 1
    return ([(rng.standard_normal((dims[k], dims[k + 1])) * scale).astype(np.float32) for k in range(K)],
            [(rng.standard_normal(dims[k + 1]) * 0.2).astype(np.float32) for k in range(K)])


def check_step(ref_csr, g, W, b, X, es, ed, n_pos):
    K = len(W)
    model = gcn_model(W, b)
    Xd = dev_f32(X)
    acts = lp.lp_sage_forward(g, model, Xd)
    a_ref = G.gcn_forward(ref_csr, W, b, X)
    for k in range(1, K + 1):
        assert_close(host(acts.A[k - 1]), a_ref.A[k], TOL_ACT, "A^%d" % k)
        assert_close(host(acts.H[k - 1]), a_ref.H[k], TOL_ACT, "H^%d" % k)
    s, loss, ds = lp.lp_score_loss(acts.H[-1], dev_i32(es), dev_i32(ed), n_pos)
    s_ref, loss_ref, ds_ref = O.score_loss(a_ref.H[K], es, ed, n_pos)
    assert_close(host(s), s_ref, TOL_ACT, "scores")
    grads = lp.lp_backward(g, model, Xd, acts, dev_i32(es), dev_i32(ed), ds, want_dX=True)
    g_ref = G.gcn_backward(ref_csr, W, a_ref, es, ed, ds_ref)
    for k in range(K):
        assert_close(host(grads.dW_neigh[k]), g_ref.dW_neigh[k], TOL_GRAD, "dW^%d" % (k + 1))
        assert_close(host(grads.dbias[k]), g_ref.dbias[k], TOL_GRAD, "dbias^%d" % (k + 1))
    assert_close(host(grads.dX), g_ref.dX, TOL_GRAD, "dX")
    return model, grads


@pytest.mark.parametrize("dims", [[4, 8], [12, 20, 4], [64, 64, 64], [128, 256, 256, 256], [100, 132, 68]])
@pytest.mark.parametrize("sym", [True, False])
def test_gcn_step_small_graphs(dims, sym):
    rng = np.random.default_rng(200 + sum(dims) + sym)
    n = 1300 + dims[-1]
    r, c = graph_with_hub_and_empty_rows(rng, n, 3500, 600)
    rl, cl = G.add_self_pairs(n, r, c)
    say("gcn dims=%s sym=%s n=%d" % (dims, sym, n))
    ref = O.build_csr(n, rl, cl, sym)
    g = lp.lp_build_csr(n, dev_i32(rl), dev_i32(cl), sym)
    W, b = toy_weights(rng, dims)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    B, n_pos = 2500, 1000
    es = rng.integers(0, n, B).astype(np.int32)
    ed = rng.integers(0, n, B).astype(np.int32)
    model, grads = check_step(ref, g, W, b, X, es, ed, n_pos)
    # the optimizer accepts a model without self weights
    state = lp.AdamState(model)
    before = host(model.W_neigh[0]).copy()
    lp.lp_adam_step(model, grads, state, 1)
    step = host(model.W_neigh[0]) - before
    gr = host(grads.dW_neigh[0])
    assert np.all(np.sign(step[np.abs(gr) > 1e-6]) == -np.sign(gr[np.abs(gr) > 1e-6]))


@pytest.mark.parametrize("dims", [[12, 20, 4], [128, 256, 256, 256]])
def test_gcn_step_with_the_training_forward(dims):
    """GCN layers through lp_sage_forward_edges on a batch small enough to be listed (no self term to gather): the
    last layer is written exactly at the end points and equals the oracle there, and the step's loss and gradients
    equal those after the full forward pass (whose parity with the oracle the tests above establish) up to the
    order of sums over hub rows."""
    from gpu_util import nan_filled_acts
    rng = np.random.default_rng(260 + sum(dims))
    n = 1300 + dims[-1]
    r, c = graph_with_hub_and_empty_rows(rng, n, 3500, 600)
    rl, cl = G.add_self_pairs(n, r, c)
    say("gcn training forward dims=%s n=%d" % (dims, n))
    ref = O.build_csr(n, rl, cl, True)
    g = lp.lp_build_csr(n, dev_i32(rl), dev_i32(cl), True)
    W, b = toy_weights(rng, dims)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    B, n_pos = 400, 150
    assert 8 * B < 3 * n
    es = rng.integers(0, n, B).astype(np.int32)
    ed = rng.integers(0, n, B).astype(np.int32)
    es[0] = 3
    K = len(W)
    model, Xd = gcn_model(W, b), dev_f32(X)
    acts = nan_filled_acts(n, model, Xd)
    lp.lp_sage_forward_edges(g, model, Xd, dev_i32(es), dev_i32(ed), acts)
    a_ref = G.gcn_forward(ref, W, b, X)
    ends = np.unique(np.concatenate([es, ed])).astype(np.int64)
    rest = np.ones(n, bool)
    rest[ends] = False
    for k in range(1, K):
        assert_close(host(acts.H[k - 1]), a_ref.H[k], TOL_ACT, "H^%d" % k)
    HK, AK = host(acts.H[K - 1]), host(acts.A[K - 1])
    assert_close(HK[ends], a_ref.H[K][ends], TOL_ACT, "H^K at the end points")
    assert_close(AK[ends], a_ref.A[K][ends], TOL_ACT, "A^K at the end points")
    assert np.isnan(HK[rest]).all() and np.isnan(AK[rest]).all()
    s, loss, ds = lp.lp_score_loss(acts.H[-1], dev_i32(es), dev_i32(ed), n_pos)
    grads = lp.lp_backward(g, model, Xd, acts, dev_i32(es), dev_i32(ed), ds, want_dX=True)
    full = lp.lp_sage_forward(g, model, Xd)
    s2, loss2, ds2 = lp.lp_score_loss(full.H[-1], dev_i32(es), dev_i32(ed), n_pos)
    g2 = lp.lp_backward(g, model, Xd, full, dev_i32(es), dev_i32(ed), ds2, want_dX=True)
    assert_close(host(s), host(s2), 1e-6, "scores after either forward pass")
    for k in range(K):
        assert_close(host(grads.dW_neigh[k]), host(g2.dW_neigh[k]), 1e-5, "dW^%d after either forward pass" % (k + 1))
        assert_close(host(grads.dbias[k]), host(g2.dbias[k]), 1e-5, "dbias^%d after either forward pass" % (k + 1))
    assert_close(host(grads.dX), host(g2.dX), 1e-5, "dX after either forward pass")


def test_gcn_step_collab_scale():
    wl = make_workload("C2")
    rl, cl = G.add_self_pairs(wl.n_nodes, wl.src, wl.dst)
    say("gcn C2 N=%d" % wl.n_nodes)
    ref = O.build_csr(wl.n_nodes, rl, cl, True)
    g = lp.lp_build_csr(wl.n_nodes, dev_i32(rl), dev_i32(cl), True)
    neg = host(lp.lp_sample_neg(g, dev_i32(wl.pos_src), wl.k_neg, wl.n_space, wl.sampler_seed, wl.sampler_step))
    es, ed = O.batch_edges(wl.pos_src, wl.pos_dst, neg, wl.k_neg)
    check_step(ref, g, wl.W_neigh, wl.bias, wl.X, es, ed, wl.n_pos)


@pytest.mark.parametrize("dims", [[24, 40, 8], [128, 512, 512, 512]])
def test_gcn_step_bf16_storage(dims):
    """bfloat16 storage of features, weights, activations and node-sized gradients (fp32 accumulation); bars as for
    the GraphSAGE bf16 path: 2^-7 on activations and scores, 2e-2 on gradients."""
    from lp_workloads import to_bf16_grid
    rng = np.random.default_rng(400 + sum(dims))
    n = 1400
    r, c = graph_with_hub_and_empty_rows(rng, n, 3500, 600)
    rl, cl = G.add_self_pairs(n, r, c)
    say("gcn bf16 dims=%s" % dims)
    ref = O.build_csr(n, rl, cl, True)
    g = lp.lp_build_csr(n, dev_i32(rl), dev_i32(cl), True)
    W, b = toy_weights(rng, dims)
    W = [to_bf16_grid(w) for w in W]
    X = to_bf16_grid(rng.standard_normal((n, dims[0])).astype(np.float32))
    B, n_pos = 2000, 800
    es, ed = rng.integers(0, n, B).astype(np.int32), rng.integers(0, n, B).astype(np.int32)
    model = gcn_model(W, b, bf16=True)
    Xd = dev_f32(X).to(torch.bfloat16)
    acts = lp.lp_sage_forward(g, model, Xd)
    a_ref = G.gcn_forward(ref, W, b, X, storage="bf16")
    K = len(W)
    for k in range(1, K + 1):
        assert_close(host(acts.H[k - 1].float()), a_ref.H[k], 2.0 ** -7, "H^%d" % k)
    s, loss, ds = lp.lp_score_loss(acts.H[-1], dev_i32(es), dev_i32(ed), n_pos)
    grads = lp.lp_backward(g, model, Xd, acts, dev_i32(es), dev_i32(ed), ds, want_dX=True)
    s_ref, loss_ref, ds_ref = O.score_loss(a_ref.H[K], es, ed, n_pos)
    g_ref = G.gcn_backward(ref, W, a_ref, es, ed, ds_ref, storage="bf16")
    assert_close(host(s), s_ref, 2.0 ** -7, "scores")
    for k in range(K):
        assert_close(host(grads.dW_neigh[k]), g_ref.dW_neigh[k], 2e-2, "dW^%d" % (k + 1))
        assert_close(host(grads.dbias[k]), g_ref.dbias[k], 2e-2, "dbias^%d" % (k + 1))
    assert_close(host(grads.dX.float()), g_ref.dX, 2e-2, "dX")
