"""GPU parity of the sampled-neighbourhood step (lp_sample_blocks, lp_sage_forward_blocks, lp_backward_blocks) with
its oracle: the blocks are integer results and must match bit for bit; activations, scores and loss within 1e-4,
gradients within 1e-3 (fp32 on the GPU, fp64 in the oracle), as for the full-graph step."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2506_20818_amd as lp
from lp_workloads import make_workload
from oracle import blocks_oracle as Bk
from oracle import lp_oracle as O
from gpu_util import assert_close, dev_f32, dev_i32, host, make_model
from test_gpu_parity import TOL_ACT, TOL_GRAD, graph_with_hub_and_empty_rows, toy_model


def say(msg):
    print("[case] " + msg, flush=True)


def check_blocks(got, ref, K):
    n = host(got.n)
    assert np.array_equal(n, ref.n), (n, ref.n)
    assert np.array_equal(host(got.nodes)[:n[0]], ref.nodes)
    index = host(got.index)
    assert np.array_equal(index[ref.nodes], np.arange(n[0])) and (index >= 0).sum() == n[0]
    assert np.array_equal(host(got.e_src_pos), ref.e_src_pos) and np.array_equal(host(got.e_dst_pos), ref.e_dst_pos)
    for k in range(1, K + 1):
        e = int(ref.ptr[k - 1][-1])
        assert np.array_equal(host(got.ptr[k - 1])[:n[k] + 1], ref.ptr[k - 1]), "ptr of block %d" % k
        assert np.array_equal(host(got.col[k - 1])[:e], ref.col[k - 1]), "col of block %d" % k
        assert np.array_equal(host(got.t_ptr[k - 1])[:n[k - 1] + 1], ref.t_ptr[k - 1]), "t_ptr of block %d" % k
        assert np.array_equal(host(got.t_col[k - 1])[:e], ref.t_col[k - 1]), "t_col of block %d" % k
        cnt = np.diff(ref.ptr[k - 1]).astype(np.float32)
        inv = np.divide(np.float32(1), cnt, out=np.zeros_like(cnt), where=cnt > 0)
        assert np.array_equal(host(got.inv_cnt[k - 1])[:n[k]], inv)


def run_case(csr_ref, g, Ws, Wn, b, X, es, ed, n_pos, fanout, seed, step):
    K = len(fanout)
    ref = Bk.sample_blocks(csr_ref, es, ed, fanout, seed, step)
    blocks = lp.lp_sample_blocks(g, dev_i32(es), dev_i32(ed), fanout, seed, step)
    check_blocks(blocks, ref, K)
    model = make_model(Ws, Wn, b)
    acts = lp.lp_sage_forward_blocks(blocks, model, dev_f32(X))
    a_ref = Bk.forward_blocks(ref, Ws, Wn, b, X)
    assert_close(host(acts.X_frontier)[:ref.n[0]], a_ref.H[0], 1e-7, "gathered features")
    for k in range(1, K + 1):
        assert_close(host(acts.A[k - 1])[:ref.n[k]], a_ref.A[k], TOL_ACT, "A^%d" % k)
        assert_close(host(acts.H[k - 1])[:ref.n[k]], a_ref.H[k], TOL_ACT, "H^%d" % k)
    s, loss, ds = lp.lp_score_loss(acts.H[-1], blocks.e_src_pos, blocks.e_dst_pos, n_pos)
    s_ref, loss_ref, ds_ref = O.score_loss(a_ref.H[K], ref.e_src_pos, ref.e_dst_pos, n_pos)
    assert_close(host(s), s_ref, TOL_ACT, "scores")
    assert abs(float(host(loss)[0]) - loss_ref) <= TOL_ACT * abs(loss_ref)
    grads = lp.lp_backward_blocks(blocks, model, acts, ds)
    g_ref = Bk.backward_blocks(ref, Ws, Wn, a_ref, ds_ref)
    for k in range(K):
        assert_close(host(grads.dW_self[k]), g_ref.dW_self[k], TOL_GRAD, "dW_self^%d" % (k + 1))
        assert_close(host(grads.dW_neigh[k]), g_ref.dW_neigh[k], TOL_GRAD, "dW_neigh^%d" % (k + 1))
        assert_close(host(grads.dbias[k]), g_ref.dbias[k], TOL_GRAD, "dbias^%d" % (k + 1))
    return blocks, ref


@pytest.mark.parametrize("dims,fanout", [([8, 16, 4], [3, 2]), ([12, 20, 16, 8], [25, 10, 5]), ([128, 256, 256, 256], [25, 10, 5]),
                                         ([64, 64], [64]), ([36, 68, 32], [1, 1]),
                                         ([8, 16, 4], [16, 17])])   # both sides of the 16-lane / 64-lane draw kernels
@pytest.mark.parametrize("sym", [True, False])
def test_sampled_step_small_graphs(dims, fanout, sym):
    rng = np.random.default_rng(sum(dims) + sum(fanout) + sym)
    n = 1200 + dims[0]
    r, c = graph_with_hub_and_empty_rows(rng, n, 6000, 700)
    say("blocks dims=%s fanout=%s sym=%s n=%d" % (dims, fanout, sym, n))
    ref = O.build_csr(n, r, c, sym)
    g = lp.lp_build_csr(n, dev_i32(r), dev_i32(c), sym)
    Ws, Wn, b = toy_model(rng, dims, scale=0.25)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    B = 300
    es, ed = rng.integers(0, n, B).astype(np.int32), rng.integers(0, n, B).astype(np.int32)
    es[:40] = 3                                                    # the hub is an end point many times over
    run_case(ref, g, Ws, Wn, b, X, es, ed, 120, fanout, seed=77, step=5)


def test_sampled_step_edge_cases():
    say("blocks: empty batch, out-of-range ids, edgeless graph")
    rng = np.random.default_rng(1)
    n, dims, fanout = 200, [8, 16, 4], [4, 3]
    r, c = rng.integers(0, n, 500).astype(np.int32), rng.integers(0, n, 500).astype(np.int32)
    g = lp.lp_build_csr(n, dev_i32(r), dev_i32(c), True)
    ref = O.build_csr(n, r, c, True)
    Ws, Wn, b = toy_model(rng, dims)
    X = rng.standard_normal((n, 8)).astype(np.float32)
    z = np.zeros(0, np.int32)
    blocks = lp.lp_sample_blocks(g, dev_i32(z), dev_i32(z), fanout, 1, 1)
    assert host(blocks.n).tolist() == [0, 0, 0]
    model = make_model(Ws, Wn, b)
    acts = lp.lp_sage_forward_blocks(blocks, model, dev_f32(X))
    grads = lp.lp_backward_blocks(blocks, model, acts, dev_f32(np.zeros(0)))
    for t in grads.dW_self + grads.dW_neigh + grads.dbias:
        assert np.all(host(t) == 0)
    # an id outside the graph is ignored: the blocks are those of the remaining end points
    es = np.array([5, 9, 300, 7], np.int32)
    ed = np.array([6, -1, 8, 7], np.int32)
    blocks = lp.lp_sample_blocks(g, dev_i32(es), dev_i32(ed), fanout, 1, 1)
    seeds = host(blocks.nodes)[:host(blocks.n)[2]]
    assert seeds.tolist() == [5, 6, 7, 8, 9]
    assert host(blocks.e_src_pos).tolist() == [0, 4, -1, 2] and host(blocks.e_dst_pos).tolist() == [1, -1, 3, 2]
    # a graph without edges: every block is empty, the model reduces to the self path
    g0 = lp.lp_build_csr(n, dev_i32(z), dev_i32(z), True)
    ref0 = O.build_csr(n, z, z, True)
    es, ed = rng.integers(0, n, 20).astype(np.int32), rng.integers(0, n, 20).astype(np.int32)
    run_case(ref0, g0, Ws, Wn, b, X, es, ed, 10, fanout, seed=3, step=3)


def test_sampled_step_collab_scale_batch():
    """The Collab-scale graph with the paper's batch size for it (10 240 positives, one negative each) and fan-outs
    25 / 10 / 5; the negatives come from lp_sample_neg."""
    wl = make_workload("C2")
    say("blocks C2: N=%d" % wl.n_nodes)
    ref_csr = O.build_csr(wl.n_nodes, wl.src, wl.dst, True)
    g = lp.lp_build_csr(wl.n_nodes, dev_i32(wl.src), dev_i32(wl.dst), True)
    n_pos = 10240
    pos_src, pos_dst = wl.pos_src[:n_pos], wl.pos_dst[:n_pos]
    neg = host(lp.lp_sample_neg(g, dev_i32(pos_src), 1, wl.n_space, wl.sampler_seed, 3))
    es, ed = O.batch_edges(pos_src, pos_dst, neg, 1)
    blocks, ref = run_case(ref_csr, g, wl.W_self, wl.W_neigh, wl.bias, wl.X, es, ed, n_pos, [25, 10, 5], seed=2024, step=9)
    say("frontiers %s, block entries %s" % (ref.n.tolist(), [int(p[-1]) for p in ref.ptr]))


@pytest.mark.parametrize("dims,fanout", [([12, 20, 8], [4, 3]), ([128, 256, 256, 256], [25, 10, 5])])
def test_sampled_step_with_mlp_predictor(dims, fanout):
    """Sampled blocks + the MLP scorer: lp_mlp_score_loss / lp_mlp_backward on frontier positions, then
    lp_backward_blocks_edge_grads; against blocks_oracle + mlp_oracle."""
    from oracle import mlp_oracle as M
    from test_gpu_mlp import mlp_weights
    rng = np.random.default_rng(1300 + sum(dims))
    n = 1200
    r, c = graph_with_hub_and_empty_rows(rng, n, 3300, 500)
    ref = O.build_csr(n, r, c, True)
    g = lp.lp_build_csr(n, dev_i32(r), dev_i32(c), True)
    Ws, Wn, b = toy_model(rng, dims, scale=0.25)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    B, n_pos = 400, 200
    es, ed = rng.integers(0, n, B).astype(np.int32), rng.integers(0, n, B).astype(np.int32)
    es[:60] = 3                                      # the hub end point is scored many times
    W, cc = mlp_weights(rng, [dims[-1], 32, 16], scale=0.4)
    K = len(fanout)
    say("sampled step with MLP predictor dims=%s fanout=%s" % (dims, fanout))
    bref = Bk.sample_blocks(ref, es, ed, fanout, 11, 2)
    blocks = lp.lp_sample_blocks(g, dev_i32(es), dev_i32(ed), fanout, 11, 2)
    check_blocks(blocks, bref, K)
    model = make_model(Ws, Wn, b)
    p = lp.Mlp([dev_f32(w) for w in W], [dev_f32(x) for x in cc])
    acts = lp.lp_sage_forward_blocks(blocks, model, dev_f32(X))
    s, loss, ds, macts = lp.lp_mlp_score_loss(acts.H[-1], blocks.e_src_pos, blocks.e_dst_pos, n_pos, p)
    mgrads, eg = lp.lp_mlp_backward(p, macts, ds)
    grads = lp.lp_backward_blocks_edge_grads(blocks, model, acts, eg)
    torch.cuda.synchronize()
    a_ref = Bk.forward_blocks(bref, Ws, Wn, b, X)
    s_ref, ma_ref = M.mlp_scores(a_ref.H[K], bref.e_src_pos, bref.e_dst_pos, W, cc)
    loss_ref, ds_ref = M.bce_mean(s_ref, n_pos)
    assert_close(host(s), s_ref, TOL_ACT, "scores")
    assert abs(float(host(loss)[0]) - loss_ref) <= TOL_ACT * max(1.0, abs(loss_ref))
    _, _, _, G_ref = M.mlp_backward(a_ref.H[K], bref.e_src_pos, bref.e_dst_pos, W, ma_ref, ds_ref)
    out = {"ref": Bk.backward_blocks(bref, Ws, Wn, a_ref, None, seed_grad=G_ref)}
    for k in range(K):
        assert_close(host(grads.dW_self[k]), out["ref"].dW_self[k], TOL_GRAD, "dW_self^%d" % (k + 1))
        assert_close(host(grads.dW_neigh[k]), out["ref"].dW_neigh[k], TOL_GRAD, "dW_neigh^%d" % (k + 1))
        assert_close(host(grads.dbias[k]), out["ref"].dbias[k], TOL_GRAD, "dbias^%d" % (k + 1))


# ------------------------------------------------------------------ full-neighbourhood hops and GCN layers on the blocks
def test_full_neighbourhood_blocks_sage():
    """Fan-out 0 = all neighbours (hub rows of several hundred entries included): blocks bit-exact, step within the
    usual bars; by construction this equals the full-graph step on the computational graph."""
    rng = np.random.default_rng(31)
    n, dims = 1100, [16, 40, 24]
    r, c = graph_with_hub_and_empty_rows(rng, n, 2600, 400)
    ref = O.build_csr(n, r, c, True)
    g = lp.lp_build_csr(n, dev_i32(r), dev_i32(c), True)
    Ws, Wn, b = toy_model(rng, dims, scale=0.25)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    es, ed = rng.integers(0, n, 150).astype(np.int32), rng.integers(0, n, 150).astype(np.int32)
    es[:20] = 3
    say("full-neighbourhood blocks (fan-out 0), GraphSAGE")
    run_case(ref, g, Ws, Wn, b, X, es, ed, 70, [0, 0], seed=5, step=9)
    run_case(ref, g, Ws, Wn, b, X, es, ed, 70, [4, 0], seed=5, step=9)       # mixed: drawn first hop, full second hop


def gcn_case(dims, fanout, bf16=False):
    from oracle import gcn_oracle as Gc
    rng = np.random.default_rng(700 + sum(dims) + sum(fanout))
    n = 1000
    r, c = graph_with_hub_and_empty_rows(rng, n, 2500, 300)
    r2, c2 = Gc.add_self_pairs(n, r, c)
    ref = O.build_csr(n, r2, c2, True)
    g = lp.lp_build_csr(n, dev_i32(r2), dev_i32(c2), True)
    K = len(dims) - 1
    W = [(rng.standard_normal((dims[k], dims[k + 1])) * 0.3).astype(np.float32) for k in range(K)]
    b = [(rng.standard_normal(dims[k + 1]) * 0.2).astype(np.float32) for k in range(K)]
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    B, n_pos = 200, 90
    es, ed = rng.integers(0, n, B).astype(np.int32), rng.integers(0, n, B).astype(np.int32)
    es[:30] = 3
    say("GCN on blocks dims=%s fanout=%s" % (dims, fanout))
    bref = Bk.sample_blocks(ref, es, ed, fanout, 21, 4)
    blocks = lp.lp_sample_blocks(g, dev_i32(es), dev_i32(ed), fanout, 21, 4)
    check_blocks(blocks, bref, K)
    inv = O.inverse_degrees(ref)
    assert np.array_equal(host(blocks.node_inv_deg)[:bref.n[0]], inv[bref.nodes[:bref.n[0]]].astype(np.float32))
    model = lp.Model(None, [dev_f32(w) for w in W], [dev_f32(x) for x in b], layer_type=lp.LP_LAYER_GCN)
    acts = lp.lp_sage_forward_blocks(blocks, model, dev_f32(X))
    a_ref = Bk.forward_blocks_gcn(bref, inv, W, b, X)
    for k in range(1, K + 1):
        assert_close(host(acts.A[k - 1])[:bref.n[k]], a_ref.A[k], TOL_ACT, "A^%d" % k)
        assert_close(host(acts.H[k - 1])[:bref.n[k]], a_ref.H[k], TOL_ACT, "H^%d" % k)
    s, loss, ds = lp.lp_score_loss(acts.H[-1], blocks.e_src_pos, blocks.e_dst_pos, n_pos)
    s_ref, loss_ref, ds_ref = O.score_loss(a_ref.H[K], bref.e_src_pos, bref.e_dst_pos, n_pos)
    assert_close(host(s), s_ref, TOL_ACT, "scores")
    grads = lp.lp_backward_blocks(blocks, model, acts, ds)
    g_ref = Bk.backward_blocks_gcn(bref, inv, W, a_ref, ds_ref)
    for k in range(K):
        assert_close(host(grads.dW_neigh[k]), g_ref.dW_neigh[k], TOL_GRAD, "dW^%d" % (k + 1))
        assert_close(host(grads.dbias[k]), g_ref.dbias[k], TOL_GRAD, "dbias^%d" % (k + 1))
    return ref, g, W, b, X, es, ed, n_pos, acts, bref


@pytest.mark.parametrize("dims,fanout", [([12, 20, 8], [0, 0]), ([12, 20, 8], [5, 3]), ([128, 256, 256, 256], [0, 0, 0]),
                                         ([128, 256, 256, 256], [25, 10, 5])])
def test_gcn_layers_on_blocks(dims, fanout):
    gcn_case(dims, fanout)


def test_gcn_full_neighbourhood_blocks_equal_the_full_graph_gcn_on_the_gpu():
    """Both GPU paths against each other as well: with all neighbours taken, the embeddings of the batch end points
    from the blocks must agree with lp_sage_forward's GCN on the whole graph (to fp32 summation-order noise)."""
    dims = [16, 32, 16]
    ref, g, W, b, X, es, ed, n_pos, acts, bref = gcn_case(dims, [0, 0])
    model = lp.Model(None, [dev_f32(w) for w in W], [dev_f32(x) for x in b], layer_type=lp.LP_LAYER_GCN)
    full = lp.lp_sage_forward(g, model, dev_f32(X))
    seeds = torch.from_numpy(bref.nodes[:bref.n[2]].astype(np.int64)).to("cuda:0")
    assert_close(host(acts.H[-1])[:bref.n[2]], host(full.H[-1][seeds]).astype(np.float64), 1e-5, "blocks vs full graph")
