"""GPU parity of the bfloat16-storage path (features, weights and activations in bf16, fp32 accumulation).

The oracle receives the same bf16-valued inputs, works in fp64 and rounds to bf16 exactly where the library stores
a bf16 matrix.  Both sides then differ by fp32-vs-fp64 accumulation noise, which now and then lands on the other
side of a bf16 rounding boundary (one bf16 ulp = 2^-8 relative).  Bars: activations, scores, loss 2^-7 relative;
gradients 2e-2 relative (per tensor, max-norm and 2-norm).  The paper fixes no precision; these bounds are this
repository's choice for the bf16 configuration.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2506_20818_amd as lp
from lp_workloads import make_workload, to_bf16_grid
from oracle import lp_oracle as O
from gpu_util import DEV, assert_close, dev_f32, dev_i32, host, rel_err
from test_gpu_parity import assert_dx_close, dx_band, graph_with_hub_and_empty_rows, hidden_of, random_pairs, say, toy_model

TOL_ACT = 2.0 ** -7
TOL_GRAD = 2e-2


def dev_bf16(a):
    return dev_f32(a).to(torch.bfloat16)        # exact: the values are already on the bf16 grid


def hostf(t):
    return host(t.float())


def bf16_model(Ws, Wn, b):
    return lp.Model([dev_bf16(w) for w in Ws], [dev_bf16(w) for w in Wn], [dev_f32(x) for x in b])


def grid(arrs):
    return [to_bf16_grid(a) for a in arrs]


@pytest.mark.parametrize("dims", [[8, 16], [24, 40, 8], [64, 64, 64], [128, 512, 512, 512], [72, 136, 24], [512, 64], [64, 1024, 8]])
@pytest.mark.parametrize("sym", [True, False])
def test_forward_parity_bf16(dims, sym):
    rng = np.random.default_rng(sum(dims) + sym)
    n = 1500 + dims[0]
    r, c = graph_with_hub_and_empty_rows(rng, n, 4000, 700)
    say("bf16 forward dims=%s sym=%s n=%d" % (dims, sym, n))
    ref = O.build_csr(n, r, c, sym)
    g = lp.lp_build_csr(n, dev_i32(r), dev_i32(c), sym)
    Ws, Wn, b = toy_model(rng, dims)
    Ws, Wn = grid(Ws), grid(Wn)
    X = to_bf16_grid(rng.standard_normal((n, dims[0])).astype(np.float32))
    acts = lp.lp_sage_forward(g, bf16_model(Ws, Wn, b), dev_bf16(X))
    assert acts.H[-1].dtype == torch.bfloat16
    exp = O.sage_forward(ref, Ws, Wn, b, X, storage="bf16")
    for k in range(1, len(dims)):
        assert_close(hostf(acts.A[k - 1]), exp.A[k], TOL_ACT, "A^%d" % k)
        assert_close(hostf(acts.H[k - 1]), exp.H[k], TOL_ACT, "H^%d" % k)


@pytest.mark.parametrize("F", [8, 64, 104, 512])
def test_score_loss_parity_bf16(F):
    rng = np.random.default_rng(F)
    n, B, n_pos = 777, 5001, 1700
    say("bf16 score_loss F=%d" % F)
    H = to_bf16_grid((rng.standard_normal((n, F)) * (2.0 / np.sqrt(F)) ** 0.5).astype(np.float32))
    es = rng.integers(0, n, B).astype(np.int32)
    ed = rng.integers(0, n, B).astype(np.int32)
    s, loss, ds = lp.lp_score_loss(dev_bf16(H), dev_i32(es), dev_i32(ed), n_pos)
    s_ref, loss_ref, ds_ref = O.score_loss(H, es, ed, n_pos)
    assert_close(host(s), s_ref, 1e-4, "scores")            # the dot product itself is fp32 on exact inputs
    assert abs(float(host(loss)[0]) - loss_ref) <= 1e-4 * abs(loss_ref)
    assert_close(host(ds), ds_ref, 1e-4, "dscore")


def check_grads(grads, ref, K, dx_band_width=None):
    for k in range(K):
        assert_close(host(grads.dW_self[k]), ref.dW_self[k], TOL_GRAD, "dW_self^%d" % (k + 1))
        assert_close(host(grads.dW_neigh[k]), ref.dW_neigh[k], TOL_GRAD, "dW_neigh^%d" % (k + 1))
        assert_close(host(grads.dbias[k]), ref.dbias[k], TOL_GRAD, "dbias^%d" % (k + 1))
    if grads.dX is not None:
        assert_dx_close(hostf(grads.dX), ref.dX, dx_band_width, TOL_GRAD, cap_on="rescued")


def check_grads_against_unrounded_backward(grads, exact, K):
    """The same gradients against a backward pass that rounds NOTHING (fp64 throughout, from the same bf16 forward
    activations): a check that does not depend on where the oracle's bf16 mode places its roundings.  Each node-sized
    matrix kept in bf16 carries a relative rounding error of at most 2^-9 per element, the gradients are linear in each
    of them, and layer k's weight gradient has at most 3 (K - k) + 1 such matrices upstream (dL/dH^K, then per layer
    the two products and their gated sum), so its relative 2-norm error is at most (3 (K - k) + 1) 2^-9, plus the
    fp32 accumulation noise of the kernels (1e-3)."""
    for k in range(1, K + 1):
        bound = (3 * (K - k) + 1) * 2.0 ** -9 + 1e-3
        for name, got, ref in (("dW_self", grads.dW_self[k - 1], exact.dW_self[k - 1]), ("dW_neigh", grads.dW_neigh[k - 1], exact.dW_neigh[k - 1]),
                               ("dbias", grads.dbias[k - 1], exact.dbias[k - 1])):
            e_l2 = rel_err(host(got), ref)[1]
            assert e_l2 <= bound, "%s^%d against the unrounded backward: 2-norm rel %.3e > %.3e" % (name, k, e_l2, bound)


@pytest.mark.parametrize("dims", [[8, 16], [24, 40, 8], [64, 64, 64], [128, 512, 512, 512], [72, 136, 24],
                                  [192, 200, 232]])   # the last: fused weight-gradient tiles that are partly empty
@pytest.mark.parametrize("sym", [True, False])
def test_backward_parity_bf16(dims, sym):
    rng = np.random.default_rng(2000 + sum(dims) + sym)
    n = 1300 + dims[-1]
    r, c = graph_with_hub_and_empty_rows(rng, n, 3500, 600)
    say("bf16 backward dims=%s sym=%s n=%d" % (dims, sym, n))
    ref = O.build_csr(n, r, c, sym)
    g = lp.lp_build_csr(n, dev_i32(r), dev_i32(c), sym)
    Ws, Wn, b = toy_model(rng, dims, scale=0.25)
    Ws, Wn = grid(Ws), grid(Wn)
    X = to_bf16_grid(rng.standard_normal((n, dims[0])).astype(np.float32))
    B, n_pos = 2500, 1000
    es = rng.integers(0, n, B).astype(np.int32)
    ed = rng.integers(0, n, B).astype(np.int32)
    model = bf16_model(Ws, Wn, b)
    Xd = dev_bf16(X)
    acts = lp.lp_sage_forward(g, model, Xd)
    s, loss, ds = lp.lp_score_loss(acts.H[-1], dev_i32(es), dev_i32(ed), n_pos)
    grads = lp.lp_backward(g, model, Xd, acts, dev_i32(es), dev_i32(ed), ds, want_dX=True)
    a_ref = O.sage_forward(ref, Ws, Wn, b, X, storage="bf16")
    s_ref, loss_ref, ds_ref = O.score_loss(a_ref.H[-1], es, ed, n_pos)
    g_ref = O.backward(ref, Ws, Wn, a_ref, es, ed, ds_ref, storage="bf16")
    assert_close(host(s), s_ref, TOL_ACT, "scores")
    assert abs(float(host(loss)[0]) - loss_ref) <= TOL_ACT * abs(loss_ref)
    K = len(dims) - 1
    check_grads(grads, g_ref, K, dx_band(ref, Ws, Wn, a_ref, es, ed, ds_ref, hidden_of(acts, K, hostf), storage="bf16"))
    check_grads_against_unrounded_backward(grads, O.backward(ref, Ws, Wn, a_ref, es, ed, ds_ref, storage="f32"), K)


@pytest.mark.parametrize("dims", [[24, 40, 8], [128, 512, 512, 512], [72, 136, 24]])
def test_training_forward_bf16_lists_the_end_points(dims):
    """lp_sage_forward_edges with bf16 storage on a batch small enough to be listed: rows of the last layer written
    exactly at the end points (everything else still NaN), equal to the oracle there; loss and gradients of the step
    against the oracle's full step."""
    from gpu_util import nan_filled_acts
    from test_gpu_parity import check_last_layer_listed
    rng = np.random.default_rng(2600 + sum(dims))
    n = 1300 + dims[-1]
    r, c = graph_with_hub_and_empty_rows(rng, n, 3500, 600)
    say("bf16 training forward dims=%s n=%d" % (dims, n))
    ref = O.build_csr(n, r, c, True)
    g = lp.lp_build_csr(n, dev_i32(r), dev_i32(c), True)
    Ws, Wn, b = toy_model(rng, dims, scale=0.25)
    Ws, Wn = grid(Ws), grid(Wn)
    X = to_bf16_grid(rng.standard_normal((n, dims[0])).astype(np.float32))
    B, n_pos = 400, 150
    assert 8 * B < 3 * n
    es = rng.integers(0, n, B).astype(np.int32)
    ed = rng.integers(0, n, B).astype(np.int32)
    es[0] = 3                                            # the 600-entry row
    model, Xd = bf16_model(Ws, Wn, b), dev_bf16(X)
    K = len(dims) - 1
    acts = nan_filled_acts(n, model, Xd)
    lp.lp_sage_forward_edges(g, model, Xd, dev_i32(es), dev_i32(ed), acts)
    a_ref = O.sage_forward(ref, Ws, Wn, b, X, storage="bf16")
    ends = check_last_layer_listed(acts, a_ref, es, ed, K, tol=TOL_ACT, to_host=hostf)
    assert 256 < ends.size <= 2 * B                      # more rows than one tile of the dense product
    s, loss, ds = lp.lp_score_loss(acts.H[-1], dev_i32(es), dev_i32(ed), n_pos)
    grads = lp.lp_backward(g, model, Xd, acts, dev_i32(es), dev_i32(ed), ds, want_dX=True)
    s_ref, loss_ref, ds_ref = O.score_loss(a_ref.H[-1], es, ed, n_pos)
    g_ref = O.backward(ref, Ws, Wn, a_ref, es, ed, ds_ref, storage="bf16")
    assert_close(host(s), s_ref, TOL_ACT, "scores")
    assert abs(float(host(loss)[0]) - loss_ref) <= TOL_ACT * abs(loss_ref)
    check_grads(grads, g_ref, K, dx_band(ref, Ws, Wn, a_ref, es, ed, ds_ref, hidden_of(acts, K, hostf), storage="bf16"))


def whole_step_bf16(name, scale=1.0):
    wl = make_workload(name, scale=scale)
    say("bf16 whole step %s scale=%g N=%d nnz~%d B=%d dims=%s" % (name, scale, wl.n_nodes, 2 * wl.src.size, wl.batch_edges, wl.dims))
    Ws, Wn, X = grid(wl.W_self), grid(wl.W_neigh), to_bf16_grid(wl.X)
    ref = O.build_csr(wl.n_nodes, wl.src, wl.dst, True)
    exp = O.train_step(ref, Ws, Wn, wl.bias, X, wl.pos_src, wl.pos_dst, wl.k_neg, wl.n_space, wl.sampler_seed,
                       wl.sampler_step, storage="bf16")
    g = lp.lp_build_csr(wl.n_nodes, dev_i32(wl.src), dev_i32(wl.dst), True)
    model = bf16_model(Ws, Wn, wl.bias)
    Xd = dev_bf16(X)
    n_pos, B = wl.n_pos, wl.batch_edges
    e_src = torch.empty(B, dtype=torch.int32, device=DEV)
    e_dst = torch.empty(B, dtype=torch.int32, device=DEV)
    e_src[:n_pos] = dev_i32(wl.pos_src)
    e_dst[:n_pos] = dev_i32(wl.pos_dst)
    lp.lp_sample_neg(g, dev_i32(wl.pos_src), wl.k_neg, wl.n_space, wl.sampler_seed, wl.sampler_step,
                     neg_dst=e_dst[n_pos:], neg_src=e_src[n_pos:])
    assert np.array_equal(host(e_dst), exp.e_dst) and np.array_equal(host(e_src), exp.e_src)
    acts = lp.lp_sage_forward(g, model, Xd)
    s, loss, ds = lp.lp_score_loss(acts.H[-1], e_src, e_dst, n_pos)
    grads = lp.lp_backward(g, model, Xd, acts, e_src, e_dst, ds)
    K = len(wl.dims) - 1
    for k in range(1, K + 1):
        assert_close(hostf(acts.A[k - 1]), exp.acts.A[k], TOL_ACT, "A^%d" % k)
        assert_close(hostf(acts.H[k - 1]), exp.acts.H[k], TOL_ACT, "H^%d" % k)
    assert_close(host(s), exp.scores, TOL_ACT, "scores")
    assert abs(float(host(loss)[0]) - exp.loss) <= TOL_ACT * abs(exp.loss)
    check_grads(grads, exp.grads, K)
    check_grads_against_unrounded_backward(grads, O.backward(ref, Ws, Wn, exp.acts, exp.e_src, exp.e_dst, exp.dscore, storage="f32"), K)


def test_whole_step_C1_bf16():
    whole_step_bf16("C1")


def test_whole_step_C5_shape_one_eighth_scale():
    # one worker's share of the partitioned graph at hidden 512 and 4 negatives per positive, on the generator
    # scaled to 1/8, every element of every saved matrix (the larger scales live in test_gpu_parity_large.py)
    whole_step_bf16("C5_keep0.2", scale=0.125)
