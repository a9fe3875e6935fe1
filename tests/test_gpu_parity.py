"""GPU parity: every call of the C ABI against the CPU oracle on the same seeded inputs.

Bars: CSR arrays and sampled negatives bit-exact; activations, scores and loss within 1e-4 relative;
gradients within 1e-3 relative (per tensor, max-norm and 2-norm), all in fp32 on the GPU vs fp64 in the oracle.
Weight and bias gradients are held to that bar as they are.  Only the input gradient dX gets an allowance for ReLU
near-ties: where the kernel's fp32 pre-activation and the oracle's fp64 one fall on different sides of zero (both
branches are valid there), the entries of dX that hinge on such units get the oracle-computed width of that
ambiguity as slack; the range of |z| is measured from the units that actually differ, the band may cover at most
0.1 % of dX, and every test prints how many units differed and how much the band covers.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2506_20818_amd as lp
from lp_workloads import make_workload
from oracle import lp_oracle as O
from gpu_util import DEV, HipStep, assert_close, dev_f32, dev_i32, host, make_model, rel_err

TOL_ACT = 1e-4
TOL_GRAD = 1e-3


def say(msg):
    print("[case] " + msg, flush=True)


def random_pairs(rng, n, e):
    return rng.integers(0, n, e).astype(np.int32), rng.integers(0, n, e).astype(np.int32)


def check_csr(g, ref):
    assert g.nnz == ref.nnz
    for name in ("rowptr", "colidx", "t_rowptr", "t_colidx"):
        assert np.array_equal(host(getattr(g, name)), getattr(ref, name)), name
    assert np.array_equal(host(g.inv_deg).view(np.uint32), ref.inv_deg.view(np.uint32)), "inv_deg bits"
    if g.t_entry_scale is not None:   # the 1/deg of every transposed entry's source row, in entry order
        assert np.array_equal(host(g.t_entry_scale).view(np.uint32), ref.inv_deg[ref.t_colidx].view(np.uint32)), "t_entry_scale bits"
    for order, rp in ((g.row_order, ref.rowptr), (g.t_row_order, ref.t_rowptr)):
        # rows of 64 and more entries by decreasing floor(log2(length)), then all shorter rows; ids ascending in a class
        deg = np.diff(rp).astype(np.int64)
        cls = np.where(deg >= 64, np.floor(np.log2(np.maximum(deg, 1))).astype(np.int64), 5)
        expect = np.lexsort((np.arange(ref.n_nodes), -cls))
        assert np.array_equal(host(order), expect), "row order"


# ------------------------------------------------------------------------------------------------ lp_build_csr
@pytest.mark.parametrize("seed", range(4))
@pytest.mark.parametrize("sym", [False, True])
def test_build_csr_small_random(seed, sym):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 3000))
    e = int(rng.integers(0, 9000))
    say("build_csr random seed=%d sym=%s n=%d e=%d" % (seed, sym, n, e))
    r, c = random_pairs(rng, n, e)                 # duplicates and self-loops included
    check_csr(lp.lp_build_csr(n, dev_i32(r), dev_i32(c), sym), O.build_csr(n, r, c, sym))


def test_build_csr_edge_cases():
    say("build_csr empty / single node / hub / out of range")
    z = np.zeros(0, np.int32)
    check_csr(lp.lp_build_csr(7, dev_i32(z), dev_i32(z), True), O.build_csr(7, z, z, True))
    one = np.zeros(3, np.int32)
    check_csr(lp.lp_build_csr(1, dev_i32(one), dev_i32(one), False), O.build_csr(1, one, one, False))
    n = 70000                                      # one hub row longer than a sort tile, 17-bit ids
    r = np.zeros(n - 1, np.int32)
    c = np.arange(1, n, dtype=np.int32)
    check_csr(lp.lp_build_csr(n, dev_i32(r), dev_i32(c), False), O.build_csr(n, r, c, False))
    check_csr(lp.lp_build_csr(n, dev_i32(r), dev_i32(c), True), O.build_csr(n, r, c, True))
    with pytest.raises(lp.LpError) as ei:
        lp.lp_build_csr(5, dev_i32([0, 5]), dev_i32([1, 1]), False)
    assert ei.value.status == -2
    with pytest.raises(lp.LpError):
        lp.lp_build_csr(5, dev_i32([0, 1]), dev_i32([1, -1]), True)


@pytest.mark.parametrize("name", ["C1", "C2"])
def test_build_csr_workloads(name):
    wl = make_workload(name, with_features=False)
    say("build_csr %s n=%d e=%d" % (name, wl.n_nodes, wl.src.size))
    check_csr(lp.lp_build_csr(wl.n_nodes, dev_i32(wl.src), dev_i32(wl.dst), True),
              O.build_csr(wl.n_nodes, wl.src, wl.dst, True))


# ------------------------------------------------------------------------------------------------ lp_sample_neg
def run_sampler(ref, g, pos, k_neg, n_space, seed, step):
    nf = torch.zeros(1, dtype=torch.int32, device=DEV)
    ns = torch.empty(pos.size * k_neg, dtype=torch.int32, device=DEV)
    got = lp.lp_sample_neg(g, dev_i32(pos), k_neg, n_space, seed, step, neg_src=ns, n_failed=nf)
    exp, exp_failed = O.sample_neg(ref, pos, k_neg, n_space, seed, step)
    assert np.array_equal(host(got), exp)
    assert np.array_equal(host(ns), np.repeat(pos, k_neg))
    assert int(host(nf)[0]) == exp_failed
    return exp


@pytest.mark.parametrize("seed", range(4))
def test_sample_neg_bit_exact_dense_small_graphs(seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(3, 60))
    r, c = random_pairs(rng, n, int(rng.integers(0, n * n // 2 + 1)))      # dense: retries and probing happen
    say("sample_neg dense seed=%d n=%d" % (seed, n))
    ref = O.build_csr(n, r, c, True)
    g = lp.lp_build_csr(n, dev_i32(r), dev_i32(c), True)
    pos = rng.integers(0, n, 3000).astype(np.int32)
    n_space = n if seed % 2 else n + 9
    run_sampler(ref, g, pos, int(rng.integers(1, 5)), n_space, int(rng.integers(0, 2 ** 63)), int(rng.integers(0, 2 ** 40)))


def test_sample_neg_degenerate_rows():
    say("sample_neg single valid destination / no valid destination / empty batch")
    r, c = np.array([0, 0], np.int32), np.array([1, 2], np.int32)
    ref, g = O.build_csr(4, r, c, True), lp.lp_build_csr(4, dev_i32(r), dev_i32(c), True)
    assert np.all(run_sampler(ref, g, np.zeros(500, np.int32), 2, 4, 99, 0) == 3)
    r, c = np.array([0, 0, 0], np.int32), np.array([1, 2, 3], np.int32)
    ref, g = O.build_csr(4, r, c, True), lp.lp_build_csr(4, dev_i32(r), dev_i32(c), True)
    run_sampler(ref, g, np.zeros(5, np.int32), 1, 4, 99, 0)
    out = lp.lp_sample_neg(g, dev_i32(np.zeros(0, np.int32)), 3, 4, 1, 1)
    assert out.numel() == 0


@pytest.mark.parametrize("name", ["C1", "C2"])
def test_sample_neg_workloads(name):
    wl = make_workload(name, with_features=False)
    say("sample_neg %s n_pos=%d k=%d" % (name, wl.n_pos, wl.k_neg))
    ref = O.build_csr(wl.n_nodes, wl.src, wl.dst, True)
    g = lp.lp_build_csr(wl.n_nodes, dev_i32(wl.src), dev_i32(wl.dst), True)
    run_sampler(ref, g, wl.pos_src, wl.k_neg, wl.n_space, wl.sampler_seed, wl.sampler_step)
    run_sampler(ref, g, wl.pos_src[:1000], 4, wl.n_space, 1, 2 ** 33 + 5)


# ------------------------------------------------------------------------------------------------ forward
def toy_model(rng, dims, scale=0.3):
    K = len(dims) - 1
    Ws = [(rng.standard_normal((dims[k], dims[k + 1])) * scale).astype(np.float32) for k in range(K)]
    Wn = [(rng.standard_normal((dims[k], dims[k + 1])) * scale).astype(np.float32) for k in range(K)]
    b = [(rng.standard_normal(dims[k + 1]) * 0.2).astype(np.float32) for k in range(K)]
    return Ws, Wn, b


def graph_with_hub_and_empty_rows(rng, n, e, hub_deg):
    r, c = random_pairs(rng, n - 50, e)             # the last 50 nodes stay isolated
    hub_c = rng.choice(n - 50, hub_deg, replace=False).astype(np.int32)
    r = np.concatenate([r, np.full(hub_deg, 3, np.int32)])
    c = np.concatenate([c, hub_c])
    return r, c


@pytest.mark.parametrize("dims", [[4, 8], [12, 20, 4], [36, 64, 32], [64, 64, 64], [128, 256, 256, 256], [100, 132, 68],
                                  [512, 64], [64, 512, 8]])
@pytest.mark.parametrize("sym", [True, False])
def test_forward_parity_widths_hub_and_empty_rows(dims, sym):
    rng = np.random.default_rng(sum(dims) + sym)
    n = 1500 + dims[0]                              # not a multiple of any tile size
    r, c = graph_with_hub_and_empty_rows(rng, n, 4000, 700)
    say("forward dims=%s sym=%s n=%d" % (dims, sym, n))
    ref = O.build_csr(n, r, c, sym)
    g = lp.lp_build_csr(n, dev_i32(r), dev_i32(c), sym)
    Ws, Wn, b = toy_model(rng, dims)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    acts = lp.lp_sage_forward(g, make_model(Ws, Wn, b), dev_f32(X))
    exp = O.sage_forward(ref, Ws, Wn, b, X)
    for k in range(1, len(dims)):
        assert_close(host(acts.A[k - 1]), exp.A[k], TOL_ACT, "A^%d" % k)
        assert_close(host(acts.H[k - 1]), exp.H[k], TOL_ACT, "H^%d" % k)
    iso = np.flatnonzero(np.diff(ref.rowptr) == 0)
    assert iso.size >= 50 and np.all(host(acts.A[0])[iso] == 0)


@pytest.mark.parametrize("x_scale,w_scale", [(1e-10, 1.0), (1e15, 1e-3), (1.0, 1e12), (1e-6, 1e-6)])
def test_products_from_bfloat16_terms_across_magnitudes(x_scale, w_scale):
    """The three-term splitting is relative: features and weights far from 1 (products from about 1e-28 up to 1e27)
    meet the same relative bar, forward and backward, with values whose exponents differ inside one row.  (Term
    products below the smallest normal fp32, 1.2e-38, are flushed by the matrix instructions, so full accuracy
    needs products above about 1e-33: the documented limit of this mode.)"""
    rng = np.random.default_rng(77)
    dims = [64, 256, 128]
    n = 900
    r, c = random_pairs(rng, n, 4000)
    say("split products x_scale=%g w_scale=%g" % (x_scale, w_scale))
    ref = O.build_csr(n, r, c, True)
    g = lp.lp_build_csr(n, dev_i32(r), dev_i32(c), True)
    Ws, Wn, b = toy_model(rng, dims)
    Ws[0], Wn[0] = (Ws[0] * w_scale).astype(np.float32), (Wn[0] * w_scale).astype(np.float32)
    b = [(bb * x_scale * w_scale).astype(np.float32) for bb in b]
    spread = np.exp2(rng.integers(-12, 13, (n, dims[0]))).astype(np.float32)       # exponents differ inside a row
    X = (rng.standard_normal((n, dims[0])) * spread * x_scale).astype(np.float32)
    model, Xd = make_model(Ws, Wn, b, lp.LP_FP32_PRODUCTS_BF16X6), dev_f32(X)
    acts = lp.lp_sage_forward(g, model, Xd)
    exp = O.sage_forward(ref, Ws, Wn, b, X)
    for k in range(1, len(dims)):
        assert_close(host(acts.H[k - 1]), exp.H[k], TOL_ACT, "H^%d" % k)
    # backward from a given dL/ds (the loss itself would saturate at these magnitudes)
    B = 1200
    es, ed = rng.integers(0, n, B).astype(np.int32), rng.integers(0, n, B).astype(np.int32)
    ds = (rng.standard_normal(B) / B).astype(np.float32)
    grads = lp.lp_backward(g, model, Xd, acts, dev_i32(es), dev_i32(ed), dev_f32(ds), want_dX=True)
    g_ref = O.backward(ref, Ws, Wn, exp, es, ed, ds.astype(np.float64))
    K = len(dims) - 1
    check_grads(grads, g_ref, K, dx_band(ref, Ws, Wn, exp, es, ed, ds.astype(np.float64), hidden_of(acts, K)))


def test_two_models_with_different_product_modes_back_to_back():
    """The way of forming fp32 products belongs to the model handed to each call: two models over the same weight
    tensors, one per mode, called alternately on one stream without any synchronisation in between, each give what
    they give when run alone, and the two modes really are different arithmetic."""
    rng = np.random.default_rng(91)
    n, dims = 2600, [64, 256, 128]
    r, c = random_pairs(rng, n, 9000)
    say("two product modes back to back n=%d dims=%s" % (n, dims))
    ref = O.build_csr(n, r, c, True)
    g = lp.lp_build_csr(n, dev_i32(r), dev_i32(c), True)
    Ws, Wn, b = toy_model(rng, dims)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    m_split = make_model(Ws, Wn, b, lp.LP_FP32_PRODUCTS_BF16X6)
    m_native = m_split.with_products(lp.LP_FP32_PRODUCTS_NATIVE)
    assert m_native.W_neigh[0].data_ptr() == m_split.W_neigh[0].data_ptr()
    Xd = dev_f32(X)
    alone = {}
    for name, m in (("split", m_split), ("native", m_native)):
        alone[name] = host(lp.lp_sage_forward(g, m, Xd).H[-1]).copy()
    outs = [lp.lp_sage_forward(g, m, Xd).H[-1] for m in (m_split, m_native, m_split, m_native, m_native, m_split)]
    for t, name in zip(outs, ("split", "native", "split", "native", "native", "split")):
        assert np.array_equal(host(t), alone[name]), name
    assert not np.array_equal(alone["split"], alone["native"])
    exp = O.sage_forward(ref, Ws, Wn, b, X).H[-1]
    assert_close(alone["split"], exp, TOL_ACT, "H^K, bfloat16 terms")
    assert_close(alone["native"], exp, TOL_ACT, "H^K, fp32 instructions")


def test_products_from_bfloat16_terms_at_the_end_of_the_fp32_range():
    """Finite inputs up to the largest fp32 value are split exactly (no NaN from a first term that would round to
    infinity) and give the oracle's result in both modes; an infinite or NaN input makes every output that depends on
    it non-finite in both modes, and no other output changes by a bit."""
    rng = np.random.default_rng(92)
    n, dims = 700, [64, 256]
    r = rng.integers(4, n, 3000).astype(np.int32)          # nodes 0..3 are nobody's neighbour (directed rows)
    c = rng.integers(4, n, 3000).astype(np.int32)
    say("end of the fp32 range n=%d dims=%s" % (n, dims))
    ref = O.build_csr(n, r, c, False)
    g = lp.lp_build_csr(n, dev_i32(r), dev_i32(c), False)
    Ws, Wn, b = toy_model(rng, dims)
    Ws[0] = (Ws[0] * 2.0 ** -12).astype(np.float32)        # keeps the sums of the huge rows finite
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    clean = X.copy()
    fmax = np.finfo(np.float32).max
    X[0, :] = 0.0
    X[0, [3, 17, 40]] = [fmax, -fmax, np.float32(3.4e38)]               # all three would round to an infinite bfloat16
    X[1, [5, 6]] = [np.float32(3.397e38), np.float32(-3.39e38)]         # just above / below the largest finite bfloat16
    exp = O.sage_forward(ref, Ws, Wn, b, X).H[-1]
    assert np.all(np.isfinite(exp[:2]))
    for mode in (lp.LP_FP32_PRODUCTS_BF16X6, lp.LP_FP32_PRODUCTS_NATIVE):
        model = make_model(Ws, Wn, b, mode)
        base = host(lp.lp_sage_forward(g, model, dev_f32(clean)).H[-1]).copy()
        got = host(lp.lp_sage_forward(g, model, dev_f32(X)).H[-1]).copy()
        for v in (0, 1):
            assert_close(got[v], exp[v], TOL_ACT, "row %d at the end of the range, mode %d" % (v, mode))
        assert np.array_equal(got[4:], base[4:])
        bad = X.copy()
        bad[2, 7], bad[3, 9] = np.inf, np.nan
        got = host(lp.lp_sage_forward(g, model, dev_f32(bad)).H[-1]).copy()
        assert not np.isfinite(got[2]).any() and not np.isfinite(got[3]).any(), "mode %d" % mode
        assert np.array_equal(got[4:], base[4:]) and np.all(np.isfinite(got[:2]))


def test_forward_without_row_order_and_single_node():
    say("forward natural row order / one-node graph")
    rng = np.random.default_rng(5)
    n, dims = 300, [8, 16, 4]
    r, c = random_pairs(rng, n, 900)
    ref = O.build_csr(n, r, c, True)
    g = lp.lp_build_csr(n, dev_i32(r), dev_i32(c), True, with_row_order=False)
    Ws, Wn, b = toy_model(rng, dims)
    X = rng.standard_normal((n, 8)).astype(np.float32)
    acts = lp.lp_sage_forward(g, make_model(Ws, Wn, b), dev_f32(X))
    assert_close(host(acts.H[-1]), O.sage_forward(ref, Ws, Wn, b, X).H[-1], TOL_ACT, "H^K")
    z = np.zeros(1, np.int32)
    ref = O.build_csr(1, z, z, False)                # a single node with a self-loop
    g = lp.lp_build_csr(1, dev_i32(z), dev_i32(z), False)
    X = rng.standard_normal((1, 8)).astype(np.float32)
    acts = lp.lp_sage_forward(g, make_model(Ws, Wn, b), dev_f32(X))
    assert_close(host(acts.H[-1]), O.sage_forward(ref, Ws, Wn, b, X).H[-1], TOL_ACT, "H^K one node")


# ------------------------------------------------------------------------------------------------ score / loss
@pytest.mark.parametrize("F", [4, 32, 64, 100, 256, 512])
def test_score_loss_parity(F):
    rng = np.random.default_rng(F)
    n, B, n_pos = 777, 5001, 1700
    say("score_loss F=%d" % F)
    H = (rng.standard_normal((n, F)) * (2.0 / np.sqrt(F)) ** 0.5).astype(np.float32)
    H[0] *= 30.0                                     # some saturated scores
    es = rng.integers(0, n, B).astype(np.int32)
    ed = rng.integers(0, n, B).astype(np.int32)
    es[:40] = 0
    ed[:20] = 0
    s, loss, ds = lp.lp_score_loss(dev_f32(H), dev_i32(es), dev_i32(ed), n_pos)
    s_ref, loss_ref, ds_ref = O.score_loss(H, es, ed, n_pos)
    assert_close(host(s), s_ref, TOL_ACT, "scores")
    assert abs(float(host(loss)[0]) - loss_ref) <= TOL_ACT * abs(loss_ref)
    assert_close(host(ds), ds_ref, TOL_ACT, "dscore")
    s2, loss2, _ = lp.lp_score_loss(dev_f32(H), dev_i32(es), dev_i32(ed), n_pos)
    assert host(loss2).tobytes() == host(loss).tobytes()        # fixed summation order


def test_score_loss_zero_embeddings_and_empty_batch():
    say("score_loss zeros / B=0")
    H = np.zeros((10, 8), np.float32)
    es, ed = np.arange(6, dtype=np.int32), np.arange(1, 7, dtype=np.int32)
    s, loss, ds = lp.lp_score_loss(dev_f32(H), dev_i32(es), dev_i32(ed), 2)
    assert np.all(host(s) == 0) and abs(float(host(loss)[0]) - np.log(2.0)) < 1e-6
    np.testing.assert_allclose(host(ds), np.array([-0.5, -0.5, 0.5, 0.5, 0.5, 0.5]) / 6, rtol=1e-6)
    z = np.zeros(0, np.int32)
    s, loss, ds = lp.lp_score_loss(dev_f32(H), dev_i32(z), dev_i32(z), 0)
    assert float(host(loss)[0]) == 0.0


def test_edges_with_ids_outside_the_graph_are_counted_and_contribute_nothing():
    """The documented contract for a corrupted batch: an edge with an end point outside [0, n_nodes) is never
    dereferenced, is scored 0 with dscore 0, stays out of the loss sum and of every gradient, still counts in B, and is
    reported through n_invalid."""
    rng = np.random.default_rng(17)
    n, dims = 900, [16, 32, 8]
    r, c = random_pairs(rng, n, 3000)
    say("edges with ids outside the graph n=%d" % n)
    ref = O.build_csr(n, r, c, True)
    g = lp.lp_build_csr(n, dev_i32(r), dev_i32(c), True)
    Ws, Wn, b = toy_model(rng, dims)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    B, n_pos = 1200, 500
    es, ed = rng.integers(0, n, B).astype(np.int32), rng.integers(0, n, B).astype(np.int32)
    bad = rng.choice(B, 37, replace=False)
    es[bad[:12]] = -1
    ed[bad[12:25]] = n
    es[bad[25:]] = n + 1000
    ed[bad[30:]] = -7
    ok = np.ones(B, bool)
    ok[bad] = False
    model, Xd = make_model(Ws, Wn, b), dev_f32(X)
    acts = lp.lp_sage_forward(g, model, Xd)
    counter = torch.zeros(1, dtype=torch.int32, device=DEV)
    s, loss, ds = lp.lp_score_loss(acts.H[-1], dev_i32(es), dev_i32(ed), n_pos, n_invalid=counter)
    assert int(host(counter)[0]) == bad.size
    a_ref = O.sage_forward(ref, Ws, Wn, b, X)
    y_pos = int(ok[:n_pos].sum())                                   # the valid edges keep their labels
    s_ref, loss_ref, ds_ref = O.score_loss(a_ref.H[-1], es[ok], ed[ok], y_pos)
    n_ok = int(ok.sum())
    assert np.all(host(s)[~ok] == 0) and np.all(host(ds)[~ok] == 0)
    assert_close(host(s)[ok], s_ref, TOL_ACT, "scores of the valid edges")
    assert abs(float(host(loss)[0]) - loss_ref * n_ok / B) <= TOL_ACT * loss_ref
    assert_close(host(ds)[ok], ds_ref * n_ok / B, TOL_ACT, "dscore of the valid edges")
    grads = lp.lp_backward(g, model, Xd, acts, dev_i32(es), dev_i32(ed), ds, want_dX=True)
    g_ref = O.backward(ref, Ws, Wn, a_ref, es[ok], ed[ok], ds_ref * n_ok / B)
    K = len(dims) - 1
    check_grads(grads, g_ref, K, dx_band(ref, Ws, Wn, a_ref, es[ok], ed[ok], ds_ref * n_ok / B, hidden_of(acts, K)))
    # the variant without a workspace counts the same
    counter.zero_()
    s2, l2 = torch.empty_like(s), torch.empty_like(loss)
    lp.lp_score_loss_noalloc(acts.H[-1], dev_i32(es), dev_i32(ed), n_pos, s2, l2, None, n_invalid=counter)
    assert int(host(counter)[0]) == bad.size and host(l2).tobytes() == host(loss).tobytes()


# ------------------------------------------------------------------------------------------------ backward
DX_BAND_CAP = 1e-3      # the near-tie band of dX may cover at most 0.1 % of its entries


def dx_band(ref_csr, Ws, Wn, acts_ref, es, ed, ds_ref, hidden_gpu, storage="f32"):
    """Near-ties of the ReLU gate, for the input gradient only.  The kernel takes relu'(z) = [z > 0] on its own
    (fp32-accumulated) pre-activation, the oracle on its fp64 one; a hidden unit whose |z| lies below the
    accumulated rounding error may take either branch, and either is a correct answer.  The width of that range is
    MEASURED here, not assumed: hidden_gpu[k-1] is the kernel's stored H^k (k = 1..K-1) and the margin is the largest
    |z| of the oracle over the units where the two sides decided differently (0 when they agree everywhere, and
    then there is no band).  Returns None, or a function that computes, per entry of dX, the oracle's
    |dX(all such units off) - dX(all on)|.  Weight and bias gradients get no such allowance."""
    K = len(Ws)
    margin, flips, units = 0.0, 0, 0
    for k in range(1, K):
        z = acts_ref.Z[k]
        differ = (np.asarray(hidden_gpu[k - 1]) > 0) != (z > 0)
        flips += int(differ.sum())
        units += z.size
        if differ.any():
            margin = max(margin, float(np.abs(z[differ]).max()))
    say("  ReLU gate: %d of %d hidden units decided differently, largest |z| among them %.3e" % (flips, units, margin))
    if flips == 0:
        return None
    margin = margin * (1.0 + 1e-9) + 1e-300

    def width():          # two more oracle backward passes: computed only if the plain bar is missed
        lo = O.backward(ref_csr, Ws, Wn, acts_ref, es, ed, ds_ref, relu_margin=margin, storage=storage)
        hi = O.backward(ref_csr, Ws, Wn, acts_ref, es, ed, ds_ref, relu_margin=-margin, storage=storage)
        return np.abs(hi.dX - lo.dX)
    return width


def assert_dx_close(got, ref, band, tol, what="dX", cap_on="covered"):
    """dX against the oracle.  The plain per-tensor bar is tried first; only if it fails is the near-tie band of
    dx_band used, and then (a) everything outside the band must meet the bar and (b) the band must stay small:
    with cap_on="covered" the entries whose band is wider than the tolerance, with cap_on="rescued" the entries
    that miss the plain bar and are excused by the band, may be at most DX_BAND_CAP of all entries.  (bf16
    storage uses the second form: there the stored activations differ by whole bf16 steps, the measured range of
    |z| is about 1e-2, so the band is wide by nature while the entries that actually move stay few.)"""
    got = np.asarray(got, np.float64)
    assert np.all(np.isfinite(got)), what
    e_max, e_l2 = rel_err(got, ref)
    if e_max <= tol and e_l2 <= tol:
        say("  %s meets the bar without any band (max-norm rel %.2e, 2-norm rel %.2e)" % (what, e_max, e_l2))
        return
    assert band is not None, "%s: max-norm rel %.3e, 2-norm rel %.3e > %.1e and no gate decision differs" % (what, e_max, e_l2, tol)
    band = band()
    diff = np.abs(got - ref)
    excess = np.maximum(diff - band, 0.0)                     # outside the near-tie band
    m, l2 = np.abs(ref).max(), np.sqrt((ref * ref).sum())
    x_max = excess.max() / m if m > 0 else excess.max()
    x_l2 = np.sqrt((excess * excess).sum()) / l2 if l2 > 0 else np.sqrt((excess * excess).sum())
    covered = float((band > tol * m).mean())
    rescued = float((diff > tol * m).mean())
    say("  %s: plain errors %.2e / %.2e; near-tie band wider than the tolerance on %.4f %% of the entries, "
        "%.4f %% of the entries miss the plain bar and lie inside it" % (what, e_max, e_l2, 100.0 * covered, 100.0 * rescued))
    assert x_max <= tol and x_l2 <= tol, "%s outside the band: max-norm rel %.3e, 2-norm rel %.3e" % (what, x_max, x_l2)
    share = covered if cap_on == "covered" else rescued
    assert share <= DX_BAND_CAP, what + ": near-tie band (%s) takes %.4f %% of the entries" % (cap_on, 100.0 * share)


def check_grads(grads, ref, K, dx_band_width=None):
    """Weight and bias gradients of every layer at the plain bar; dX (when computed) with the measured near-tie band."""
    for k in range(K):
        assert_close(host(grads.dW_self[k]), ref.dW_self[k], TOL_GRAD, "dW_self^%d" % (k + 1))
        assert_close(host(grads.dW_neigh[k]), ref.dW_neigh[k], TOL_GRAD, "dW_neigh^%d" % (k + 1))
        assert_close(host(grads.dbias[k]), ref.dbias[k], TOL_GRAD, "dbias^%d" % (k + 1))
    if grads.dX is not None:
        assert_dx_close(host(grads.dX), ref.dX, dx_band_width, TOL_GRAD)


def hidden_of(acts, K, to_host=host):
    return [to_host(acts.H[k - 1]) for k in range(1, K)]


@pytest.mark.parametrize("dims", [[4, 8], [12, 20, 4], [64, 64, 64], [128, 256, 256, 256], [100, 132, 68], [64, 512, 8],
                                  [192, 200, 232],    # fused weight-gradient tiles that are partly empty
                                  [64, 512, 128], [48, 80, 144]])   # 128-column tiles; K parts of 48 and 80 values
@pytest.mark.parametrize("sym", [True, False])
def test_backward_parity(dims, sym, products=lp.LP_FP32_PRODUCTS_BF16X6):
    rng = np.random.default_rng(1000 + sum(dims) + sym)
    n = 1300 + dims[-1]
    r, c = graph_with_hub_and_empty_rows(rng, n, 3500, 600)
    say("backward dims=%s sym=%s n=%d" % (dims, sym, n))
    ref = O.build_csr(n, r, c, sym)
    g = lp.lp_build_csr(n, dev_i32(r), dev_i32(c), sym)
    Ws, Wn, b = toy_model(rng, dims, scale=0.25)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    B, n_pos = 2500, 1000
    es = rng.integers(0, n, B).astype(np.int32)
    ed = rng.integers(0, n, B).astype(np.int32)      # repeated nodes and u == v included
    model = make_model(Ws, Wn, b, products)
    Xd = dev_f32(X)
    acts = lp.lp_sage_forward(g, model, Xd)
    s, loss, ds = lp.lp_score_loss(acts.H[-1], dev_i32(es), dev_i32(ed), n_pos)
    grads = lp.lp_backward(g, model, Xd, acts, dev_i32(es), dev_i32(ed), ds, want_dX=True)
    a_ref = O.sage_forward(ref, Ws, Wn, b, X)
    s_ref, loss_ref, ds_ref = O.score_loss(a_ref.H[-1], es, ed, n_pos)
    g_ref = O.backward(ref, Ws, Wn, a_ref, es, ed, ds_ref)
    K = len(dims) - 1
    assert_close(host(s), s_ref, TOL_ACT, "scores")
    check_grads(grads, g_ref, K, dx_band(ref, Ws, Wn, a_ref, es, ed, ds_ref, hidden_of(acts, K)))
    # without dX the weight gradients are the same
    grads2 = lp.lp_backward(g, model, Xd, acts, dev_i32(es), dev_i32(ed), ds, want_dX=False)
    check_grads(grads2, g_ref, K)
    # a graph without the per-entry scales of its transpose (the backward pass then looks them up in inv_deg): same bits
    g3 = lp.lp_build_csr(n, dev_i32(r), dev_i32(c), sym, with_entry_scale=False)
    grads3 = lp.lp_backward(g3, model, Xd, acts, dev_i32(es), dev_i32(ed), ds, want_dX=True)
    for k in range(K):
        assert torch.equal(grads3.dW_self[k], grads.dW_self[k]) and torch.equal(grads3.dW_neigh[k], grads.dW_neigh[k])
    assert torch.equal(grads3.dX, grads.dX)


@pytest.mark.parametrize("dims", [[128, 256, 256, 256], [192, 200, 232], [64, 512, 128], [48, 80, 144]])
def test_backward_parity_with_fp32_matrix_instructions(dims):
    """The same bar with LP_FP32_PRODUCTS_NATIVE (the other tests build their models with products from bfloat16
    terms)."""
    test_backward_parity(dims, True, lp.LP_FP32_PRODUCTS_NATIVE)


@pytest.mark.parametrize("dims", [[16, 32, 8], [128, 256, 64], [64, 520, 8]])
def test_hub_rows_served_by_a_whole_workgroup(dims):
    """Rows of 512 or more entries take the workgroup-per-row path of the aggregation: hubs of 511 (stays on the
    wavefront path), 512, 1023, 1025 and 3000 neighbours in the graph (rows, and columns of the transpose), and a
    node that is an endpoint of 1700 scored edges in the batch."""
    rng = np.random.default_rng(77 + dims[0])
    n = 3300
    r, c = random_pairs(rng, n, 5000)
    for hub, deg in ((5, 511), (9, 512), (100, 1023), (2000, 1025), (3299, 3000)):
        r = np.concatenate([r, np.full(deg, hub, np.int32)])
        c = np.concatenate([c, rng.choice(n, deg, replace=False).astype(np.int32)])
    say("hub rows dims=%s n=%d" % (dims, n))
    ref = O.build_csr(n, r, c, False)
    assert np.diff(ref.rowptr).max() >= 3000
    g = lp.lp_build_csr(n, dev_i32(r), dev_i32(c), False)
    Ws, Wn, b = toy_model(rng, dims, scale=0.2)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    B, n_pos = 4000, 1500
    es = rng.integers(0, n, B).astype(np.int32)
    ed = rng.integers(0, n, B).astype(np.int32)
    es[:1200] = 7                                    # batch hub: 1200 times a source, 500 times a destination
    ed[3500:] = 7
    model = make_model(Ws, Wn, b)
    Xd = dev_f32(X)
    acts = lp.lp_sage_forward(g, model, Xd)
    a_ref = O.sage_forward(ref, Ws, Wn, b, X)
    for k in range(1, len(dims)):
        assert_close(host(acts.A[k - 1]), a_ref.A[k], TOL_ACT, "A^%d" % k)
        assert_close(host(acts.H[k - 1]), a_ref.H[k], TOL_ACT, "H^%d" % k)
    s, loss, ds = lp.lp_score_loss(acts.H[-1], dev_i32(es), dev_i32(ed), n_pos)
    grads = lp.lp_backward(g, model, Xd, acts, dev_i32(es), dev_i32(ed), ds, want_dX=True)
    s_ref, loss_ref, ds_ref = O.score_loss(a_ref.H[-1], es, ed, n_pos)
    g_ref = O.backward(ref, Ws, Wn, a_ref, es, ed, ds_ref)
    K = len(dims) - 1
    check_grads(grads, g_ref, K, dx_band(ref, Ws, Wn, a_ref, es, ed, ds_ref, hidden_of(acts, K)))
    # same bits when repeated: the hub sums do not depend on which workgroup serves which row
    again = lp.lp_backward(g, model, Xd, acts, dev_i32(es), dev_i32(ed), ds, want_dX=True)
    assert np.array_equal(host(again.dX), host(grads.dX)) and np.array_equal(host(again.dW_neigh[0]), host(grads.dW_neigh[0]))


def test_backward_empty_batch_gives_zero_gradients():
    say("backward B=0")
    rng = np.random.default_rng(3)
    n, dims = 200, [8, 16, 4]
    r, c = random_pairs(rng, n, 500)
    g = lp.lp_build_csr(n, dev_i32(r), dev_i32(c), True)
    Ws, Wn, b = toy_model(rng, dims)
    model = make_model(Ws, Wn, b)
    Xd = dev_f32(rng.standard_normal((n, 8)))
    acts = lp.lp_sage_forward(g, model, Xd)
    z = dev_i32(np.zeros(0, np.int32))
    grads = lp.lp_backward(g, model, Xd, acts, z, z, dev_f32(np.zeros(0)), want_dX=True)
    for t in grads.dW_self + grads.dW_neigh + grads.dbias + [grads.dX]:
        assert np.all(host(t) == 0)


# ------------------------------------------------------------------------------------------------ training forward
def oracle_acts_with_the_kernel_gates(acts_ref, hidden_gpu, K, max_abs_z=1e-5, max_share=1e-5):
    """relu'(z) = [z > 0] is a decision taken in floating point; where the kernel's fp32 pre-activation and the oracle's
    fp64 one fall on different sides of 0 both answers are correct, and a comparison of what follows has to take the
    decision in one precision: the kernel's.  Returns the oracle's activations with the sign of Z flipped at exactly
    those units (nothing else changes), after checking that they are genuine near-ties (|z| <= max_abs_z) and few."""
    Z = list(acts_ref.Z)
    flips = 0
    for k in range(1, K):
        z = acts_ref.Z[k]
        differ = (np.asarray(hidden_gpu[k - 1]) > 0) != (z > 0)
        if differ.any():
            assert float(np.abs(z[differ]).max()) <= max_abs_z, "gate decisions differ away from 0"
            Z[k] = np.where(differ, -z, z)
            Z[k][differ & (z == 0)] = 1e-300          # the oracle's exact 0 (gate closed), the kernel's gate open
            flips += int(differ.sum())
    assert flips <= max(1, int(max_share * sum(acts_ref.Z[k].size for k in range(1, K))))
    return O.Activations(acts_ref.H, acts_ref.A, Z), flips


def check_last_layer_listed(acts, a_ref, es, ed, K, tol=TOL_ACT, to_host=host, what=""):
    """After lp_sage_forward_edges into NaN-filled matrices: the lower layers complete; rows of A^K and H^K of the end
    points of the scored edges against the oracle; with 8 B < 3 n every other row still NaN (never written), else every
    row evaluated.  Returns the end points."""
    n = a_ref.H[K].shape[0]
    ok = (es >= 0) & (es < n) & (ed >= 0) & (ed < n)
    ends = np.unique(np.concatenate([es[ok], ed[ok]])).astype(np.int64)
    rest = np.ones(n, bool)
    rest[ends] = False
    for k in range(1, K):
        assert_close(to_host(acts.A[k - 1]), a_ref.A[k], tol, what + "A^%d" % k)
        assert_close(to_host(acts.H[k - 1]), a_ref.H[k], tol, what + "H^%d" % k)
    A, H = to_host(acts.A[K - 1]), to_host(acts.H[K - 1])
    if 8 * es.size < 3 * n:
        if ends.size:
            assert_close(A[ends], a_ref.A[K][ends], tol, what + "A^K at the end points")
            assert_close(H[ends], a_ref.H[K][ends], tol, what + "H^K at the end points")
        assert np.isnan(A[rest]).all() and np.isnan(H[rest]).all(), "a row of a node that is no end point was written"
    else:
        assert_close(A, a_ref.A[K], tol, what + "A^K")
        assert_close(H, a_ref.H[K], tol, what + "H^K")
    return ends


@pytest.mark.parametrize("dims", [[12, 8], [12, 20, 4], [128, 256, 256, 256], [100, 132, 68], [64, 512, 128]])
@pytest.mark.parametrize("B,bad_ids", [(1, False), (150, False), (345, False), (6000, False), (345, True)])
def test_training_forward_evaluates_the_last_layer_at_the_end_points_only(dims, B, bad_ids):
    """lp_sage_forward_edges, then the loss and the backward pass on the same edges: everything against the oracle's
    full pass.  B = 345 lists about 600 nodes (more than the rows of one tile of the dense product, the hub row 3 among
    them); B = 6000 is beyond 3 n / 8, where every node is evaluated.  With bad_ids two edges carry an id outside the graph: they list nothing, and the loss and the
    gradients are those the library gives after the full forward pass."""
    rng = np.random.default_rng(4100 + sum(dims) + B + bad_ids)
    n = 1400 + dims[0]
    r, c = graph_with_hub_and_empty_rows(rng, n, 3500, 700)
    say("training forward dims=%s B=%d n=%d" % (dims, B, n))
    ref = O.build_csr(n, r, c, True)
    g = lp.lp_build_csr(n, dev_i32(r), dev_i32(c), True)
    Ws, Wn, b = toy_model(rng, dims, scale=0.25)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    es = rng.integers(0, n, B).astype(np.int32)
    ed = rng.integers(0, n, B).astype(np.int32)
    es[0] = 3                                            # the 700-entry row
    if bad_ids:
        es[5], ed[7] = -1, n
    n_pos = max(1, B // 3)
    model, Xd = make_model(Ws, Wn, b), dev_f32(X)
    K = len(dims) - 1
    from gpu_util import nan_filled_acts
    acts = nan_filled_acts(n, model, Xd)
    lp.lp_sage_forward_edges(g, model, Xd, dev_i32(es), dev_i32(ed), acts)
    a_ref = O.sage_forward(ref, Ws, Wn, b, X)
    ends = check_last_layer_listed(acts, a_ref, es, ed, K)
    assert ends.size <= 2 * B
    # what follows reads only rows that were written
    s, loss, ds = lp.lp_score_loss(acts.H[-1], dev_i32(es), dev_i32(ed), n_pos)
    grads = lp.lp_backward(g, model, Xd, acts, dev_i32(es), dev_i32(ed), ds, want_dX=True)
    valid = (es >= 0) & (es < n) & (ed >= 0) & (ed < n)
    # the same step after the full forward pass: equal up to the order of the sums over hub rows
    full = lp.lp_sage_forward(g, model, Xd)
    s2, loss2, ds2 = lp.lp_score_loss(full.H[-1], dev_i32(es), dev_i32(ed), n_pos)
    assert_close(host(s), host(s2), 1e-6, "scores after either forward pass")
    assert abs(float(host(loss)[0]) - float(host(loss2)[0])) <= 1e-6 * abs(float(host(loss2)[0]))
    g2 = lp.lp_backward(g, model, Xd, full, dev_i32(es), dev_i32(ed), ds2, want_dX=True)
    for k in range(K):
        assert_close(host(grads.dW_self[k]), host(g2.dW_self[k]), 1e-5, "dW_self^%d after either forward pass" % (k + 1))
        assert_close(host(grads.dW_neigh[k]), host(g2.dW_neigh[k]), 1e-5, "dW_neigh^%d after either forward pass" % (k + 1))
        assert_close(host(grads.dbias[k]), host(g2.dbias[k]), 1e-5, "dbias^%d after either forward pass" % (k + 1))
    assert_close(host(grads.dX), host(g2.dX), 1e-5, "dX after either forward pass")
    if bad_ids:
        assert not valid.all()
    else:
        s_ref, loss_ref, ds_ref = O.score_loss(a_ref.H[-1], es, ed, n_pos)
        assert_close(host(s), s_ref, TOL_ACT, "scores")
        assert abs(float(host(loss)[0]) - loss_ref) <= TOL_ACT * abs(loss_ref)
        # a batch this small hangs every gradient on a few thousand hidden units, so a single unit whose gate the two
        # sides decide differently (|z| below 1e-6) moves a weight gradient by more than the bar: the oracle's backward
        # pass takes the kernel's decision at such units
        gated, flips = oracle_acts_with_the_kernel_gates(a_ref, hidden_of(acts, K), K)
        say("  %d hidden unit(s) take the kernel's gate decision in the oracle's backward pass" % flips)
        g_ref = O.backward(ref, Ws, Wn, gated, es, ed, ds_ref)
        check_grads(grads, g_ref, K)


def test_training_forward_with_an_empty_batch_and_around_the_largest_listed_batch():
    say("training forward B=0 / B around 3n/8")
    rng = np.random.default_rng(4242)
    n, dims = 900, [16, 32, 8]
    r, c = random_pairs(rng, n, 3000)
    ref = O.build_csr(n, r, c, True)
    g = lp.lp_build_csr(n, dev_i32(r), dev_i32(c), True)
    Ws, Wn, b = toy_model(rng, dims)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    model, Xd = make_model(Ws, Wn, b), dev_f32(X)
    a_ref = O.sage_forward(ref, Ws, Wn, b, X)
    from gpu_util import nan_filled_acts
    z = dev_i32(np.zeros(0, np.int32))
    acts = nan_filled_acts(n, model, Xd)
    lp.lp_sage_forward_edges(g, model, Xd, z, z, acts)
    check_last_layer_listed(acts, a_ref, np.zeros(0, np.int32), np.zeros(0, np.int32), 2)
    # a batch whose every edge carries an id outside the graph lists nothing: the last layer stays untouched
    bad = np.full(50, n, np.int32)
    acts = nan_filled_acts(n, model, Xd)
    lp.lp_sage_forward_edges(g, model, Xd, dev_i32(bad), dev_i32(-bad), acts)
    check_last_layer_listed(acts, a_ref, bad, -bad, 2)
    assert np.isnan(host(acts.H[-1])).all() and np.isnan(host(acts.A[-1])).all()
    every = np.arange(n, dtype=np.int32)
    Bmax = (3 * n - 1) // 8                              # the longest list: 2 Bmax distinct end points
    acts = nan_filled_acts(n, model, Xd)
    lp.lp_sage_forward_edges(g, model, Xd, dev_i32(every[:Bmax]), dev_i32(every[n - Bmax:]), acts)
    assert check_last_layer_listed(acts, a_ref, every[:Bmax], every[n - Bmax:], 2).size == 2 * Bmax
    acts = nan_filled_acts(n, model, Xd)                 # one edge more: every node is evaluated
    lp.lp_sage_forward_edges(g, model, Xd, dev_i32(every[:Bmax + 1]), dev_i32(every[n - Bmax - 1:]), acts)
    check_last_layer_listed(acts, a_ref, every[:Bmax + 1], every[n - Bmax - 1:], 2)
    assert not np.isnan(host(acts.H[-1])).any()
    # a GCN model takes the same path (no self term to gather)
    gl = O.build_csr(n, np.concatenate([r, every]), np.concatenate([c, every]), True)
    gg = lp.lp_build_csr(n, dev_i32(np.concatenate([r, every])), dev_i32(np.concatenate([c, every])), True)
    gm = lp.Model(None, [dev_f32(w) for w in Wn], [dev_f32(x) for x in b], layer_type=lp.LP_LAYER_GCN)
    es, ed = rng.integers(0, n, 200).astype(np.int32), rng.integers(0, n, 200).astype(np.int32)
    acts = nan_filled_acts(n, gm, Xd)
    lp.lp_sage_forward_edges(gg, gm, Xd, dev_i32(es), dev_i32(ed), acts)
    full = lp.lp_sage_forward(gg, gm, Xd)
    ends = torch.from_numpy(np.unique(np.concatenate([es, ed])).astype(np.int64)).to(DEV)
    assert_close(host(acts.H[-1][ends]), host(full.H[-1][ends]), 1e-6, "GCN H^K at the end points")
    assert int(torch.isnan(acts.H[-1]).any(dim=1).sum()) == n - ends.numel()


# ------------------------------------------------------------------------------------------------ whole step
def whole_step(name):
    run_whole_step(make_workload(name))


BOTH_PRODUCT_MODES = (lp.LP_FP32_PRODUCTS_BF16X6, lp.LP_FP32_PRODUCTS_NATIVE)


def run_whole_step(wl, modes=(lp.LP_FP32_PRODUCTS_BF16X6,)):
    """One step against the oracle, once per way of forming the fp32 products; returns, per mode, the 2-norm relative
    errors of the embeddings and of the first layer's weight gradient (the two ends of the chain of products)."""
    say("whole step %s N=%d nnz~%d B=%d" % (wl.name, wl.n_nodes, 2 * wl.src.size, wl.batch_edges))
    ref = O.build_csr(wl.n_nodes, wl.src, wl.dst, True)
    exp = O.train_step(ref, wl.W_self, wl.W_neigh, wl.bias, wl.X, wl.pos_src, wl.pos_dst, wl.k_neg, wl.n_space,
                       wl.sampler_seed, wl.sampler_step)
    g = lp.lp_build_csr(wl.n_nodes, dev_i32(wl.src), dev_i32(wl.dst), True)
    check_csr(g, ref)
    K = len(wl.dims) - 1
    errs = {}
    for mode in modes:
        say("  fp32 products mode %d" % mode)
        model, Xd = make_model(wl.W_self, wl.W_neigh, wl.bias, mode), dev_f32(wl.X)
        # the step as the benchmark runs it: the training forward (last layer at the end points of the batch only)
        got = HipStep(g, model, Xd, dev_i32(wl.pos_src), dev_i32(wl.pos_dst), wl.k_neg, wl.n_space, wl.sampler_seed,
                      wl.sampler_step, forward="edges")
        assert np.array_equal(host(got.e_src), exp.e_src) and np.array_equal(host(got.e_dst), exp.e_dst)
        check_last_layer_listed(got.acts, exp.acts, exp.e_src, exp.e_dst, K)
        assert_close(host(got.scores), exp.scores, TOL_ACT, "scores")
        assert abs(float(host(got.loss)[0]) - exp.loss) <= TOL_ACT * abs(exp.loss)
        assert_close(host(got.dscore), exp.dscore, TOL_ACT, "dscore")
        check_grads(got.grads, exp.grads, K, dx_band(ref, wl.W_self, wl.W_neigh, exp.acts, exp.e_src, exp.e_dst, exp.dscore,
                                                     hidden_of(got.acts, K)))
        # the embeddings of every node (evaluation, inference): the full forward pass
        full = lp.lp_sage_forward(g, model, Xd)
        for k in range(1, K + 1):
            assert_close(host(full.A[k - 1]), exp.acts.A[k], TOL_ACT, "A^%d" % k)
            assert_close(host(full.H[k - 1]), exp.acts.H[k], TOL_ACT, "H^%d" % k)
        errs[mode] = (rel_err(host(full.H[-1]), exp.acts.H[K])[1], rel_err(host(got.grads.dW_neigh[0]), exp.grads.dW_neigh[0])[1])
    return errs


def test_whole_step_C1():
    whole_step("C1")


def test_whole_step_C2_full_size():
    """Both ways of forming the fp32 products meet the bar at full size, and the products taken from bfloat16 terms
    are as close to the fp64 oracle as those of the fp32 matrix instructions (embeddings; the weight gradients go
    through ReLU gates whose flips dominate either error)."""
    errs = run_whole_step(make_workload("C2"), BOTH_PRODUCT_MODES)
    say("  2-norm relative errors (H^K, dW_neigh^1): split %s native %s" % (errs[lp.LP_FP32_PRODUCTS_BF16X6], errs[lp.LP_FP32_PRODUCTS_NATIVE]))
    assert errs[lp.LP_FP32_PRODUCTS_BF16X6][0] <= 1.5 * errs[lp.LP_FP32_PRODUCTS_NATIVE][0] + 1e-7
