"""GPU parity at the larger benchmark shapes.

C3 (one worker's view of a partitioned 1 M-node graph, 3 negatives per positive): the whole step, element by
element.  C4 (2.9 M nodes, 29 M directed entries), the configuration the benchmark times: CSR and negatives
bit-exact in full, and the whole three-layer step against a full fp64 oracle step of the same size (every weight and
bias gradient of every layer, every score and loss-gradient scalar, the loss, and the rows of every A^k and H^k on
a sample of random, hub and empty rows), in both ways of forming the fp32 products; plus one-layer pieces whose
input gradient is checked on sampled rows.  C5 (bf16 storage, hidden 512, one worker's view of C4's graph, cross
edges kept w.p. 1.0, 0.5 and 0.2): for every setting the CSR bit-exact and the whole step against a full fp64 oracle
step, both at full size (the generator scaled to 1/8, with every element of every saved matrix compared, is in
test_gpu_parity_bf16.py).
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2506_20818_amd as lp
from lp_workloads import CONFIGS, init_features, make_workload
from oracle import lp_oracle as O
from gpu_util import DEV, HipStep, assert_close, dev_f32, dev_i32, host, make_model
from test_gpu_parity import TOL_ACT, TOL_GRAD, check_csr, check_grads, run_sampler, say, whole_step


def test_whole_step_C3_worker_view():
    whole_step("C3")


@pytest.fixture(scope="module")
def c4():
    wl = make_workload("C4", with_features=False)
    say("C4 graph: N=%d E=%d" % (wl.n_nodes, wl.src.size))
    ref = O.build_csr(wl.n_nodes, wl.src, wl.dst, True)
    g = lp.lp_build_csr(wl.n_nodes, dev_i32(wl.src), dev_i32(wl.dst), True)
    return wl, ref, g


def test_C4_csr_and_negatives_bit_exact(c4):
    wl, ref, g = c4
    say("C4 csr + sampler")
    check_csr(g, ref)
    run_sampler(ref, g, wl.pos_src, wl.k_neg, wl.n_space, wl.sampler_seed, wl.sampler_step)


def sample_rows(ref, rng, n_random=1500, n_hubs=20):
    deg = np.diff(ref.rowptr)
    hubs = np.argsort(deg)[-n_hubs:]
    empty = np.flatnonzero(deg == 0)[:20]
    return np.unique(np.concatenate([rng.integers(0, ref.n_nodes, n_random), hubs, empty]))


def oracle_step_in_stages(ref, Ws, Wn, bias, X, wl, storage="f32"):
    """O.train_step written out call by call, so that a long run names the stage it is in."""
    say("  oracle: negatives")
    neg, _ = O.sample_neg(ref, wl.pos_src, wl.k_neg, wl.n_space, wl.sampler_seed, wl.sampler_step)
    es, ed = O.batch_edges(wl.pos_src, wl.pos_dst, neg, wl.k_neg)
    say("  oracle: forward (fp64, %d nodes)" % ref.n_nodes)
    acts = O.sage_forward(ref, Ws, Wn, bias, X, storage)
    s, loss, ds = O.score_loss(acts.H[-1], es, ed, wl.pos_src.size)
    say("  oracle: backward")
    grads = O.backward(ref, Ws, Wn, acts, es, ed, ds, storage=storage)
    say("  oracle: done")
    return O.StepResult(neg, es, ed, acts, s, loss, ds, grads)


def check_sampled_rows_of_a_training_step(got, exp, ref, rows, K, tol, to_host):
    """A step whose forward pass was lp_sage_forward_edges into NaN-filled matrices: layers below K on the sampled
    rows; layer K on a sample of the end points of the batch (hubs among them).  With 8 B < 3 n every row of a node that
    is no end point is still NaN; a larger batch has every row evaluated (checked on the sampled rows)."""
    ridx = torch.from_numpy(rows).to(DEV)
    for k in range(1, K):
        assert_close(to_host(got.acts.A[k - 1][ridx]), exp.acts.A[k][rows], tol, "A^%d rows" % k)
        assert_close(to_host(got.acts.H[k - 1][ridx]), exp.acts.H[k][rows], tol, "H^%d rows" % k)
    ends = np.unique(np.concatenate([exp.e_src, exp.e_dst])).astype(np.int64)
    deg = np.diff(ref.rowptr)
    pick = np.unique(np.concatenate([np.random.default_rng(7).choice(ends, min(3000, ends.size), replace=False),
                                     ends[np.argsort(deg[ends])[-40:]]]))
    pidx = torch.from_numpy(pick).to(DEV)
    assert_close(to_host(got.acts.A[K - 1][pidx]), exp.acts.A[K][pick], tol, "A^K at end points")
    assert_close(to_host(got.acts.H[K - 1][pidx]), exp.acts.H[K][pick], tol, "H^K at end points")
    listed = 8 * exp.e_src.size < 3 * ref.n_nodes
    say("  last layer of the training forward: %s, %d end points of %d nodes" % ("listed rows" if listed else "every row", ends.size, ref.n_nodes))
    is_end = torch.zeros(ref.n_nodes, dtype=torch.bool, device=DEV)
    is_end[torch.from_numpy(ends).to(DEV)] = True
    for t in (got.acts.A[K - 1], got.acts.H[K - 1]):
        nan_rows = torch.isnan(t).any(dim=1)
        if listed:
            assert bool((nan_rows == ~is_end).all()), "rows written by the training forward are not exactly the end points"
        else:
            assert not bool(nan_rows.any())
    if not listed:
        assert_close(to_host(got.acts.A[K - 1][ridx]), exp.acts.A[K][rows], tol, "A^K rows")
        assert_close(to_host(got.acts.H[K - 1][ridx]), exp.acts.H[K][rows], tol, "H^K rows")


@pytest.mark.timeout(900)
def test_whole_step_C4_full_size(c4):
    """The configuration the benchmark times, all three layers, at full size and in the launch configuration of the
    benchmark (same entry points, same workspaces, no dX): this is where the gated transposed aggregation over 2.9 M
    rows with 15 000-entry hub columns, the fused weight gradients with 2.9 M reduction rows and their fold, and
    the rotation of the backward buffers across layers are checked."""
    wl, ref, g = c4
    say("C4 whole step, full size: N=%d nnz=%d B=%d dims=%s" % (wl.n_nodes, ref.nnz, wl.batch_edges, wl.dims))
    X = init_features(wl.n_nodes, wl.dims[0], CONFIGS["C4"]["seeds"]["x"])
    exp = oracle_step_in_stages(ref, wl.W_self, wl.W_neigh, wl.bias, X, wl)
    K = len(wl.dims) - 1
    rng = np.random.default_rng(404)
    rows = sample_rows(ref, rng, n_random=3000, n_hubs=40)
    ridx = torch.from_numpy(rows).to(DEV)
    Xd = dev_f32(X)
    for mode in (lp.LP_FP32_PRODUCTS_BF16X6, lp.LP_FP32_PRODUCTS_NATIVE):
        say("  fp32 products mode %d" % mode)
        model = make_model(wl.W_self, wl.W_neigh, wl.bias, mode)
        got = HipStep(g, model, Xd, dev_i32(wl.pos_src), dev_i32(wl.pos_dst), wl.k_neg, wl.n_space, wl.sampler_seed,
                      wl.sampler_step, want_dX=False, forward="edges")
        assert np.array_equal(host(got.e_src), exp.e_src) and np.array_equal(host(got.e_dst), exp.e_dst)
        check_sampled_rows_of_a_training_step(got, exp, ref, rows, K, TOL_ACT, host)
        assert_close(host(got.scores), exp.scores, TOL_ACT, "scores")
        assert abs(float(host(got.loss)[0]) - exp.loss) <= TOL_ACT * abs(exp.loss)
        assert_close(host(got.dscore), exp.dscore, TOL_ACT, "dscore")
        check_grads(got.grads, exp.grads, K)
        say("  the full forward pass, last layer on the sampled rows")
        lp.lp_sage_forward(g, model, Xd, got.acts)
        assert_close(host(got.acts.A[K - 1][ridx]), exp.acts.A[K][rows], TOL_ACT, "A^K rows (full pass)")
        assert_close(host(got.acts.H[K - 1][ridx]), exp.acts.H[K][rows], TOL_ACT, "H^K rows (full pass)")
        assert bool(torch.isfinite(got.acts.H[-1]).all())
        del got


@pytest.mark.parametrize("F", [128, 256])
def test_C4_forward_one_layer_sampled_rows(c4, F):
    wl, ref, g = c4
    say("C4 forward F=%d sampled rows" % F)
    rng = np.random.default_rng(40 + F)
    X = init_features(wl.n_nodes, F, 500 + F)
    Ws = (rng.standard_normal((F, 256)) / np.sqrt(2 * F)).astype(np.float32)
    Wn = (rng.standard_normal((F, 256)) / np.sqrt(2 * F)).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, 256).astype(np.float32)
    # two layers so that the first one is rectified: rows of A^1 and H^1 are checked
    W2 = np.zeros((256, 4), np.float32)
    acts = lp.lp_sage_forward(g, make_model([Ws, W2], [Wn, W2], [b, np.zeros(4, np.float32)]), dev_f32(X))
    rows = sample_rows(ref, rng)
    a_ref = O.mean_aggregate(ref, X, rows)
    h_ref = np.maximum(X[rows].astype(np.float64) @ Ws.astype(np.float64) + a_ref @ Wn.astype(np.float64) + b, 0.0)
    ridx = torch.from_numpy(rows).to(DEV)
    assert_close(host(acts.A[0][ridx]), a_ref, TOL_ACT, "A^1 rows")
    assert_close(host(acts.H[0][ridx]), h_ref, TOL_ACT, "H^1 rows")
    # invariants at full size: rows without neighbours aggregate to zero, everything is finite
    iso = torch.from_numpy(np.flatnonzero(np.diff(ref.rowptr) == 0)).to(DEV)
    assert float(acts.A[0][iso].abs().max()) == 0.0
    assert bool(torch.isfinite(acts.H[0]).all())


def test_C4_score_and_one_layer_backward(c4):
    wl, ref, g = c4
    say("C4 score + backward, one layer 256->256")
    rng = np.random.default_rng(77)
    F = 256
    N = wl.n_nodes
    X = init_features(N, F, 901)
    Ws = (rng.standard_normal((F, F)) / np.sqrt(2 * F) * F ** -0.25).astype(np.float32)
    Wn = (rng.standard_normal((F, F)) / np.sqrt(2 * F) * F ** -0.25).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, F).astype(np.float32)
    neg, _ = O.sample_neg(ref, wl.pos_src, wl.k_neg, wl.n_space, wl.sampler_seed, wl.sampler_step)
    es, ed = O.batch_edges(wl.pos_src, wl.pos_dst, neg, wl.k_neg)
    model = make_model([Ws], [Wn], [b])
    Xd = dev_f32(X)
    acts = lp.lp_sage_forward(g, model, Xd)
    s, loss, ds = lp.lp_score_loss(acts.H[-1], dev_i32(es), dev_i32(ed), wl.n_pos)
    grads = lp.lp_backward(g, model, Xd, acts, dev_i32(es), dev_i32(ed), ds, want_dX=True)

    # oracle on the rows the batch touches (dL/dH is zero elsewhere)
    touched = np.unique(np.concatenate([es, ed]))
    pos_of = np.full(N, -1, np.int64)
    pos_of[touched] = np.arange(touched.size)
    a_t = O.mean_aggregate(ref, X, touched)
    x_t = X[touched].astype(np.float64)
    h_t = x_t @ Ws.astype(np.float64) + a_t @ Wn.astype(np.float64) + b          # single layer: not rectified
    s_ref, loss_ref, ds_ref = O.score_loss(h_t, pos_of[es], pos_of[ed], wl.n_pos)
    assert_close(host(s), s_ref, TOL_ACT, "scores")
    assert abs(float(host(loss)[0]) - loss_ref) <= TOL_ACT * abs(loss_ref)
    assert_close(host(ds), ds_ref, TOL_ACT, "dscore")
    dZ_t = O.edge_grad_scatter(h_t, pos_of[es], pos_of[ed], ds_ref)             # rows of dL/dZ, compact
    assert_close(host(grads.dbias[0]), dZ_t.sum(0), TOL_GRAD, "dbias")
    assert_close(host(grads.dW_self[0]), x_t.T @ dZ_t, TOL_GRAD, "dW_self")
    assert_close(host(grads.dW_neigh[0]), a_t.T @ dZ_t, TOL_GRAD, "dW_neigh")
    # dX on sampled rows: dZ[u] W_self^T + sum over v with u in N(v) of dZ[v] W_neigh^T / |N(v)|
    rows = sample_rows(ref, rng, n_random=400, n_hubs=5)
    deg = np.diff(ref.rowptr).astype(np.float64)
    T_t = dZ_t @ Wn.astype(np.float64).T
    dX_ref = np.zeros((rows.size, F))
    for i, u in enumerate(rows):
        if pos_of[u] >= 0:
            dX_ref[i] = dZ_t[pos_of[u]] @ Ws.astype(np.float64).T
        vs = ref.t_colidx[ref.t_rowptr[u]:ref.t_rowptr[u + 1]]
        vs = vs[pos_of[vs] >= 0]
        if vs.size:
            dX_ref[i] += (T_t[pos_of[vs]] / deg[vs, None]).sum(0)
    assert_close(host(grads.dX[torch.from_numpy(rows).to(DEV)]), dX_ref, TOL_GRAD, "dX rows")


def whole_step_bf16_sampled_rows(wl, ref, g):
    """A bf16 whole step against the oracle (bf16 bars: 2^-7 on activations, scores and loss, 2e-2 on gradients):
    every gradient, score and the loss; A^k and H^k on sampled, hub and empty rows."""
    from lp_workloads import to_bf16_grid
    from test_gpu_parity_bf16 import TOL_ACT as BF_ACT, bf16_model, check_grads as bf_check_grads, dev_bf16, hostf
    Ws, Wn = [to_bf16_grid(w) for w in wl.W_self], [to_bf16_grid(w) for w in wl.W_neigh]
    X = to_bf16_grid(wl.X)
    exp = oracle_step_in_stages(ref, Ws, Wn, wl.bias, X, wl, storage="bf16")
    K = len(wl.dims) - 1
    model, Xd = bf16_model(Ws, Wn, wl.bias), dev_bf16(X)
    got = HipStep(g, model, Xd, dev_i32(wl.pos_src), dev_i32(wl.pos_dst), wl.k_neg, wl.n_space, wl.sampler_seed,
                  wl.sampler_step, want_dX=False, forward="edges")
    assert np.array_equal(host(got.e_src), exp.e_src) and np.array_equal(host(got.e_dst), exp.e_dst)
    rows = sample_rows(ref, np.random.default_rng(505), n_random=3000, n_hubs=40)
    ridx = torch.from_numpy(rows).to(DEV)
    check_sampled_rows_of_a_training_step(got, exp, ref, rows, K, BF_ACT, hostf)
    assert_close(host(got.scores), exp.scores, BF_ACT, "scores")
    assert abs(float(host(got.loss)[0]) - exp.loss) <= BF_ACT * abs(exp.loss)
    bf_check_grads(got.grads, exp.grads, K)
    say("  the full forward pass, last layer on the sampled rows")
    lp.lp_sage_forward(g, model, Xd, got.acts)
    assert_close(hostf(got.acts.A[K - 1][ridx]), exp.acts.A[K][rows], BF_ACT, "A^K rows (full pass)")
    assert_close(hostf(got.acts.H[K - 1][ridx]), exp.acts.H[K][rows], BF_ACT, "H^K rows (full pass)")
    assert bool(torch.isfinite(got.acts.H[-1].float()).all())
    if ref.n_nodes < 600000:    # (one more fp64 backward pass: left out at full size)
        from test_gpu_parity_bf16 import check_grads_against_unrounded_backward
        check_grads_against_unrounded_backward(got.grads, O.backward(ref, Ws, Wn, exp.acts, exp.e_src, exp.e_dst, exp.dscore, storage="f32"), K)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("keep,scale", [("1", 1.0), ("0.5", 1.0), ("0.2", 1.0)])
def test_whole_step_C5_bf16(keep, scale):
    """One worker's share of C4's graph under a 4-way partition, cross edges kept w.p. `keep`, bf16 storage, hidden
    512, four negatives per positive.  CSR bit-exact at full size; the whole step at `scale` (1.0 = full size)."""
    name = "C5_keep" + keep
    full = make_workload(name, with_features=False)
    say("%s: N=%d E=%d, CSR at full size" % (name, full.n_nodes, full.src.size))
    ref = O.build_csr(full.n_nodes, full.src, full.dst, True)
    g = lp.lp_build_csr(full.n_nodes, dev_i32(full.src), dev_i32(full.dst), True)
    check_csr(g, ref)
    if scale == 1.0:
        wl = full
        wl.X = init_features(wl.n_nodes, wl.dims[0], CONFIGS[name]["seeds"]["x"])
    else:
        del ref, g
        wl = make_workload(name, scale=scale)
        ref = O.build_csr(wl.n_nodes, wl.src, wl.dst, True)
        g = lp.lp_build_csr(wl.n_nodes, dev_i32(wl.src), dev_i32(wl.dst), True)
    say("%s whole step at scale %g: N=%d nnz=%d B=%d dims=%s max degree %d" % (
        name, scale, wl.n_nodes, ref.nnz, wl.batch_edges, wl.dims, int(np.diff(ref.rowptr).max())))
    whole_step_bf16_sampled_rows(wl, ref, g)


@pytest.mark.parametrize("storage,n", [("f32", 40000), ("bf16", 40000)])
def test_hidden_512_persistent_tiles(storage, n):
    """Hidden width 512 on 40 000 nodes (enough 128-row tiles for one persistent workgroup per CU): layer transforms
    with two column tiles and the input-gradient transform of layer 2 with two outputs of 512 columns, with fp32
    products from bfloat16 terms and with bf16 storage; forward and backward against the oracle on every element."""
    from test_gpu_parity import check_grads, dx_band, hidden_of, random_pairs, toy_model
    rng = np.random.default_rng(4242)
    dims = [64, 512, 512]
    r, c = random_pairs(rng, n, 120000)
    say("hidden 512 %s: n=%d dims=%s" % (storage, n, dims))
    ref = O.build_csr(n, r, c, True)
    g = lp.lp_build_csr(n, dev_i32(r), dev_i32(c), True)
    Ws, Wn, b = toy_model(rng, dims, scale=0.25)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    B, n_pos = 6000, 2500
    es, ed = rng.integers(0, n, B).astype(np.int32), rng.integers(0, n, B).astype(np.int32)
    if storage == "bf16":
        from lp_workloads import to_bf16_grid
        from test_gpu_parity_bf16 import TOL_ACT as BF_ACT, bf16_model, check_grads as bf_check_grads, dev_bf16, hostf
        Ws, Wn, X = [to_bf16_grid(w) for w in Ws], [to_bf16_grid(w) for w in Wn], to_bf16_grid(X)
        model, Xd = bf16_model(Ws, Wn, b), dev_bf16(X)
        acts = lp.lp_sage_forward(g, model, Xd)
        s, loss, ds = lp.lp_score_loss(acts.H[-1], dev_i32(es), dev_i32(ed), n_pos)
        grads = lp.lp_backward(g, model, Xd, acts, dev_i32(es), dev_i32(ed), ds, want_dX=True)
        a_ref = O.sage_forward(ref, Ws, Wn, b, X, storage="bf16")
        s_ref, loss_ref, ds_ref = O.score_loss(a_ref.H[-1], es, ed, n_pos)
        g_ref = O.backward(ref, Ws, Wn, a_ref, es, ed, ds_ref, storage="bf16")
        for k in (1, 2):
            assert_close(hostf(acts.H[k - 1]), a_ref.H[k], BF_ACT, "H^%d" % k)
        assert_close(host(s), s_ref, BF_ACT, "scores")
        bf_check_grads(grads, g_ref, 2, dx_band(ref, Ws, Wn, a_ref, es, ed, ds_ref, hidden_of(acts, 2, hostf), storage="bf16"))
    else:
        model, Xd = make_model(Ws, Wn, b, lp.LP_FP32_PRODUCTS_BF16X6), dev_f32(X)
        acts = lp.lp_sage_forward(g, model, Xd)
        s, loss, ds = lp.lp_score_loss(acts.H[-1], dev_i32(es), dev_i32(ed), n_pos)
        grads = lp.lp_backward(g, model, Xd, acts, dev_i32(es), dev_i32(ed), ds, want_dX=True)
        a_ref = O.sage_forward(ref, Ws, Wn, b, X)
        s_ref, loss_ref, ds_ref = O.score_loss(a_ref.H[-1], es, ed, n_pos)
        g_ref = O.backward(ref, Ws, Wn, a_ref, es, ed, ds_ref)
        for k in (1, 2):
            assert_close(host(acts.H[k - 1]), a_ref.H[k], TOL_ACT, "H^%d" % k)
        assert_close(host(s), s_ref, TOL_ACT, "scores")
        check_grads(grads, g_ref, 2, dx_band(ref, Ws, Wn, a_ref, es, ed, ds_ref, hidden_of(acts, 2)))


@pytest.mark.parametrize("n,dims", [(65535, [48, 256]), (65537, [48, 256]), (65536 + 255, [64, 192, 320]), (131072 + 1, [32, 272])])
def test_row_counts_around_the_256_row_tile_switch(n, dims):
    """Node counts just below and above 256 rows x 256 compute units (where the persistent NT kernels change from
    128-row to 256-row tiles), K parts of 48, 64 and 192 values (3, 4 and 12 steps per part), output widths that
    leave the second column tile three quarters empty (320) or almost empty (272): forward and backward, every
    element against the oracle."""
    from test_gpu_parity import check_grads, dx_band, hidden_of, random_pairs, toy_model
    rng = np.random.default_rng(n + sum(dims))
    r, c = random_pairs(rng, n, 3 * n)
    say("tile switch: n=%d dims=%s" % (n, dims))
    ref = O.build_csr(n, r, c, True)
    g = lp.lp_build_csr(n, dev_i32(r), dev_i32(c), True)
    Ws, Wn, b = toy_model(rng, dims, scale=0.25)
    X = rng.standard_normal((n, dims[0])).astype(np.float32)
    B, n_pos = 5000, 2000
    es, ed = rng.integers(0, n, B).astype(np.int32), rng.integers(0, n, B).astype(np.int32)
    model, Xd = make_model(Ws, Wn, b), dev_f32(X)
    acts = lp.lp_sage_forward(g, model, Xd)
    s, loss, ds = lp.lp_score_loss(acts.H[-1], dev_i32(es), dev_i32(ed), n_pos)
    grads = lp.lp_backward(g, model, Xd, acts, dev_i32(es), dev_i32(ed), ds, want_dX=True)
    a_ref = O.sage_forward(ref, Ws, Wn, b, X)
    s_ref, loss_ref, ds_ref = O.score_loss(a_ref.H[-1], es, ed, n_pos)
    g_ref = O.backward(ref, Ws, Wn, a_ref, es, ed, ds_ref)
    K = len(dims) - 1
    for k in range(1, K + 1):
        assert_close(host(acts.H[k - 1]), a_ref.H[k], TOL_ACT, "H^%d" % k)
    assert_close(host(s), s_ref, TOL_ACT, "scores")
    check_grads(grads, g_ref, K, dx_band(ref, Ws, Wn, a_ref, es, ed, ds_ref, hidden_of(acts, K)))
