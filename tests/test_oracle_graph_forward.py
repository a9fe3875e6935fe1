"""Pins for the oracle's graph construction and forward pass.

None of these re-use the oracle's own formulas: they compare against dense
0/1 adjacency matrices built entry by entry, closed forms on named graphs, and
invariants that hold for any correct mean aggregation.
"""
import numpy as np
import pytest

from oracle import lp_oracle as O


def dense_adj(n, rows, cols, symmetrize):
    A = np.zeros((n, n))
    for r, c in zip(rows, cols):
        A[r, c] = 1.0
        if symmetrize:
            A[c, r] = 1.0
    return A


def csr_to_dense(n, rowptr, colidx):
    A = np.zeros((n, n))
    for v in range(n):
        for p in range(rowptr[v], rowptr[v + 1]):
            A[v, colidx[p]] += 1.0
    return A


def random_pairs(rng, n, e):
    return rng.integers(0, n, e).astype(np.int32), rng.integers(0, n, e).astype(np.int32)


# ---------------------------------------------------------------- CSR
@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("sym", [False, True])
def test_csr_equals_dense_bruteforce(seed, sym):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 64))
    r, c = random_pairs(rng, n, int(rng.integers(0, 300)))   # has duplicates and self-loops
    g = O.build_csr(n, r, c, sym)
    A = dense_adj(n, r, c, sym)
    assert np.array_equal(csr_to_dense(n, g.rowptr, g.colidx), A)        # a set: entries are 0/1
    assert np.array_equal(csr_to_dense(n, g.t_rowptr, g.t_colidx), A.T)
    # canonical form
    assert g.rowptr[0] == 0 and g.rowptr[-1] == g.colidx.size == int(A.sum())
    assert np.all(np.diff(g.rowptr) >= 0)
    for v in range(n):
        row = g.colidx[g.rowptr[v]:g.rowptr[v + 1]]
        assert np.all(np.diff(row) > 0)
    deg = A.sum(1)
    expect = np.where(deg > 0, 1.0 / np.maximum(deg, 1), 0.0).astype(np.float32)
    assert np.array_equal(g.inv_deg, expect)
    assert g.inv_deg.dtype == np.float32 and g.rowptr.dtype == np.int32 and g.colidx.dtype == np.int32


def test_csr_symmetric_input_equals_its_transpose_and_transpose_is_involution():
    rng = np.random.default_rng(3)
    r, c = random_pairs(rng, 40, 200)
    g = O.build_csr(40, r, c, True)
    assert np.array_equal(g.rowptr, g.t_rowptr) and np.array_equal(g.colidx, g.t_colidx)
    d = O.build_csr(40, r, c, False)
    rows_t = np.repeat(np.arange(40), np.diff(d.t_rowptr))
    back = O.build_csr(40, d.t_colidx, rows_t, False)      # transpose of the transpose, as pairs
    assert np.array_equal(back.rowptr, d.rowptr) and np.array_equal(back.colidx, d.colidx)
    assert np.array_equal(back.t_rowptr, d.t_rowptr) and np.array_equal(back.t_colidx, d.t_colidx)


def test_csr_empty_and_out_of_range():
    g = O.build_csr(5, np.zeros(0, np.int32), np.zeros(0, np.int32), True)
    assert g.nnz == 0 and np.array_equal(g.rowptr, np.zeros(6, np.int32)) and np.all(g.inv_deg == 0)
    with pytest.raises(ValueError):
        O.build_csr(5, np.array([5]), np.array([0]), False)
    with pytest.raises(ValueError):
        O.build_csr(5, np.array([0]), np.array([-1]), False)


# ---------------------------------------------------------------- aggregation
@pytest.mark.parametrize("seed", range(4))
def test_mean_aggregate_equals_dense_rownormalised_matmul(seed):
    rng = np.random.default_rng(10 + seed)
    n, f = 37, 5
    r, c = random_pairs(rng, n, 90)
    g = O.build_csr(n, r, c, seed % 2 == 0)
    A = dense_adj(n, r, c, seed % 2 == 0)
    deg = A.sum(1, keepdims=True)
    M = np.divide(A, deg, out=np.zeros_like(A), where=deg > 0)
    H = rng.standard_normal((n, f))
    np.testing.assert_allclose(O.mean_aggregate(g, H), M @ H, rtol=1e-13, atol=1e-13)
    rows = [5, 0, 36, 5]
    np.testing.assert_allclose(O.mean_aggregate(g, H, rows), (M @ H)[rows], rtol=1e-13, atol=1e-13)
    # adjoint is the transposed matrix
    T = rng.standard_normal((n, f))
    np.testing.assert_allclose(O.mean_aggregate_adjoint(g, T), M.T @ T, rtol=1e-13, atol=1e-13)


def test_mean_aggregate_constant_and_isolated():
    # path 0-1-2 plus isolated node 3
    g = O.build_csr(4, np.array([0, 1]), np.array([1, 2]), True)
    H = np.full((4, 3), 7.25)
    out = O.mean_aggregate(g, H)
    assert np.array_equal(out[:3], H[:3]) and np.array_equal(out[3], np.zeros(3))
    # values by hand: row 1 averages nodes 0 and 2
    H = np.array([[1.0], [10.0], [5.0], [100.0]])
    assert np.array_equal(O.mean_aggregate(g, H), np.array([[10.0], [3.0], [10.0], [0.0]]))


def test_mean_aggregate_complete_graph_and_star_closed_forms():
    n, f = 9, 4
    rng = np.random.default_rng(0)
    H = rng.standard_normal((n, f))
    iu = np.triu_indices(n, 1)
    g = O.build_csr(n, iu[0], iu[1], True)
    np.testing.assert_allclose(O.mean_aggregate(g, H), (H.sum(0) - H) / (n - 1), rtol=1e-13)
    # star with centre 0: centre gets the mean of the leaves, each leaf gets the centre
    g = O.build_csr(n, np.zeros(n - 1, np.int64), np.arange(1, n), True)
    out = O.mean_aggregate(g, H)
    np.testing.assert_allclose(out[0], H[1:].mean(0), rtol=1e-13)
    assert np.array_equal(out[1:], np.repeat(H[:1], n - 1, 0))


def test_mean_aggregate_directed_rows_aggregate_from_their_columns():
    # a single directed pair (0 -> 1): row 0 lists node 1, so node 0 reads h_1; node 1 reads nothing
    g = O.build_csr(2, np.array([0]), np.array([1]), False)
    H = np.array([[2.0], [3.0]])
    assert np.array_equal(O.mean_aggregate(g, H), np.array([[3.0], [0.0]]))
    assert np.array_equal(O.mean_aggregate_adjoint(g, H), np.array([[0.0], [2.0]]))


def test_relabelling_equivariance():
    rng = np.random.default_rng(5)
    n, f = 30, 6
    r, c = random_pairs(rng, n, 80)
    perm = rng.permutation(n)
    H = rng.standard_normal((n, f))
    g = O.build_csr(n, r, c, True)
    gp = O.build_csr(n, perm[r], perm[c], True)
    Hp = np.empty_like(H)
    Hp[perm] = H
    np.testing.assert_allclose(O.mean_aggregate(gp, Hp)[perm], O.mean_aggregate(g, H), rtol=1e-13, atol=1e-15)


# ---------------------------------------------------------------- layers
def _toy_model(rng, dims):
    Ws = [rng.standard_normal((dims[k], dims[k + 1])) for k in range(len(dims) - 1)]
    Wn = [rng.standard_normal((dims[k], dims[k + 1])) for k in range(len(dims) - 1)]
    b = [rng.standard_normal(dims[k + 1]) for k in range(len(dims) - 1)]
    return Ws, Wn, b


def test_forward_without_edges_or_with_zero_neighbour_weights_is_an_mlp():
    rng = np.random.default_rng(1)
    dims = [5, 7, 6, 3]
    Ws, Wn, b = _toy_model(rng, dims)
    X = rng.standard_normal((12, 5))
    mlp = X
    for k in range(3):
        mlp = mlp @ Ws[k] + b[k]
        if k < 2:
            mlp = np.maximum(mlp, 0)
    edgeless = O.build_csr(12, np.zeros(0, np.int32), np.zeros(0, np.int32), True)
    np.testing.assert_allclose(O.sage_forward(edgeless, Ws, Wn, b, X).H[-1], mlp, rtol=1e-12)
    r, c = random_pairs(rng, 12, 30)
    g = O.build_csr(12, r, c, True)
    zero = [np.zeros_like(w) for w in Wn]
    np.testing.assert_allclose(O.sage_forward(g, Ws, zero, b, X).H[-1], mlp, rtol=1e-12)


def test_forward_single_layer_identity_neighbour_weight_is_pure_mean_and_no_relu_on_last_layer():
    rng = np.random.default_rng(2)
    n, f = 15, 4
    r, c = random_pairs(rng, n, 40)
    g = O.build_csr(n, r, c, True)
    X = rng.standard_normal((n, f))
    acts = O.sage_forward(g, [np.zeros((f, f))], [np.eye(f)], [np.zeros(f)], X)
    np.testing.assert_array_equal(acts.H[1], O.mean_aggregate(g, X))
    assert (acts.H[1] < 0).any()             # the last layer is not rectified
    # two layers: the hidden layer is rectified
    acts = O.sage_forward(g, [np.eye(f), np.eye(f)], [np.zeros((f, f))] * 2, [np.zeros(f)] * 2, X)
    np.testing.assert_array_equal(acts.H[1], np.maximum(X, 0))
    np.testing.assert_array_equal(acts.H[2], np.maximum(X, 0))


def test_forward_matches_dense_formula_on_small_graph():
    rng = np.random.default_rng(4)
    n, dims = 20, [3, 5, 4]
    r, c = random_pairs(rng, n, 50)
    g = O.build_csr(n, r, c, False)
    A = dense_adj(n, r, c, False)
    deg = A.sum(1, keepdims=True)
    M = np.divide(A, deg, out=np.zeros_like(A), where=deg > 0)
    Ws, Wn, b = _toy_model(rng, dims)
    X = rng.standard_normal((n, 3))
    h1 = np.maximum(X @ Ws[0] + (M @ X) @ Wn[0] + b[0], 0)
    h2 = h1 @ Ws[1] + (M @ h1) @ Wn[1] + b[1]
    acts = O.sage_forward(g, Ws, Wn, b, X)
    np.testing.assert_allclose(acts.H[1], h1, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(acts.H[2], h2, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(acts.A[2], M @ h1, rtol=1e-12, atol=1e-13)


def test_bf16_storage_rounding_is_nearest_even():
    # 1 + 2^-8 is exactly halfway between bf16 neighbours 1 and 1 + 2^-7: ties go to even (1.0)
    a = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -3.140625])
    out = O._round_bf16(a)
    assert np.array_equal(out, np.array([1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -3.140625]))
