"""CPU oracle for one worker's GNN link-prediction training step.

TEST INFRASTRUCTURE ONLY.  This file is the plain, slow definition of what the
HIP library must compute.  It is imported by the tests, by the smoke check and
by the benchmark's cpu_baseline leg, and by nothing else; it shares no code
with the HIP path and never calls it.

All floating-point work is done in float64 from the given inputs; integer work
(CSR construction, negative sampling) is exact.  Every function follows the
paper's training step (Algorithm 1, "Distributed Model Training" part, the
per-worker body), with the concrete layer, scorer and loss chosen as follows,
since the paper keeps them generic:

* Eq. (1) is instantiated as the GraphSAGE layer with mean aggregator named in
  the paper's "Hyperparameters" paragraph:
      a_v = (1/|N(v)|) * sum_{u in N(v)} h_u      (0 when N(v) is empty)
      z_v = h_v W_self + a_v W_neigh + b
      h'_v = relu(z_v) between layers, z_v after the last layer.
* Eq. (2) is the dot product s_(u,v) = <h_u, h_v> (one of the two predictors the
  paper names).
* The loss is binary cross-entropy on sigmoid(s) with labels 1/0 and the batch
  mean L = (1/N) sum l(s, y), N = |P| + |N| (Sec. IV-B, last paragraph).
* Negatives follow the per-source uniform rule of Sec. II-B: the source is
  kept, the destination is uniform over the sample space among nodes that are
  neither the source nor one of its neighbours.

Parity pins for every function here live in tests/test_oracle_*.py.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

U32 = np.uint64(0xFFFFFFFF)


# ==========================================================================
# Graph: canonical CSR of the visible edge set (Sec. II-A: E is a set of pairs)
# ==========================================================================
@dataclass
class CSR:
    n_nodes: int
    rowptr: np.ndarray      # int32 [n_nodes+1]
    colidx: np.ndarray      # int32 [nnz], ascending and distinct inside each row
    t_rowptr: np.ndarray    # CSR of the reversed pairs
    t_colidx: np.ndarray
    inv_deg: np.ndarray     # float32 [n_nodes], 1/|N(v)|, 0 for empty rows

    @property
    def nnz(self) -> int:
        return int(self.colidx.size)


def _csr_of_pairs(n_nodes: int, r: np.ndarray, c: np.ndarray):
    """Rows of the pair set {(r_i, c_i)}: repeated pairs collapse (E is a set),
    pairs are ordered by (row, column), rowptr[v] counts pairs with row < v."""
    key = np.unique(r.astype(np.int64) * np.int64(n_nodes) + c.astype(np.int64))
    rows = key // n_nodes
    cols = key % n_nodes
    counts = np.bincount(rows, minlength=n_nodes)
    rowptr = np.zeros(n_nodes + 1, np.int64)
    rowptr[1:] = np.cumsum(counts)
    return rowptr.astype(np.int32), cols.astype(np.int32)


def build_csr(n_nodes: int, rows: np.ndarray, cols: np.ndarray, symmetrize: bool) -> CSR:
    """Row v of the result lists N(v), the nodes v aggregates from.  With
    ``symmetrize`` every input pair also counts reversed (undirected graphs,
    Sec. IV-A: "undirected, unweighted").  The transposed CSR lists, for node u,
    the rows v with u in N(v)."""
    rows = np.asarray(rows, np.int64)
    cols = np.asarray(cols, np.int64)
    if rows.size and (rows.min() < 0 or cols.min() < 0 or rows.max() >= n_nodes or cols.max() >= n_nodes):
        raise ValueError("node id out of range")
    if symmetrize:
        rows, cols = np.concatenate([rows, cols]), np.concatenate([cols, rows])
    rowptr, colidx = _csr_of_pairs(n_nodes, rows, cols)
    t_rowptr, t_colidx = _csr_of_pairs(n_nodes, cols, rows)
    deg = np.diff(rowptr.astype(np.int64))
    inv_deg = np.zeros(n_nodes, np.float32)
    nz = deg > 0
    inv_deg[nz] = (np.float32(1.0) / deg[nz].astype(np.float32)).astype(np.float32)
    return CSR(n_nodes, rowptr, colidx, t_rowptr, t_colidx, inv_deg)


# ==========================================================================
# Storage rounding (only the bf16 configuration rounds anything)
# ==========================================================================
def _round_bf16(a: np.ndarray) -> np.ndarray:
    f = np.ascontiguousarray(a, dtype=np.float32)     # fp64 -> fp32, nearest even
    bits = f.view(np.uint32).astype(np.uint64)
    bits = (bits + np.uint64(0x7FFF) + ((bits >> np.uint64(16)) & np.uint64(1))) & np.uint64(0xFFFF0000)
    return bits.astype(np.uint32).view(np.float32).reshape(f.shape).astype(np.float64)


def _store(a: np.ndarray, storage: str) -> np.ndarray:
    if storage == "f32":
        return a            # fp32 rounding of stored activations (6e-8) is far below every tolerance
    if storage == "bf16":
        return _round_bf16(a)
    raise ValueError(storage)


# ==========================================================================
# Forward: K layers of Eq. (1)
# ==========================================================================
def mean_aggregate(csr: CSR, H: np.ndarray, rows: Optional[Sequence[int]] = None) -> np.ndarray:
    """a_v = mean of h_u over u in N(v); zero vector for a node without
    neighbours.  With ``rows`` only those rows are computed (and returned in
    that order)."""
    H = np.asarray(H, np.float64)
    sel = range(csr.n_nodes) if rows is None else rows
    out = np.zeros((len(sel), H.shape[1]), np.float64)
    rp, ci = csr.rowptr, csr.colidx
    for i, v in enumerate(sel):
        lo, hi = rp[v], rp[v + 1]
        if hi > lo:
            out[i] = H[ci[lo:hi]].sum(axis=0) / float(hi - lo)
    return out


@dataclass
class Activations:
    H: List[np.ndarray]     # H[0] = X, H[k] for k = 1..K
    A: List[np.ndarray]     # A[0] = None, A[k] = aggregated H[k-1]
    Z: List[np.ndarray]     # Z[0] = None, Z[k] = pre-activation of layer k


def sage_forward(csr: CSR, W_self, W_neigh, bias, X, storage: str = "f32") -> Activations:
    K = len(W_self)
    H = [np.asarray(X, np.float64)]
    A: List[Optional[np.ndarray]] = [None]
    Z: List[Optional[np.ndarray]] = [None]
    for k in range(1, K + 1):
        a = _store(mean_aggregate(csr, H[k - 1]), storage)
        z = (H[k - 1] @ np.asarray(W_self[k - 1], np.float64)
             + a @ np.asarray(W_neigh[k - 1], np.float64)
             + np.asarray(bias[k - 1], np.float64))
        h = np.maximum(z, 0.0) if k < K else z
        A.append(a)
        Z.append(z)
        H.append(_store(h, storage))
    return Activations(H, A, Z)


# ==========================================================================
# Negative sampling: per-source uniform (Sec. II-B) with a counter-based RNG
# ==========================================================================
PHILOX_M0 = 0xD2511F53
PHILOX_M1 = 0xCD9E8D57
PHILOX_W0 = 0x9E3779B9
PHILOX_W1 = 0xBB67AE85
MAX_ATTEMPTS = 16


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11).  Works on
    Python ints or on numpy uint64 arrays holding 32-bit values; returns the
    four 32-bit output words."""
    m = 0xFFFFFFFF
    arr = isinstance(c0, np.ndarray)
    if arr:
        M0, M1, m = np.uint64(PHILOX_M0), np.uint64(PHILOX_M1), U32
        sh = np.uint64(32)
        k0 = np.uint64(k0)
        k1 = np.uint64(k1)
    else:
        M0, M1, sh = PHILOX_M0, PHILOX_M1, 32
    for rnd in range(10):
        if rnd:
            k0 = (k0 + (np.uint64(PHILOX_W0) if arr else PHILOX_W0)) & m
            k1 = (k1 + (np.uint64(PHILOX_W1) if arr else PHILOX_W1)) & m
        p0 = M0 * c0
        p1 = M1 * c2
        hi0, lo0 = p0 >> sh, p0 & m
        hi1, lo1 = p1 >> sh, p1 & m
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return c0, c1, c2, c3


def sample_neg(csr: CSR, pos_src: np.ndarray, k_neg: int, n_space: int, seed: int, step: int):
    """For positive i and j < k_neg, sample q = i*k_neg + j keeps the source
    u = pos_src[i] and draws a destination uniformly from [0, n_space) that is
    not u and not in N(u).

    Randomness: attempt t of sample q uses 32-bit word (t mod 4) of
    Philox4x32-10(counter = (q, t div 4, step_lo, step_hi), key = (seed_lo, seed_hi));
    the candidate is floor(word * n_space / 2^32).  The first valid candidate
    among attempts 0..15 wins.  If all sixteen are rejected, candidates
    c+1, c+2, ... (mod n_space) after the last one are tried in turn; if no node
    is valid at all the last candidate is returned and counted in ``n_failed``.

    Returns (neg_dst int32 [n_pos*k_neg], n_failed)."""
    pos_src = np.asarray(pos_src, np.int64)
    n_q = pos_src.size * k_neg
    N = csr.n_nodes
    span = np.int64(max(N, n_space))
    rows = np.repeat(np.arange(N, dtype=np.int64), np.diff(csr.rowptr.astype(np.int64)))
    edge_key = rows * span + csr.colidx.astype(np.int64)          # ascending by construction

    def is_edge(u, c):
        k = u * span + c
        pos = np.searchsorted(edge_key, k)
        pos = np.minimum(pos, max(edge_key.size - 1, 0))
        return (edge_key[pos] == k) if edge_key.size else np.zeros(k.shape, bool)

    q = np.arange(n_q, dtype=np.uint64)
    u = np.repeat(pos_src, k_neg)
    out = np.full(n_q, -1, np.int64)
    last = np.zeros(n_q, np.int64)
    todo = np.arange(n_q)
    s_lo, s_hi = seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF
    st_lo, st_hi = np.uint64(step & 0xFFFFFFFF), np.uint64((step >> 32) & 0xFFFFFFFF)
    for t in range(MAX_ATTEMPTS):
        if todo.size == 0:
            break
        qq = q[todo]
        words = philox4x32_10(qq, np.full(qq.shape, t >> 2, np.uint64),
                              np.full(qq.shape, st_lo), np.full(qq.shape, st_hi), s_lo, s_hi)
        r = words[t & 3]
        c = ((r * np.uint64(n_space)) >> np.uint64(32)).astype(np.int64)
        uu = u[todo]
        ok = (c != uu) & ~is_edge(uu, c)
        out[todo[ok]] = c[ok]
        last[todo[~ok]] = c[~ok]
        todo = todo[~ok]
    n_failed = 0
    for idx in todo:                      # rare: sixteen rejections in a row
        c, uu = int(last[idx]), int(u[idx])
        found = False
        for _ in range(n_space):
            c = (c + 1) % n_space
            if c != uu and not bool(is_edge(np.array([uu]), np.array([c]))[0]):
                found = True
                break
        if not found:
            c = int(last[idx])
            n_failed += 1
        out[idx] = c
    return out.astype(np.int32), n_failed


# ==========================================================================
# Scores and loss: Eq. (2) with the dot product, BCE, batch mean
# ==========================================================================
def score_loss(HK: np.ndarray, e_src: np.ndarray, e_dst: np.ndarray, n_pos_edges: int):
    """Edges 0..n_pos_edges-1 carry label 1, the rest label 0.
    Returns (scores [B], loss scalar, dscore [B] = dL/ds)."""
    HK = np.asarray(HK, np.float64)
    B = e_src.size
    s = np.einsum("ef,ef->e", HK[e_src], HK[e_dst]) if B else np.zeros(0)
    y = np.zeros(B)
    y[:n_pos_edges] = 1.0
    # -[y ln sigma(s) + (1-y) ln(1-sigma(s))], written so that exp never overflows
    ell = np.maximum(s, 0.0) - y * s + np.log1p(np.exp(-np.abs(s)))
    loss = ell.sum() / B if B else 0.0
    e = np.exp(-np.abs(s))
    sig = np.where(s >= 0, 1.0 / (1.0 + e), e / (1.0 + e))
    dscore = (sig - y) / B if B else np.zeros(0)
    return s, float(loss), dscore


# ==========================================================================
# Backward: chain rule through scorer, layers and aggregation
# ==========================================================================
def neighbour_sum_adjoint(csr: CSR, T: np.ndarray) -> np.ndarray:
    """Adjoint of the plain neighbour sum: node u receives T[v] from every v that aggregates from u.  Written
    as the scatter dual of the forward loop, from the forward CSR alone."""
    T = np.asarray(T, np.float64)
    out = np.zeros_like(T)
    rp, ci = csr.rowptr, csr.colidx
    for v in range(csr.n_nodes):
        lo, hi = rp[v], rp[v + 1]
        if hi > lo:
            out[ci[lo:hi]] += T[v]      # columns are distinct inside a row
    return out


def inverse_degrees(csr: CSR) -> np.ndarray:
    deg = np.diff(csr.rowptr.astype(np.int64)).astype(np.float64)
    return np.divide(1.0, deg, out=np.zeros_like(deg), where=deg > 0)


def mean_aggregate_adjoint(csr: CSR, T: np.ndarray) -> np.ndarray:
    """Adjoint of mean_aggregate: node u receives T[v]/|N(v)| from every v that aggregates from u."""
    return neighbour_sum_adjoint(csr, np.asarray(T, np.float64) * inverse_degrees(csr)[:, None])


@dataclass
class Grads:
    dW_self: List[np.ndarray]
    dW_neigh: List[np.ndarray]
    dbias: List[np.ndarray]
    dX: np.ndarray


def edge_grad_scatter(HK: np.ndarray, e_src, e_dst, dscore) -> np.ndarray:
    """dL/dH^K: each scored edge sends g_e * h_v to u and g_e * h_u to v."""
    HK = np.asarray(HK, np.float64)
    G = np.zeros_like(HK)
    np.add.at(G, e_src, dscore[:, None] * HK[e_dst])
    np.add.at(G, e_dst, dscore[:, None] * HK[e_src])
    return G


def backward(csr: CSR, W_self, W_neigh, acts: Activations, e_src, e_dst, dscore, relu_margin: float = 0.0,
             storage: str = "f32", seed_grad: Optional[np.ndarray] = None) -> Grads:
    """``relu_margin`` is 0 for the method itself: relu'(z) = [z > 0].  A test may pass +t and -t to find the
    gradient entries that depend on hidden units whose pre-activation lies within t of the kink, where a
    lower-precision implementation may legitimately take the other branch.

    With ``storage="bf16"`` every node-sized matrix that a bf16 implementation keeps in memory is rounded to
    bfloat16 where it is stored: dL/dH^K, the two products dZ W_self^T and (dZ W_neigh^T)/|N(v)|, and each
    dL/dH^(k-1).  Weight and bias gradients are sums over those stored values and are not rounded.

    ``seed_grad``: dL/dH^K given directly by a scorer other than the dot product (e_src, e_dst and dscore are then
    not used); the walk through the layers is the same."""
    K = len(W_self)
    inv_d = inverse_degrees(csr)
    if seed_grad is not None:
        G = _store(np.asarray(seed_grad, np.float64), storage)
    else:
        G = _store(edge_grad_scatter(acts.H[K], e_src, e_dst, np.asarray(dscore, np.float64)), storage)
    dWs, dWn, db = [None] * K, [None] * K, [None] * K
    for k in range(K, 0, -1):
        dZ = G if k == K else G * (acts.Z[k] > relu_margin)
        db[k - 1] = dZ.sum(axis=0)
        dWs[k - 1] = acts.H[k - 1].T @ dZ
        dWn[k - 1] = acts.A[k].T @ dZ
        T = _store((dZ @ np.asarray(W_neigh[k - 1], np.float64).T) * inv_d[:, None], storage)
        S = _store(dZ @ np.asarray(W_self[k - 1], np.float64).T, storage)
        G = _store(S + neighbour_sum_adjoint(csr, T), storage)
    return Grads(dWs, dWn, db, G)


# ==========================================================================
# Whole step
# ==========================================================================
@dataclass
class StepResult:
    neg_dst: np.ndarray
    e_src: np.ndarray
    e_dst: np.ndarray
    acts: Activations
    scores: np.ndarray
    loss: float
    dscore: np.ndarray
    grads: Grads


def batch_edges(pos_src, pos_dst, neg_dst, k_neg):
    """Scored edge list: the positives, then negative q = i*k_neg + j with the
    source of positive i."""
    e_src = np.concatenate([pos_src, np.repeat(pos_src, k_neg)]).astype(np.int32)
    e_dst = np.concatenate([pos_dst, neg_dst]).astype(np.int32)
    return e_src, e_dst


def train_step(csr: CSR, W_self, W_neigh, bias, X, pos_src, pos_dst, k_neg, n_space,
               seed, step, storage: str = "f32") -> StepResult:
    neg_dst, _ = sample_neg(csr, pos_src, k_neg, n_space, seed, step)
    e_src, e_dst = batch_edges(pos_src, pos_dst, neg_dst, k_neg)
    acts = sage_forward(csr, W_self, W_neigh, bias, X, storage)
    s, loss, ds = score_loss(acts.H[-1], e_src, e_dst, pos_src.size)
    grads = backward(csr, W_self, W_neigh, acts, e_src, e_dst, ds, storage=storage)
    return StepResult(neg_dst, e_src, e_dst, acts, s, loss, ds, grads)
