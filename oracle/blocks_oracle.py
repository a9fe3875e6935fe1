"""CPU oracle for the sampled-neighbourhood form of the training step (the paper's own training mode).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's cpu_baseline leg; shares no code
with the HIP path.

What the paper fixes (Sec. II-B, last paragraph; Fig. 1b; "Hyperparameters"): for every mini-batch the sampler builds
the computational graph of the endpoints of the batch's positive and negative edges, sampling a bounded number of
neighbours per node and hop (25, 10 and 5 for the first, second and third hop), and the K layers of Eq. (1) are
evaluated on that graph only.

Reading taken here (the paper leaves the mechanics to its graph library):
  * D_K = the nodes that are an endpoint of a scored edge, ascending.  Hop h = 1..K belongs to layer k = K+1-h:
    every v in D_k draws S_k(v), min(|N(v)|, fanout[h-1]) distinct neighbours, uniformly without replacement.
    D_{k-1} = D_k followed by the nodes of the samples that are not in D_k yet, ascending; so every frontier is a
    prefix of D_0 and a node keeps one position through all layers.
  * a_v = mean over S_k(v) (zero if empty), z_v = h_v W_self + a_v W_neigh + b for v in D_k; ReLU between layers.
  * the draw: a partial Fisher-Yates shuffle of the positions 0..d-1 of the sorted neighbour list; swap t exchanges
    position t with position t + floor(word * (d - t) / 2^32), where word is word (t mod 4) of Philox4x32-10 with
    counter (v, hop * 2^16 + t div 4, step_lo, step_hi) and key (seed_lo, seed_hi); the sample is positions
    0..f-1 after f swaps, in that order.  A node with d <= f takes all its neighbours in list order.
  * a fan-out of 0 stands for "all neighbours" (a full-neighbourhood mini-batch): no draw, the whole list in order.
With a fan-out at least as large as every degree the computational graph is the exact K-hop neighbourhood, and
embeddings, loss and weight gradients coincide with the full-graph step: that is the main pin of this file.

GCN layers on the blocks ("Hyperparameters" names a 3-layer GCN trained in mini-batches; the neighbour sampling is
stated for GraphSAGE only).  Reading: the Kipf-Welling propagation of the full visible graph, restricted to the
computational graph, with the degrees d^ of the FULL graph in the normalisation,
    a_v = (d^_v / |S(v)|) * sum_{u in S(v)} h_u / sqrt(d^_v d^_u),    z_v = a_v W + b,
where the factor d^_v / |S(v)| makes a drawn subset an unbiased estimate of the full sum and is 1 for a
full-neighbourhood block, for which the layer equals the full-graph GCN exactly on the computational graph.  The
self-pair is an ordinary entry of the caller's CSR (as in the full-graph GCN), so there is no separate self path.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np

from oracle import lp_oracle as O


@dataclass
class Blocks:
    n: np.ndarray                 # int32 [K+1]: frontier sizes, n[K] <= ... <= n[0]
    nodes: np.ndarray             # int32 [n[0]]: global ids; frontier k = nodes[:n[k]]
    ptr: List[np.ndarray]         # ptr[k-1]: int32 [n[k]+1], block of layer k
    col: List[np.ndarray]         # col[k-1]: int32 [E_k], positions in frontier k-1, rows in draw order
    t_ptr: List[np.ndarray]       # transposed block: int32 [n[k-1]+1]
    t_col: List[np.ndarray]       # int32 [E_k]: destination positions, by (source position, entry index)
    e_src_pos: np.ndarray         # batch edges in positions of frontier K
    e_dst_pos: np.ndarray


def sample_row(neigh: np.ndarray, f: int, v: int, hop: int, seed: int, step: int) -> np.ndarray:
    """S(v): the draw described in the header, one node, Python integers."""
    d = int(neigh.size)
    if f == 0 or d <= f:
        return neigh.copy()
    a = list(range(d))
    words = None
    for t in range(f):
        if t % 4 == 0:
            words = O.philox4x32_10(v, (hop << 16) + t // 4, step & 0xFFFFFFFF, (step >> 32) & 0xFFFFFFFF,
                                    seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
        r = t + ((words[t % 4] * (d - t)) >> 32)
        a[t], a[r] = a[r], a[t]
    return neigh[np.array(a[:f], np.int64)]


def sample_blocks(csr: O.CSR, e_src: np.ndarray, e_dst: np.ndarray, fanout: List[int], seed: int, step: int) -> Blocks:
    K = len(fanout)
    e_src = np.asarray(e_src, np.int64)
    e_dst = np.asarray(e_dst, np.int64)
    seeds = np.unique(np.concatenate([e_src, e_dst]))
    index = np.full(csr.n_nodes, -1, np.int64)
    index[seeds] = np.arange(seeds.size)
    nodes = list(seeds.tolist())
    n = [0] * (K + 1)
    n[K] = len(nodes)
    ptr, col, t_ptr, t_col = [None] * K, [None] * K, [None] * K, [None] * K
    for hop in range(1, K + 1):
        k = K + 1 - hop
        rows = [sample_row(csr.colidx[csr.rowptr[v]:csr.rowptr[v + 1]], fanout[hop - 1], v, hop, seed, step)
                for v in nodes[:n[k]]]
        glob = np.concatenate(rows).astype(np.int64) if rows else np.zeros(0, np.int64)
        new = np.unique(glob[index[glob] < 0]) if glob.size else np.zeros(0, np.int64)
        index[new] = len(nodes) + np.arange(new.size)
        nodes.extend(new.tolist())
        n[k - 1] = len(nodes)
        p = np.zeros(n[k] + 1, np.int64)
        p[1:] = np.cumsum([r.size for r in rows])
        ptr[k - 1] = p.astype(np.int32)
        col[k - 1] = index[glob].astype(np.int32)
        # transposed block: entries grouped by source position, in entry order inside a group
        dst_of_entry = np.repeat(np.arange(n[k]), np.diff(p))
        order = np.argsort(col[k - 1], kind="stable")
        tp = np.zeros(n[k - 1] + 1, np.int64)
        tp[1:] = np.cumsum(np.bincount(col[k - 1], minlength=n[k - 1]))
        t_ptr[k - 1] = tp.astype(np.int32)
        t_col[k - 1] = dst_of_entry[order].astype(np.int32)
    return Blocks(np.array(n, np.int32), np.array(nodes, np.int32), ptr, col, t_ptr, t_col,
                  index[e_src].astype(np.int32), index[e_dst].astype(np.int32))


def block_mean(ptr: np.ndarray, col: np.ndarray, H: np.ndarray) -> np.ndarray:
    """a_i = mean of H[col[p]] over the entries p of row i; zero for an empty row."""
    out = np.zeros((ptr.size - 1, H.shape[1]))
    for i in range(ptr.size - 1):
        lo, hi = ptr[i], ptr[i + 1]
        if hi > lo:
            out[i] = H[col[lo:hi]].sum(axis=0) / float(hi - lo)
    return out


@dataclass
class BlockActs:
    H: List[np.ndarray]      # H[k]: [n[k], F_k], k = 0..K (H[0] = X rows of frontier 0)
    A: List[np.ndarray]      # A[k]: [n[k], F_{k-1}], k = 1..K
    Z: List[np.ndarray]


def forward_blocks(b: Blocks, W_self, W_neigh, bias, X) -> BlockActs:
    K = len(W_self)
    H = [np.asarray(X, np.float64)[b.nodes[:b.n[0]]]]
    A, Z = [None], [None]
    for k in range(1, K + 1):
        nk = int(b.n[k])
        a = block_mean(b.ptr[k - 1], b.col[k - 1], H[k - 1])
        z = H[k - 1][:nk] @ np.asarray(W_self[k - 1], np.float64) + a @ np.asarray(W_neigh[k - 1], np.float64) \
            + np.asarray(bias[k - 1], np.float64)
        A.append(a)
        Z.append(z)
        H.append(np.maximum(z, 0.0) if k < K else z)
    return BlockActs(H, A, Z)


def backward_blocks(b: Blocks, W_self, W_neigh, acts: BlockActs, dscore, relu_margin: float = 0.0, seed_grad=None) -> O.Grads:
    """Chain rule through scorer, layers and sampled aggregation; dX is not formed.

    ``seed_grad``: dL/dH^K on frontier K given directly by a scorer other than the dot product (dscore is then unused).
    """
    K = len(W_self)
    if seed_grad is not None:
        G = np.asarray(seed_grad, np.float64)
    else:
        G = O.edge_grad_scatter(acts.H[K], b.e_src_pos, b.e_dst_pos, np.asarray(dscore, np.float64))
    dWs, dWn, db = [None] * K, [None] * K, [None] * K
    for k in range(K, 0, -1):
        nk = int(b.n[k])
        dZ = G if k == K else G * (acts.Z[k] > relu_margin)
        db[k - 1] = dZ.sum(axis=0)
        dWs[k - 1] = acts.H[k - 1][:nk].T @ dZ
        dWn[k - 1] = acts.A[k].T @ dZ
        if k == 1:
            break
        ptr, col = b.ptr[k - 1], b.col[k - 1]
        cnt = np.diff(ptr).astype(np.float64)
        T = (dZ @ np.asarray(W_neigh[k - 1], np.float64).T) * np.divide(1.0, cnt, out=np.zeros_like(cnt), where=cnt > 0)[:, None]
        Gn = np.zeros((int(b.n[k - 1]), acts.H[k - 1].shape[1]))
        Gn[:nk] = dZ @ np.asarray(W_self[k - 1], np.float64).T
        for i in range(nk):
            lo, hi = ptr[i], ptr[i + 1]
            if hi > lo:
                np.add.at(Gn, col[lo:hi], T[i])       # a sampled node can only occur once per row, add.at is for safety
        G = Gn
    return O.Grads(dWs, dWn, db, None)


# ---------------------------------------------------------------------------------------------- GCN layers on blocks
def gcn_block_aggregate(ptr: np.ndarray, col: np.ndarray, inv_deg_pos: np.ndarray, H: np.ndarray) -> np.ndarray:
    """a_i = (d_i / |row i|) * sum over the entries p of row i of H[col[p]] / sqrt(d_i d_col[p]); d = full-graph degrees
    of the nodes at the frontier positions (inv_deg_pos = 1 / d, 0 for a node without entries)."""
    out = np.zeros((ptr.size - 1, H.shape[1]))
    c = np.sqrt(inv_deg_pos)
    for i in range(ptr.size - 1):
        lo, hi = ptr[i], ptr[i + 1]
        if hi > lo:
            d_i = 1.0 / inv_deg_pos[i]
            out[i] = (d_i / float(hi - lo)) * c[i] * (c[col[lo:hi]][:, None] * H[col[lo:hi]]).sum(axis=0)
    return out


def forward_blocks_gcn(b: Blocks, inv_deg: np.ndarray, W, bias, X) -> BlockActs:
    """inv_deg: the full graph's 1 / d^ per node (O.inverse_degrees of the CSR that holds the self-pairs)."""
    K = len(W)
    ipos = np.asarray(inv_deg, np.float64)[b.nodes[:b.n[0]]]
    H = [np.asarray(X, np.float64)[b.nodes[:b.n[0]]]]
    A, Z = [None], [None]
    for k in range(1, K + 1):
        a = gcn_block_aggregate(b.ptr[k - 1], b.col[k - 1], ipos, H[k - 1])
        z = a @ np.asarray(W[k - 1], np.float64) + np.asarray(bias[k - 1], np.float64)
        A.append(a)
        Z.append(z)
        H.append(np.maximum(z, 0.0) if k < K else z)
    return BlockActs(H, A, Z)


def backward_blocks_gcn(b: Blocks, inv_deg: np.ndarray, W, acts: BlockActs, dscore, relu_margin: float = 0.0,
                        seed_grad=None) -> O.Grads:
    """Weight and bias gradients through the GCN blocks (dW is reported as dW_neigh, as in the full-graph GCN)."""
    K = len(W)
    ipos = np.asarray(inv_deg, np.float64)[b.nodes[:b.n[0]]]
    c = np.sqrt(ipos)
    if seed_grad is not None:
        G = np.asarray(seed_grad, np.float64)
    else:
        G = O.edge_grad_scatter(acts.H[K], b.e_src_pos, b.e_dst_pos, np.asarray(dscore, np.float64))
    dW, db = [None] * K, [None] * K
    for k in range(K, 0, -1):
        nk = int(b.n[k])
        dZ = G if k == K else G * (acts.Z[k] > relu_margin)
        db[k - 1] = dZ.sum(axis=0)
        dW[k - 1] = acts.A[k].T @ dZ
        if k == 1:
            break
        ptr, col = b.ptr[k - 1], b.col[k - 1]
        T = dZ @ np.asarray(W[k - 1], np.float64).T
        Gn = np.zeros((int(b.n[k - 1]), acts.H[k - 1].shape[1]))
        for i in range(nk):
            lo, hi = ptr[i], ptr[i + 1]
            if hi > lo:
                w_i = (1.0 / ipos[i]) / float(hi - lo) * c[i]
                np.add.at(Gn, col[lo:hi], (w_i * c[col[lo:hi]])[:, None] * T[i])
        G = Gn
    return O.Grads([None] * K, dW, db, None)
