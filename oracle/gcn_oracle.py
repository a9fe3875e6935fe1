"""CPU oracle for the GCN instance of Eq. (1) (the paper's second representative model, "Hyperparameters").

TEST INFRASTRUCTURE ONLY: imported by tests and the benchmark's cpu_baseline leg; shares no code with the HIP path.

Reading (the paper names the model, not its formula): the graph convolution of Kipf and Welling (ICLR 2017),
  h'_v = act( sum_{u in N^(v)} h_u / sqrt(d^_u d^_v) W + b ),
on the visible graph with every self-pair present (N^(v) = N(v) with v itself added, d^_v = |N^(v)|); ReLU between
layers, none after the last.  The caller supplies a CSR that already contains the self-pairs (build it from the
edge list with one (v, v) pair per node appended), so d^ is simply the row length.  For a CSR that is not symmetric
the same row lengths normalise both sides: S[v, u] = 1 / sqrt(d^_v d^_u) for u in N^(v).
"""
from __future__ import annotations

from typing import List

import numpy as np

from oracle import lp_oracle as O


def add_self_pairs(n_nodes: int, rows: np.ndarray, cols: np.ndarray):
    """The edge list with one (v, v) pair per node appended (input marshalling, no arithmetic)."""
    loop = np.arange(n_nodes, dtype=np.int32)
    return np.concatenate([np.asarray(rows, np.int32), loop]), np.concatenate([np.asarray(cols, np.int32), loop])


def normalised_aggregate(csr: O.CSR, H: np.ndarray) -> np.ndarray:
    """a_v = sum over the row of v of h_u / sqrt(d^_v d^_u)."""
    H = np.asarray(H, np.float64)
    c = np.sqrt(O.inverse_degrees(csr))
    out = np.zeros_like(H)
    rp, ci = csr.rowptr, csr.colidx
    for v in range(csr.n_nodes):
        lo, hi = rp[v], rp[v + 1]
        if hi > lo:
            out[v] = c[v] * (c[ci[lo:hi]][:, None] * H[ci[lo:hi]]).sum(axis=0)
    return out


def normalised_aggregate_adjoint(csr: O.CSR, T: np.ndarray) -> np.ndarray:
    """Adjoint of normalised_aggregate, written as the scatter dual of its loop."""
    T = np.asarray(T, np.float64)
    c = np.sqrt(O.inverse_degrees(csr))
    out = np.zeros_like(T)
    rp, ci = csr.rowptr, csr.colidx
    for v in range(csr.n_nodes):
        lo, hi = rp[v], rp[v + 1]
        if hi > lo:
            out[ci[lo:hi]] += (c[v] * c[ci[lo:hi]])[:, None] * T[v]      # columns are distinct inside a row
    return out


def gcn_forward(csr: O.CSR, W, bias, X, storage: str = "f32") -> O.Activations:
    K = len(W)
    H = [np.asarray(X, np.float64)]
    A, Z = [None], [None]
    for k in range(1, K + 1):
        a = O._store(normalised_aggregate(csr, H[k - 1]), storage)
        z = a @ np.asarray(W[k - 1], np.float64) + np.asarray(bias[k - 1], np.float64)
        A.append(a)
        Z.append(z)
        H.append(O._store(np.maximum(z, 0.0) if k < K else z, storage))
    return O.Activations(H, A, Z)


def gcn_backward(csr: O.CSR, W, acts: O.Activations, e_src, e_dst, dscore, relu_margin: float = 0.0,
                 storage: str = "f32") -> O.Grads:
    """Gradients of the batch loss (dot-product scorer) with respect to W, b and X.  dW_self stays None: the layer
    has a single weight matrix, reported as dW_neigh."""
    K = len(W)
    G = O._store(O.edge_grad_scatter(acts.H[K], e_src, e_dst, np.asarray(dscore, np.float64)), storage)
    dW, db = [None] * K, [None] * K
    for k in range(K, 0, -1):
        dZ = G if k == K else G * (acts.Z[k] > relu_margin)
        db[k - 1] = dZ.sum(axis=0)
        dW[k - 1] = acts.A[k].T @ dZ
        T = O._store(dZ @ np.asarray(W[k - 1], np.float64).T, storage)
        G = O._store(normalised_aggregate_adjoint(csr, T), storage)
    return O.Grads([None] * K, dW, db, G)
