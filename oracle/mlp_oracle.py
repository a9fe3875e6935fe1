"""CPU oracle for the MLP edge predictor (Eq. 2 with "MLP" as the predictor; "Hyperparameters": a 3-layer MLP).

TEST INFRASTRUCTURE ONLY: imported by tests and the benchmark's cpu_baseline leg; shares no code with the HIP path.

The paper says the pairwise node embeddings "are aggregated and go through an edge predictor" and names the
MLP without a formula.  Reading: the pair (h_u, h_v) is combined by the element-wise product (symmetric in u and v,
and the dot-product predictor is then the special case of summing it), followed by L linear layers with ReLU between
them and a single output:
    x_e = h_u * h_v,   u^0 = x_e,   u^j = relu(u^(j-1) W_j + c_j) for j < L,   s_e = u^(L-1) W_L + c_L.
Loss and labels are those of the dot-product path.  All arithmetic in float64.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np

from oracle import lp_oracle as O


@dataclass
class MlpActs:
    X: np.ndarray            # [B, F] products of the end-point embeddings
    U: List[np.ndarray]      # U[j]: output of hidden layer j = 1..L-1 (U[0] = X)
    Zs: List[np.ndarray]     # pre-activations of the hidden layers (index 0 unused)


def mlp_scores(HK, e_src, e_dst, W, c, storage: str = "f32"):
    HK = np.asarray(HK, np.float64)
    X = O._store(HK[e_src] * HK[e_dst], storage)
    U, Zs = [X], [None]
    L = len(W)
    for j in range(1, L):
        z = U[j - 1] @ np.asarray(W[j - 1], np.float64) + np.asarray(c[j - 1], np.float64)
        Zs.append(z)
        U.append(O._store(np.maximum(z, 0.0), storage))
    s = (U[L - 1] @ np.asarray(W[L - 1], np.float64)).reshape(-1) + float(np.asarray(c[L - 1], np.float64).reshape(-1)[0])
    return s, MlpActs(X, U, Zs)


def bce_mean(s: np.ndarray, n_pos_edges: int):
    """Batch-mean binary cross-entropy on logits and its derivative (same as the dot-product path)."""
    B = s.size
    y = np.zeros(B)
    y[:n_pos_edges] = 1.0
    ell = np.maximum(s, 0.0) - y * s + np.log1p(np.exp(-np.abs(s)))
    e = np.exp(-np.abs(s))
    sig = np.where(s >= 0, 1.0 / (1.0 + e), e / (1.0 + e))
    return (float(ell.sum() / B) if B else 0.0), ((sig - y) / B if B else np.zeros(0))


def mlp_backward(HK, e_src, e_dst, W, acts: MlpActs, dscore, relu_margin: float = 0.0, storage: str = "f32"):
    """Returns (dW list, dc list, edge_grad [B, F] = dL/dx_e, G = dL/dH^K [N, F])."""
    HK = np.asarray(HK, np.float64)
    L = len(W)
    dW, dc = [None] * L, [None] * L
    ds = np.asarray(dscore, np.float64)
    dW[L - 1] = (acts.U[L - 1].T @ ds).reshape(-1, 1)
    dc[L - 1] = np.array([ds.sum()])
    dU = ds[:, None] * np.asarray(W[L - 1], np.float64).reshape(1, -1)
    for j in range(L - 1, 0, -1):
        dZ = O._store(dU * (acts.Zs[j] > relu_margin), storage)
        dW[j - 1] = acts.U[j - 1].T @ dZ
        dc[j - 1] = dZ.sum(axis=0)
        dU = dZ @ np.asarray(W[j - 1], np.float64).T
    edge_grad = O._store(dU, storage)
    G = np.zeros_like(HK)
    np.add.at(G, e_src, edge_grad * HK[e_dst])
    np.add.at(G, e_dst, edge_grad * HK[e_src])
    return dW, dc, edge_grad, O._store(G, storage)
