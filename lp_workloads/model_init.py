"""Seeded random node features and model parameters (inputs only)."""
from __future__ import annotations

from typing import List, Tuple

import numpy as np


def init_features(n_nodes: int, f0: int, seed: int) -> np.ndarray:
    """Node-major feature matrix [n_nodes, f0], standard normal, float32."""
    rng = np.random.default_rng(seed)
    return rng.standard_normal((n_nodes, f0), dtype=np.float32)


def init_model(dims: List[int], seed: int) -> Tuple[list, list, list]:
    """Per layer k=1..K: W_self, W_neigh of shape [F_{k-1}, F_k] ~ N(0, 1/(2 F_{k-1}))
    and a bias ~ U(-0.1, 0.1).  The last layer is additionally scaled by
    F_K^(-1/4) so that dot-product scores stay O(1) and the sigmoids in the loss
    are not saturated."""
    rng = np.random.default_rng(seed)
    K = len(dims) - 1
    W_self, W_neigh, bias = [], [], []
    for k in range(1, K + 1):
        fi, fo = dims[k - 1], dims[k]
        s = np.sqrt(1.0 / (2.0 * fi))
        if k == K:
            s *= fo ** -0.25
        W_self.append((rng.standard_normal((fi, fo)) * s).astype(np.float32))
        W_neigh.append((rng.standard_normal((fi, fo)) * s).astype(np.float32))
        bias.append(rng.uniform(-0.1, 0.1, size=fo).astype(np.float32))
    return W_self, W_neigh, bias


def to_bf16_grid(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 value (ties to even) and
    return them as float32 again, so that an input can be handed to a bf16 path
    and to a wider-precision checker as the same numbers."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    rounded = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
    return rounded.astype(np.uint32).view(np.float32).reshape(a.shape)
