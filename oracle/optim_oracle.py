"""CPU oracle for the weight update that closes a training step (Algorithm 1, "Update W <- W - eta grad L(W)").

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's cpu_baseline leg.

The algorithm box writes plain gradient descent; the experiments ("Hyperparameters") use the Adam optimizer with
learning rate 0.001.  Both are given here, in float64, one tensor at a time:

  sgd:   w <- w - lr * g
  adam (Kingma and Ba, 2015, Algorithm 1 there), step count t = 1, 2, ...:
         m <- b1 m + (1 - b1) g,   v <- b2 v + (1 - b2) g^2,
         w <- w - lr * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps)

With storage == "bf16" the updated weight is rounded to bfloat16 (nearest even), as the stored weights of the
bf16 configuration are; the moments stay unrounded.
"""
from __future__ import annotations

import numpy as np

from oracle.lp_oracle import _store


def sgd_step(w, g, lr: float, storage: str = "f32"):
    return _store(np.asarray(w, np.float64) - lr * np.asarray(g, np.float64), storage)


def adam_step(w, g, m, v, t: int, lr: float = 1e-3, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
              storage: str = "f32"):
    """Returns (w, m, v) after step t (t counts from 1)."""
    w, g = np.asarray(w, np.float64), np.asarray(g, np.float64)
    m = beta1 * np.asarray(m, np.float64) + (1.0 - beta1) * g
    v = beta2 * np.asarray(v, np.float64) + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** t)
    v_hat = v / (1.0 - beta2 ** t)
    return _store(w - lr * m_hat / (np.sqrt(v_hat) + eps), storage), m, v
