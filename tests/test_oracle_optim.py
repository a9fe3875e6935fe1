"""Pins for the optimizer oracle: closed forms (first Adam step, constant gradients, a quadratic bowl under plain
gradient descent) and an independent library implementation of the same published algorithm (torch.optim on the
CPU in float64)."""
import numpy as np
import torch

from oracle import optim_oracle as P


def test_sgd_is_a_linear_step_and_contracts_a_quadratic():
    rng = np.random.default_rng(0)
    w = rng.standard_normal(50)
    g = rng.standard_normal(50)
    np.testing.assert_allclose(P.sgd_step(w, g, 0.1), w - 0.1 * g, rtol=0, atol=1e-15)
    # L(w) = |w|^2 / 2 has gradient w: every step multiplies w by (1 - lr)
    x = w.copy()
    for _ in range(10):
        x = P.sgd_step(x, x, 0.25)
    np.testing.assert_allclose(x, w * 0.75 ** 10, rtol=1e-12)


def test_adam_first_step_and_constant_gradient_closed_forms():
    rng = np.random.default_rng(1)
    w = rng.standard_normal(40)
    g = rng.standard_normal(40) * 10.0 ** rng.integers(-6, 3, 40)
    lr, eps = 1e-3, 1e-8
    # with a constant gradient the bias-corrected moments are exactly g and g^2 at every step
    x, m, v = w.copy(), np.zeros(40), np.zeros(40)
    for t in range(1, 6):
        x, m, v = P.adam_step(x, g, m, v, t, lr=lr, eps=eps)
        np.testing.assert_allclose(x, w - t * lr * g / (np.abs(g) + eps), rtol=1e-9, atol=1e-15)
    # a zero gradient leaves the weight where it is
    x0, _, _ = P.adam_step(w, np.zeros(40), np.zeros(40), np.zeros(40), 1)
    assert np.array_equal(x0, w)


def test_adam_and_sgd_match_torch_optim_over_a_gradient_sequence():
    rng = np.random.default_rng(2)
    w0 = rng.standard_normal((7, 5))
    grads = [rng.standard_normal((7, 5)) * s for s in (1.0, 0.1, 3.0, 1e-3, 0.5, 2.0)]
    for name in ("adam", "sgd"):
        p = torch.nn.Parameter(torch.tensor(w0, dtype=torch.float64))
        opt = (torch.optim.Adam([p], lr=2e-3, betas=(0.8, 0.95), eps=1e-7) if name == "adam"
               else torch.optim.SGD([p], lr=0.05))
        x, m, v = w0.copy(), np.zeros_like(w0), np.zeros_like(w0)
        for t, g in enumerate(grads, start=1):
            p.grad = torch.tensor(g, dtype=torch.float64)
            opt.step()
            if name == "adam":
                x, m, v = P.adam_step(x, g, m, v, t, lr=2e-3, beta1=0.8, beta2=0.95, eps=1e-7)
            else:
                x = P.sgd_step(x, g, 0.05)
            np.testing.assert_allclose(x, p.detach().numpy(), rtol=1e-11, atol=1e-14)


def test_bf16_storage_rounds_the_updated_weight_only():
    w = np.array([1.0, -2.0, 0.3])
    g = np.array([0.5, 0.25, -1.0])
    x, m, v = P.adam_step(w, g, np.zeros(3), np.zeros(3), 1, storage="bf16")
    bits = x.astype(np.float32).view(np.uint32)
    assert np.all(bits & 0xFFFF == 0)                          # representable in bfloat16
    exact, m2, v2 = P.adam_step(w, g, np.zeros(3), np.zeros(3), 1)
    assert np.all(np.abs(x - exact) <= np.abs(exact) * 2.0 ** -8) and np.array_equal(m, m2) and np.array_equal(v, v2)
