"""Pins for oracle/optimizer_oracle.py: closed forms of the two update rules and an independent
library implementation (torch.optim on the CPU, float64).  CPU only."""
import numpy as np
import pytest

from oracle import optimizer_oracle as oo

torch = pytest.importorskip("torch")


def test_first_adamw_step_is_a_signed_step_of_size_lr():
    """t = 1: mhat = g, vhat = g^2, so the step is lr * g / (|g| + eps) (+ decay)."""
    rng = np.random.default_rng(0)
    w, g = rng.standard_normal(100), rng.standard_normal(100)
    w1, m1, v1 = oo.adamw_step(w, np.zeros(100), np.zeros(100), g, 1, lr=1e-2, eps=1e-8, weight_decay=0.1)
    np.testing.assert_allclose(w1, w - 1e-2 * (g / (np.abs(g) + 1e-8) + 0.1 * w), rtol=1e-12)
    np.testing.assert_allclose(m1, 0.1 * g, rtol=1e-12)
    np.testing.assert_allclose(v1, 0.001 * g * g, rtol=1e-12)


def test_constant_gradient_keeps_the_bias_corrected_moments_constant():
    g = np.array([0.5, -2.0, 3.0])
    w, m, v = np.zeros(3), np.zeros(3), np.zeros(3)
    for t in range(1, 20):
        w_prev = w
        w, m, v = oo.adamw_step(w, m, v, g, t, lr=1e-3, eps=0.0)
        np.testing.assert_allclose(m / (1 - 0.9 ** t), g, rtol=1e-12)
        np.testing.assert_allclose(v / (1 - 0.999 ** t), g * g, rtol=1e-12)
        np.testing.assert_allclose(w - w_prev, -1e-3 * np.sign(g), rtol=1e-10)


def test_zero_gradient_only_decays():
    w = np.array([1.0, -4.0])
    w1, m1, v1 = oo.adamw_step(w, np.zeros(2), np.zeros(2), np.zeros(2), 1, lr=0.1, eps=1e-8, weight_decay=0.5)
    np.testing.assert_allclose(w1, w * (1 - 0.05), rtol=1e-12)
    assert not m1.any() and not v1.any()
    np.testing.assert_allclose(oo.sgd_step(w, np.zeros(2), 0.1, 0.5), w * 0.95, rtol=1e-12)


def test_sgd_on_a_quadratic_contracts_geometrically():
    w = np.array([3.0, -1.0])
    for _ in range(10):
        w = oo.sgd_step(w, w, lr=0.25)          # gradient of |w|^2 / 2
    np.testing.assert_allclose(w, np.array([3.0, -1.0]) * 0.75 ** 10, rtol=1e-12)


@pytest.mark.parametrize("wd", [0.0, 0.05])
def test_against_the_library_optimizers(wd):
    rng = np.random.default_rng(1)
    w0 = rng.standard_normal(64)
    grads = [rng.standard_normal(64) for _ in range(5)]
    # AdamW
    p = torch.nn.Parameter(torch.tensor(w0, dtype=torch.float64))
    opt = torch.optim.AdamW([p], lr=3e-3, betas=(0.9, 0.95), eps=1e-6, weight_decay=wd)
    w, m, v = w0.copy(), np.zeros(64), np.zeros(64)
    for t, g in enumerate(grads, start=1):
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        w, m, v = oo.adamw_step(w, m, v, g, t, lr=3e-3, beta1=0.9, beta2=0.95, eps=1e-6, weight_decay=wd)
        np.testing.assert_allclose(w, p.detach().numpy(), rtol=1e-10, atol=1e-12)
    # SGD with L2 term
    p = torch.nn.Parameter(torch.tensor(w0, dtype=torch.float64))
    opt = torch.optim.SGD([p], lr=0.05, weight_decay=wd)
    w = w0.copy()
    for g in grads:
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        w = oo.sgd_step(w, g, 0.05, wd)
        np.testing.assert_allclose(w, p.detach().numpy(), rtol=1e-12, atol=1e-14)
