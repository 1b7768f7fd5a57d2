"""Pins of the update oracles: textbook properties that a wrong sign, a missing bias correction
or swapped moments would break."""
import numpy as np

from oracle import optim as P


def test_gd_update_descends_a_quadratic():
    rng = np.random.default_rng(0)
    A = rng.standard_normal((20, 5))
    y = rng.standard_normal(20)
    beta = rng.standard_normal(5)
    loss = lambda b: 0.5 * np.sum((A @ b - y) ** 2)
    g = A.T @ (A @ beta - y)
    lr = 1.0 / np.linalg.norm(A, 2) ** 2
    assert loss(P.gd_update(beta, g, lr)) < loss(beta)
    assert np.allclose(P.gd_update(beta, g, 0.0), beta)


def test_adam_first_step_has_magnitude_lr_and_moves_against_the_gradient():
    """With zero initial moments the bias-corrected first step is lr * g / (|h| + eps): for
    h = g its magnitude is lr whatever the scale of g (the optimizer's defining property)."""
    g = np.array([1e-6, -3.0, 250.0, -1e3])
    beta = np.zeros(4)
    b1, m1, m2 = P.adam_update(beta, np.zeros(4), np.zeros(4), g, g, 1e-2, 0.9, 0.999, 1e-12, 1)
    assert np.allclose(b1, -1e-2 * np.sign(g), rtol=1e-5)
    assert np.allclose(m1, 0.1 * g) and np.allclose(m2, 0.001 * g * g)
    # the second track only enters the denominator: doubling it halves the step
    b2, _, _ = P.adam_update(beta, np.zeros(4), np.zeros(4), g, 2 * g, 1e-2, 0.9, 0.999, 1e-12, 1)
    assert np.allclose(b2, 0.5 * b1, rtol=1e-5)


def test_adam_constant_gradient_keeps_unit_steps():
    g = np.array([0.5, -2.0])
    beta, m1, m2 = np.zeros(2), np.zeros(2), np.zeros(2)
    for t in range(1, 30):
        new, m1, m2 = P.adam_update(beta, m1, m2, g, g, 1e-3, 0.9, 0.999, 1e-12, t)
        assert np.allclose(new - beta, -1e-3 * np.sign(g), rtol=1e-6)      # bias corrections cancel exactly
        beta = new
