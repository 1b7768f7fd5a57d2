"""Pins of the least-squares oracle (CPU only): gradient of the loss by finite differences,
the normal equations, additivity over partitions, bfloat16 conversion."""
import numpy as np

from oracle import lsq as LS
from paper_2605_15890_amd import inputs as I


def test_bf16_roundtrip_and_rounding():
    x = np.array([1.0, -2.5, 3.140625, 1.0 + 2 ** -8, 1.0 + 2 ** -9, 1.0 + 3 * 2 ** -9], dtype=np.float32)
    bits = LS.f32_to_bf16_bits(x)
    back = LS.bf16_bits_to_f64(bits)
    assert back[0] == 1.0 and back[1] == -2.5 and back[2] == 3.140625
    assert back[3] == 1.0 + 2 ** -7 or back[3] == 1.0          # tie -> even
    assert back[3] == 1.0                                       # 1+2^-8 is a tie between 1 and 1+2^-7: even is 1
    assert back[4] == 1.0 and back[5] == 1.0 + 2 ** -7
    Xb, _, _ = I.least_squares_numpy(64, 128)
    assert np.array_equal(LS.f32_to_bf16_bits(LS.bf16_bits_to_f64(Xb).astype(np.float32)), Xb)


def test_gradient_matches_finite_differences_and_partitions_add_up():
    Xb, y, w_star = I.least_squares_numpy(256, 128)
    rng = np.random.default_rng(0)
    beta = rng.standard_normal(128)
    G, r = LS.partial_gradients(Xb, y, beta, 8)
    g = G.sum(axis=0)
    X = LS.bf16_bits_to_f64(Xb)
    assert np.allclose(g, X.T @ (X @ beta - y), rtol=1e-12, atol=1e-12)
    for j in (0, 17, 127):
        e = np.zeros(128)
        e[j] = 1e-5
        fd = (LS.loss(Xb, y, beta + e) - LS.loss(Xb, y, beta - e)) / 2e-5
        assert abs(fd - g[j]) < 1e-6 * max(1.0, abs(g[j]))
    # each partition's gradient is the gradient of that partition's own loss
    rows = 256 // 8
    for p in (0, 5):
        sl = slice(p * rows, (p + 1) * rows)
        e = np.zeros(128)
        e[3] = 1e-5
        fd = (LS.loss(Xb[sl], y[sl], beta + e) - LS.loss(Xb[sl], y[sl], beta - e)) / 2e-5
        assert abs(fd - G[p, 3]) < 1e-6


def test_gradient_vanishes_at_the_least_squares_solution():
    Xb, y, w_star = I.least_squares_numpy(512, 128)
    X = LS.bf16_bits_to_f64(Xb)
    sol = np.linalg.lstsq(X, y.astype(np.float64), rcond=None)[0]
    G, r = LS.partial_gradients(Xb, y, sol, 4)
    assert np.linalg.norm(G.sum(axis=0)) < 1e-9 * np.linalg.norm(X.T @ y)
    assert np.linalg.norm(sol - w_star) < 0.05 * np.linalg.norm(w_star)
