"""Monte-Carlo pins of the whole oracle path on the tiny configuration: unbiasedness
(constraint of problem P1) and the residual error against its exact expression (proof of
Lemma 1 before bounding).  CPU only; 1000 iterations with fresh arrivals and fresh draws."""
import numpy as np
import pytest

from oracle import agc_oracle as O
from oracle import design as D
from paper_2605_15890_amd import inputs as I


def _setup(scale_mode):
    cfg = I.CONFIGS["tiny"]
    p = I.straggler_probs(cfg)
    bits = I.random_bits(cfg)
    c = D.c_weights(p, bits, D.phi_coef_balanced(p, int(bits.sum())))
    alpha, supp = D.cyclic_code(c, cfg.k, cfg.s)
    B, w = D.physical_code(alpha, p)
    row_ptr = np.arange(0, cfg.n * cfg.s + 1, cfg.s)
    col = np.array(supp).ravel()
    val = np.array([B[i, j] for i in range(cfg.n) for j in supp[i]], dtype=np.float32)
    csr = O.Csr(row_ptr, col, val, cfg.k)
    G = I.partial_gradients_numpy(cfg)
    return cfg, p, bits, csr, w.astype(np.float32), G


def _exact_error(cfg, G, csr, bits, w, p, scale_mode):
    f = np.array([O.encode(G, csr, i) for i in range(cfg.n)])
    scales = O.scales(G, csr, scale_mode)
    var_q = []
    for i in range(cfg.n):
        inv = O.inv16(scales[i], int(bits[i]))
        L = O.levels(int(bits[i]))
        unit = float(scales[i]) / L
        tot = 0.0
        for x in f[i]:
            lo, pu = O.quantize_prob(x, inv, int(bits[i]))
            tot += unit * unit * pu * (1 - pu) if lo < L else 0.0
        var_q.append(tot)
    return D.exact_moments(f.astype(np.float64), var_q, w.astype(np.float64), p)


@pytest.mark.parametrize("scale_mode", [O.SCALE_MAXABS, O.SCALE_L2])
def test_worker_moments_equal_the_per_coordinate_sums(scale_mode):
    """The whole-vector moment routine used by the large Monte-Carlo checks against a plain
    loop over the per-coordinate round-up probabilities (themselves pinned by brute force over
    all primary fields), and against a direct variance of the two-point outcome of every
    coordinate; the clamp case (|f| = scale has no randomness) is part of the max-abs run."""
    cfg, p, bits, csr, w, G = _setup(scale_mode)
    scales = O.scales(G, csr, scale_mode)
    for i in range(cfg.n):
        b = int(bits[i])
        f = O.encode(G, csr, i)
        inv, L = O.inv16(scales[i], b), O.levels(b)
        unit = float(scales[i]) / L
        m0 = min(max(0, int(np.argmax(np.abs(f))) - 100), cfg.d - 1500)   # the window holds |f| = max|f|
        win = f[m0:m0 + 1500]
        tot, clamped = 0.0, 0
        for x in win:
            lo, pu = O.quantize_prob(x, inv, b)
            up = min(lo + 1, L)
            clamped += lo >= L
            mean = unit * ((1 - pu) * lo + pu * up)
            tot += (1 - pu) * (unit * lo - mean) ** 2 + pu * (unit * up - mean) ** 2
        if scale_mode == O.SCALE_MAXABS:
            assert clamped >= 1
        ss, vq = O.worker_moments(G[:, m0:m0 + 1500], csr, i, b, scales[i])
        assert ss == pytest.approx(float(np.sum(win.astype(np.float64) ** 2)), rel=1e-13)
        assert vq == pytest.approx(tot, rel=1e-11)
    with pytest.raises(ValueError):
        O.worker_moments(G, csr, 0, 1, 1.0)


@pytest.mark.parametrize("scale_mode", [O.SCALE_MAXABS, O.SCALE_L2])
def test_montecarlo_unbiased_and_residual(scale_mode):
    cfg, p, bits, csr, w, G = _setup(scale_mode)
    T = cfg.iters
    g = G.astype(np.float64).sum(axis=0)
    mean_exact, V = _exact_error(cfg, G, csr, bits, w, p, scale_mode)
    assert np.allclose(mean_exact, g, rtol=0, atol=1e-5)          # the code is unbiased
    rng = np.random.default_rng(77)
    dirs = rng.standard_normal((8, cfg.d))
    dirs /= np.linalg.norm(dirs, axis=1, keepdims=True)
    proj = np.zeros((T, 8))
    sq = np.zeros(T)
    acc = np.zeros(cfg.d)
    batch_means = []
    bacc = np.zeros(cfg.d)
    for t in range(T):
        mask = I.arrival_mask(cfg, p, t)
        _, _, gh = O.step(G, csr, bits, w, mask, cfg.philox_seed, t, scale_mode)
        e = gh.astype(np.float64) - g
        proj[t] = dirs @ e
        sq[t] = e @ e
        acc += e
        bacc += e
        if (t + 1) % 50 == 0:
            batch_means.append(float((bacc / 50) @ (bacc / 50)))
            bacc[:] = 0
    # (i) projections of the mean error on fixed directions: within 3 standard errors of 0
    z = proj.mean(axis=0) / (proj.std(axis=0, ddof=1) / np.sqrt(T))
    assert np.all(np.abs(z) < 3.0), z
    # (ii) residual error E||g_hat - g||^2 against the exact expression
    se = sq.std(ddof=1) / np.sqrt(T)
    assert abs(sq.mean() - V) < 3.0 * se, (sq.mean(), V, se)
    # (iii) the error of a 50-iteration average shrinks like V/50
    bm = np.array(batch_means)
    assert abs(bm.mean() - V / 50) < 3.0 * bm.std(ddof=1) / np.sqrt(len(bm)), (bm.mean(), V / 50)
    # arrival frequencies follow 1 - p_i
    arr = np.array([I.arrival_mask(cfg, p, t) for t in range(T)]).mean(axis=0)
    assert np.all(np.abs(arr - (1 - p)) < 4 * np.sqrt(p * (1 - p) / T))
