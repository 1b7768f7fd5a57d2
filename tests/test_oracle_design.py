"""Pins of the oracle's host-side design maths: code structure (Sec. III-A), bit allocation
(Sec. III-B), error bounds (Lemmas 1 and 2), second-moment decoder (Sec. V-E).  CPU only."""
import numpy as np
import pytest
from scipy import optimize

from oracle import agc_oracle as O
from oracle import design as D


def _rand_instance(rng, n, zmax=8):
    p = rng.uniform(0.05, 0.6, n)
    z = rng.integers(2, zmax + 1, n)
    return p, z


# ------------------------------------------------------------------ Theorem 1 / construction
@pytest.mark.parametrize("n,k", [(3, 3), (5, 8), (8, 5), (10, 10), (64, 64)])
def test_interval_code_structure(n, k):
    rng = np.random.default_rng(n * 100 + k)
    p, z = _rand_instance(rng, n)
    c = D.c_weights(p, z, 0.3)
    Y = D.row_targets(c, k)
    assert Y.sum() == pytest.approx(k, rel=1e-13)            # sum_i Y_i = #partitions
    assert np.all(Y > 0)
    alpha = D.interval_code(Y, k)
    assert np.all(alpha >= 0)
    assert np.allclose(alpha.sum(axis=0), 1.0, atol=1e-12)   # unbiasedness: column sums 1
    assert np.allclose(alpha.sum(axis=1), Y, atol=1e-12)     # optimal structure: row sums Y_i
    assert np.count_nonzero(alpha) <= n + k - 1              # sparsity of the construction
    assert np.count_nonzero(alpha) / k <= 1 + (n - 1) / k + 1e-12   # computation load
    # objective at the optimum equals k^2 / sum c^-1 (proofs of Theorem 1 and Lemma 2)
    assert D.csp2_objective(c, alpha) == pytest.approx(k * k / np.sum(1 / c), rel=1e-12)
    B, w = D.physical_code(alpha, p)
    assert D.unbiased_residual(B, w, p) < 1e-12
    # each row's support is one contiguous run of partitions
    for i in range(n):
        nz = np.nonzero(alpha[i])[0]
        assert nz.size >= 1 and np.array_equal(nz, np.arange(nz[0], nz[-1] + 1))


def test_homogeneous_gives_identity():
    alpha = D.interval_code(D.row_targets(D.c_weights([0.2] * 6, [4] * 6, 0.1), 6), 6)
    assert np.allclose(alpha, np.eye(6), atol=1e-12)


def test_row_targets_solve_csp2_numerically():
    """The closed form against a numerical solve of c-SP2 (minimise sum_i c_i (sum_j alpha_ij)^2
    subject to unit column sums) with a generic constrained optimiser."""
    rng = np.random.default_rng(7)
    n, k = 4, 3
    p, z = _rand_instance(rng, n)
    c = D.c_weights(p, z, 0.2)

    def obj(a):
        return float(np.sum(c * a.reshape(n, k).sum(axis=1) ** 2))

    cons = [{"type": "eq", "fun": (lambda a, j=j: a.reshape(n, k)[:, j].sum() - 1.0)} for j in range(k)]
    res = optimize.minimize(obj, np.full(n * k, 1.0 / n), constraints=cons, method="SLSQP",
                            options={"ftol": 1e-14, "maxiter": 500})
    assert res.success
    assert np.allclose(res.x.reshape(n, k).sum(axis=1), D.row_targets(c, k), atol=1e-5)
    assert res.fun == pytest.approx(k * k / np.sum(1 / c), rel=1e-8)
    # any other feasible point is no better: the interval code and a perturbed one
    alpha = D.interval_code(D.row_targets(c, k), k)
    pert = alpha.copy()
    pert[0, 0] += 0.05
    pert[1, 0] -= 0.05
    assert D.csp2_objective(c, pert) > D.csp2_objective(c, alpha)


def test_cyclic_code_is_unbiased_on_its_support():
    rng = np.random.default_rng(9)
    for n, s in [(4, 2), (16, 3), (64, 4)]:
        p, z = _rand_instance(rng, n)
        c = D.c_weights(p, z, 0.3)
        alpha, supp = D.cyclic_code(c, n, s)
        assert np.allclose(alpha.sum(axis=0), 1.0, atol=1e-12)
        assert all(np.count_nonzero(alpha[i]) == s for i in range(n))
        assert supp[n - 1] == [(n - 1 + u) % n for u in range(s)]
        B, w = D.physical_code(alpha, p)
        assert D.unbiased_residual(B, w, p) < 1e-12
        # a heuristic: never better than the optimal structure
        assert D.csp2_objective(c, alpha) >= n * n / np.sum(1 / c) * (1 - 1e-12)


# ------------------------------------------------------------------ bounds
def test_lemma_bounds_dominate_exact_error():
    """exact E||g - g_hat||^2 <= Lemma 1 bound; with the optimal structure Lemma 1's bound
    equals Lemma 2's closed form (Euclidean-norm scale, phi with the true dimension)."""
    rng = np.random.default_rng(11)
    n = k = 6
    d = 400
    p, z = _rand_instance(rng, n)
    z = z.astype(np.uint8)
    pc = D.phi_coef_paper(d)
    c = D.c_weights(p, z, pc)
    alpha = D.interval_code(D.row_targets(c, k), k)
    B, w = D.physical_code(alpha, p)
    csr = O.Csr.from_dense(B.astype(np.float32))
    G = rng.standard_normal((k, d)).astype(np.float32)
    Cg = float(np.max(np.sum(G.astype(np.float64) ** 2, axis=1)))
    f = np.array([O.encode(G, csr, i) for i in range(n)], dtype=np.float64)
    var_q = []
    for i in range(n):
        sc = O.scale_l2(f[i].astype(np.float32))
        inv = O.inv16(sc, int(z[i]))
        L = O.levels(int(z[i]))
        tot = 0.0
        for x in f[i].astype(np.float32):
            lo, pu = O.quantize_prob(x, inv, int(z[i]))
            tot += (float(sc) / L) ** 2 * pu * (1 - pu)
        var_q.append(tot)
        assert tot <= float(D.phi(z[i], pc)) * float(np.sum(f[i] ** 2)) * (1 + 1e-9)
    _, err = D.exact_moments(f, var_q, w, p)
    b1 = D.lemma1_bound(Cg, p, z, pc, w, B)
    b2 = D.lemma2_bound(Cg, c, k)
    assert err <= b1 * (1 + 1e-9)
    assert b1 == pytest.approx(b2, rel=1e-9)


# ------------------------------------------------------------------ bit allocation
def test_dp_equals_bruteforce():
    rng = np.random.default_rng(13)
    for trial in range(30):
        n = int(rng.integers(2, 6))
        z_res = int(rng.integers(0, 9))
        p = rng.uniform(0.02, 0.7, n)
        pc = 10 ** rng.uniform(-2, 2)
        cap = None if trial % 2 else 6
        r_dp, f_dp = D.alloc_dp(p, pc, z_res, cap)
        r_bf, f_bf = D.alloc_bruteforce(p, pc, z_res, cap)
        assert f_dp == pytest.approx(f_bf, rel=1e-13)
        assert r_dp.sum() == z_res and np.all(r_dp >= 0)
        assert D.objective(p, r_dp, pc) == pytest.approx(f_dp, rel=1e-13)


def test_lowcomplexity_feasible_and_near_optimal():
    """Algorithm 1 never beats the DP optimum and stays within 0.1 % of it on random
    instances (the paper reports it as consistently matching the optimum, Sec. VI)."""
    rng = np.random.default_rng(17)
    worst = 1.0
    for trial in range(25):
        n = int(rng.integers(3, 13))
        z_res = int(rng.integers(1, 4 * n))
        p = rng.uniform(0.05, 0.6, n)
        z_tot = z_res + 2 * n
        pc = D.phi_coef_balanced(p, z_tot) if trial % 2 else 10 ** rng.uniform(-1, 2)
        cap = 6
        if n * cap < z_res:
            continue
        r, f = D.alloc_lowcomplexity(p, pc, z_res, cap)
        r_dp, f_dp = D.alloc_dp(p, pc, z_res, cap)
        assert r.sum() == z_res and np.all(r >= 0) and np.all(r <= cap)
        assert D.objective(p, r, pc) == pytest.approx(f, rel=1e-12)
        assert f <= f_dp * (1 + 1e-12)
        worst = min(worst, f / f_dp)
    assert worst >= 1 - 1e-3


def test_utility_monotone_in_p():
    # dh/dp < 0: more reliable workers contribute more (Sec. III-B.2)
    for r in range(0, 7):
        hs = [D.utility(p, r, 0.5) for p in np.linspace(0.01, 0.9, 30)]
        assert all(a > b for a, b in zip(hs, hs[1:]))


# ------------------------------------------------------------------ two-track decoder
def test_second_moment_decoder_minimises_objective():
    rng = np.random.default_rng(19)
    n = k = 5
    p, z = _rand_instance(rng, n)
    c = D.c_weights(p, z, 0.4)
    alpha = D.interval_code(D.row_targets(c, k), k)
    B, w = D.physical_code(alpha, p)
    for Lam in (0.1, 1.0, 10.0):
        v = D.second_moment_decoder(p, z, 0.4, B, Lam)
        m0 = D.second_moment_objective(v, p, z, 0.4, B, Lam)
        res = optimize.minimize(lambda x: D.second_moment_objective(x, p, z, 0.4, B, Lam), w,
                                method="BFGS", options={"gtol": 1e-12})
        assert m0 <= res.fun * (1 + 1e-6)
        assert m0 <= D.second_moment_objective(w, p, z, 0.4, B, Lam)      # beats the unbiased decoder
        for _ in range(20):
            assert m0 <= D.second_moment_objective(v + 1e-3 * rng.standard_normal(n), p, z, 0.4, B, Lam)


# ------------------------------------------------------------------ optimum on a prescribed cyclic support
def _kkt_gap(c, alpha, supp, k):
    """Optimality conditions of the support-restricted problem: inside every column the
    holders that carry weight share the smallest marginal cost 2 c_i r_i."""
    r = alpha.sum(axis=1)
    worst = 0.0
    for j in range(k):
        holders = [i for i in range(len(c)) if j in supp[i]]
        m = np.array([2 * c[i] * r[i] for i in holders])
        a = np.array([alpha[i, j] for i in holders])
        lo = m.min()
        worst = max(worst, float(np.max((m - lo) * (a > 1e-7)) / max(lo, 1e-300)))
    return worst


def test_cyclic_optimum_full_support_reaches_theorem_1():
    rng = np.random.default_rng(31)
    n = k = 6
    p, z = _rand_instance(rng, n)
    c = D.c_weights(p, z, 0.4)
    ok, a_lp = D.cyclic_row_sum_feasible(c, k, k)          # s = k: every worker may hold everything
    assert ok
    assert np.allclose(a_lp.sum(axis=1), D.row_targets(c, k), atol=1e-9)
    assert np.allclose(a_lp.sum(axis=0), 1.0, atol=1e-9)
    a_qp, supp = D.cyclic_code_optimal(c, k, k)
    best = k * k / np.sum(1.0 / c)                          # Lemma 2 / Theorem 1 value
    assert abs(D.csp2_objective(c, a_qp) - best) <= 1e-8 * best
    assert abs(D.csp2_objective(c, a_lp) - best) <= 1e-9 * best


def test_cyclic_optimum_equal_workers_is_uniform():
    n = k = 8
    c = np.full(n, 0.7)
    for s in (1, 2, 3):
        a, supp = D.cyclic_code_optimal(c, k, s)
        assert np.allclose(a.sum(axis=1), 1.0, atol=1e-7)             # Y_i = 1 for equal workers
        assert abs(D.csp2_objective(c, a) - n * 0.7) <= 1e-9 * n


def test_cyclic_optimum_narrow_band_is_between_bound_and_heuristic_and_satisfies_kkt():
    rng = np.random.default_rng(32)
    hit_infeasible = False
    for trial in range(6):
        n = k = 10
        s = 2 + trial % 2
        p = rng.uniform(0.02, 0.7, n)
        z = rng.integers(2, 9, n)
        c = D.c_weights(p, z, 0.4)
        a, supp = D.cyclic_code_optimal(c, k, s)
        assert np.allclose(a.sum(axis=0), 1.0, atol=1e-9) and a.min() >= 0
        for i in range(n):
            assert all(a[i, j] == 0 for j in range(k) if j not in supp[i])
        obj = D.csp2_objective(c, a)
        bound = k * k / np.sum(1.0 / c)
        heur = D.csp2_objective(c, D.cyclic_code(c, k, s)[0])
        assert bound * (1 - 1e-9) <= obj <= heur * (1 + 1e-9)
        assert _kkt_gap(c, a, supp, k) < 1e-5
        ok, _ = D.cyclic_row_sum_feasible(c, k, s)
        if ok:
            assert abs(obj - bound) <= 1e-7 * bound
        else:
            hit_infeasible = True
            assert obj > bound * (1 + 1e-6)
    assert hit_infeasible                                     # the narrow band does bind somewhere
