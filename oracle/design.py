"""Oracle for the host-side design maths of the scheme, binary64 / numpy.

TEST INFRASTRUCTURE (see agc_oracle.c).  Everything here is the paper's formula
written out; nothing is shared with the product's C++ host routines.

Symbols: n workers, k partitions (the paper swaps the two letters), p_i the
straggling probabilities, z_i the bit-widths, r_i = z_i - z_min the residual
bits, phi(z) = phi_coef / (2^(z-1) - 1)^2 with phi_coef = l/4 in the paper
(Sec. II-B) or eta*l/4 with the error-balance factor of Sec. V-B.
"""
import itertools
import math

import numpy as np


# ----------------------------------------------------------------------------
# quantization-variance constant and worker utility  (Sec. II-B, Sec. III-B)
# ----------------------------------------------------------------------------
def phi(z, phi_coef):
    return phi_coef / (2.0 ** (np.asarray(z, dtype=np.float64) - 1.0) - 1.0) ** 2


def phi_coef_paper(l):
    """phi(z) = l / (4 (2^(z-1)-1)^2)   (Sec. II-B)."""
    return l / 4.0


def phi_coef_balanced(p, z_tot):
    """Error-balance scaling of Sec. V-B: eta = mean(p) * 4 (2^(Z_tot/n - 1) - 1)^2 / l,
    so eta * l / 4 = mean(p) * (2^(Z_tot/n - 1) - 1)^2."""
    p = np.asarray(p, dtype=np.float64)
    return float(np.mean(p)) * (2.0 ** (z_tot / len(p) - 1.0) - 1.0) ** 2


def c_weights(p, z, phi_coef):
    """c_i = (p_i + phi(z_i)) / (1 - p_i)   (Sec. III-A; with Sec. V-B's eta folded
    into phi_coef this is p/(1-p) + eta*phi/(1-p))."""
    p = np.asarray(p, dtype=np.float64)
    return (p + phi(z, phi_coef)) / (1.0 - p)


def utility(p_i, r, phi_coef, z_min=2):
    """h_i(r) = (1-p_i) / (p_i + phi(r + z_min))   (problem b-SP1)."""
    return (1.0 - p_i) / (p_i + phi(r + z_min, phi_coef))


def objective(p, r, phi_coef, z_min=2):
    """F(r) = sum_i h_i(r_i)."""
    return float(sum(utility(pi, ri, phi_coef, z_min) for pi, ri in zip(p, r)))


# ----------------------------------------------------------------------------
# bit allocation  (Sec. III-B)
# ----------------------------------------------------------------------------
def alloc_bruteforce(p, phi_coef, z_res, r_max=None, z_min=2):
    """Global optimum of b-SP1 by enumerating every composition (tiny n only)."""
    n = len(p)
    cap = z_res if r_max is None else r_max
    best, best_r = -math.inf, None
    for r in itertools.product(range(0, min(cap, z_res) + 1), repeat=n):
        if sum(r) != z_res:
            continue
        f = objective(p, r, phi_coef, z_min)
        if f > best:
            best, best_r = f, r
    return (None if best_r is None else np.array(best_r)), best


def alloc_dp(p, phi_coef, z_res, r_max=None, z_min=2):
    """Bellman recurrence V[i,r] = max_{0<=a<=r} V[i-1,r-a] + h_i(a), V[0,0]=0,
    V[0,r>0] = -inf (Sec. III-B.1).  r_max caps a single worker (the paper has no
    cap; None reproduces it)."""
    n = len(p)
    cap = z_res if r_max is None else r_max
    V = np.full((n + 1, z_res + 1), -np.inf)
    arg = np.zeros((n + 1, z_res + 1), dtype=np.int64)
    V[0, 0] = 0.0
    for i in range(1, n + 1):
        for r in range(z_res + 1):
            for a in range(0, min(r, cap) + 1):
                v = V[i - 1, r - a] + utility(p[i - 1], a, phi_coef, z_min)
                if v > V[i, r]:
                    V[i, r], arg[i, r] = v, a
    if not np.isfinite(V[n, z_res]):
        return None, -math.inf
    r_out = np.zeros(n, dtype=np.int64)
    rem = z_res
    for i in range(n, 0, -1):
        r_out[i - 1] = arg[i, rem]
        rem -= arg[i, rem]
    return r_out, float(V[n, z_res])


def _dutility(p_i, r, phi_coef, z_min=2):
    """d h_i / d r for real r: with x = 2^(r+z_min-1) - 1,
    h = (1-p) x^2 / (p x^2 + A),  dh/dx = (1-p) 2 x A / (p x^2 + A)^2,  dx/dr = ln2 (x+1)."""
    x = 2.0 ** (r + z_min - 1.0) - 1.0
    return (1.0 - p_i) * 2.0 * phi_coef * x * (x + 1.0) * math.log(2.0) / (p_i * x * x + phi_coef) ** 2


def _concave_root(p_i, lam, phi_coef, r_cap, z_min=2):
    """Largest r in [0, r_cap] with h_i'(r) = lam (the root on the concave branch of the
    sigmoid), r_cap if h_i' is still above lam there, 0 if h_i' never reaches lam."""
    grid = np.linspace(0.0, r_cap, 257)
    vals = np.array([_dutility(p_i, r, phi_coef, z_min) for r in grid])
    top = int(np.argmax(vals))
    if vals[top] < lam:
        return 0.0
    if _dutility(p_i, r_cap, phi_coef, z_min) >= lam:
        return float(r_cap)
    lo, hi = grid[top], float(r_cap)
    for _ in range(80):
        mid = 0.5 * (lo + hi)
        if _dutility(p_i, mid, phi_coef, z_min) >= lam:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def _round_to_sum(r_real, total, cap):
    """floor, then hand the missing units to the largest remainders (ties: lowest index)."""
    r = np.minimum(np.floor(r_real + 1e-12).astype(np.int64), cap)
    rem = r_real - r
    missing = int(total - r.sum())
    order = sorted(range(len(r)), key=lambda i: (-rem[i], i))
    t = 0
    while missing > 0 and t < 10 * len(r) + 10:
        i = order[t % len(r)]
        if r[i] < cap:
            r[i] += 1
            missing -= 1
        t += 1
    while missing < 0:
        i = int(np.argmax(r))
        r[i] -= 1
        missing += 1
    return r


def alloc_lowcomplexity(p, phi_coef, z_res, r_max=None, z_min=2):
    """Algorithm 1 (Sec. III-B.2) under this build's reading of the steps the paper
    leaves open: Lagrangian candidate = continuous relaxation on the top-kappa set solved
    by bisection on the multiplier, each worker on the concave branch, rounded by
    largest remainder; equal candidate = floor(Z/kappa) each, the most reliable
    Z mod kappa workers one more; one-bit local search = best-improvement swaps inside
    the active set until no swap has positive gain."""
    p = np.asarray(p, dtype=np.float64)
    n = len(p)
    cap = z_res if r_max is None else r_max
    order = sorted(range(n), key=lambda i: (p[i], i))
    best_f, best_r = -math.inf, None
    for kappa in range(1, min(n, z_res) + 1):
        if kappa * cap < z_res:
            continue
        S = order[:kappa]
        # equal allocation
        r_eq = np.full(kappa, z_res // kappa, dtype=np.int64)
        r_eq[: z_res % kappa] += 1
        cands = [r_eq] if r_eq.max() <= cap else []
        # Lagrangian relaxation
        lam_hi = max(max(_dutility(p[i], r, phi_coef, z_min) for r in np.linspace(0, cap, 65))
                     for i in S) * 1.01 + 1e-300
        lam_lo = 0.0
        for _ in range(100):
            lam = 0.5 * (lam_lo + lam_hi)
            tot = sum(_concave_root(p[i], lam, phi_coef, cap, z_min) for i in S)
            if tot > z_res:
                lam_lo = lam
            else:
                lam_hi = lam
        r_real = np.array([_concave_root(p[i], lam_hi, phi_coef, cap, z_min) for i in S])
        cands.append(_round_to_sum(r_real, z_res, cap))
        best_c, best_cf = None, -math.inf
        for c in cands:
            if c.sum() != z_res:
                continue
            f = sum(utility(p[i], ri, phi_coef, z_min) for i, ri in zip(S, c))
            if f > best_cf:
                best_c, best_cf = c.copy(), f
        if best_c is None:
            continue
        # one-bit swaps
        for _ in range(100000):
            gain_best, pair = 0.0, None
            for a in range(kappa):
                if best_c[a] >= cap:
                    continue
                up = utility(p[S[a]], best_c[a] + 1, phi_coef, z_min) - utility(p[S[a]], best_c[a], phi_coef, z_min)
                for b in range(kappa):
                    if b == a or best_c[b] < 1:
                        continue
                    down = utility(p[S[b]], best_c[b] - 1, phi_coef, z_min) - utility(p[S[b]], best_c[b], phi_coef, z_min)
                    if up + down > gain_best:
                        gain_best, pair = up + down, (a, b)
            if pair is None:
                break
            best_c[pair[0]] += 1
            best_c[pair[1]] -= 1
        f = sum(utility(p[i], ri, phi_coef, z_min) for i, ri in zip(S, best_c))
        # workers outside the active set keep r = 0 and still contribute h_i(0)
        f += sum(utility(p[i], 0, phi_coef, z_min) for i in order[kappa:])
        if f > best_f:
            best_f = f
            best_r = np.zeros(n, dtype=np.int64)
            for i, ri in zip(S, best_c):
                best_r[i] = ri
    return best_r, best_f


# ----------------------------------------------------------------------------
# code structure  (Sec. III-A)
# ----------------------------------------------------------------------------
def row_targets(c, k):
    """Theorem 1: Y_i = c_i^{-1} * k / sum_m c_m^{-1}  (k = number of partitions)."""
    inv = 1.0 / np.asarray(c, dtype=np.float64)
    return inv * k / inv.sum()


def interval_code(Y, k):
    """Sparse construction of Sec. III-A: R_i = sum_{m<=i} Y_m and
    alpha_i^j = [min(R_i, j) - max(R_{i-1}, j-1)]_+ for partitions j = 1..k."""
    n = len(Y)
    R = np.concatenate([[0.0], np.cumsum(np.asarray(Y, dtype=np.float64))])
    R[n] = float(k)
    alpha = np.zeros((n, k))
    for i in range(1, n + 1):
        for j in range(1, k + 1):
            alpha[i - 1, j - 1] = max(min(R[i], j) - max(R[i - 1], j - 1), 0.0)
    return alpha


def cyclic_support(n, k, s):
    """supp(i) = {i, i+1, ..., i+s-1 mod k} in that order (replication factor s)."""
    return [[(i + u) % k for u in range(s)] for i in range(n)]


def cyclic_code(c, k, s):
    """Column-normalised weights on the cyclic support: alpha_i^j = c_i^{-1} / sum of
    c^{-1} over the workers that hold j.  Satisfies the unbiasedness condition exactly;
    it is a heuristic on a prescribed support, not Theorem 1's optimum."""
    n = len(c)
    inv = 1.0 / np.asarray(c, dtype=np.float64)
    supp = cyclic_support(n, k, s)
    colsum = np.zeros(k)
    for i in range(n):
        for j in supp[i]:
            colsum[j] += inv[i]
    alpha = np.zeros((n, k))
    for i in range(n):
        for j in supp[i]:
            alpha[i, j] = inv[i] / colsum[j]
    return alpha, supp


def cyclic_row_sum_feasible(c, k, s):
    """Is Theorem 1's structure reachable on the cyclic support?  Linear feasibility of
    alpha >= 0 on the support with row sums Y_i and column sums 1 (a transportation problem),
    decided with a library LP solver.  Returns (feasible, alpha or None)."""
    from scipy.optimize import linprog
    n = len(c)
    supp = cyclic_support(n, k, s)
    Y = row_targets(c, k)
    nv = n * s
    A_eq = np.zeros((n + k, nv))
    b_eq = np.concatenate([Y, np.ones(k)])
    for i in range(n):
        for u, j in enumerate(supp[i]):
            A_eq[i, i * s + u] = 1.0
            A_eq[n + j, i * s + u] = 1.0
    res = linprog(np.zeros(nv), A_eq=A_eq, b_eq=b_eq, bounds=[(0, None)] * nv, method="highs")
    if res.status != 0:
        return False, None
    alpha = np.zeros((n, k))
    for i in range(n):
        for u, j in enumerate(supp[i]):
            alpha[i, j] = res.x[i * s + u]
    return True, alpha


def cyclic_code_optimal(c, k, s):
    """Problem c-SP2 restricted to the cyclic support: minimise sum_i c_i (sum_j alpha_i^j)^2
    subject to column sums 1, alpha >= 0, alpha = 0 off the support.  The objective depends on
    the row sums only, so it is a convex quadratic programme in them; solved here with a
    library routine (SLSQP from the column-normalised start, analytic gradient).  When the row
    sums of Theorem 1 are reachable the minimum is k^2 / sum c^-1."""
    from scipy.optimize import minimize
    c = np.asarray(c, dtype=np.float64)
    n = len(c)
    supp = cyclic_support(n, k, s)
    a0, _ = cyclic_code(c, k, s)
    x0 = np.array([a0[i, j] for i in range(n) for j in supp[i]])
    cols = np.array([j for i in range(n) for j in supp[i]])
    rows = np.repeat(np.arange(n), s)

    def f(x):
        r = np.bincount(rows, weights=x, minlength=n)
        return float(np.sum(c * r * r))

    def g(x):
        r = np.bincount(rows, weights=x, minlength=n)
        return 2.0 * (c * r)[rows]

    Ac = np.zeros((k, n * s))
    Ac[cols, np.arange(n * s)] = 1.0
    res = minimize(f, x0, jac=g, method="SLSQP", bounds=[(0.0, None)] * (n * s),
                   constraints=[{"type": "eq", "fun": lambda x: Ac @ x - 1.0, "jac": lambda x: Ac}],
                   options={"ftol": 1e-15, "maxiter": 2000})
    alpha = np.zeros((n, k))
    alpha[rows, cols] = np.maximum(res.x, 0.0)
    return alpha, supp


def physical_code(alpha, p):
    """a_ij = alpha_i^j / w~_i, w_i = w~_i / (1 - p_i) with the free w~_i := 1."""
    p = np.asarray(p, dtype=np.float64)
    return alpha.copy(), 1.0 / (1.0 - p)


def unbiased_residual(B, w, p):
    """max_j | sum_i (1-p_i) w_i a_ij - 1 |   (unbiasedness condition, Sec. III)."""
    p = np.asarray(p, dtype=np.float64)
    return float(np.max(np.abs(((1.0 - p) * np.asarray(w, dtype=np.float64)) @ np.asarray(B, dtype=np.float64) - 1.0)))


def csp2_objective(c, alpha):
    """sum_i c_i (sum_j alpha_i^j)^2   (problem c-SP2)."""
    return float(np.sum(np.asarray(c) * alpha.sum(axis=1) ** 2))


def lemma1_bound(Cg, p, z, phi_coef, w, B):
    """C * sum_i (1-p_i) (p_i + phi(z_i)) w_i^2 (sum_j a_ij)^2   (Lemma 1)."""
    p = np.asarray(p, dtype=np.float64)
    return float(Cg * np.sum((1 - p) * (p + phi(z, phi_coef)) * np.asarray(w) ** 2 * np.asarray(B).sum(axis=1) ** 2))


def lemma2_bound(Cg, c, k):
    """k^2 C / sum_i c_i^{-1}   (Lemma 2)."""
    return float(k * k * Cg / np.sum(1.0 / np.asarray(c)))


def second_moment_decoder(p, z, phi_coef, B, Lam):
    """Two-track decoding (Sec. V-E): v_i = k Lam / ((p_i+phi_i) (sum_j a_ij) (1 + Lam sum_m c_m^-1))."""
    p = np.asarray(p, dtype=np.float64)
    k = np.asarray(B).shape[1]
    ph = phi(z, phi_coef)
    c = (p + ph) / (1 - p)
    return k * Lam / ((p + ph) * np.asarray(B).sum(axis=1) * (1.0 + Lam * np.sum(1.0 / c)))


def second_moment_objective(v, p, z, phi_coef, B, Lam):
    """Lam [sum_j (1 - sum_i (1-p_i) v_i a_ij)]^2 + sum_i (1-p_i)(p_i+phi_i) v_i^2 (sum_j a_ij)^2."""
    p = np.asarray(p, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    bias = np.sum(1.0 - ((1 - p) * v) @ B)
    var = np.sum((1 - p) * (p + phi(z, phi_coef)) * v ** 2 * B.sum(axis=1) ** 2)
    return float(Lam * bias ** 2 + var)


# ----------------------------------------------------------------------------
# exact first and second moments of the estimator (proof of Lemma 1, before bounding)
# ----------------------------------------------------------------------------
def exact_moments(f, var_q, w, p):
    """f: (n, d) coded gradients (binary64), var_q[i] = E||Q_i(f_i) - E Q_i(f_i)||^2.
    Returns E[g_hat] and E||g_hat - E g_hat||^2 under independent Bernoulli arrivals:
      E g_hat = sum_i (1-p_i) w_i f_i
      E||.||^2 = sum_i (1-p_i) w_i^2 ( p_i ||f_i||^2 + var_q_i )."""
    f = np.asarray(f, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    p = np.asarray(p, dtype=np.float64)
    mean = ((1 - p) * w) @ f
    err = float(np.sum((1 - p) * w ** 2 * (p * np.sum(f * f, axis=1) + np.asarray(var_q))))
    return mean, err
