// Host-side design routines of the scheme: bit allocation (Sec. III-B) and code construction
// (Sec. III-A).  They run once per change of the system statistics and touch no GPU state.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <numeric>
#include <vector>

#include "../../include/agc.h"

namespace {

// phi(z) = phi_coef / (2^(z-1) - 1)^2 for real z  (Sec. II-B, variance constant)
inline double phi_of(double z, double phi_coef)
{
    const double x = std::exp2(z - 1.0) - 1.0;
    return phi_coef / (x * x);
}

// h_i(z) = (1 - p_i) / (p_i + phi(z))  (utility of worker i in problem b-SP1)
inline double util(double p, double z, double phi_coef) { return (1.0 - p) / (p + phi_of(z, phi_coef)); }

// derivative of h_i with respect to z:  x = 2^(z-1)-1, h = (1-p) x^2 / (p x^2 + A),
// dh/dx = 2 (1-p) A x / (p x^2 + A)^2, dx/dz = ln2 (x + 1)
inline double dutil(double p, double z, double A)
{
    const double x = std::exp2(z - 1.0) - 1.0;
    const double den = p * x * x + A;
    return 2.0 * (1.0 - p) * A * x * (x + 1.0) * M_LN2 / (den * den);
}

struct Problem {
    int n;
    const double* p;
    double A;  // phi_coef
    int zmin, zmax;
};

// h_i' rises then falls in z (sigmoid utility).  Largest z in [zmin, zmax] with h_i'(z) = lam:
// the stationary point of the relaxation on the concave branch.  zmax when the slope is still
// above lam there, zmin when the slope never reaches lam.
double concave_root(const Problem& P, int i, double lam)
{
    const int G = 256;
    double best = -1.0, zbest = P.zmin;
    for (int t = 0; t <= G; ++t) {
        const double z = P.zmin + (P.zmax - P.zmin) * (double)t / G;
        const double v = dutil(P.p[i], z, P.A);
        if (v > best) { best = v; zbest = z; }
    }
    if (best < lam) return P.zmin;
    if (dutil(P.p[i], P.zmax, P.A) >= lam) return P.zmax;
    double lo = zbest, hi = P.zmax;
    for (int it = 0; it < 80; ++it) {
        const double mid = 0.5 * (lo + hi);
        if (dutil(P.p[i], mid, P.A) >= lam) lo = mid; else hi = mid;
    }
    return 0.5 * (lo + hi);
}

double objective_subset(const Problem& P, const std::vector<int>& S, const std::vector<int>& z)
{
    double f = 0.0;
    for (size_t a = 0; a < S.size(); ++a) f += util(P.p[S[a]], z[a], P.A);
    return f;
}

}  // namespace

extern "C" {

double agc_phi_coef_balanced(int n, const double* p, int z_total)
{
    if (n <= 0 || !p) return 0.0;
    double mean = 0.0;
    for (int i = 0; i < n; ++i) mean += p[i];
    mean /= n;
    const double x = std::exp2((double)z_total / n - 1.0) - 1.0;
    return mean * x * x;
}

double agc_alloc_objective(int n, const double* p, double phi_coef, const uint8_t* bits)
{
    double f = 0.0;
    for (int i = 0; i < n; ++i) f += util(p[i], bits[i], phi_coef);
    return f;
}

static agc_status check_alloc_args(int n, const double* p, int z_total, int z_min, int z_max,
                                   const uint8_t* out)
{
    if (!p || !out || n <= 0) return AGC_EINVAL;
    if (z_min < 2 || z_max < z_min || z_max > AGC_MAX_BITS) return AGC_EBITS;
    if (z_total < (int64_t)n * z_min || z_total > (int64_t)n * z_max) return AGC_EBITS;
    for (int i = 0; i < n; ++i)
        if (!(p[i] >= 0.0 && p[i] < 1.0)) return AGC_EINVAL;
    return AGC_OK;
}

agc_status agc_alloc_bits_dp(int n, const double* p, double phi_coef, int z_total, int z_min,
                             int z_max, uint8_t* bits_out)
{
    agc_status st = check_alloc_args(n, p, z_total, z_min, z_max, bits_out);
    if (st != AGC_OK) return st;
    const int zres = z_total - n * z_min, cap = z_max - z_min;
    const double NEG = -std::numeric_limits<double>::infinity();
    // V[i][r]: best utility of workers 1..i with residual budget r  (Bellman recurrence)
    std::vector<std::vector<double>> V(n + 1, std::vector<double>(zres + 1, NEG));
    std::vector<std::vector<int>> arg(n + 1, std::vector<int>(zres + 1, 0));
    V[0][0] = 0.0;
    for (int i = 1; i <= n; ++i)
        for (int r = 0; r <= zres; ++r)
            for (int a = 0; a <= std::min(r, cap); ++a) {
                if (V[i - 1][r - a] == NEG) continue;
                const double v = V[i - 1][r - a] + util(p[i - 1], z_min + a, phi_coef);
                if (v > V[i][r]) { V[i][r] = v; arg[i][r] = a; }
            }
    if (V[n][zres] == NEG) return AGC_EBITS;
    int rem = zres;
    for (int i = n; i >= 1; --i) {
        bits_out[i - 1] = (uint8_t)(z_min + arg[i][rem]);
        rem -= arg[i][rem];
    }
    return AGC_OK;
}

agc_status agc_alloc_bits(int n, const double* p, double phi_coef, int z_total, int z_min,
                          int z_max, uint8_t* bits_out)
{
    agc_status st = check_alloc_args(n, p, z_total, z_min, z_max, bits_out);
    if (st != AGC_OK) return st;
    const Problem P{n, p, phi_coef, z_min, z_max};
    const int zres = z_total - n * z_min, cap = z_max - z_min;
    // line 1 of Algorithm 1: most reliable workers first
    std::vector<int> order(n);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return p[a] < p[b]; });

    double f_best = -std::numeric_limits<double>::infinity();
    std::vector<int> z_best(n, z_min);
    if (zres == 0) f_best = 0.0;  // nothing to distribute
    for (int kappa = 1; kappa <= std::min(n, zres); ++kappa) {
        if ((int64_t)kappa * cap < zres) continue;  // the active set cannot absorb the budget
        const std::vector<int> S(order.begin(), order.begin() + kappa);
        // (2) equal allocation, the first zres mod kappa workers one bit more
        std::vector<int> z_eq(kappa, z_min + zres / kappa);
        for (int a = 0; a < zres % kappa; ++a) z_eq[a] += 1;
        // (1) Lagrangian relaxation: bisection on the multiplier
        double lam_lo = 0.0, lam_hi = 0.0;
        for (int i : S)
            for (int t = 0; t <= 64; ++t)
                lam_hi = std::max(lam_hi, dutil(p[i], z_min + cap * (double)t / 64, phi_coef));
        lam_hi = lam_hi * 1.01 + 1e-300;
        std::vector<double> zr(kappa);
        for (int it = 0; it < 100; ++it) {
            const double lam = 0.5 * (lam_lo + lam_hi);
            double tot = 0.0;
            for (int a = 0; a < kappa; ++a) tot += concave_root(P, S[a], lam) - z_min;
            if (tot > zres) lam_lo = lam; else lam_hi = lam;
        }
        for (int a = 0; a < kappa; ++a) zr[a] = concave_root(P, S[a], lam_hi) - z_min;
        // round: floor, then largest remainders (ties: more reliable first)
        std::vector<int> z_lag(kappa);
        std::vector<double> rem(kappa);
        int have = 0;
        for (int a = 0; a < kappa; ++a) {
            int fl = std::min((int)std::floor(zr[a] + 1e-12), cap);
            z_lag[a] = z_min + fl;
            rem[a] = zr[a] - fl;
            have += fl;
        }
        std::vector<int> by_rem(kappa);
        std::iota(by_rem.begin(), by_rem.end(), 0);
        std::stable_sort(by_rem.begin(), by_rem.end(), [&](int a, int b) { return rem[a] > rem[b]; });
        for (int t = 0; have < zres && t < 16 * kappa + 16; ++t) {
            const int a = by_rem[t % kappa];
            if (z_lag[a] < z_max) { z_lag[a] += 1; have += 1; }
        }
        while (have > zres) {
            const int a = (int)(std::max_element(z_lag.begin(), z_lag.end()) - z_lag.begin());
            z_lag[a] -= 1;
            have -= 1;
        }
        // (3) hybrid selection
        std::vector<int> z = z_eq;
        double f = *std::max_element(z_eq.begin(), z_eq.end()) <= z_max ? objective_subset(P, S, z_eq)
                                                                       : -std::numeric_limits<double>::infinity();
        if (have == zres) {
            const double fl = objective_subset(P, S, z_lag);
            if (fl > f) { f = fl; z = z_lag; }
        }
        if (!std::isfinite(f)) continue;
        // (4) one-bit local search: best-improvement swaps while some swap has positive gain
        for (int guard = 0; guard < 100000; ++guard) {
            double gain_best = 0.0;
            int ia = -1, ib = -1;
            for (int a = 0; a < kappa; ++a) {
                if (z[a] >= z_max) continue;
                const double up = util(p[S[a]], z[a] + 1, phi_coef) - util(p[S[a]], z[a], phi_coef);
                for (int b = 0; b < kappa; ++b) {
                    if (b == a || z[b] <= z_min) continue;
                    const double down = util(p[S[b]], z[b] - 1, phi_coef) - util(p[S[b]], z[b], phi_coef);
                    if (up + down > gain_best) { gain_best = up + down; ia = a; ib = b; }
                }
            }
            if (ia < 0) break;
            z[ia] += 1;
            z[ib] -= 1;
        }
        f = objective_subset(P, S, z);
        for (int t = kappa; t < n; ++t) f += util(p[order[t]], z_min, phi_coef);  // inactive workers keep z_min
        if (f > f_best) {
            f_best = f;
            std::fill(z_best.begin(), z_best.end(), z_min);
            for (int a = 0; a < kappa; ++a) z_best[S[a]] = z[a];
        }
    }
    if (!std::isfinite(f_best)) return AGC_EBITS;
    for (int i = 0; i < n; ++i) bits_out[i] = (uint8_t)z_best[i];
    return AGC_OK;
}

static agc_status code_weights(int n, const double* p, const uint8_t* bits, double phi_coef,
                               std::vector<double>& cinv)
{
    cinv.resize(n);
    for (int i = 0; i < n; ++i) {
        if (!(p[i] >= 0.0 && p[i] < 1.0)) return AGC_EINVAL;
        if (bits[i] < 2 || bits[i] > AGC_MAX_BITS) return AGC_EBITS;
        const double c = (p[i] + phi_of(bits[i], phi_coef)) / (1.0 - p[i]);
        if (!(c > 0.0) || !std::isfinite(c)) return AGC_EINVAL;
        cinv[i] = 1.0 / c;
    }
    return AGC_OK;
}

agc_status agc_build_code(int n, int k, const double* p, const uint8_t* bits, double phi_coef,
                          int32_t* row_ptr, int32_t* col, float* val, float* w_out, int cap,
                          int* nnz)
{
    if (!p || !bits || !row_ptr || !col || !val || !w_out || !nnz) return AGC_EINVAL;
    if (n <= 0 || k <= 0) return AGC_ESHAPE;
    std::vector<double> cinv;
    agc_status st = code_weights(n, p, bits, phi_coef, cinv);
    if (st != AGC_OK) return st;
    double tot = 0.0;
    for (double v : cinv) tot += v;
    // Theorem 1: target mass of worker i; allocation segment [R_{i-1}, R_i] on the axis [0, k]
    int count = 0;
    double R_prev = 0.0;
    row_ptr[0] = 0;
    for (int i = 0; i < n; ++i) {
        const double Y = cinv[i] * (double)k / tot;
        double R = (i == n - 1) ? (double)k : R_prev + Y;
        // A segment end that should fall on a partition boundary lands a few units in the last
        // place beside it after the running sum; left there it would add an entry of ~1e-16 (one
        // more partition for the worker to compute, one more row in its window).  Ends within
        // 1e-12 * k of an integer are moved onto it; the segments still tile [0, k], so every
        // column still sums to 1.
        const double R_int = std::nearbyint(R);
        if (std::fabs(R - R_int) <= 1e-12 * (double)k) R = R_int;
        // overlap of [R_prev, R] with the unit segment [j-1, j] of partition j (1-based)
        int j_first = (int)std::floor(R_prev) + 1;
        int j_last = std::min(k, (int)std::ceil(R));
        for (int j = j_first; j <= j_last; ++j) {
            const double ov = std::min(R, (double)j) - std::max(R_prev, (double)(j - 1));
            if (ov > 0.0) {
                if (count >= cap) return AGC_ESHAPE;
                col[count] = j - 1;
                val[count] = (float)ov;
                ++count;
            }
        }
        row_ptr[i + 1] = count;
        w_out[i] = (float)(1.0 / (1.0 - p[i]));
        R_prev = R;
    }
    *nnz = count;
    return AGC_OK;
}

agc_status agc_build_cyclic_code(int n, int k, int s, const double* p, const uint8_t* bits,
                                 double phi_coef, int32_t* row_ptr, int32_t* col, float* val,
                                 float* w_out)
{
    if (!p || !bits || !row_ptr || !col || !val || !w_out) return AGC_EINVAL;
    if (n <= 0 || k <= 0 || n != k || s < 1 || s > k) return AGC_ESHAPE;
    std::vector<double> cinv;
    agc_status st = code_weights(n, p, bits, phi_coef, cinv);
    if (st != AGC_OK) return st;
    std::vector<double> colsum(k, 0.0);
    for (int i = 0; i < n; ++i)
        for (int u = 0; u < s; ++u) colsum[(i + u) % k] += cinv[i];
    for (int i = 0; i < n; ++i) {
        row_ptr[i] = i * s;
        for (int u = 0; u < s; ++u) {
            const int j = (i + u) % k;
            col[i * s + u] = j;
            val[i * s + u] = (float)(cinv[i] / colsum[j]);
        }
        w_out[i] = (float)(1.0 / (1.0 - p[i]));
    }
    row_ptr[n] = n * s;
    return AGC_OK;
}

// Problem c-SP2 on the cyclic support {i, .., i+s-1 mod k} (n == k):  minimise
// sum_i c_i r_i^2, r_i = sum_j alpha_i^j, subject to column sums 1 and alpha >= 0.  The objective
// is convex and its constraints are one simplex per column, so exact minimisation over one column
// at a time converges to the optimum.  One column step: with a_i the row sums without this
// column's entries, the unit mass goes to the holders in order of increasing marginal cost
// 2 c_i a_i until they share one level mu (x_i = max(0, mu / (2 c_i) - a_i), sum x_i = 1).
agc_status agc_build_cyclic_code_opt(int n, int k, int s, const double* p, const uint8_t* bits,
                                     double phi_coef, int32_t* row_ptr, int32_t* col, float* val,
                                     float* w_out, double* objective, int* reaches_bound)
{
    if (!p || !bits || !row_ptr || !col || !val || !w_out) return AGC_EINVAL;
    if (n <= 0 || k <= 0 || n != k || s < 1 || s > k) return AGC_ESHAPE;
    std::vector<double> cinv;
    agc_status st = code_weights(n, p, bits, phi_coef, cinv);
    if (st != AGC_OK) return st;
    // start from the column-normalised weights
    std::vector<double> alpha((size_t)n * s), r(n, 0.0), colsum(k, 0.0);
    for (int i = 0; i < n; ++i)
        for (int u = 0; u < s; ++u) colsum[(i + u) % k] += cinv[i];
    for (int i = 0; i < n; ++i)
        for (int u = 0; u < s; ++u) {
            alpha[(size_t)i * s + u] = cinv[i] / colsum[(i + u) % k];
            r[i] += alpha[(size_t)i * s + u];
        }
    std::vector<int> order(s);
    std::vector<double> a(s), x(s);
    const int max_sweeps = 200000;
    for (int sweep = 0; sweep < max_sweeps; ++sweep) {
        double moved = 0.0;
        for (int j = 0; j < k; ++j) {
            // holders of column j: worker (j - u) mod n holds it at position u
            for (int u = 0; u < s; ++u) {
                const int i = ((j - u) % n + n) % n;
                a[u] = r[i] - alpha[(size_t)i * s + u];
                order[u] = u;
            }
            std::sort(order.begin(), order.end(), [&](int u1, int u2) {
                const int i1 = ((j - u1) % n + n) % n, i2 = ((j - u2) % n + n) % n;
                return a[u1] / cinv[i1] < a[u2] / cinv[i2];  // marginal cost c_i a_i
            });
            // level mu/2 = (1 + sum_{active} a_i) / sum_{active} c_i^-1 over the cheapest m holders
            double sum_a = 0.0, sum_cinv = 0.0, level = 0.0;
            int m = 0;
            for (; m < s; ++m) {
                const int u = order[m], i = ((j - u) % n + n) % n;
                if (m > 0 && a[u] / cinv[i] >= level) break;  // this holder is already above the level
                sum_a += a[u];
                sum_cinv += cinv[i];
                level = (1.0 + sum_a) / sum_cinv;
            }
            for (int u = 0; u < s; ++u) x[u] = 0.0;
            for (int q = 0; q < m; ++q) {
                const int u = order[q], i = ((j - u) % n + n) % n;
                x[u] = std::max(0.0, level * cinv[i] - a[u]);
            }
            double tot = 0.0;
            for (int u = 0; u < s; ++u) tot += x[u];
            for (int u = 0; u < s; ++u) {
                const int i = ((j - u) % n + n) % n;
                const double nx = x[u] / tot;  // rounding left the sum a few ulps off 1
                moved = std::max(moved, std::fabs(nx - alpha[(size_t)i * s + u]));
                alpha[(size_t)i * s + u] = nx;
                r[i] = a[u] + nx;
            }
        }
        if (moved < 1e-15) break;
    }
    double obj = 0.0, inv_sum = 0.0;
    for (int i = 0; i < n; ++i) {
        obj += r[i] * r[i] / cinv[i];
        inv_sum += cinv[i];
        row_ptr[i] = i * s;
        for (int u = 0; u < s; ++u) {
            col[i * s + u] = (i + u) % k;
            val[i * s + u] = (float)alpha[(size_t)i * s + u];
        }
        w_out[i] = (float)(1.0 / (1.0 - p[i]));
    }
    row_ptr[n] = n * s;
    if (objective) *objective = obj;
    // Theorem 1's row sums are reachable on this support iff the minimum equals k^2 / sum c^-1
    if (reaches_bound) *reaches_bound = obj <= (double)k * k / inv_sum * (1.0 + 1e-9) ? 1 : 0;
    return AGC_OK;
}

agc_status agc_check_unbiased(int n, int k, const int32_t* row_ptr, const int32_t* col,
                              const float* val, const float* w, const double* p, double tol,
                              double* residual)
{
    if (!row_ptr || !col || !val || !w || !p || n <= 0 || k <= 0) return AGC_EINVAL;
    std::vector<double> acc(k, 0.0);
    for (int i = 0; i < n; ++i)
        for (int e = row_ptr[i]; e < row_ptr[i + 1]; ++e) {
            if (col[e] < 0 || col[e] >= k) return AGC_ESHAPE;
            acc[col[e]] += (1.0 - p[i]) * (double)w[i] * (double)val[e];
        }
    double worst = 0.0;
    for (int j = 0; j < k; ++j) worst = std::max(worst, std::fabs(acc[j] - 1.0));
    if (residual) *residual = worst;
    return worst <= tol ? AGC_OK : AGC_EINVAL;
}

agc_status agc_second_moment_decoder(int n, int k, const int32_t* row_ptr, const int32_t* col,
                                     const float* val, const double* p, const uint8_t* bits,
                                     double phi_coef, double lambda, float* v)
{
    if (!row_ptr || !col || !val || !p || !bits || !v || n <= 0 || k <= 0 || !(lambda > 0.0)) return AGC_EINVAL;
    // stationarity of  lambda * (k - sum_i u_i)^2 + sum_i c_i u_i^2  in u_i = (1-p_i) v_i A_i,
    // A_i the row sum of the code, c_i = (p_i + phi(z_i)) / (1 - p_i)
    double inv_c_sum = 0.0;
    for (int i = 0; i < n; ++i) {
        if (!(p[i] >= 0.0 && p[i] < 1.0)) return AGC_EINVAL;
        inv_c_sum += (1.0 - p[i]) / (p[i] + phi_of((double)bits[i], phi_coef));
    }
    for (int i = 0; i < n; ++i) {
        double row_sum = 0.0;
        for (int e = row_ptr[i]; e < row_ptr[i + 1]; ++e) {
            if (col[e] < 0 || col[e] >= k) return AGC_ESHAPE;
            row_sum += (double)val[e];
        }
        if (row_sum == 0.0) return AGC_EINVAL;
        v[i] = (float)((double)k * lambda /
                       ((p[i] + phi_of((double)bits[i], phi_coef)) * row_sum * (1.0 + lambda * inv_c_sum)));
    }
    return AGC_OK;
}

}  // extern "C"
