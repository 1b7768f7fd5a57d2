"""Pins of the oracle's quantizer against what the paper fixes (Sec. II-B): grid, number of
levels, unbiasedness by exhaustive enumeration, exact variance and the phi(z) bound."""
from fractions import Fraction
import itertools

import numpy as np
import pytest

from oracle import agc_oracle as O
from oracle import design as D


def test_levels():
    # Sec. II-B: s_i = 2^(z_i - 1) - 1, at least one magnitude level at z = 2
    assert [O.levels(b) for b in (2, 3, 4, 8, 16)] == [1, 3, 7, 127, 32767]
    assert O.levels(1) == 1  # one-bit extension: two-point grid


@pytest.mark.parametrize("bits", [2, 3, 5, 8, 12])
def test_values_on_grid_and_zero(bits):
    """Every code dequantizes to sign * q/L * scale with q in 0..L; zero maps to code 0;
    a coordinate already on the grid is reproduced whatever the draw is."""
    L = O.levels(bits)
    scale = np.float32(8.0)
    inv = O.inv16(scale, bits)
    rng = np.random.default_rng(bits)
    for _ in range(200):
        f = np.float32(rng.uniform(-8, 8))
        code = O.quantize_one(f, inv, bits, int(rng.integers(0, 65536)), int(rng.integers(0, 1 << 32)))
        assert 0 <= code < (1 << bits)
        level = code & ((1 << (bits - 1)) - 1)
        assert level <= L
        v = float(O.code_value(code, bits))
        assert abs(v) == level and (v < 0) == (f < 0) or level == 0
        # nearest two grid points bracket |f|
        assert level in (int(np.floor(abs(f) / 8.0 * L)), int(np.floor(abs(f) / 8.0 * L)) + 1)
    for u16, r2 in [(0, 0), (65535, 0xFFFFFFFF), (12345, 999)]:
        assert O.quantize_one(0.0, inv, bits, u16, r2) == 0
        if L >= 2:
            q = L // 2 + 1
            f_on = np.float32(-8.0 * q / L) if (8.0 * q / L) == float(np.float32(8.0 * q / L)) else None
            if f_on is not None and float(O.grid_pos(f_on, inv, bits)) == q * 65536.0:
                assert O.quantize_one(f_on, inv, bits, u16, r2) == ((1 << (bits - 1)) | q)


@pytest.mark.parametrize("bits", [1, 2, 3, 4, 8])
def test_decision_counts_match_probability(bits):
    """Brute force over all 2^16 primary fields: the number that round up is exactly the
    integer part Fi of the scaled probability, plus the tie resolved by the secondary word;
    over a lattice of secondary words the tie rounds up in exactly the fraction g."""
    rng = np.random.default_rng(100 + bits)
    scale = np.float32(3.0)
    inv = O.inv16(scale, bits)
    L = O.levels(bits)
    for f in [np.float32(x) for x in (0.37, -1.234567, 2.999, 1e-3, -0.5)] + [np.float32(rng.uniform(-3, 3))]:
        lo, p_up = O.quantize_prob(f, inv, bits)
        T = float(O.grid_pos(f, inv, bits))
        assert lo == int(T) >> 16
        assert p_up == pytest.approx((T - lo * 65536.0) / 65536.0, abs=0)
        Fi = int(T) & 0xFFFF
        g = T - int(T)
        base = None
        ups = 0
        for u16 in range(65536):
            code = O.quantize_one(f, inv, bits, u16, 0xFFFFFFFF)  # ties resolve down unless g*2^32 > r2
            level = code & ((1 << (bits - 1)) - 1) if bits >= 2 else code
            if base is None:
                base = min(lo, L)
            ups += int(level > min(lo, L))
        if lo < L:
            assert ups == Fi + (1 if g * 2.0 ** 32 > 0xFFFFFFFF else 0)
        # tie-break lattice: r2 = j * 2^20, j < 4096
        if lo < L and g > 0:
            cnt = 0
            for j in range(4096):
                code = O.quantize_one(f, inv, bits, Fi, j << 20)
                level = code & ((1 << (bits - 1)) - 1) if bits >= 2 else code
                cnt += int(level == lo + 1)
            assert cnt == int(np.ceil(g * 4096))


@pytest.mark.parametrize("bits", [1, 2, 3, 6, 8])
def test_unbiased_single_coordinate(bits):
    """E[Q(x)_m | x] = x_m (Sec. II-B): probability-weighted sum of the two reachable values."""
    rng = np.random.default_rng(bits)
    for _ in range(300):
        scale = np.float32(rng.uniform(0.5, 4.0))
        f = np.float32(rng.uniform(-1, 1) * scale)
        inv = O.inv16(scale, bits)
        lo, p_up = O.quantize_prob(f, inv, bits)
        L = O.levels(bits)
        unit = float(scale) / L
        if bits >= 2:
            mean = unit * (lo + p_up) * (-1 if f < 0 else 1)
        else:
            mean = float(scale) * (2 * (lo + p_up) - 1)
        assert mean == pytest.approx(float(f), rel=4e-7, abs=4e-7 * float(scale))


def test_clamp_at_full_scale():
    """|f| == scale must give level L, never L+1 (which would spill into the sign bit)."""
    rng = np.random.default_rng(5)
    for bits in range(2, 17):
        L = O.levels(bits)
        for _ in range(200):
            scale = np.float32(rng.uniform(1e-3, 1e3))
            inv = O.inv16(scale, bits)
            for sgn in (1, -1):
                code = O.quantize_one(np.float32(sgn) * scale, inv, bits, 0, 0)
                assert code & ((1 << (bits - 1)) - 1) == L
                assert code >> (bits - 1) == (1 if sgn < 0 else 0)
    for _ in range(200):
        scale = np.float32(rng.uniform(1e-3, 1e3))
        inv = O.inv16(scale, 1)
        assert O.quantize_one(scale, inv, 1, 0, 0) == 1
        assert O.quantize_one(-scale, inv, 1, 65535, 0xFFFFFFFF) == 0


def test_zero_and_tiny_scale():
    assert O.inv16(0.0, 4) == 0.0
    assert O.inv16(1e-45, 8) == 0.0          # quotient overflows binary32: treated as zero vector
    assert O.quantize_one(0.0, 0.0, 4, 0, 0) == 0
    # sign of a negative zero is kept in the sign bit (decodes to -0.0)
    assert O.quantize_one(np.float32(-0.0), O.inv16(1.0, 4), 4, 5, 5) == 8
    assert float(O.code_value(8, 4)) == 0.0


def _var_q(f, scale, bits):
    """exact quantization variance of one vector from the oracle's own probabilities"""
    inv = O.inv16(scale, bits)
    L = O.levels(bits)
    unit = float(scale) / L if bits >= 2 else 2.0 * float(scale)
    tot = 0.0
    for x in f:
        lo, p = O.quantize_prob(x, inv, bits)
        if lo >= L:
            p = 0.0
        tot += unit * unit * p * (1 - p)
    return tot


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_variance_bound_l2(bits):
    """E||Q(x)-x||^2 <= phi(z) ||x||^2 with phi(z) = l / (4 (2^(z-1)-1)^2) when the scale is
    the Euclidean norm (Sec. II-B)."""
    rng = np.random.default_rng(bits)
    for d in (7, 64, 500):
        f = rng.standard_normal(d).astype(np.float32)
        scale = O.scale_l2(f)
        var = _var_q(f, scale, bits)
        bound = float(D.phi(bits, D.phi_coef_paper(d))) * float(np.sum(f.astype(np.float64) ** 2))
        assert var <= bound * (1 + 1e-6)
        assert var > 0


def _enumerate_estimator(G, csr, bits, w, p, scales):
    """All 2^n arrival patterns x all up/down outcomes of every coordinate, each decoded by
    the oracle, weighted by its exact probability.  Returns E[g_hat] and E||g_hat - g||^2 as
    Fractions / floats, with g = sum_j g_j."""
    n, d = csr.n, G.shape[1]
    f = [O.encode(G, csr, i) for i in range(n)]
    cells = []      # per (i, m): list of (prob Fraction, forcing draw)
    for i in range(n):
        inv = O.inv16(scales[i], int(bits[i]))
        for m in range(d):
            lo, p_up = O.quantize_prob(f[i][m], inv, int(bits[i]))
            opts = []
            P = Fraction(p_up)
            if P > 0:
                opts.append((P, (0, 0)))                      # forces "up"
            if P < 1:
                opts.append((1 - P, (65535, 0xFFFFFFFF)))     # forces "down"
            cells.append(opts)
    g = np.sum(G.astype(np.float64), axis=0)
    mean = [Fraction(0)] * d
    err = Fraction(0)
    total_prob = Fraction(0)
    for outcome in itertools.product(*cells):
        pq = Fraction(1)
        streams = []
        idx = 0
        for i in range(n):
            inv = O.inv16(scales[i], int(bits[i]))
            codes = []
            for m in range(d):
                pr, (u16, r2) = outcome[idx]
                idx += 1
                pq *= pr
                codes.append(O.quantize_one(f[i][m], inv, int(bits[i]), u16, r2))
            streams.append(O.pack(np.array(codes, dtype=np.uint32), int(bits[i])))
        for mask in itertools.product((0, 1), repeat=n):
            pm = Fraction(1)
            for i in range(n):
                pm *= (1 - Fraction(p[i])) if mask[i] else Fraction(p[i])
            gh = O.decode(streams, scales, bits, w, np.array(mask, dtype=np.uint8), d)
            pr = pq * pm
            total_prob += pr
            for m in range(d):
                mean[m] += pr * Fraction(float(gh[m]))
                err += pr * (Fraction(float(gh[m])) - Fraction(float(g[m]))) ** 2
    assert total_prob == 1
    return mean, err, f


def test_exhaustive_unbiasedness_exact_dyadic():
    """n=3 workers, k=3 partitions, d=2: with dyadic p, code, gradients and power-of-two scales
    every operation of the path is exact, so E[g_hat] must equal sum_j g_j EXACTLY
    (Sec. III, unbiasedness constraint of P1 with condition sum_i (1-p_i) w_i a_ij = 1)."""
    p = [0.5, 0.75, 0.5]
    alpha = np.array([[0.5, 0.25, 0.0], [0.5, 0.5, 0.25], [0.0, 0.25, 0.75]])
    B, w = D.physical_code(alpha, p)
    assert D.unbiased_residual(B, w, p) == 0.0
    csr = O.Csr.from_dense(B)
    G = np.array([[0.25, -0.5], [1.0, 0.375], [-0.75, 0.125]], dtype=np.float32)
    bits = np.array([2, 2, 1], dtype=np.uint8)
    scales = np.array([1.0, 2.0, 1.0], dtype=np.float32)   # >= max|f_i|, powers of two
    for i in range(3):
        assert float(np.max(np.abs(O.encode(G, csr, i)))) <= scales[i]
    mean, err, f = _enumerate_estimator(G, csr, bits, w.astype(np.float32), p, scales)
    g = G.astype(np.float64).sum(axis=0)
    assert [float(x) for x in mean] == [float(x) for x in g]
    # exact residual error against the closed form (proof of Lemma 1, before bounding)
    var_q = [_var_q(f[i], scales[i], int(bits[i])) for i in range(3)]
    _, err_closed = D.exact_moments(np.array(f, dtype=np.float64), var_q, w, p)
    assert float(err) == pytest.approx(err_closed, rel=1e-12)


@pytest.mark.parametrize("scale_mode", [O.SCALE_MAXABS, O.SCALE_L2])
def test_exhaustive_unbiasedness_general(scale_mode):
    """Same enumeration with generic reals, mixed bit-widths and the oracle's own scales;
    binary32 rounding of T and of the decode leaves a relative error of a few 1e-7."""
    rng = np.random.default_rng(3)
    p = np.array([0.1, 0.3, 0.45])
    bits = np.array([3, 2, 4], dtype=np.uint8)
    c = D.c_weights(p, bits, 0.05)
    alpha = D.interval_code(D.row_targets(c, 3), 3)
    B, w = D.physical_code(alpha, p)
    assert D.unbiased_residual(B, w, p) < 1e-12
    csr = O.Csr.from_dense(B)
    G = rng.standard_normal((3, 2)).astype(np.float32)
    scales = O.scales(G, csr, scale_mode)
    mean, err, f = _enumerate_estimator(G, csr, bits, w.astype(np.float32), p, scales)
    g = G.astype(np.float64).sum(axis=0)
    Bf = csr.dense()                       # the binary32-rounded code actually used
    wf = w.astype(np.float32).astype(np.float64)
    expect = ((1 - p) * wf) @ Bf @ G.astype(np.float64)
    assert np.allclose([float(x) for x in mean], expect, rtol=2e-6, atol=1e-7)
    assert np.allclose([float(x) for x in mean], g, rtol=2e-6, atol=1e-6)
    var_q = [_var_q(f[i], scales[i], int(bits[i])) for i in range(3)]
    mean_c, err_c = D.exact_moments(np.array(f, dtype=np.float64), var_q, wf, p)
    # enumeration measures the error around g; closed form around E[g_hat]; they differ by
    # ||E g_hat - g||^2 ~ 1e-13
    assert float(err) == pytest.approx(err_c, rel=1e-5)


def test_onebit_extension_unbiased_enumeration():
    """One-bit codes (outside the paper's z >= 2) decode to +-scale with mean f."""
    p = [0.5, 0.5]
    alpha = np.array([[0.5, 0.5], [0.5, 0.5]])
    B, w = D.physical_code(alpha, p)
    csr = O.Csr.from_dense(B)
    G = np.array([[0.25, -0.5], [0.5, 0.125]], dtype=np.float32)
    bits = np.array([1, 1], dtype=np.uint8)
    scales = np.array([0.5, 0.5], dtype=np.float32)
    mean, err, f = _enumerate_estimator(G, csr, bits, w.astype(np.float32), p, scales)
    assert [float(x) for x in mean] == [float(x) for x in G.astype(np.float64).sum(axis=0)]
