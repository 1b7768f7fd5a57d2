"""Pins of the layer-wise composition in oracle/agc_oracle.py (Sec. II-B: the quantizer applied
"at layer-wise or bucket-wise granularity").  The composition has no arithmetic of its own; these
tests fix what it must compose: which scale goes with which coordinate, and that the draws stay
those of the whole vector."""
import numpy as np
import pytest

from oracle import agc_oracle as O


def _cyclic(rng, n, s, integer=False):
    row_ptr = np.arange(n + 1, dtype=np.int32) * s
    col = np.array([(i + u) % n for i in range(n) for u in range(s)], dtype=np.int32)
    if integer:
        val = rng.integers(-3, 4, n * s).astype(np.float32)
    else:
        val = rng.uniform(0.2, 1.0, n * s).astype(np.float32)
    return row_ptr, col, val


def test_one_layer_is_the_per_vector_step():
    rng = np.random.default_rng(1)
    n = k = 5
    d = 777
    row_ptr, col, val = _cyclic(rng, n, 3)
    csr = O.Csr(row_ptr, col, val, k)
    G = rng.standard_normal((k, d)).astype(np.float32)
    bits = np.array([2, 3, 5, 8, 16], dtype=np.uint8)
    w = rng.uniform(0.5, 2.0, n).astype(np.float32)
    mask = np.array([1, 1, 0, 1, 1], dtype=np.uint8)
    s1, c1, g1 = O.step(G, csr, bits, w, mask, 9, 4, O.SCALE_MAXABS)
    s2, c2, g2 = O.step_layers(G, csr, bits, w, mask, 9, 4, [d])
    assert c2.shape == (n, 1) and np.array_equal(c1.view(np.uint32), c2[:, 0].view(np.uint32))
    for a, b in zip(s1, s2):
        assert np.array_equal(a, b)
    assert np.array_equal(g1.view(np.uint32), g2.view(np.uint32))


def test_one_layer_is_the_per_vector_step_also_with_the_euclidean_scale():
    rng = np.random.default_rng(11)
    n = k = 4
    d = 2500
    row_ptr, col, val = _cyclic(rng, n, 2)
    csr = O.Csr(row_ptr, col, val, k)
    G = rng.standard_normal((k, d)).astype(np.float32)
    bits = np.array([2, 4, 6, 9], dtype=np.uint8)
    w = rng.uniform(0.5, 2.0, n).astype(np.float32)
    mask = np.ones(n, dtype=np.uint8)
    s1, c1, g1 = O.step(G, csr, bits, w, mask, 1, 2, O.SCALE_L2)
    s2, c2, g2 = O.step_layers(G, csr, bits, w, mask, 1, 2, [d], scale_mode=O.SCALE_L2)
    assert np.array_equal(c1.view(np.uint32), c2[:, 0].view(np.uint32))
    assert all(np.array_equal(a, b) for a, b in zip(s1, s2))
    assert np.array_equal(g1.view(np.uint32), g2.view(np.uint32))


def test_layer_norms_are_the_norms_of_the_slices():
    """Every layer's Euclidean scale against an exactly rounded sum of the slice's squares
    (math.fsum over the binary64 squares, which are exact), to the last few units of binary32."""
    import math
    rng = np.random.default_rng(12)
    n = k = 3
    d = 5000
    row_ptr, col, val = _cyclic(rng, n, 2)
    csr = O.Csr(row_ptr, col, val, k)
    G = rng.standard_normal((k, d)).astype(np.float32)
    ends = [256, 1280, 4864, 5000]
    sc = O.scales_layers(G, csr, ends, scale_mode=O.SCALE_L2)
    for i in range(n):
        f = O.encode(G, csr, i).astype(np.float64)
        for l, (m0, m1) in enumerate(O.layer_ranges(ends, d)):
            exact = math.sqrt(math.fsum(float(x) * float(x) for x in f[m0:m1]))
            assert abs(float(sc[i, l]) - exact) <= 2e-7 * exact, (i, l)
    # and a layer that starts off the origin uses a tree of its own: equal slices, equal norms
    G2 = np.concatenate([G[:, 1280:4864], G[:, 1280:4864]], axis=1)
    sc2 = O.scales_layers(G2, csr, [3584, 7168], scale_mode=O.SCALE_L2)
    assert np.array_equal(sc2[:, 0].view(np.uint32), sc2[:, 1].view(np.uint32))
    assert np.array_equal(sc2[:, 0].view(np.uint32), sc[:, 2].view(np.uint32))


def test_layer_scales_are_the_exact_maxima_of_integer_data():
    """Integer code and integer gradients: every f_i[m] is an exact integer, so the scales must
    equal the maxima numpy finds in the integer product, layer by layer."""
    rng = np.random.default_rng(2)
    n = k = 6
    d = 1000
    row_ptr, col, val = _cyclic(rng, n, 3, integer=True)
    csr = O.Csr(row_ptr, col, val, k)
    G = rng.integers(-50, 51, (k, d)).astype(np.float32)
    B = np.zeros((n, k), dtype=np.int64)
    for i in range(n):
        for e in range(row_ptr[i], row_ptr[i + 1]):
            B[i, col[e]] += int(val[e])
    F = B @ G.astype(np.int64)
    ends = [7, 256, 300, 999, 1000]
    sc = O.scales_layers(G, csr, ends)
    for l, (m0, m1) in enumerate(O.layer_ranges(ends, d)):
        assert np.array_equal(sc[:, l], np.abs(F[:, m0:m1]).max(axis=1).astype(np.float32)), l


def test_every_coordinate_is_quantized_on_the_grid_of_its_own_layer():
    """Layers whose magnitudes differ by 10^3: the decoded value of an arrived worker differs from
    f_i[m] by less than one cell of the layer's grid, scale_il / L_i, and reaches the layer's scale
    somewhere; with the scale of any other layer one of the two would fail."""
    rng = np.random.default_rng(3)
    n = k = 4
    d = 900
    ends = [300, 600, 900]
    row_ptr, col, val = _cyclic(rng, n, 2)
    csr = O.Csr(row_ptr, col, val, k)
    G = rng.standard_normal((k, d)).astype(np.float32)
    G[:, :300] *= np.float32(1e-3)
    G[:, 600:] *= np.float32(1e3)
    bits = np.array([3, 4, 6, 8], dtype=np.uint8)
    streams, sc = O.encode_quantize_layers(G, csr, bits, 5, 0, ends)
    for i in range(n):
        f = O.encode(G, csr, i).astype(np.float64)
        L = O.levels(int(bits[i]))
        one = np.zeros(n, dtype=np.uint8)
        one[i] = 1
        wone = np.ones(n, dtype=np.float32)
        dec = O.decode_layers(streams, sc, bits, wone, one, d, ends).astype(np.float64)
        for l, (m0, m1) in enumerate(O.layer_ranges(ends, d)):
            cell = float(sc[i, l]) / L
            err = np.abs(dec[m0:m1] - f[m0:m1])
            assert err.max() < cell * (1 + 1e-5), (i, l)
            assert np.abs(dec[m0:m1]).max() <= float(sc[i, l]) * (1 + 1e-6)
            assert np.abs(f[m0:m1]).max() == float(sc[i, l])
        # the scales themselves are three orders of magnitude apart, layer to layer
        assert sc[i, 0] * 100 < sc[i, 1] < sc[i, 2] / 100


def test_layer_codes_use_the_draws_of_the_whole_vector():
    """With the same scale in every layer the cut must not show: the codes equal those of the
    per-vector quantizer given that scale."""
    rng = np.random.default_rng(4)
    n = k = 3
    d = 700
    row_ptr, col, val = _cyclic(rng, n, 2)
    csr = O.Csr(row_ptr, col, val, k)
    G = rng.standard_normal((k, d)).astype(np.float32)
    bits = np.array([2, 4, 7], dtype=np.uint8)
    base = O.scales(G, csr, O.SCALE_MAXABS)
    ends = [256, 512, 700]
    same = np.repeat(base[:, None], len(ends), axis=1)
    s_layers, _ = O.encode_quantize_layers(G, csr, bits, 12, 3, ends, scales_in=same)
    s_vector, _ = O.encode_quantize(G, csr, bits, 12, 3, O.SCALE_MAXABS, scales_in=base)
    for a, b in zip(s_layers, s_vector):
        assert np.array_equal(a, b)


def test_layerwise_estimator_is_unbiased_monte_carlo():
    """E[g_hat] = sum_j g_j for a code with unit column sums and w_i = 1 when everybody arrives
    (constraint of problem P1 with p = 0): 4000 steps, every coordinate within 4.5 standard errors."""
    rng = np.random.default_rng(5)
    n = k = 3
    d = 6
    row_ptr = np.array([0, 2, 4, 6], dtype=np.int32)
    col = np.array([0, 1, 1, 2, 2, 0], dtype=np.int32)
    val = np.array([0.25, 0.5, 0.5, 0.75, 0.25, 0.75], dtype=np.float32)   # column sums 1
    csr = O.Csr(row_ptr, col, val, k)
    G = rng.standard_normal((k, d)).astype(np.float32)
    G[:, :2] *= np.float32(0.01)
    G[:, 4:] *= np.float32(30.0)
    bits = np.array([2, 3, 4], dtype=np.uint8)
    w = np.ones(n, dtype=np.float32)
    mask = np.ones(n, dtype=np.uint8)
    T = 4000
    acc = np.zeros((T, d))
    for t in range(T):
        acc[t] = O.step_layers(G, csr, bits, w, mask, 77, t, [2, 4, 6])[2]
    g = G.astype(np.float64).sum(axis=0)
    z = (acc.mean(axis=0) - g) / (acc.std(axis=0, ddof=1) / np.sqrt(T) + 1e-300)
    assert np.all(np.abs(z) < 4.5), z
    # and the small layer is not lost: under one scale per vector a two-bit worker would round
    # almost all of it to zero; here its estimate carries signal in every coordinate
    assert np.all(np.abs(acc.mean(axis=0)[:2] - g[:2]) < 0.5 * np.abs(g[:2]) + 4.5 * acc.std(axis=0, ddof=1)[:2] / np.sqrt(T))


def test_layer_ranges_reject_bad_ends():
    for bad in ([], [5, 5, 10], [10, 5], [3, 9]):
        with pytest.raises(AssertionError):
            O.layer_ranges(bad, 10)
