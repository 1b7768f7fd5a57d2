"""Pins of the oracle's bucket-wise quantizer (Sec. II-B names the extension; its arithmetic is
this build's reading).  They tie it to things fixed elsewhere: the per-vector quantizer (itself
pinned by the paper's definitions) on inputs where the two must coincide, the unbiasedness of
the rounding rule, a brute-force decode, and the reason buckets exist (small layers survive)."""
import numpy as np
import pytest

from oracle import agc_oracle as O
from paper_2605_15890_amd import inputs as I


def _cyclic(n, s, rng):
    row_ptr = np.arange(n + 1, dtype=np.int32) * s
    col = np.array([[(i + u) % n for u in range(s)] for i in range(n)], dtype=np.int32).ravel()
    val = rng.uniform(0.2, 1.0, n * s).astype(np.float32)
    return O.Csr(row_ptr, col, val, n)


def test_bucket_scales_are_the_per_bucket_norms():
    rng = np.random.default_rng(0)
    f = rng.standard_normal(1000).astype(np.float32)
    for u in range(4):
        seg = f[256 * u:256 * (u + 1)]
        assert O.bucket_scale(f, u, O.SCALE_MAXABS) == float(np.max(np.abs(seg)))
        l2 = float(np.sqrt(np.sum(seg.astype(np.float64) ** 2)))
        assert abs(O.bucket_scale(f, u, O.SCALE_L2) - l2) <= 1.2e-7 * l2      # one binary32 rounding
    assert O.num_buckets(1000) == 4 and O.num_buckets(1024) == 4 and O.num_buckets(1025) == 5


def test_multiplier_and_weight_agree_with_the_per_vector_ones_on_powers_of_two():
    for bits in (1, 2, 3, 8, 16):
        for e in (-20, -3, 0, 5):
            s = float(2.0 ** e)
            assert O.inv16_bucket(s, bits) == O.inv16(s, bits)
            for w in (0.3, 1.0, 1.7):
                assert np.float32(O.wl_bucket(w, bits)) * np.float32(s) == np.float32(O.coef(w, s, bits))
    assert O.inv16_bucket(0.0, 4) == 0.0
    assert O.inv16_bucket(1e-45, 16) == 0.0           # quotient overflows binary32: treated as a zero bucket
    for bits in (2, 5, 11):                           # one rounding of the exact quotient
        for s in (0.3, 1.7, 123.456):
            L = O.levels(bits)
            exact = L * 65536.0 / float(np.float32(s))
            assert abs(O.inv16_bucket(s, bits) - exact) <= 6e-8 * exact


@pytest.mark.parametrize("scale_mode", [O.SCALE_MAXABS])
@pytest.mark.parametrize("d", [1, 100, 256])
def test_single_bucket_with_power_of_two_scale_equals_the_per_vector_quantizer(d, scale_mode):
    """d <= 256 is one bucket; when every worker's largest magnitude is a power of two both
    multipliers and both decode weights are the same numbers, so the whole step must coincide
    with the per-vector path."""
    rng = np.random.default_rng(d)
    n = 4
    csr = O.Csr(np.arange(n + 1, dtype=np.int32), np.arange(n, dtype=np.int32), np.ones(n, np.float32), n)
    G = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    G[np.arange(n), rng.integers(0, d, n)] = [1.0, -0.5, 2.0, -0.25]          # the largest magnitudes
    for j, top in enumerate([1.0, 0.5, 2.0, 0.25]):
        G[j] = np.clip(G[j], -top, top)
    bits = np.array([1, 2, 5, 9], dtype=np.uint8)
    w = np.array([1.0, 1.3, 0.7, 2.0], dtype=np.float32)
    mask = np.array([1, 1, 0, 1], dtype=np.uint8)
    a_streams, a_scales, a_ghat = O.step(G, csr, bits, w, mask, 11, 3, scale_mode)
    b_streams, b_scales, b_ghat = O.step_bucket(G, csr, bits, w, mask, 11, 3, scale_mode)
    assert b_scales.shape == (n, 1) and np.array_equal(b_scales[:, 0], a_scales)
    assert all(np.array_equal(x, y) for x, y in zip(a_streams, b_streams))
    assert np.array_equal(a_ghat.view(np.uint32), b_ghat.view(np.uint32))


@pytest.mark.parametrize("scale_mode", [O.SCALE_MAXABS, O.SCALE_L2])
def test_expected_value_of_every_coordinate_is_the_coded_gradient(scale_mode):
    """Exact expectation from the rounding probabilities: scale_u * (lo + P(up)) / L = |f|."""
    rng = np.random.default_rng(5)
    n, d = 3, 700
    csr = _cyclic(n, 2, rng)
    G = (rng.standard_normal((n, d)) * np.repeat(10.0 ** rng.uniform(-3, 1, (n, 1)), d, axis=1)).astype(np.float32)
    for i, bits in enumerate((2, 4, 9)):
        f = O.encode(G, csr, i, 0, d)
        L = O.levels(bits)
        for u in range(O.num_buckets(d)):
            scale = O.bucket_scale(f, u, scale_mode)
            inv = O.inv16_bucket(scale, bits)
            for m in range(256 * u, min(d, 256 * u + 256), 7):
                lo, p_up = O.quantize_prob(float(f[m]), inv, bits)
                assert lo + p_up <= L + 1e-9
                want = abs(float(f[m]))
                got = scale * (lo + p_up) / L
                assert abs(got - want) <= 3e-7 * scale, (i, m)


def test_codes_are_drawn_with_the_global_coordinate_index():
    """The bucket path must use the same counter-based draws as the per-vector path: with the
    bucket's scale handed to the per-vector routine as that worker's scale, and a power-of-two
    scale so that the multipliers coincide, the codes inside the bucket are identical."""
    rng = np.random.default_rng(9)
    n, d = 2, 1000
    csr = O.Csr(np.arange(n + 1, dtype=np.int32), np.arange(n, dtype=np.int32), np.ones(n, np.float32), n)
    G = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    G[:, 300] = 4.0
    G[:, 600] = -0.125
    G[:, 512:768] = np.clip(G[:, 512:768], -0.125, 0.125)
    for i, bits in enumerate((3, 7)):
        codes, sc = O.codes_bucket_range(G, csr, i, bits, O.SCALE_MAXABS, 5, 2, 256, 768)
        assert list(sc) == [4.0, 0.125]
        ref1 = O.codes_range(G, csr, i, bits, 4.0, 5, 2, 256, 512)
        ref2 = O.codes_range(G, csr, i, bits, 0.125, 5, 2, 512, 768)
        assert np.array_equal(codes, np.concatenate([ref1, ref2]))


def test_decode_is_the_weighted_sum_of_dequantized_codes():
    rng = np.random.default_rng(2)
    n, d = 4, 900
    bits = np.array([1, 3, 6, 12], dtype=np.uint8)
    nb = O.num_buckets(d)
    scales = rng.uniform(0.1, 3, (n, nb)).astype(np.float32)
    w = rng.uniform(0.5, 2, n).astype(np.float32)
    mask = np.array([1, 0, 1, 1], dtype=np.uint8)
    streams, vals = [], []
    for i in range(n):
        b = int(bits[i])
        codes = rng.integers(0, 1 << b, d).astype(np.uint32)
        if b >= 2:
            L = O.levels(b)
            lev = np.minimum(codes & ((1 << (b - 1)) - 1), L)
            sign = np.where(codes >> (b - 1) & 1, -1.0, 1.0)
            codes = (lev | ((sign < 0).astype(np.uint32) << (b - 1))).astype(np.uint32)
            vals.append(sign * lev / L)
        else:
            vals.append(np.where(codes == 1, 1.0, -1.0))
        streams.append(O.pack(codes, b))
    got = O.decode_bucket(streams, scales, bits, w, mask, d)
    per_coord_scale = np.repeat(scales.astype(np.float64), 256, axis=1)[:, :d]
    want = sum(float(w[i]) * per_coord_scale[i] * vals[i] for i in range(n) if mask[i])
    assert np.allclose(got, want, rtol=0, atol=2e-6 * np.max(np.abs(want)))


def test_small_layers_survive_with_bucket_scales():
    """The reason for buckets: with per-layer magnitudes spread over three decades a single
    scale per vector rounds the small layers to noise; per-bucket scales keep their relative
    error at the level of the large ones."""
    cfg = I.CONFIGS["resnet18"]
    d = 60 * 1024
    rng = np.random.default_rng(1)
    n = k = 4
    csr = _cyclic(n, 2, rng)
    G = rng.standard_normal((k, d)).astype(np.float32)
    sig, edges = I.layer_sigmas(cfg, d)
    for l in range(len(sig)):
        G[:, edges[l]:edges[l + 1]] *= np.float32(sig[l])
    bits = np.full(n, 4, dtype=np.uint8)
    w = np.ones(n, dtype=np.float32)
    mask = np.ones(n, dtype=np.uint8)
    f_sum = sum(O.encode(G, csr, i, 0, d).astype(np.float64) for i in range(n))
    _, _, g_vec = O.step(G, csr, bits, w, mask, 1, 0, O.SCALE_MAXABS)
    _, _, g_bkt = O.step_bucket(G, csr, bits, w, mask, 1, 0, O.SCALE_MAXABS)
    small = np.argmin(sig)
    sl = slice(edges[small], edges[small + 1])
    rel = lambda g: np.linalg.norm(g[sl] - f_sum[sl]) / np.linalg.norm(f_sum[sl])
    assert rel(g_bkt) < 0.5
    assert rel(g_vec) > 10 * rel(g_bkt)
