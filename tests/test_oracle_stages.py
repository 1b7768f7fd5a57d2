"""Pins of the oracle's encode, scale, pack and decode stages (CPU only)."""
import math

import numpy as np
import pytest

from oracle import agc_oracle as O


# ---------------------------------------------------------------- encode (Sec. II-A)
def test_encode_matches_dense_product():
    """f_i = sum_j a_ij g_j: against a binary64 matrix product, and exactly on integers."""
    rng = np.random.default_rng(0)
    n, k, d = 5, 6, 300
    B = rng.standard_normal((n, k)) * (rng.random((n, k)) < 0.5)
    csr = O.Csr.from_dense(B.astype(np.float32))
    G = rng.standard_normal((k, d)).astype(np.float32)
    ref = csr.dense() @ G.astype(np.float64)
    for i in range(n):
        f = O.encode(G, csr, i)
        assert np.allclose(f, ref[i], rtol=0, atol=1e-5)
    Bi = rng.integers(-3, 4, (n, k)).astype(np.float32)
    Gi = rng.integers(-50, 50, (k, d)).astype(np.float32)
    csr = O.Csr.from_dense(Bi)
    for i in range(n):
        assert np.array_equal(O.encode(Gi, csr, i), (Bi.astype(np.float64) @ Gi.astype(np.float64))[i])


def test_encode_uses_stored_order_and_fma():
    """Summation follows the stored order of the row with one rounding per further term:
    1e8 + 1 - 1e8 gives 0 or 1 depending on the order; a fused multiply-add keeps the low
    bits of the product that a separate multiply would lose."""
    G = np.array([[1e8], [1.0], [-1e8]], dtype=np.float32)
    a = O.Csr([0, 3], [0, 1, 2], [1, 1, 1], 3)
    b = O.Csr([0, 3], [0, 2, 1], [1, 1, 1], 3)
    assert float(O.encode(G, a, 0)[0]) == 0.0
    assert float(O.encode(G, b, 0)[0]) == 1.0
    x = np.float32(1 + 2 ** -12)
    G2 = np.array([[-(x * x)], [x]], dtype=np.float32)          # -(rounded x^2), x
    c = O.Csr([0, 2], [0, 1], [1.0, x], 2)
    exact_low = float(np.float64(x) * np.float64(x) - np.float64(np.float32(x * x)))
    assert exact_low != 0.0
    assert float(O.encode(G2, c, 0)[0]) == exact_low
    assert float(O.encode(np.zeros((2, 1), np.float32), O.Csr([0, 0], [], [], 2), 0)[0]) == 0.0


# ---------------------------------------------------------------- scale (Sec. II-B)
@pytest.mark.parametrize("d", [1, 3, 255, 256, 257, 4096, 4097, 70000, 300001])
def test_scales(d):
    rng = np.random.default_rng(d)
    f = (rng.standard_normal(d) * 10 ** rng.uniform(-3, 3)).astype(np.float32)
    assert float(O.scale_maxabs(f)) == float(np.max(np.abs(f)))
    exact = math.fsum(float(x) * float(x) for x in f)
    assert O.sumsq_tree(f) == pytest.approx(exact, rel=1e-13)
    assert float(O.scale_l2(f)) == float(np.float32(math.sqrt(O.sumsq_tree(f))))
    assert float(O.scale_l2(f)) >= float(O.scale_maxabs(f))


def test_l2_tree_is_a_fixed_tree():
    """The norm's accumulation order is part of the definition: a vector built so that
    orders disagree in the last place must reproduce the documented tree, here checked on a
    case small enough to follow by hand: slots 0 and 1 of one block."""
    f = np.zeros(8, dtype=np.float32)
    f[0], f[1], f[2], f[3] = 1.0, 2.0 ** -27, 2.0 ** -27, 2.0 ** -27
    # slot 0: (1 + 2^-54) + (2^-54 + 2^-54) = 1 + 2^-53 -> rounds to even = 1.0 ; exact sum is 1+3*2^-54
    assert O.sumsq_tree(f) == 1.0
    f2 = np.zeros(8, dtype=np.float32)
    f2[0], f2[2], f2[3], f2[4] = 1.0, 2.0 ** -26.5, 2.0 ** -26.5, 0.0
    x2 = float(np.float32(2.0 ** -26.5)) ** 2
    assert O.sumsq_tree(f2) == (1.0 + 0.0) + (x2 + x2)


# ---------------------------------------------------------------- pack (Sec. II-B payload)
@pytest.mark.parametrize("bits", list(range(1, 17)))
def test_pack_layout_and_roundtrip(bits):
    """The stream is the little-endian integer sum_m code_m << (m*b), zero-padded to whole
    groups of 128 codes."""
    rng = np.random.default_rng(bits)
    for d in [1, 2, 7, 31, 32, 33, 127, 128, 129, 300, 1000]:
        codes = rng.integers(0, 1 << bits, d).astype(np.uint32)
        stream = O.pack(codes, bits)
        assert stream.size == O.code_bytes(d, bits) == -(-d // 128) * 16 * bits
        big = 0
        for m, c in enumerate(codes):
            big |= int(c) << (m * bits)
        assert stream.tobytes() == big.to_bytes(stream.size, "little")
        assert np.array_equal(O.unpack(stream, d, bits), codes)


# ---------------------------------------------------------------- decode (Sec. II-A)
def test_decode_on_grid_equals_weighted_sum():
    """With every coded value on its worker's grid the quantizer is the identity, so the
    estimate is sum_i I_i w_i f_i, checked against a binary64 product; no arrival gives 0."""
    rng = np.random.default_rng(2)
    n, k, d = 6, 6, 777
    bits = np.array([2, 3, 4, 5, 8, 8], dtype=np.uint8)
    # partial gradients are integers and the code is the identity, so f_i = g_i; scale = L_i
    G = np.stack([rng.integers(-O.levels(int(b)), O.levels(int(b)) + 1, d) for b in bits]).astype(np.float32)
    G[np.arange(n), 0] = [O.levels(int(b)) for b in bits]        # make max|f_i| == L_i
    csr = O.Csr.from_dense(np.eye(n, dtype=np.float32))
    streams, scales = O.encode_quantize(G, csr, bits, seed=11, step=3, scale_mode=O.SCALE_MAXABS)
    assert np.array_equal(scales, [O.levels(int(b)) for b in bits])
    w = rng.uniform(0.5, 2.0, n).astype(np.float32)
    for mask in ([1] * n, [1, 0, 1, 0, 0, 1], [0] * n):
        mask = np.array(mask, dtype=np.uint8)
        gh = O.decode(streams, scales, bits, w, mask, d)
        ref = (mask * w.astype(np.float64)) @ G.astype(np.float64)
        assert np.allclose(gh, ref, rtol=1e-6, atol=2e-4)   # six binary32 terms of size ~250
        if not mask.any():
            assert np.all(gh == 0)


def test_step_is_encode_quantize_then_decode():
    rng = np.random.default_rng(4)
    n, k, d = 4, 4, 1000
    B = np.zeros((n, k), dtype=np.float32)
    for i in range(n):
        B[i, i], B[i, (i + 1) % k] = 0.6, 0.4
    csr = O.Csr.from_dense(B)
    G = rng.standard_normal((k, d)).astype(np.float32)
    bits = np.array([8, 6, 4, 2], dtype=np.uint8)
    w = np.ones(n, dtype=np.float32)
    mask = np.array([1, 1, 0, 1], dtype=np.uint8)
    for mode in (O.SCALE_L2, O.SCALE_MAXABS):
        s1, sc1, gh1 = O.step(G, csr, bits, w, mask, 99, 5, mode)
        s2, sc2 = O.encode_quantize(G, csr, bits, 99, 5, mode)
        assert all(np.array_equal(a, b) for a, b in zip(s1, s2)) and np.array_equal(sc1, sc2)
        assert np.array_equal(gh1, O.decode(s2, sc2, bits, w, mask, d))
        for i in range(n):
            f = O.encode(G, csr, i)
            assert sc1[i] == (O.scale_l2(f) if mode == O.SCALE_L2 else O.scale_maxabs(f))
            assert np.array_equal(O.unpack(s1[i], d, int(bits[i])),
                                  O.codes_range(G, csr, i, int(bits[i]), sc1[i], 99, 5, 0, d))
        # a window computed on its own equals the same window of the full run
        assert np.array_equal(O.codes_range(G, csr, 1, 6, sc1[1], 99, 5, 300, 340),
                              O.unpack(s1[1], d, 6)[300:340])
