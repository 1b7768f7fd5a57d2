"""Pins of the oracle's counter-based generator and of the draw layout (CPU only)."""
import os

import numpy as np

from oracle import agc_oracle as O

MUL_A, MUL_B = 0xD2511F53, 0xCD9E8D57
WEYL = (0x9E3779B9, 0xBB67AE85)
MASK = 0xFFFFFFFF


def test_known_answers(golden_dir):
    """Published known answers of Philox4x32-10 (tests/golden/philox4x32_10_kat.txt)."""
    rows = 0
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            v = [int(t, 16) for t in line.split()]
            out = O.philox4x32_10(v[0:4], v[4:6])
            assert [int(x) for x in out] == v[6:10]
            rows += 1
    assert rows == 3


def _inverse(out, key):
    """Run the ten rounds backwards: each round is a bijection of the counter because the
    multipliers are odd (invertible mod 2^32).  Written from the round's algebra, not from
    the forward code."""
    inv_a, inv_b = pow(MUL_A, -1, 1 << 32), pow(MUL_B, -1, 1 << 32)
    c = [int(x) for x in out]
    for rnd in range(9, -1, -1):
        k0 = (key[0] + rnd * WEYL[0]) & MASK
        k1 = (key[1] + rnd * WEYL[1]) & MASK
        p2 = (c[1] * inv_b) & MASK          # word 2 before the round
        p0 = (c[3] * inv_a) & MASK          # word 0 before the round
        p1 = c[0] ^ ((MUL_B * p2) >> 32) ^ k0
        p3 = c[2] ^ ((MUL_A * p0) >> 32) ^ k1
        c = [p0, p1, p2, p3]
    return c


def test_bijection_roundtrip():
    rng = np.random.default_rng(1)
    for _ in range(200):
        ctr = [int(x) for x in rng.integers(0, 1 << 32, 4)]
        key = [int(x) for x in rng.integers(0, 1 << 32, 2)]
        assert _inverse(O.philox4x32_10(ctr, key), key) == ctr


def test_uniformity_of_fields():
    """16-bit primary fields over many counters: mean, variance and byte chi-square."""
    seed, step = 0x1234567890ABCDEF, 7
    vals = np.array([O.draw(seed, step, w, m)[0] for w in range(4) for m in range(20000)],
                    dtype=np.float64)
    n = vals.size
    assert abs(vals.mean() - 32767.5) < 5 * 65536 / np.sqrt(12 * n)
    assert abs(vals.var() / (65536.0 ** 2 / 12) - 1) < 0.03
    hist = np.bincount((vals.astype(np.int64) >> 8), minlength=256)
    chi2 = ((hist - n / 256) ** 2 / (n / 256)).sum()
    assert chi2 < 255 + 6 * np.sqrt(2 * 255)


def test_draw_layout():
    """One primary block serves coordinates 4g..4g+3 of workers 2q and 2q+1 as eight
    distinct 16-bit fields; the secondary word comes from a block of its own."""
    seed, step = 0xDEADBEEF12345678, (5 << 32) | 9
    key = [seed & MASK, seed >> 32]
    for q in (0, 3):
        for g in (0, 11):
            blk = O.philox4x32_10([g, q, step & MASK, step >> 32], key)
            fields = []
            for wd in blk:
                fields += [int(wd) & 0xFFFF, int(wd) >> 16]
            got = [O.draw(seed, step, 2 * q + wi, 4 * g + c)[0] for wi in range(2) for c in range(4)]
            assert got == fields
            for wi in range(2):
                blk2 = O.philox4x32_10([g, 0x80000000 | (2 * q + wi), step & MASK, step >> 32], key)
                assert [O.draw(seed, step, 2 * q + wi, 4 * g + c)[1] for c in range(4)] == [int(x) for x in blk2]


def test_streams_differ_by_seed_step_worker():
    base = [O.draw(1, 1, 0, m)[0] for m in range(64)]
    assert base != [O.draw(2, 1, 0, m)[0] for m in range(64)]
    assert base != [O.draw(1, 2, 0, m)[0] for m in range(64)]
    assert base != [O.draw(1, 1, 2, m)[0] for m in range(64)]
    assert base == [O.draw(1, 1, 0, m)[0] for m in range(64)]
