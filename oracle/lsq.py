"""Oracle of the least-squares stage that produces the partial gradients (Sec. II-A:
g_j = grad L(D_j, beta) with L(D_j, beta) = 0.5 * ||X_j beta - y_j||^2), binary64 / numpy.

TEST INFRASTRUCTURE (see agc_oracle.c).  X is stored as bfloat16, i.e. as the upper 16 bits of
a binary32 number; every bfloat16 value is exactly representable in binary64.
"""
import numpy as np


def bf16_bits_to_f64(bits):
    """uint16 array of bfloat16 bit patterns -> binary64 values (exact)."""
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def f32_to_bf16_bits(x):
    """binary32 -> bfloat16 bit patterns, round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return rounded.astype(np.uint16)


def residual(X_bits, y, beta):
    return bf16_bits_to_f64(X_bits) @ np.asarray(beta, dtype=np.float64) - np.asarray(y, dtype=np.float64)


def loss(X_bits, y, beta):
    r = residual(X_bits, y, beta)
    return 0.5 * float(r @ r)


def partial_gradients(X_bits, y, beta, k):
    """G[p] = X_p^T (X_p beta - y_p) for k equal contiguous partitions; returns (G, residual)."""
    X = bf16_bits_to_f64(X_bits)
    r = X @ np.asarray(beta, dtype=np.float64) - np.asarray(y, dtype=np.float64)
    n = X.shape[0]
    rows = n // k
    G = np.stack([X[p * rows:(p + 1) * rows].T @ r[p * rows:(p + 1) * rows] for p in range(k)])
    return G, r
