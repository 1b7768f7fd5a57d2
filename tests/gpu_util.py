"""Helpers shared by the GPU parity tests: run the HIP path through the C ABI binding and the
oracle on the same inputs, and compare element by element."""
import numpy as np

from oracle import agc_oracle as O
from paper_2605_15890_amd import api


def to_device(G_host):
    """k x d float32 on the GPU with a row stride that is a multiple of 4 elements."""
    import torch
    k, d = G_host.shape
    G = api.padded_rows(k, d)
    G.copy_(torch.from_numpy(np.ascontiguousarray(G_host)))
    return G


def run_hip(G_dev, n, k, d, row_ptr, col, val, bits, w, mask, seed, step, scale_mode,
            allow_1bit=False, force_generic=False, expect_path=None):
    """One agc_step on the GPU.  Returns (streams, scales, ghat) as host numpy arrays."""
    import torch
    ctx = api.Context(n, k, d, scale_mode=scale_mode, allow_1bit=allow_1bit, force_generic=force_generic)
    try:
        ctx.agc_set_code(row_ptr, col, val)
        if expect_path is not None:
            assert ctx.agc_code_path() == expect_path, (ctx.agc_code_path(), expect_path)
        codes, scales, ghat = ctx.alloc_outputs(bits)
        for c in codes:
            c.fill_(0xA5)          # the kernels must overwrite every byte, padding included
        ghat.fill_(float("nan"))
        ctx.agc_step(G_dev, bits, w, mask, seed, step, codes, scales, ghat)
        torch.cuda.synchronize()
        return [c.cpu().numpy() for c in codes], scales.cpu().numpy(), ghat.cpu().numpy()
    finally:
        ctx.close()


def compare_with_oracle(G_host, k, row_ptr, col, val, bits, w, mask, seed, step, scale_mode,
                        hip_out, tag=""):
    """Bit-exact codes (flip count 0), equal scales, decode within 1e-5 relative L2 (and, as
    the arithmetic is specified operation by operation, in fact identical)."""
    streams, scales, ghat = hip_out
    csr = O.Csr(row_ptr, col, val, k)
    o_streams, o_scales, o_ghat = O.step(G_host, csr, bits, w, mask, seed, step, scale_mode)
    assert np.array_equal(scales.view(np.uint32), o_scales.view(np.uint32)), (tag, scales, o_scales)
    d = G_host.shape[1]
    flips = 0
    for i in range(csr.n):
        assert streams[i].shape == o_streams[i].shape, (tag, i)
        if not np.array_equal(streams[i], o_streams[i]):
            a = O.unpack(streams[i], d, int(bits[i]))
            b = O.unpack(o_streams[i], d, int(bits[i]))
            diff = int(np.count_nonzero(a != b))
            assert diff > 0, (tag, "padding bytes differ for worker", i)
            flips += diff
    assert flips == 0, (tag, "code flips", flips)
    den = float(np.linalg.norm(o_ghat.astype(np.float64)))
    err = float(np.linalg.norm(ghat.astype(np.float64) - o_ghat.astype(np.float64)))
    assert err <= 1e-5 * den or (den == 0.0 and err == 0.0), (tag, err, den)
    assert np.array_equal(ghat.view(np.uint32), o_ghat.view(np.uint32)), (tag, "decode not identical")
    return o_streams, o_scales, o_ghat


def random_csr(rng, n, k, max_nnz_per_row=5, allow_empty=True):
    row_ptr, col, val = [0], [], []
    for i in range(n):
        cnt = int(rng.integers(0 if allow_empty else 1, min(k, max_nnz_per_row) + 1))
        cols = rng.choice(k, size=cnt, replace=False)
        col += [int(c) for c in cols]
        val += [float(v) for v in rng.standard_normal(cnt)]
        row_ptr.append(len(col))
    return (np.array(row_ptr, dtype=np.int32), np.array(col, dtype=np.int32),
            np.array(val, dtype=np.float32))


def cyclic_csr(rng, n, s):
    row_ptr = np.arange(n + 1, dtype=np.int32) * s
    col = np.array([(i + u) % n for i in range(n) for u in range(s)], dtype=np.int32)
    val = rng.uniform(0.1, 1.0, n * s).astype(np.float32) * rng.choice([-1.0, 1.0], n * s).astype(np.float32)
    return row_ptr, col, val


def monotone_csr(rng, n, k, max_len):
    """Random code of the monotone-interval shape: runs of consecutive columns whose two ends
    never decrease; several workers may start at the same column, columns may be skipped."""
    row_ptr, col, val = [0], [], []
    lo = hi = 0
    for i in range(n):
        lo = min(k - 1, max(lo, hi - int(rng.integers(0, 2))) + (int(rng.integers(0, 2)) if i else 0))
        length = int(rng.integers(1, max_len + 1))
        new_hi = min(k - 1, max(hi, lo + length - 1))
        if new_hi - lo + 1 > max_len:
            lo = new_hi - max_len + 1
        hi = new_hi
        cols = list(range(lo, hi + 1))
        col += cols
        val += list(rng.uniform(-1.0, 1.0, len(cols)).astype(np.float32))
        row_ptr.append(len(col))
    return np.array(row_ptr, np.int32), np.array(col, np.int32), np.array(val, np.float32)
