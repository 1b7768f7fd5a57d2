"""Randomised sweep of valid problem shapes on the GPU against the oracle: worker / partition
counts, band widths, monotone-interval and general sparse codes, ragged lengths, bit-widths 1..16, arrival masks,
both scale kinds, per-vector and bucket-wise scales, fused and two-pass steps.  Every case is
seeded; codes must be bit-exact, scales and estimates identical."""
import numpy as np
import pytest

from oracle import agc_oracle as O
from paper_2605_15890_amd import api

from gpu_util import cyclic_csr, monotone_csr, random_csr, to_device

pytestmark = pytest.mark.gpu


def _case(seed):
    rng = np.random.default_rng(seed)
    kind = rng.random()
    if kind < 0.45:      # cyclic band
        n = k = int(rng.integers(1, 40))
        s = int(rng.integers(1, min(8, k) + 1))
        code = cyclic_csr(rng, n, s)
        path = s
    elif kind < 0.75:    # monotone intervals (window drivers)
        n, k = int(rng.integers(1, 70)), int(rng.integers(1, 70))
        code = monotone_csr(rng, n, k, int(rng.choice([1, 2, 3, 4, 6, 8])))
        longest = int(np.diff(code[0]).max())
        path = 100 + (2 if longest <= 2 else 4 if longest <= 4 else 8)
        if n == k and np.array_equal(code[1], np.arange(n)) and longest == 1:
            path = 1     # a diagonal code is also a cyclic band of width 1, which is looked for first
    else:
        n, k = int(rng.integers(1, 40)), int(rng.integers(1, 40))
        code = random_csr(rng, n, k, int(rng.choice([1, 2, 3, 4, 5, 8, 12])))
        path = None
    d = int(rng.choice([1, 2, 7, 64, 255, 256, 257, 511, 1024, 1500, 4096, 5000, 12345]))
    allow_1bit = rng.random() < 0.5
    bits = rng.integers(1 if allow_1bit else 2, 17, n).astype(np.uint8)
    w = rng.uniform(0.2, 3.0, n).astype(np.float32)
    mask = (rng.random(n) < 0.7).astype(np.uint8)
    scale = float(10.0 ** rng.uniform(-6, 4))
    G = (rng.standard_normal((k, d)) * scale).astype(np.float32)
    if rng.random() < 0.3:
        G[rng.integers(0, k)] = 0.0                        # an all-zero partition
    return dict(n=n, k=k, d=d, code=code, path=path, bits=bits, w=w, mask=mask, G=G, allow_1bit=allow_1bit,
                scale_mode=int(rng.integers(0, 2)), bucket=int(rng.choice([0, 256])), unfused=bool(rng.integers(0, 2)),
                seed=int(rng.integers(0, 2 ** 62)), step=int(rng.integers(0, 2 ** 40)))


@pytest.mark.parametrize("seed", range(72))
def test_random_case(seed):
    import torch
    c = _case(1000 + seed)
    n, k, d = c["n"], c["k"], c["d"]
    ctx = api.Context(n, k, d, scale_mode=c["scale_mode"], allow_1bit=c["allow_1bit"], bucket=c["bucket"],
                      unfused_step=c["unfused"])
    try:
        ctx.agc_set_code(*c["code"])
        if c["path"] is not None:
            assert ctx.agc_code_path() == c["path"]
        codes, scales, ghat = ctx.alloc_outputs(c["bits"])
        for t in codes:
            t.fill_(0x5A)
        ghat.fill_(float("nan"))
        ctx.agc_step(to_device(c["G"]), c["bits"], c["w"], c["mask"], c["seed"], c["step"], codes, scales, ghat)
        torch.cuda.synchronize()
        csr = O.Csr(*c["code"], k)
        oracle_step = O.step_bucket if c["bucket"] else O.step
        o_streams, o_scales, o_ghat = oracle_step(c["G"], csr, c["bits"], c["w"], c["mask"], c["seed"], c["step"],
                                                  c["scale_mode"])
        tag = {kk: vv for kk, vv in c.items() if kk not in ("G", "code")}
        assert np.array_equal(scales.cpu().numpy().view(np.uint32), o_scales.view(np.uint32)), tag
        for i in range(n):
            assert np.array_equal(codes[i].cpu().numpy(), o_streams[i]), (tag, i)
        assert np.array_equal(ghat.cpu().numpy().view(np.uint32), o_ghat.view(np.uint32)), tag
    finally:
        ctx.close()
