"""GPU test of agc_decode_noalloc, the decode entry point for callers that cannot allocate device
memory: through the C ABI, its estimate must equal agc_decode's bit for bit (and therefore the
oracle's decode) on two calls in a row, the second with a smaller input, so that whatever the
first call left in the library's fixed device array cannot leak into the second."""
import numpy as np
import pytest

from oracle import agc_oracle as O
from paper_2605_15890_amd import api

from gpu_util import cyclic_csr, to_device

pytestmark = pytest.mark.gpu


def _problem(rng, n, d, bits, bucket):
    """Codes and scales of one encode (through a context, which is what produces payloads), the
    context's own decode of them, and the oracle's."""
    import torch
    k, s = n, min(3, n)
    row_ptr, col, val = cyclic_csr(rng, n, s)
    w = rng.uniform(0.5, 2.0, n).astype(np.float32)
    G = rng.standard_normal((k, d)).astype(np.float32)
    ctx = api.Context(n, k, d, scale_mode=api.AGC_SCALE_MAXABS, allow_1bit=True, bucket=bucket)
    ctx.agc_set_code(row_ptr, col, val)
    codes, scales, ghat = ctx.alloc_outputs(bits)
    ctx.agc_encode_quantize(to_device(G), bits, 4242, 9, codes, scales)
    torch.cuda.synchronize()
    return ctx, codes, scales, ghat, w


def _check(ctx, n, d, bucket, codes, scales, bits, w, mask, ghat):
    import torch
    ctx.agc_decode(codes, scales, bits, w, mask, ghat)
    got = torch.full_like(ghat, float("nan"))
    api.agc_decode_noalloc(n, d, bucket, codes, scales, bits, w, mask, got)
    torch.cuda.synchronize()
    assert torch.equal(ghat.view(torch.int32), got.view(torch.int32)), (n, d, bucket, mask)
    streams = [c.cpu().numpy() for c in codes]
    sc = scales.cpu().numpy()
    want = (O.decode_bucket if bucket else O.decode)(streams, sc, bits, w, mask, d, 0, d)
    assert np.array_equal(want.view(np.uint32), got.cpu().numpy().view(np.uint32)), (n, d, bucket, mask)


@pytest.mark.parametrize("bucket", [0, 256])
def test_noalloc_decode_equals_context_decode_twice(bucket):
    rng = np.random.default_rng(7 + bucket)
    # first call: 9 workers, several tiles and a ragged tail; all arrive, so all 9 table slots are written
    n1, d1 = 9, 70001
    bits1 = np.array([1, 2, 3, 4, 5, 7, 9, 12, 16], dtype=np.uint8)
    ctx1, codes1, scales1, ghat1, w1 = _problem(rng, n1, d1, bits1, bucket)
    _check(ctx1, n1, d1, bucket, codes1, scales1, bits1, w1, np.ones(n1, np.uint8), ghat1)
    # second call, smaller in every respect: 4 workers of which 2 arrive, 1000 coordinates
    n2, d2 = 4, 1000
    bits2 = np.array([8, 2, 1, 6], dtype=np.uint8)
    ctx2, codes2, scales2, ghat2, w2 = _problem(rng, n2, d2, bits2, bucket)
    _check(ctx2, n2, d2, bucket, codes2, scales2, bits2, w2, np.array([0, 1, 0, 1], np.uint8), ghat2)
    # nobody arrives: the estimate is exactly zero, whatever the array still holds
    _check(ctx2, n2, d2, bucket, codes2, scales2, bits2, w2, np.zeros(n2, np.uint8), ghat2)
    # and the larger problem once more
    _check(ctx1, n1, d1, bucket, codes1, scales1, bits1, w1, np.array([1, 0, 1, 1, 0, 1, 1, 1, 0], np.uint8), ghat1)
    ctx1.close()
    ctx2.close()


def test_noalloc_decode_rejects_bad_arguments_without_touching_the_gpu_state():
    import torch
    rng = np.random.default_rng(3)
    n, d = 3, 513
    bits = np.array([2, 4, 8], dtype=np.uint8)
    ctx, codes, scales, ghat, w = _problem(rng, n, d, bits, 0)
    mask = np.ones(n, np.uint8)
    bad = bits.copy()
    bad[1] = 17
    assert api.agc_decode_noalloc(n, d, 0, codes, scales, bad, w, mask, ghat, check=False) == api.AGC_EBITS
    assert api.agc_decode_noalloc(n, d, 128, codes, scales, bits, w, mask, ghat, check=False) == api.AGC_EINVAL
    off = torch.empty(d + 1, dtype=torch.float32, device="cuda")[1:]
    assert api.agc_decode_noalloc(n, d, 0, codes, scales, bits, w, mask, off, check=False) == api.AGC_EALIGN
    _check(ctx, n, d, 0, codes, scales, bits, w, mask, ghat)     # still works afterwards
    ctx.close()
