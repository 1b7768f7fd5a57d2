"""GPU checks of the measurement hooks of include/agc_debug.h: the calibration copy copies, and the
access-pattern probe reads and writes exactly the region its header documents."""
import numpy as np
import pytest

from paper_2605_15890_amd import api

pytestmark = pytest.mark.gpu


def test_calibration_copy_copies():
    import torch
    src = torch.arange(1 << 16, dtype=torch.float32, device="cuda")
    dst = torch.zeros_like(src)
    api.agc_calibration_copy(dst, src, src.numel() * 4)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)


@pytest.mark.parametrize("k,d,piece", [(5, 2048 + 300, 96), (3, 256, 16), (64, 4096, 1024), (2, 255, 96)])
def test_stream_rows_touches_exactly_its_output_region(k, d, piece):
    """Per-wave mode writes, for row j and block u, the first piece/16 float4 of the block's row data
    to stream j; the workgroup-flush mode writes the same region (other values); nothing beyond the
    k * floor(d/256) * piece bytes is touched, and piece = 0 writes nothing."""
    import torch
    rng = np.random.default_rng(k * 1000 + d)
    G_host = rng.standard_normal((k, d)).astype(np.float32)
    G = api.padded_rows(k, d)
    G.copy_(torch.from_numpy(G_host))
    nblocks = d // 256
    region = max(4, k * nblocks * piece // 4)            # floats
    canary = 12345.0
    for flush, occ, fma in ((False, 0, 0), (True, 0, 0), (True, 4, 0), (True, 4, 100), (True, 4, 40), (False, 4, 0)):
        out = torch.full((region + 1024,), canary, dtype=torch.float32, device="cuda")
        api.agc_debug_stream_rows(G, piece, out, wg_flush=flush, waves_per_simd=occ, fma_per_row=fma)
        torch.cuda.synchronize()
        o = out.cpu().numpy()
        assert np.all(o[k * nblocks * piece // 4:] == canary)          # nothing past the region
        if nblocks:
            assert not np.any(o[:k * nblocks * piece // 4] == canary)  # all of the region written
        if not flush and nblocks:
            per = piece // 4                                           # floats per piece
            want = np.stack([G_host[j, :nblocks * 256].reshape(nblocks, 256)[:, :per].reshape(-1) for j in range(k)])
            assert np.array_equal(o[:k * nblocks * per].reshape(k, nblocks * per), want)
    for per_wave in (1, 2):
        out = torch.full((1024,), canary, dtype=torch.float32, device="cuda")
        api.agc_debug_stream_rows(G, 0, out, blocks_per_wave=per_wave)
        torch.cuda.synchronize()
        assert bool((out == canary).all())
    for bad in (dict(waves_per_simd=3), dict(fma_per_row=8, waves_per_simd=4), dict(fma_per_row=100)):
        with pytest.raises(api.AgcError):
            api.agc_debug_stream_rows(G, 0, out, **bad)
    with pytest.raises(api.AgcError):     # the two-block walk is a reads-only form
        api.agc_debug_stream_rows(G, piece, torch.empty(region + 1024, dtype=torch.float32, device="cuda"),
                                  blocks_per_wave=2)
