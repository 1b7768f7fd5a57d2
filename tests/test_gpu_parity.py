"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Codes must be bit-exact (flip count 0), scales equal, decode within 1e-5 relative L2
(checked, and in fact identical because both sides follow one operation-by-operation
definition)."""
import numpy as np
import pytest

from oracle import agc_oracle as O
from paper_2605_15890_amd import api
from paper_2605_15890_amd import inputs as I

from gpu_util import compare_with_oracle, cyclic_csr, monotone_csr, random_csr, run_hip, to_device

pytestmark = pytest.mark.gpu

MODES = [api.AGC_SCALE_MAXABS, api.AGC_SCALE_L2]


def _config_code(cfg, p, bits):
    """Cyclic code of the configuration from the library's host routine."""
    pc = api.agc_phi_coef_balanced(p, int(np.sum(bits)))
    return api.agc_build_cyclic_code(cfg.n, cfg.k, cfg.s, p, np.maximum(bits, 2), pc)


@pytest.mark.parametrize("scale_mode", MODES)
@pytest.mark.parametrize("force_generic", [False, True])
def test_tiny_config_full_parity(scale_mode, force_generic):
    cfg = I.CONFIGS["tiny"]
    p, bits = I.straggler_probs(cfg), I.random_bits(cfg)
    row_ptr, col, val, w = _config_code(cfg, p, bits)
    G = I.partial_gradients_numpy(cfg)
    Gd = to_device(G)
    for it in range(3):
        mask = I.arrival_mask(cfg, p, it)
        out = run_hip(Gd, cfg.n, cfg.k, cfg.d, row_ptr, col, val, bits, w, mask, cfg.philox_seed, it,
                      scale_mode, force_generic=force_generic, expect_path=0 if force_generic else cfg.s)
        compare_with_oracle(G, cfg.k, row_ptr, col, val, bits, w, mask, cfg.philox_seed, it, scale_mode,
                            out, tag=f"tiny it={it}")


@pytest.mark.parametrize("d", [1, 3, 4, 5, 127, 128, 129, 255, 256, 257, 1000, 1023, 1025, 4097, 70001])
def test_ragged_sizes_cyclic_and_generic(d):
    """Sizes around every tile boundary (float4, 128-code group, 256-coordinate block, 1024
    segment/workgroup), mixed bit-widths including 1 and 16."""
    rng = np.random.default_rng(d)
    n = k = 6
    s = 1 + d % 4
    row_ptr, col, val = cyclic_csr(rng, n, s)
    bits = np.array([1, 2, 3, 5, 8, 16], dtype=np.uint8)
    w = rng.uniform(0.5, 2, n).astype(np.float32)
    mask = np.array([1, 0, 1, 1, 1, 1], dtype=np.uint8)
    G = rng.standard_normal((k, d)).astype(np.float32)
    Gd = to_device(G)
    for scale_mode in MODES:
        for force_generic in (False, True):
            out = run_hip(Gd, n, k, d, row_ptr, col, val, bits, w, mask, 42, 7, scale_mode, allow_1bit=True,
                          force_generic=force_generic, expect_path=0 if force_generic else s)
            compare_with_oracle(G, k, row_ptr, col, val, bits, w, mask, 42, 7, scale_mode, out,
                                tag=f"d={d} mode={scale_mode} generic={force_generic}")


@pytest.mark.parametrize("s", [1, 2, 3, 4, 5, 6, 7, 8])
def test_every_band_width(s):
    rng = np.random.default_rng(100 + s)
    n = k = 11 if s <= 5 else 9
    d = 3000 + 37 * s
    row_ptr, col, val = cyclic_csr(rng, n, s)
    bits = rng.integers(2, 13, n).astype(np.uint8)
    w = rng.uniform(0.5, 2, n).astype(np.float32)
    mask = (rng.random(n) < 0.7).astype(np.uint8)
    G = (rng.standard_normal((k, d)) * 10 ** rng.uniform(-3, 3)).astype(np.float32)
    out = run_hip(to_device(G), n, k, d, row_ptr, col, val, bits, w, mask, 5, 1 << 40, api.AGC_SCALE_MAXABS,
                  expect_path=s)
    compare_with_oracle(G, k, row_ptr, col, val, bits, w, mask, 5, 1 << 40, api.AGC_SCALE_MAXABS, out,
                        tag=f"s={s}")


@pytest.mark.parametrize("n,k", [(1, 1), (1, 7), (7, 1), (5, 9), (9, 5), (33, 20), (64, 64), (200, 17)])
def test_general_codes(n, k):
    """Arbitrary sparse codes (empty rows, long rows, n != k, repeated use of one partition) take
    the gather path; the optimally structured interval code of Sec. III-A follows."""
    rng = np.random.default_rng(n * 1000 + k)
    d = int(rng.integers(1500, 6000))
    G = rng.standard_normal((k, d)).astype(np.float32)
    Gd = to_device(G)
    bits = rng.integers(2, 9, n).astype(np.uint8)
    w = rng.uniform(0.5, 2, n).astype(np.float32)
    mask = (rng.random(n) < 0.6).astype(np.uint8)
    for max_nnz in (4, 8, 13):
        row_ptr, col, val = random_csr(rng, n, k, max_nnz)
        outs = []
        for force_generic in (False, True):
            out = run_hip(Gd, n, k, d, row_ptr, col, val, bits, w, mask, 77, 3, api.AGC_SCALE_L2,
                          force_generic=force_generic,
                          # a tiny random code may happen to be a band or a run of intervals
                          expect_path=0 if force_generic or n >= 30 else None)
            compare_with_oracle(G, k, row_ptr, col, val, bits, w, mask, 77, 3, api.AGC_SCALE_L2, out,
                                tag=f"random csr max_nnz={max_nnz} generic={force_generic}")
            outs.append(out)
        assert all(np.array_equal(a, b) for a, b in zip(outs[0][0], outs[1][0]))
    p = rng.uniform(0.05, 0.6, n)
    row_ptr, col, val, w2 = api.agc_build_code(n, k, p, bits, 0.3)
    out = run_hip(Gd, n, k, d, row_ptr, col, val, bits, w2, mask, 78, 4, api.AGC_SCALE_MAXABS)
    compare_with_oracle(G, k, row_ptr, col, val, bits, w2, mask, 78, 4, api.AGC_SCALE_MAXABS, out,
                        tag="interval code")


@pytest.mark.parametrize("kind", ["cyclic8", "cyclic3", "window", "general_wide"])
def test_maximum_worker_count(kind):
    """n = 256 workers, the most the library takes (their arguments fill the kernel argument
    block), with every driver: cyclic bands, monotone intervals, and a general code over k = 4096
    partitions.  Bit-widths cover 1..16, both scale kinds, ragged d."""
    rng = np.random.default_rng({"cyclic8": 1, "cyclic3": 2, "window": 3, "general_wide": 4}[kind])
    n = api.AGC_MAX_WORKERS
    if kind.startswith("cyclic"):
        k, s = n, int(kind[-1])
        row_ptr, col, val = cyclic_csr(rng, n, s)
        path = s
    elif kind == "window":
        k = 300
        row_ptr, col, val = monotone_csr(rng, n, k, 8)
        path = 108
    else:
        k = 4096
        row_ptr, col, val = random_csr(rng, n, k, 5)
        path = 0
    d = 777
    bits = ((np.arange(n) % 16) + 1).astype(np.uint8)
    rng.shuffle(bits)
    w = rng.uniform(0.5, 2, n).astype(np.float32)
    mask = (rng.random(n) < 0.8).astype(np.uint8)
    G = rng.standard_normal((k, d)).astype(np.float32)
    Gd = to_device(G)
    for scale_mode in MODES:
        out = run_hip(Gd, n, k, d, row_ptr, col, val, bits, w, mask, 11, 12, scale_mode, allow_1bit=True,
                      expect_path=path)
        compare_with_oracle(G, k, row_ptr, col, val, bits, w, mask, 11, 12, scale_mode, out,
                            tag=f"n=256 {kind} mode={scale_mode}")


def test_degenerate_inputs():
    """All stragglers (estimate exactly 0), everyone arrived, an all-zero coded vector
    (scale 0), and max-abs coordinates that sit exactly on the top level."""
    rng = np.random.default_rng(9)
    n = k = 4
    d = 2049
    row_ptr, col, val = cyclic_csr(rng, n, 2)
    G = rng.standard_normal((k, d)).astype(np.float32)
    G[1] = 0.0
    G[2] = 0.0          # worker 1 = f(g_1, g_2) is identically zero
    bits = np.array([2, 4, 8, 3], dtype=np.uint8)
    w = np.ones(n, dtype=np.float32)
    Gd = to_device(G)
    for mask in ([0, 0, 0, 0], [1, 1, 1, 1], [0, 1, 0, 0]):
        mask = np.array(mask, dtype=np.uint8)
        out = run_hip(Gd, n, k, d, row_ptr, col, val, bits, w, mask, 1, 2, api.AGC_SCALE_MAXABS)
        _, o_scales, o_ghat = compare_with_oracle(G, k, row_ptr, col, val, bits, w, mask, 1, 2,
                                                  api.AGC_SCALE_MAXABS, out, tag=f"mask={mask}")
        assert o_scales[1] == 0.0
        if mask.sum() == 0 or list(mask) == [0, 1, 0, 0]:
            assert np.all(out[2] == 0)
    # the coordinate that carries the maximum is coded as +-L, never L+1
    streams, scales, _ = out
    csr = O.Csr(row_ptr, col, val, k)
    for i in (0, 2, 3):
        f = O.encode(G, csr, i)
        m = int(np.argmax(np.abs(f)))
        code = int(O.unpack(streams[i], d, int(bits[i]))[m])
        assert code & ((1 << (bits[i] - 1)) - 1) == O.levels(int(bits[i]))


def test_config2_full_parity():
    """n = k = 16, s = 3, d = 2^20, bits from the allocator at 4 bits per coordinate."""
    cfg = I.CONFIGS["n16_d1m"]
    p = I.straggler_probs(cfg)
    z_tot = cfg.bits_law[1] * cfg.n
    bits = api.agc_alloc_bits(p, api.agc_phi_coef_balanced(p, z_tot), z_tot, 2, 8)
    row_ptr, col, val, w = _config_code(cfg, p, bits)
    G = I.partial_gradients_numpy(cfg)
    Gd = to_device(G)
    for scale_mode in MODES:
        mask = I.arrival_mask(cfg, p, 0)
        out = run_hip(Gd, cfg.n, cfg.k, cfg.d, row_ptr, col, val, bits, w, mask, cfg.philox_seed, 0,
                      scale_mode, expect_path=cfg.s)
        compare_with_oracle(G, cfg.k, row_ptr, col, val, bits, w, mask, cfg.philox_seed, 0, scale_mode,
                            out, tag=f"config2 mode={scale_mode}")


def test_stage_calls_equal_step_and_are_deterministic():
    import torch
    rng = np.random.default_rng(21)
    n = k = 8
    d = 5000
    row_ptr, col, val = cyclic_csr(rng, n, 3)
    bits = rng.integers(2, 9, n).astype(np.uint8)
    w = rng.uniform(0.5, 2, n).astype(np.float32)
    mask = (rng.random(n) < 0.6).astype(np.uint8)
    G = rng.standard_normal((k, d)).astype(np.float32)
    Gd = to_device(G)
    a = run_hip(Gd, n, k, d, row_ptr, col, val, bits, w, mask, 3, 9, api.AGC_SCALE_L2)
    b = run_hip(Gd, n, k, d, row_ptr, col, val, bits, w, mask, 3, 9, api.AGC_SCALE_L2)
    assert all(np.array_equal(x, y) for x, y in zip(a[0], b[0]))
    assert np.array_equal(a[1], b[1]) and np.array_equal(a[2].view(np.uint32), b[2].view(np.uint32))
    ctx = api.Context(n, k, d, scale_mode=api.AGC_SCALE_L2)
    ctx.agc_set_code(row_ptr, col, val)
    codes, scales, ghat = ctx.alloc_outputs(bits)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):       # a non-default stream, passed explicitly
        ctx.agc_encode_quantize(Gd, bits, 3, 9, codes, scales, stream=side.cuda_stream)
        ctx.agc_decode(codes, scales, bits, w, mask, ghat, stream=side.cuda_stream)
    side.synchronize()
    assert all(np.array_equal(x.cpu().numpy(), y) for x, y in zip(codes, a[0]))
    assert np.array_equal(ghat.cpu().numpy().view(np.uint32), a[2].view(np.uint32))
    # different step -> different draws
    c = run_hip(Gd, n, k, d, row_ptr, col, val, bits, w, mask, 3, 10, api.AGC_SCALE_L2)
    assert any(not np.array_equal(x, y) for x, y in zip(a[0], c[0]))
    ctx.close()


def test_argument_errors_are_reported_not_launched():
    import torch
    n = k = 4
    d = 1024
    ctx = api.Context(n, k, d)
    bits = np.array([2, 3, 4, 5], dtype=np.uint8)
    codes, scales, ghat = ctx.alloc_outputs(bits)
    G = api.padded_rows(k, d)
    w = np.ones(n, dtype=np.float32)
    mask = np.ones(n, dtype=np.uint8)
    assert ctx.agc_step(G, bits, w, mask, 1, 1, codes, scales, ghat, check=False) == api.AGC_ESTATE
    rng = np.random.default_rng(0)
    ctx.agc_set_code(*cyclic_csr(rng, n, 2))
    assert ctx.agc_step(G, np.array([1, 3, 4, 5], np.uint8), w, mask, 1, 1, codes, scales, ghat, check=False) == api.AGC_EBITS
    assert ctx.agc_step(G, np.array([2, 3, 4, 17], np.uint8), w, mask, 1, 1, codes, scales, ghat, check=False) == api.AGC_EBITS
    Gbad = torch.zeros((k, d + 1), dtype=torch.float32, device="cuda")[:, 1:]     # base off by 4 bytes
    assert ctx.agc_step(Gbad, bits, w, mask, 1, 1, codes, scales, ghat, check=False) == api.AGC_EALIGN
    Gld = torch.zeros((k, d + 2), dtype=torch.float32, device="cuda")[:, :d]      # ldg % 4 != 0
    assert ctx.agc_step(Gld, bits, w, mask, 1, 1, codes, scales, ghat, check=False) == api.AGC_EALIGN
    gh_bad = torch.zeros(d + 1, dtype=torch.float32, device="cuda")[1:]
    assert ctx.agc_step(G, bits, w, mask, 1, 1, codes, scales, gh_bad, check=False) == api.AGC_EALIGN
    with pytest.raises(api.AgcError) as e:
        ctx.agc_set_code(np.array([0, 1, 2, 3, 4], np.int32), np.array([0, 1, 2, 9], np.int32),
                         np.ones(4, np.float32))
    assert e.value.status == api.AGC_ESHAPE
    assert ctx.agc_step(G, bits, w, mask, 1, 1, codes, scales, ghat, check=False) == api.AGC_OK
    torch.cuda.synchronize()
    # the binding knows the tensors behind the pointers and refuses buffers that are too small
    small = [c[: c.numel() // 2] for c in codes]
    for call in (lambda: ctx.agc_step(G, bits, w, mask, 1, 1, small, scales, ghat),
                 lambda: ctx.agc_step(G, bits + 1, w, mask, 1, 1, codes, scales, ghat),
                 lambda: ctx.agc_step(G[:, : d - 4], bits, w, mask, 1, 1, codes, scales, ghat),
                 lambda: ctx.agc_step(G, bits, w, mask, 1, 1, codes, scales, ghat[: d - 1]),
                 lambda: ctx.agc_decode(small, scales, bits, w, mask, ghat)):
        with pytest.raises(api.AgcError) as e:
            call()
        assert e.value.status == api.AGC_ESHAPE
    ctx.close()


@pytest.mark.parametrize("unfused", [True, False])
def test_per_kernel_timing_counts_launches(unfused):
    import torch
    rng = np.random.default_rng(3)
    n = k = 4
    d = 1 << 16
    ctx = api.Context(n, k, d, unfused_step=unfused)
    ctx.agc_set_code(*cyclic_csr(rng, n, 2))
    bits = np.array([2, 3, 4, 5], dtype=np.uint8)
    codes, scales, ghat = ctx.alloc_outputs(bits)
    G = to_device(rng.standard_normal((k, d)).astype(np.float32))
    ctx.agc_profile_enable(True)
    for it in range(150):           # more than the ring holds: the oldest pairs are drained on the way
        ctx.agc_step(G, bits, np.ones(n, np.float32), np.ones(n, np.uint8), 1, it, codes, scales, ghat)
    prof = ctx.agc_profile_read()
    for name in api.KERNEL_NAMES:
        ms, cnt = prof[name]
        if name == "decode" and not unfused:      # the fused step has no separate decode launch
            assert cnt == 0
        else:
            assert cnt == 150 and 0 < ms < 10_000
    ctx.agc_profile_enable(False)
    ctx.agc_step(G, bits, np.ones(n, np.float32), np.ones(n, np.uint8), 1, 0, codes, scales, ghat)
    torch.cuda.synchronize()
    assert all(c == 0 for _, c in ctx.agc_profile_read().values())
    ctx.close()


def test_montecarlo_unbiased_on_gpu():
    """1000 GPU steps on the tiny configuration with fresh arrivals: projections of the mean
    error on fixed directions stay within 3 standard errors of zero."""
    import torch
    cfg = I.CONFIGS["tiny"]
    p, bits = I.straggler_probs(cfg), I.random_bits(cfg)
    row_ptr, col, val, w = _config_code(cfg, p, bits)
    G = I.partial_gradients_numpy(cfg)
    Gd = to_device(G)
    g = torch.from_numpy(G.astype(np.float64).sum(axis=0)).cuda()
    rng = np.random.default_rng(77)
    dirs = rng.standard_normal((8, cfg.d))
    dirs /= np.linalg.norm(dirs, axis=1, keepdims=True)
    dirs_d = torch.from_numpy(dirs).cuda()
    ctx = api.Context(cfg.n, cfg.k, cfg.d)
    ctx.agc_set_code(row_ptr, col, val)
    codes, scales, ghat = ctx.alloc_outputs(bits)
    T = cfg.iters
    proj = torch.zeros((T, 8), dtype=torch.float64, device="cuda")
    for t in range(T):
        ctx.agc_step(Gd, bits, w, I.arrival_mask(cfg, p, t), cfg.philox_seed, t, codes, scales, ghat)
        proj[t] = dirs_d @ (ghat.double() - g)
    proj = proj.cpu().numpy()
    z = proj.mean(axis=0) / (proj.std(axis=0, ddof=1) / np.sqrt(T))
    assert np.all(np.abs(z) < 3.0), z
    ctx.close()


def test_optimal_cyclic_code_runs_on_the_band_path():
    """Weights from the support-restricted optimum (some stored entries are exactly zero): the
    layout is still cyclic, so the register-ring path must take it, with the oracle's bits."""
    cfg = I.CONFIGS["n16_d1m"]
    d = (1 << 16) + 77
    p = I.straggler_probs(cfg)
    z_tot = cfg.bits_law[1] * cfg.n
    bits = api.agc_alloc_bits(p, api.agc_phi_coef_balanced(p, z_tot), z_tot, 2, 8)
    pc = api.agc_phi_coef_balanced(p, int(bits.sum()))
    row_ptr, col, val, w, obj, reach = api.agc_build_cyclic_code_opt(cfg.n, cfg.k, cfg.s, p, bits, pc)
    assert (val == 0).any()
    G = I.partial_gradients_numpy(cfg, d=d)
    Gd = to_device(G)
    for scale_mode in MODES:
        mask = I.arrival_mask(cfg, p, 1)
        out = run_hip(Gd, cfg.n, cfg.k, d, row_ptr, col, val, bits, w, mask, cfg.philox_seed, 1, scale_mode,
                      expect_path=cfg.s)
        compare_with_oracle(G, cfg.k, row_ptr, col, val, bits, w, mask, cfg.philox_seed, 1, scale_mode, out,
                            tag=f"optimal cyclic mode={scale_mode}")


@pytest.mark.parametrize("bucket", [0, 256])
def test_fused_step_equals_two_pass_step(bucket):
    """agc_step forms the estimate inside the quantize pass; with unfused_step it runs the
    stand-alone decode kernel.  Codes, scales and estimate must agree bit for bit (ragged size,
    mixed widths including one bit, a straggler, band and generic path, both scale kinds)."""
    import torch
    rng = np.random.default_rng(21)
    n = k = 7
    d = 3 * 1024 + 333
    bits = np.array([1, 2, 3, 4, 7, 9, 16], dtype=np.uint8)
    w = rng.uniform(0.5, 2, n).astype(np.float32)
    G = to_device(rng.standard_normal((k, d)).astype(np.float32))
    for code in (cyclic_csr(rng, n, 3), random_csr(rng, n, k, 4)):
        for scale_mode in MODES:
            for mask in (np.array([1, 1, 0, 1, 0, 1, 1], np.uint8), np.zeros(n, np.uint8)):
                outs = []
                for unfused in (False, True):
                    ctx = api.Context(n, k, d, scale_mode=scale_mode, allow_1bit=True, bucket=bucket,
                                      unfused_step=unfused)
                    ctx.agc_set_code(*code)
                    codes, scales, ghat = ctx.alloc_outputs(bits)
                    ghat.fill_(float("nan"))
                    ctx.agc_step(G, bits, w, mask, 9, 4, codes, scales, ghat)
                    torch.cuda.synchronize()
                    outs.append((codes, scales, ghat))
                    ctx.close()
                (c0, s0, g0), (c1, s1, g1) = outs
                assert all(torch.equal(a, b) for a, b in zip(c0, c1))
                assert torch.equal(s0.view(torch.int32), s1.view(torch.int32))
                assert torch.equal(g0.view(torch.int32), g1.view(torch.int32))


@pytest.mark.parametrize("n,k,max_len,d", [(3, 1, 1, 300), (5, 9, 2, 1000), (9, 5, 2, 4097), (33, 20, 4, 2048),
                                           (40, 64, 4, 70001), (64, 64, 8, 5000), (200, 17, 8, 1025), (17, 200, 8, 3000)])
def test_monotone_interval_codes_take_the_window_path(n, k, max_len, d):
    rng = np.random.default_rng(n * 1000 + k)
    row_ptr, col, val = monotone_csr(rng, n, k, max_len)
    longest = int(np.diff(row_ptr).max())
    want_path = 100 + (2 if longest <= 2 else 4 if longest <= 4 else 8)
    bits = rng.integers(1, 17, n).astype(np.uint8)
    w = rng.uniform(0.5, 2, n).astype(np.float32)
    mask = (rng.random(n) < 0.7).astype(np.uint8)
    G = rng.standard_normal((k, d)).astype(np.float32)
    Gd = to_device(G)
    for scale_mode in MODES:
        out = run_hip(Gd, n, k, d, row_ptr, col, val, bits, w, mask, 5, 9, scale_mode, allow_1bit=True,
                      expect_path=want_path)
        compare_with_oracle(G, k, row_ptr, col, val, bits, w, mask, 5, 9, scale_mode, out,
                            tag=f"window n={n} k={k} len={longest} mode={scale_mode}")


@pytest.mark.parametrize("name", ["n16_d1m", "resnet18"])
def test_paper_interval_code_on_named_configs(name):
    """The sparse construction of Sec. III-A (contiguous allocation segments) for the named
    configurations, first 2^16+5 coordinates: window path, oracle bits, and the same bits as the
    generic path."""
    cfg = I.CONFIGS[name]
    d = (1 << 16) + 5
    p = I.straggler_probs(cfg)
    bits = I.random_bits(cfg)
    if bits is None:
        z_tot = cfg.bits_law[1] * cfg.n
        bits = api.agc_alloc_bits(p, api.agc_phi_coef_balanced(p, z_tot), z_tot, 2, 8)
    pc = api.agc_phi_coef_balanced(p, int(bits.sum()))
    row_ptr, col, val, w = api.agc_build_code(cfg.n, cfg.k, p, np.maximum(bits, 2), pc)
    G = I.partial_gradients_numpy(cfg, d=d)
    Gd = to_device(G)
    mask = I.arrival_mask(cfg, p, 2)
    outs = []
    for force_generic in (False, True):
        out = run_hip(Gd, cfg.n, cfg.k, d, row_ptr, col, val, bits, w, mask, cfg.philox_seed, 2,
                      api.AGC_SCALE_MAXABS, allow_1bit=cfg.allow_1bit, force_generic=force_generic)
        compare_with_oracle(G, cfg.k, row_ptr, col, val, bits, w, mask, cfg.philox_seed, 2, api.AGC_SCALE_MAXABS,
                            out, tag=f"{name} interval generic={force_generic}")
        outs.append(out)
    assert all(np.array_equal(a, b) for a, b in zip(outs[0][0], outs[1][0]))


# ---------------------------------------------------------------------------------------------
# Max-abs scale pass, two blocks of 256 coordinates per wave (engaged from 20480 blocks on, for
# codes served by a register-ring driver): whole step against the oracle at sizes whose tail is
# a lone full block, a full block followed by a ragged one, or a ragged first block of a pair;
# each row of G carries one dominant entry at a place that only one part of the kernel sees.
# ---------------------------------------------------------------------------------------------
TWO_BLOCK_MIN = 20480


@pytest.mark.parametrize("kind", ["cyclic3", "window4"])
@pytest.mark.parametrize("tail", [0, 256, 300, 513, 767])
def test_two_block_scale_pass_matches_oracle(kind, tail):
    rng = np.random.default_rng(4100 + tail)
    d = TWO_BLOCK_MIN * 256 + tail
    if kind == "cyclic3":
        n = k = 5
        row_ptr, col, val = cyclic_csr(rng, n, 3)
        path = 3
    else:
        n, k = 6, 5
        row_ptr, col, val = monotone_csr(rng, n, k, 4)
        path = None
    G_host = (rng.standard_normal((k, d)) * 0.01).astype(np.float32)
    # dominant entries: second block of a pair, last coordinate, the block before the tail,
    # first block of the last whole pair, a middle pair's second block
    spots = [300, d - 1, (d - 1) // 256 * 256 - 3, (d // 512 - 1) * 512 + 17, 512 * 4097 + 511]
    for j in range(k):
        G_host[j, spots[j % len(spots)]] = np.float32(3.0 + j)
    bits = rng.integers(2, 9, n).astype(np.uint8)
    w = rng.uniform(0.5, 1.5, n).astype(np.float32)
    mask = (rng.uniform(size=n) < 0.8).astype(np.uint8)
    mask[0] = 1
    G = to_device(G_host)
    out = run_hip(G, n, k, d, row_ptr, col, val, bits, w, mask, 77, 3, api.AGC_SCALE_MAXABS, expect_path=path)
    compare_with_oracle(G_host, k, row_ptr, col, val, bits, w, mask, 77, 3, api.AGC_SCALE_MAXABS, out,
                          tag=f"two-block {kind} tail={tail}")


# ---------------------------------------------------------------------------------------------
# The hot calls enqueue kernel launches only, so a caller may record them into a HIP graph.  A
# replay repeats the recorded step (same seed and step counter): every replay must reproduce the
# eager result bit for bit, with eager work and synchronisations between the replays.
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("unfused,scale_mode", [(False, api.AGC_SCALE_MAXABS), (True, api.AGC_SCALE_MAXABS),
                                                (False, api.AGC_SCALE_L2)])
def test_step_recorded_in_a_hip_graph_replays_the_eager_result(unfused, scale_mode):
    import torch
    rng = np.random.default_rng(909)
    n = k = 8
    d = 70001
    row_ptr, col, val = cyclic_csr(rng, n, 3)
    G_host = rng.standard_normal((k, d)).astype(np.float32)
    bits = rng.integers(2, 9, n).astype(np.uint8)
    w = rng.uniform(0.5, 1.5, n).astype(np.float32)
    mask = np.array([1, 0, 1, 1, 1, 0, 1, 1], dtype=np.uint8)
    G = to_device(G_host)
    ctx = api.Context(n, k, d, scale_mode=scale_mode, unfused_step=unfused)
    try:
        ctx.agc_set_code(row_ptr, col, val)
        codes, scales, ghat = ctx.alloc_outputs(bits)
        ctx.agc_step(G, bits, w, mask, 5, 11, codes, scales, ghat)
        torch.cuda.synchronize()
        want = [c.clone() for c in codes], scales.clone(), ghat.clone()
        # the eager result is the oracle's
        compare_with_oracle(G_host, k, row_ptr, col, val, bits, w, mask, 5, 11, scale_mode,
                            ([c.cpu().numpy() for c in codes], scales.cpu().numpy(), ghat.cpu().numpy()), tag="eager")
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):      # one untimed run on the capture stream first
            ctx.agc_step(G, bits, w, mask, 5, 11, codes, scales, ghat)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            ctx.agc_step(G, bits, w, mask, 5, 11, codes, scales, ghat)
        for replay in range(3):
            for c in codes:
                c.fill_(0x5A)
            scales.fill_(-1.0)
            ghat.fill_(float("nan"))
            ctx.agc_step(G, bits, w, mask, 6, 12 + replay, codes, scales, ghat)   # eager work in between, other draws
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for i in range(n):
                assert torch.equal(codes[i], want[0][i]), (replay, i)
            assert torch.equal(scales.view(torch.int32), want[1].view(torch.int32)), replay
            assert torch.equal(ghat.view(torch.int32), want[2].view(torch.int32)), replay
        del graph
    finally:
        ctx.close()


def test_two_block_scale_pass_with_the_maximum_worker_count():
    """n = 256 workers over k = 8 partitions (interval code, window driver) at a size where the
    max-abs scale pass takes two blocks per wave: every worker's scale against the oracle, and the
    codes of a few workers in a window that straddles the last whole pair of blocks."""
    import torch
    rng = np.random.default_rng(4242)
    n, k = api.AGC_MAX_WORKERS, 8
    d = TWO_BLOCK_MIN * 256 + 300
    row_ptr, col, val = monotone_csr(rng, n, k, 4)
    G_host = (rng.standard_normal((k, d)) * 0.01).astype(np.float32)
    spots = [300, d - 1, (d - 1) // 256 * 256 - 3, (d // 512 - 1) * 512 + 17, 512 * 4097 + 511, 7, 511, d - 301]
    for j in range(k):
        G_host[j, spots[j]] = np.float32(2.0 + j)
    bits = np.full(n, 2, dtype=np.uint8)
    G = to_device(G_host)
    ctx = api.Context(n, k, d, scale_mode=api.AGC_SCALE_MAXABS)
    try:
        ctx.agc_set_code(row_ptr, col, val)
        assert ctx.agc_code_path() > 100
        codes, scales, _ = ctx.alloc_outputs(bits)
        ctx.agc_encode_quantize(G, bits, 31, 2, codes, scales)
        torch.cuda.synchronize()
        csr = O.Csr(row_ptr, col, val, k)
        o_scales = O.scales(G_host, csr, api.AGC_SCALE_MAXABS)
        assert np.array_equal(scales.cpu().numpy().view(np.uint32), o_scales.view(np.uint32))
        m0, m1 = (d // 512 - 1) * 512 - 256, d
        for i in (0, 1, 100, n - 1):
            want = O.codes_range(G_host, csr, i, 2, o_scales[i], 31, 2, m0, m1)
            got = O.unpack(codes[i].cpu().numpy(), d, 2)[m0:m1]
            assert np.array_equal(got, want), i
    finally:
        ctx.close()


@pytest.mark.parametrize("kind", ["cyclic1", "cyclic2", "cyclic4", "cyclic5", "cyclic8", "window2", "window8"])
def test_two_block_scale_pass_every_driver_width(kind):
    """Scales of the two-block max-abs pass for every width of the ring and window drivers that the
    other two-block tests do not reach (they take widths 3 and 4), against the oracle."""
    import torch
    width = int(kind[6:])
    rng = np.random.default_rng(5200 + width + (100 if kind.startswith("window") else 0))
    d = TWO_BLOCK_MIN * 256 + 300
    if kind.startswith("cyclic"):
        n = k = 9
        row_ptr, col, val = cyclic_csr(rng, n, width)
        path = width
    else:
        n, k = 11, 9
        row_ptr, col, val = monotone_csr(rng, n, k, width)
        longest = int(np.max(np.diff(row_ptr)))
        path = 100 + (2 if longest <= 2 else 4 if longest <= 4 else 8)
    G_host = (rng.standard_normal((k, d)) * 0.01).astype(np.float32)
    spots = [300, d - 1, (d - 1) // 256 * 256 - 3, (d // 512 - 1) * 512 + 17, 512 * 4097 + 511, 7, 511, d - 301, 256]
    for j in range(k):
        G_host[j, spots[j]] = np.float32(2.0 + j)
    bits = np.full(n, 2, dtype=np.uint8)
    G = to_device(G_host)
    ctx = api.Context(n, k, d, scale_mode=api.AGC_SCALE_MAXABS)
    try:
        ctx.agc_set_code(row_ptr, col, val)
        assert ctx.agc_code_path() == path
        codes, scales, _ = ctx.alloc_outputs(bits)
        ctx.agc_encode_quantize(G, bits, 31, 2, codes, scales)
        torch.cuda.synchronize()
        o_scales = O.scales(G_host, O.Csr(row_ptr, col, val, k), api.AGC_SCALE_MAXABS)
        assert np.array_equal(scales.cpu().numpy().view(np.uint32), o_scales.view(np.uint32))
    finally:
        ctx.close()
