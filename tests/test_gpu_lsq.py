"""GPU tests of the least-squares stage (partial gradients on the matrix cores, model update)
and of the whole loop  partial gradients -> encode/quantize -> decode -> update  against the
binary64 oracle, through the C ABI."""
import numpy as np
import pytest

from oracle import agc_oracle as O
from oracle import lsq as LS
from oracle import optim as P
from paper_2605_15890_amd import api
from paper_2605_15890_amd import inputs as I

pytestmark = pytest.mark.gpu

# binary32 accumulation of exact products: a row dot of F terms and a column sum of N/k terms;
# the measured error sits near 1e-6, the bound below leaves a margin of one order of magnitude
REL_L2_TOL = 2e-5


def _device_problem(n_rows, n_feat):
    import torch
    Xb, y, w_star = I.least_squares_numpy(n_rows, n_feat)
    X = torch.from_numpy(Xb.view(np.int16)).cuda().view(torch.bfloat16)
    return Xb, y, w_star, X, torch.from_numpy(y).cuda()


def _rel(a, b):
    return float(np.linalg.norm(a.astype(np.float64) - b) / np.linalg.norm(b))


@pytest.mark.parametrize("n_rows,n_feat,k", [(1024, 128, 4), (4096, 512, 8), (3 * 16 * 7, 1280, 3),
                                             (8192, 4096, 32), (2048, 8192, 2), (512, 4224, 4), (256, 384, 1)])
def test_partial_gradients_match_fp64(n_rows, n_feat, k):
    import torch
    Xb, y, w_star, X, y_d = _device_problem(n_rows, n_feat)
    rng = np.random.default_rng(n_feat)
    beta = rng.standard_normal(n_feat).astype(np.float32)
    beta_d = torch.from_numpy(beta).cuda()
    G = api.padded_rows(k, n_feat)
    G.fill_(float("nan"))
    resid = torch.full((n_rows,), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(api.agc_ls_workspace_floats(n_rows, n_feat, k), dtype=torch.float32, device="cuda")
    api.agc_ls_partial_gradients(X, y_d, beta_d, k, G, resid, ws)
    torch.cuda.synchronize()
    G_o, r_o = LS.partial_gradients(Xb, y, beta, k)
    assert _rel(resid.cpu().numpy(), r_o) <= REL_L2_TOL
    for p in range(k):
        assert _rel(G[p].cpu().numpy(), G_o[p]) <= REL_L2_TOL, p
    # a second call gives the same bits (fixed reduction order)
    G2 = api.padded_rows(k, n_feat)
    resid2 = torch.empty_like(resid)
    api.agc_ls_partial_gradients(X, y_d, beta_d, k, G2, resid2, ws)
    torch.cuda.synchronize()
    assert torch.equal(G.view(torch.int32), G2.view(torch.int32))
    assert torch.equal(resid.view(torch.int32), resid2.view(torch.int32))


def test_rejects_shapes_the_kernel_does_not_cover():
    import torch
    X = torch.zeros((64, 128), dtype=torch.bfloat16, device="cuda")
    y = torch.zeros(64, device="cuda")
    b = torch.zeros(128, device="cuda")
    G = api.padded_rows(4, 128)
    ws = torch.zeros(1 << 16, device="cuda")
    assert api.agc_ls_partial_gradients(X, y, b, 3, G, y, ws, check=False) == api.AGC_ESHAPE   # 64 % (16*3)
    X2 = torch.zeros((64, 96), dtype=torch.bfloat16, device="cuda")
    assert api.agc_ls_partial_gradients(X2, y, b, 4, G, y, ws, check=False) == api.AGC_ESHAPE  # 96 % 128


def test_gd_update():
    import torch
    rng = np.random.default_rng(1)
    b = rng.standard_normal(5001).astype(np.float32)
    g = rng.standard_normal(5001).astype(np.float32)
    bd, gd = torch.from_numpy(b).cuda(), torch.from_numpy(g).cuda()
    api.agc_gd_update(bd, gd, 0.125)
    torch.cuda.synchronize()
    want = P.gd_update(b, g, 0.125).astype(np.float32)                                 # single rounding (fma)
    assert np.array_equal(bd.cpu().numpy(), want)


def test_end_to_end_loop_follows_the_oracle_loop():
    """Gradient descent on the least-squares loss with coded, quantized, straggler-hit gradient
    transport.  Each iteration the GPU's partial gradients are also handed to the oracle's step,
    whose estimate must equal the GPU's bit for bit; the loss must fall by orders of magnitude
    and track an all-oracle loop (binary64 gradients rounded to binary32) closely."""
    import torch
    n = k = 8
    s = 3
    n_rows, n_feat = 8192, 512
    Xb, y, w_star, X, y_d = _device_problem(n_rows, n_feat)
    p = np.linspace(0.05, 0.4, n)
    bits = np.array([4, 4, 5, 3, 4, 6, 3, 3], dtype=np.uint8)
    pc = api.agc_phi_coef_balanced(p, int(bits.sum()))
    row_ptr, col, val, w = api.agc_build_cyclic_code(n, k, s, p, bits, pc)
    csr = O.Csr(row_ptr, col, val, k)
    ctx = api.Context(n, k, n_feat, scale_mode=api.AGC_SCALE_MAXABS)
    ctx.agc_set_code(row_ptr, col, val)
    codes, scales, ghat = ctx.alloc_outputs(bits)
    G = api.padded_rows(k, n_feat)
    resid = torch.empty(n_rows, dtype=torch.float32, device="cuda")
    ws = torch.empty(api.agc_ls_workspace_floats(n_rows, n_feat, k), dtype=torch.float32, device="cuda")
    beta_d = torch.zeros(n_feat, dtype=torch.float32, device="cuda")
    beta_o = np.zeros(n_feat, dtype=np.float32)
    lam = n_rows / n_feat * (1 + np.sqrt(n_feat / n_rows)) ** 2
    lr = np.float32(0.5 / lam)
    seed = 0x5EED
    cfg = I.Config(5, "lsq", n, k, s, n_feat, "normal", ("fixed", list(p)), ("fixed", list(bits)), 60)
    loss_d, loss_o = [], []
    for t in range(cfg.iters):
        mask = I.arrival_mask(cfg, p, t)
        api.agc_ls_partial_gradients(X, y_d, beta_d, k, G, resid, ws)
        ctx.agc_step(G, bits, w, mask, seed, t, codes, scales, ghat)
        torch.cuda.synchronize()
        # the oracle, given the GPU's partial gradients, reproduces the GPU's estimate exactly
        _, _, gh_same = O.step(G.cpu().numpy(), csr, bits, w, mask, seed, t, O.SCALE_MAXABS)
        assert np.array_equal(gh_same.view(np.uint32), ghat.cpu().numpy().view(np.uint32)), t
        loss_d.append(0.5 * float((resid.double() ** 2).sum()))
        api.agc_gd_update(beta_d, ghat, float(lr))
        # the all-oracle loop
        G_o, r_o = LS.partial_gradients(Xb, y, beta_o, k)
        loss_o.append(0.5 * float(r_o @ r_o))
        _, _, gh_o = O.step(G_o.astype(np.float32), csr, bits, w, mask, seed, t, O.SCALE_MAXABS)
        beta_o = P.gd_update(beta_o, gh_o, float(lr)).astype(np.float32)
    torch.cuda.synchronize()
    ctx.close()
    loss_d, loss_o = np.array(loss_d), np.array(loss_o)
    assert loss_d[-1] < 0.02 * loss_d[0], (loss_d[0], loss_d[-1])
    assert np.all(np.abs(loss_d - loss_o) <= 0.02 * loss_o), np.max(np.abs(loss_d - loss_o) / loss_o)
    assert _rel(beta_d.cpu().numpy(), beta_o.astype(np.float64)) < 0.02


def test_full_size_loop_sampled_parity():
    """N = 2^20 samples, 4096 features, k = n = 32, s = 3, 500 iterations, all on the GPU.  The
    oracle cannot run that loop, so it checks, at three iterations, whole partitions of the
    partial-gradient stage (binary64, given the GPU's current model) and the complete
    encode/quantize/decode step on the GPU's partial gradients (bit for bit); the loss curve must
    fall to the noise floor of the data."""
    import torch
    cfg = I.CONFIGS["lsq"]
    n, k, s, F, N = cfg.n, cfg.k, cfg.s, cfg.d, cfg.extra["n_rows"]
    dev = torch.device("cuda:0")
    X, y_d, w_star = I.least_squares_torch(N, F, dev)
    p = I.straggler_probs(cfg)
    z_tot = cfg.bits_law[1] * n
    bits = api.agc_alloc_bits(p, api.agc_phi_coef_balanced(p, z_tot), z_tot, 2, 8)
    pc = api.agc_phi_coef_balanced(p, int(bits.sum()))
    row_ptr, col, val, w = api.agc_build_cyclic_code(n, k, s, p, bits, pc)
    csr = O.Csr(row_ptr, col, val, k)
    ctx = api.Context(n, k, F, scale_mode=api.AGC_SCALE_MAXABS)
    ctx.agc_set_code(row_ptr, col, val)
    codes, scales, ghat = ctx.alloc_outputs(bits)
    G = api.padded_rows(k, F)
    resid = torch.empty(N, dtype=torch.float32, device=dev)
    ws = torch.empty(api.agc_ls_workspace_floats(N, F, k), dtype=torch.float32, device=dev)
    beta = torch.zeros(F, dtype=torch.float32, device=dev)
    lam = N / F * (1 + np.sqrt(F / N)) ** 2
    lr = float(np.float32(0.5 / lam))
    rows = N // k
    losses = torch.zeros(cfg.iters, dtype=torch.float64, device=dev)
    checked = 0
    for t in range(cfg.iters):
        mask = I.arrival_mask(cfg, p, t)
        api.agc_ls_partial_gradients(X, y_d, beta, k, G, resid, ws)
        ctx.agc_step(G, bits, w, mask, cfg.philox_seed, t, codes, scales, ghat)
        losses[t] = 0.5 * (resid.double() ** 2).sum()
        if t in (0, 7, cfg.iters - 1):
            torch.cuda.synchronize()
            print(f"[lsq] oracle check at iteration {t}", flush=True)
            beta_h = beta.cpu().numpy()
            G_h = G.cpu().numpy()
            for part in ((0, 13, 31) if t == 0 else (t % k,)):
                sl = slice(part * rows, (part + 1) * rows)
                Xp = X[sl].view(torch.int16).cpu().numpy().view(np.uint16)
                G_o, r_o = LS.partial_gradients(Xp, y_d[sl].cpu().numpy(), beta_h, 1)
                assert _rel(resid[sl].cpu().numpy(), r_o) <= REL_L2_TOL, (t, part)
                assert _rel(G_h[part], G_o[0]) <= REL_L2_TOL, (t, part)
            _, o_scales, o_ghat = O.step(G_h, csr, bits, w, mask, cfg.philox_seed, t, O.SCALE_MAXABS)
            assert np.array_equal(o_scales.view(np.uint32), scales.cpu().numpy().view(np.uint32)), t
            assert np.array_equal(o_ghat.view(np.uint32), ghat.cpu().numpy().view(np.uint32)), t
            checked += 1
        api.agc_gd_update(beta, ghat, lr)
    torch.cuda.synchronize()
    ctx.close()
    L = losses.cpu().numpy()
    floor = 0.5 * N * 1e-4          # the noise in y has standard deviation 0.01
    err = float(torch.linalg.norm(beta - w_star) / torch.linalg.norm(w_star))
    print(f"[lsq] loss {L[0]:.4g} -> {L[-1]:.4g} (noise floor {floor:.4g}), |beta-w*|/|w*| = {err:.3g}", flush=True)
    assert checked == 3
    assert L[-1] < 1e-3 * L[0] and L[-1] < 3.0 * floor, (L[0], L[-1], floor)
    assert err < 0.02
