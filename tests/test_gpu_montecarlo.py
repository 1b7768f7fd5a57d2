"""Monte-Carlo unbiasedness of the GPU path at the iteration counts the named configurations
state (1000 / 200 / 100 steps, a fresh Bernoulli arrival mask and fresh Philox draws per step):

  (i)  projections of mean_T(g_hat) - g on 8 fixed unit directions lie within 3 standard errors
       of zero (constraint of problem P1: E[g_hat] = sum_j g_j);
  (ii) mean_T ||g_hat - g||^2 lies within 3 standard errors of the exact residual error
       sum_i (1-p_i) w_i^2 (p_i ||f_i||^2 + sum_m Var Q_i(f_i)_m)  (proof of Lemma 1 before any
       bounding), whose two sums the CPU oracle evaluates over ALL d coordinates of every worker
       (no sampling, also at d = 25.6 M), from the scales the oracle computes itself.

All per-step statistics stay on the device; the steps run through the C ABI exactly as the
benchmark runs them (fused step) or as two passes (stand-alone decode kernel)."""
import numpy as np
import pytest

from oracle import agc_oracle as O
from oracle import design as D
from paper_2605_15890_amd import api
from paper_2605_15890_amd import inputs as I

pytestmark = pytest.mark.gpu


def _problem(cfg):
    p = I.straggler_probs(cfg)
    bits = I.random_bits(cfg)
    if bits is None:
        z_tot = cfg.bits_law[1] * cfg.n
        bits = api.agc_alloc_bits(p, api.agc_phi_coef_balanced(p, z_tot), z_tot, 2, 8)
    pc = api.agc_phi_coef_balanced(p, int(bits.sum()))
    row_ptr, col, val, w = api.agc_build_cyclic_code(cfg.n, cfg.k, cfg.s, p, bits, pc)
    return p, bits, (row_ptr, col, val), w


@pytest.mark.parametrize("name,unfused", [("tiny", False), ("tiny", True), ("n16_d1m", True), ("n16_d1m", False),
                                          ("resnet50", False)])
def test_montecarlo_unbiased_and_residual_error_on_gpu(name, unfused):
    import torch
    cfg = I.CONFIGS[name]
    n, k, d, T = cfg.n, cfg.k, cfg.d, cfg.iters
    p, bits, code, w = _problem(cfg)
    dev = torch.device("cuda:0")
    G = I.partial_gradients_torch(cfg, dev)
    g = torch.zeros(d, dtype=torch.float64, device=dev)
    for j in range(k):
        g += G[j].double()
    gen = torch.Generator(device=dev).manual_seed(770 + cfg.index)
    dirs = torch.randn((8, d), generator=gen, device=dev, dtype=torch.float64)
    dirs /= dirs.norm(dim=1, keepdim=True)

    ctx = api.Context(n, k, d, scale_mode=api.AGC_SCALE_MAXABS, unfused_step=unfused)
    ctx.agc_set_code(*code)
    assert ctx.agc_code_path() == cfg.s
    codes, scales, ghat = ctx.alloc_outputs(bits)
    proj = torch.zeros((T, 8), dtype=torch.float64, device=dev)
    sq = torch.zeros(T, dtype=torch.float64, device=dev)
    arrivals = np.zeros(n)
    e = torch.empty(d, dtype=torch.float64, device=dev)
    for t in range(T):
        mask = I.arrival_mask(cfg, p, t)
        arrivals += mask
        ctx.agc_step(G, bits, w, mask, cfg.philox_seed, t, codes, scales, ghat)
        torch.sub(ghat, g, out=e)            # binary64: promotes ghat
        proj[t] = dirs @ e
        sq[t] = e @ e
    torch.cuda.synchronize()
    print(f"[{name}] {T} steps done", flush=True)
    proj_h, sq_h = proj.cpu().numpy(), sq.cpu().numpy()
    scales_h = scales.cpu().numpy()
    G_host = G.cpu().numpy()
    ctx.close()
    del G, dirs, e, codes, ghat
    torch.cuda.empty_cache()

    # exact residual error from the oracle, all coordinates of all workers
    csr = O.Csr(code[0], code[1], code[2], k)
    o_scales = O.scales(G_host, csr, O.SCALE_MAXABS)
    assert np.array_equal(o_scales.view(np.uint32), scales_h.view(np.uint32))
    sumsq, var_q = np.zeros(n), np.zeros(n)
    for i in range(n):
        sumsq[i], var_q[i] = O.worker_moments(G_host, csr, i, int(bits[i]), o_scales[i])
    w64 = w.astype(np.float64)
    V = float(np.sum((1 - p) * w64 ** 2 * (p * sumsq + var_q)))
    # the closed-form helper agrees (it takes the coded vectors themselves; feed it their norms)
    _, V2 = D.exact_moments(np.sqrt(sumsq)[:, None], var_q, w64, p)
    assert V == pytest.approx(V2, rel=1e-12)

    # (i) unbiasedness along fixed directions
    z = proj_h.mean(axis=0) / (proj_h.std(axis=0, ddof=1) / np.sqrt(T))
    print(f"[{name}] z(projections) = {np.round(z, 2)}", flush=True)
    assert np.all(np.abs(z) < 3.0), z
    # (ii) residual error against the exact expression
    se = sq_h.std(ddof=1) / np.sqrt(T)
    zr = (sq_h.mean() - V) / se
    print(f"[{name}] mean ||g_hat-g||^2 = {sq_h.mean():.6g}, exact = {V:.6g}, z = {zr:.2f}", flush=True)
    assert abs(zr) < 3.0, (sq_h.mean(), V, se)
    # the masks really were fresh Bernoulli(1 - p_i) draws
    assert np.all(np.abs(arrivals / T - (1 - p)) < 4 * np.sqrt(p * (1 - p) / T))
