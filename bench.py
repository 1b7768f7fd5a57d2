#!/usr/bin/env python3
"""Benchmark of the approximate-gradient-coding hot path on one MI355X.

One step = one agc_step: scale pass -> scale finalize -> encode+quantize+pack -> decode over
one batch of synthetic partial gradients that is already resident in HBM.  Prints ONE JSON
line: throughput in GB/s of gradient traffic (4*k*d bytes per step), the roofline view of the
dominant kernel (HIP-event durations measured in the timed region) and the CPU oracle timed
on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload resnet50] [--scale maxabs|l2]
                    [--code cyclic|interval] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
VALU_PEAK_GLANEOPS = 256 * 64 * 2.4   # 256 CUs x 64 lanes x 2.4 GHz = 39 321.6 G lane-ops/s


def build_problem(cfg, api, code_kind):
    from paper_2605_15890_amd import inputs as I
    p = I.straggler_probs(cfg)
    bits = I.random_bits(cfg)
    if bits is None:        # bits from the low-complexity allocator at the configured mean budget
        z_tot = cfg.bits_law[1] * cfg.n
        bits = api.agc_alloc_bits(p, api.agc_phi_coef_balanced(p, z_tot), z_tot, 2, 8)
    pc = api.agc_phi_coef_balanced(p, int(bits.sum()))
    if code_kind == "cyclic":
        row_ptr, col, val, w = api.agc_build_cyclic_code(cfg.n, cfg.k, cfg.s, p, np.maximum(bits, 2), pc)
    else:
        row_ptr, col, val, w = api.agc_build_code(cfg.n, cfg.k, p, np.maximum(bits, 2), pc)
    ok, res = api.agc_check_unbiased(cfg.k, row_ptr, col, val, w, p, 1e-5)
    assert ok, res
    return p, bits, (row_ptr, col, val), w


def stored_valu(tag, kernel):
    """Vector-ALU lane-operations per launch of `kernel` (rocprofv3 --pmc SQ_INSTS_VALU x 64),
    recorded in the same profiles/traffic_<tag>.txt; None when absent."""
    path = os.path.join(ROOT, "profiles", f"traffic_{tag}.txt")
    if not os.path.exists(path):
        return None
    with open(path) as fh:
        for line in fh:
            f = line.split()
            if len(f) >= 3 and f[0] == "valu_lane_ops_per_launch" and f[1] == kernel:
                return float(f[2])
    return None


def stored_traffic(tag, kernel):
    """HBM bytes per launch of `kernel` as measured offline with rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE (scaled by the calibration copy) and recorded in profiles/traffic_<tag>.txt;
    None when no such record exists.  bench.py itself never runs the profiler."""
    path = os.path.join(ROOT, "profiles", f"traffic_{tag}.txt")
    if not os.path.exists(path):
        return None, None
    with open(path) as fh:
        for line in fh:
            f = line.split()
            if len(f) >= 3 and f[0] == "traffic_bytes_per_launch" and f[1] == kernel:
                return float(f[2]), os.path.relpath(path, ROOT)
    return None, None


def bench_lsq(args):
    """--workload lsq: one step = partial gradients of the least-squares loss (MFMA kernel, X
    resident in HBM) -> agc_step -> model update.  Not the headline workload: the line it prints
    reports the rate at which the step streams X and the roofline of the partial-gradient kernel."""
    import torch
    from paper_2605_15890_amd import api
    from paper_2605_15890_amd import inputs as I
    cfg = I.CONFIGS["lsq"]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    n, k, F, N = cfg.n, cfg.k, cfg.d, cfg.extra["n_rows"]
    p, bits, code, w = build_problem(cfg, api, "cyclic")
    X, y, w_star = I.least_squares_torch(N, F, dev)
    ctx = api.Context(n, k, F, scale_mode=api.AGC_SCALE_MAXABS)
    ctx.agc_set_code(*code)
    codes, scales, ghat = ctx.alloc_outputs(bits)
    G = api.padded_rows(k, F)
    resid = torch.empty(N, dtype=torch.float32, device=dev)
    ws = torch.empty(api.agc_ls_workspace_floats(N, F, k), dtype=torch.float32, device=dev)
    beta = torch.zeros(F, dtype=torch.float32, device=dev)
    lr = float(np.float32(0.5 / (N / F * (1 + np.sqrt(F / N)) ** 2)))
    K, W = args.steps, args.warmup
    masks = [I.arrival_mask(cfg, p, t) for t in range(W + K)]
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(K)]

    def step(t, pair=None):
        if pair:
            pair[0].record()
        api.agc_ls_partial_gradients(X, y, beta, k, G, resid, ws)     # on torch's current stream
        if pair:
            pair[1].record()
        ctx.agc_step(G, bits, w, masks[t], cfg.philox_seed, t, codes, scales, ghat)
        api.agc_gd_update(beta, ghat, lr)

    for t in range(W):
        step(t)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(W, W + K):
        step(t, ev[t - W])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K
    ls_ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))    # partial kernel + its small reduction
    x_bytes = 2.0 * N * F
    alg = x_bytes + 4.0 * N * 2 + 4.0 * F      # X once, y in, residual out, model in
    traffic, traffic_src = stored_traffic("lsq", "ls_partial_gradients")
    cpu_baseline = None
    if not args.no_cpu_baseline:
        from oracle import lsq as LS
        rows = N // k
        Xp = X[:rows].view(torch.int16).cpu().numpy().view(np.uint16)
        yp, bh = y[:rows].cpu().numpy(), beta.cpu().numpy()
        c0 = time.perf_counter()
        LS.partial_gradients(Xp, yp, bh, 1)
        c1 = time.perf_counter()
        cpu_baseline = {"value": round(2.0 * rows * F / (c1 - c0) / 1e9, 4), "unit": "GB/s",
                        "cores": os.cpu_count(), "kind": "oracle",
                        "sample": f"binary64 numpy partial gradient of one partition ({rows} of {N} samples), "
                                  f"{c1 - c0:.2f} s wall"}
    out = {
        "metric": "least-squares GD step (partial gradients + encode/quantize/decode + update): GB/s of X streamed",
        "value": round(x_bytes / (ms_per_step * 1e-3) / 1e9, 1), "unit": "GB/s", "n_gpus": 1, "steps": K,
        "warmup": W, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"lsq: N={N} samples, {F} features (bf16), k={k} partitions, n={n} workers, "
                               f"s={cfg.s}, bits sum {int(bits.sum())}, cyclic code, maxabs scale"},
        "roofline": {"kernel": "ls_partial_gradients", "bound": "hbm",
                     "achieved": round(alg / (ls_ms * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(alg / (ls_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "traffic_source": traffic_src, "avg_launch_ms": round(ls_ms, 4),
                     "alg_bytes_per_launch": alg},
        "cpu_baseline": cpu_baseline,
    }
    print(json.dumps(out))
    ctx.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="resnet50")
    ap.add_argument("--scale", default="maxabs", choices=["maxabs", "l2"])
    ap.add_argument("--code", default="cyclic", choices=["cyclic", "interval"])
    ap.add_argument("--bucket", type=int, default=0, choices=[0, 256],
                    help="256: one scale per 256-coordinate bucket (single pass over G); 0: one per vector")
    ap.add_argument("--unfused", action="store_true",
                    help="run the step as two passes (stand-alone decode kernel) instead of the fused pass")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-log2", type=int, default=23,
                    help="the oracle is timed on the first 2^this coordinates (all partitions)")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run one plain 1 GiB copy kernel (reference for the traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; there is no multi-GPU path (it would shard the "
              "coordinate axis d, exchanging only the per-worker scale partials). Run with --gpus 1.",
              file=sys.stderr)
        sys.exit(2)

    if args.workload == "lsq":
        return bench_lsq(args)

    import torch
    from paper_2605_15890_amd import api
    from paper_2605_15890_amd import inputs as I

    cfg = I.CONFIGS[args.workload]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    scale_mode = api.AGC_SCALE_MAXABS if args.scale == "maxabs" else api.AGC_SCALE_L2
    p, bits, code, w = build_problem(cfg, api, args.code)
    n, k, d = cfg.n, cfg.k, cfg.d

    G = I.partial_gradients_torch(cfg, dev)
    assert G.stride(0) % 4 == 0 and G.data_ptr() % 16 == 0
    ctx = api.Context(n, k, d, scale_mode=scale_mode, allow_1bit=cfg.allow_1bit, bucket=args.bucket,
                      unfused_step=args.unfused)
    ctx.agc_set_code(*code)
    codes, scales, ghat = ctx.alloc_outputs(bits)
    nb = ctx.agc_scales_per_worker() if args.bucket else 0
    K, W = args.steps, args.warmup
    masks = [I.arrival_mask(cfg, p, t) for t in range(W + K)]     # sampled outside the timed region
    seed = cfg.philox_seed

    if args.calibrate:   # known traffic: reads 2^30 bytes, writes 2^30 bytes
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        api.agc_calibration_copy(dst, src, 1 << 30)
        torch.cuda.synchronize()
        del src, dst
    for t in range(W):
        ctx.agc_step(G, bits, w, masks[t], seed, t, codes, scales, ghat)
    torch.cuda.synchronize()
    ctx.agc_profile_enable(True)
    ctx.agc_profile_read()
    t0 = time.perf_counter()
    for t in range(W, W + K):
        ctx.agc_step(G, bits, w, masks[t], seed, t, codes, scales, ghat)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = ctx.agc_profile_read()
    ctx.agc_profile_enable(False)

    ms_per_step = (t1 - t0) * 1e3 / K
    grad_bytes = 4.0 * k * d
    value = grad_bytes / (ms_per_step * 1e-3) / 1e9

    # algorithmic bytes per launch of each kernel (what the method must move)
    sum_b = float(np.sum(bits))
    arrived_b = float(np.mean([np.sum(bits[m.astype(bool)]) for m in masks[W:]]))
    n_arr = float(np.mean([m.sum() for m in masks[W:]]))
    alg_bytes = {
        "scale_pass": 0.0 if args.bucket else 4.0 * k * d,
        "scale_finalize": 0.0,
        "quantize": 4.0 * k * d + d * sum_b / 8.0 + 4.0 * n * nb + (0.0 if args.unfused else 4.0 * d),
        "decode": (d * arrived_b / 8.0 + 4.0 * d + 4.0 * n_arr * nb) if args.unfused else 0.0,
    }
    kernels = {}
    for name, (ms, cnt) in prof.items():
        if cnt == 0:
            continue
        avg = ms / max(cnt, 1)
        kernels[name] = {"avg_ms": round(avg, 4), "launches": cnt,
                         "alg_GBps": round(alg_bytes[name] / (avg * 1e-3) / 1e9, 1) if avg > 0 else None}
    dominant = max(kernels, key=lambda nm: kernels[nm]["avg_ms"])
    dom_avg_s = kernels[dominant]["avg_ms"] * 1e-3
    achieved = alg_bytes[dominant] / dom_avg_s / 1e9
    step_alg_bytes = sum(alg_bytes.values())
    tag = (f"{cfg.name}_{args.code}_{args.scale}" + (f"_bucket{args.bucket}" if args.bucket else "")
           + ("_unfused" if args.unfused else ""))
    traffic, traffic_src = stored_traffic(tag, dominant)
    roofline = {
        "kernel": dominant, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
        "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
        "traffic_source": traffic_src,
        "avg_launch_ms": kernels[dominant]["avg_ms"],
        "alg_bytes_per_launch": alg_bytes[dominant],
        "step_alg_bytes": step_alg_bytes,
        "step_hbm_frac": round(step_alg_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
    }
    valu_ops = stored_valu(tag, dominant)
    if valu_ops:   # the kernel is co-bound by plain vector ALU work: say how close to that peak it runs
        roofline["valu"] = {"lane_ops_per_launch": valu_ops,
                            "achieved_Tlaneops": round(valu_ops / dom_avg_s / 1e12, 2),
                            "peak_Tlaneops": round(VALU_PEAK_GLANEOPS / 1e3, 2),
                            "frac": round(valu_ops / dom_avg_s / 1e9 / VALU_PEAK_GLANEOPS, 4)}

    cpu_baseline = None
    if not args.no_cpu_baseline:
        from oracle import agc_oracle as O
        ds = min(d, 1 << args.cpu_sample_log2)
        Gs = G[:, :ds].contiguous().cpu().numpy()
        csr = O.Csr(code[0], code[1], code[2], k)
        c0 = time.perf_counter()
        o_mode = O.SCALE_MAXABS if args.scale == "maxabs" else O.SCALE_L2
        (O.step_bucket if args.bucket else O.step)(Gs, csr, bits, w, masks[W], seed, W, o_mode)
        c1 = time.perf_counter()
        cpu_baseline = {
            "value": round(4.0 * k * ds / (c1 - c0) / 1e9, 4), "unit": "GB/s", "cores": O.threads(),
            "kind": "oracle",
            "sample": f"one oracle step on the first {ds} of {d} coordinates of all {k} partitions "
                      f"({n * ds} coded elements), {c1 - c0:.2f} s wall",
        }

    out = {
        "metric": "encode+quantize+decode GB/s of gradient traffic",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: n={n} workers, k={k} partitions, s={cfg.s}, d={d}, "
                               f"{cfg.law} gradients, bits sum {int(sum_b)} (mean {sum_b / n:.2f}), "
                               f"{args.code} code, {args.scale} scale"
                               + (f" per {args.bucket}-coordinate bucket" if args.bucket else " per vector")
                               + (", two-pass step" if args.unfused else ", fused step"),
                   "code_path": ctx.agc_code_path()},
        "coded_elements_per_s": round(n * d / (ms_per_step * 1e-3), 1),
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "kernels": kernels,
    }
    print(json.dumps(out))
    ctx.close()


if __name__ == "__main__":
    main()
