#!/usr/bin/env python3
"""Benchmark of the approximate-gradient-coding hot path on one MI355X.

One step = one agc_step: scale pass -> scale finalize -> encode+quantize+pack -> decode over
one batch of synthetic partial gradients that is already resident in HBM.  Prints ONE JSON
line: throughput in GB/s of gradient traffic (4*k*d bytes per step), the roofline view of the
dominant kernel (HIP-event durations measured in the timed region) and the CPU oracle timed
on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload resnet50] [--scale maxabs|l2]
                    [--code cyclic|interval] [--bucket 0|256] [--layers N] [--two-pass] [--no-variants]
                    [--no-cpu-baseline]

The default run (no flags) times the metric configuration (resnet50-sized: n = k = 64, s = 4,
d = 25.6 M, cyclic code, max-abs scale per vector, fused step) and then, in the same process and
on the same inputs, the other forms the library offers at that size (two-pass step, Euclidean
scale, the paper's interval code, layer-wise and bucket-wise scales), a plain copy and the bare access pattern of
the two streaming passes, so that every number quoted anywhere comes from one timed line.
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


def tag_of(cfg, code, scale, bucket, two_pass, layers=0):
    return (f"{cfg.name}_{code}_{scale}" + (f"_bucket{bucket}" if bucket else "") + (f"_layers{layers}" if layers else "")
            + ("_two_pass" if two_pass else ""))


def alg_bytes_of(n, k, d, bits, masks, bucket, two_pass):
    """Algorithmic bytes per launch of each kernel: what the method must move."""
    nb = (d + 255) // 256 if bucket else 0
    sum_b = float(np.sum(bits))
    arrived_b = float(np.mean([np.sum(bits[m.astype(bool)]) for m in masks]))
    n_arr = float(np.mean([m.sum() for m in masks]))
    return {
        "scale_pass": 0.0 if bucket else 4.0 * k * d,
        "scale_finalize": 0.0,
        "quantize": 4.0 * k * d + d * sum_b / 8.0 + 4.0 * n * nb + (0.0 if two_pass else 4.0 * d),
        "decode": (d * arrived_b / 8.0 + 4.0 * d + 4.0 * n_arr * nb) if two_pass else 0.0,
    }


def equal_layers(d, count):
    """Ends of `count` layers of near-equal size, all but the last multiples of 256."""
    ends = sorted({int(round(d * (l + 1) / count)) // 256 * 256 for l in range(count - 1)} - {0})
    return np.array([e for e in ends if e < d] + [d], dtype=np.int64)


def time_variant(api, I, cfg, G, bufs, p, bits, code, w, scale, bucket, two_pass, K, W, seed, layers=0):
    """W warm-up steps, K timed steps without any event between the kernels (wall clock bracketed by
    device synchronisation: this is the step time), then K more steps with a HIP-event pair around
    every kernel on the stream the kernels run on (their average durations; the event records
    themselves cost about 20 us per step, which is why the two are separate regions)."""
    import torch
    n, k, d = cfg.n, cfg.k, cfg.d
    scale_mode = api.AGC_SCALE_MAXABS if scale == "maxabs" else api.AGC_SCALE_L2
    ctx = api.Context(n, k, d, scale_mode=scale_mode, allow_1bit=cfg.allow_1bit, bucket=bucket, unfused_step=two_pass)
    ctx.agc_set_code(*code)
    if layers:
        ctx.agc_set_layers(equal_layers(d, layers))
    codes, ghat = bufs
    per = ctx.agc_scales_per_worker()
    scales = torch.empty((n, per) if per > 1 else n, dtype=torch.float32, device=G.device)
    masks = [I.arrival_mask(cfg, p, t) for t in range(W + 2 * K)]     # sampled outside the timed regions
    for t in range(W):
        ctx.agc_step(G, bits, w, masks[t], seed, t, codes, scales, ghat)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(W, W + K):
        ctx.agc_step(G, bits, w, masks[t], seed, t, codes, scales, ghat)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ctx.agc_profile_enable(True)
    ctx.agc_profile_read()
    for t in range(W + K, W + 2 * K):
        ctx.agc_step(G, bits, w, masks[t], seed, t, codes, scales, ghat)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    prof = ctx.agc_profile_read()
    ctx.agc_profile_enable(False)
    path = ctx.agc_code_path()
    ctx.close()
    del scales
    ms_per_step = (t1 - t0) * 1e3 / K
    alg = alg_bytes_of(n, k, d, bits, masks[W:W + K], bucket, two_pass)
    kernels = {}
    for name, (ms, cnt) in prof.items():
        if cnt == 0:
            continue
        avg = ms / cnt
        kernels[name] = {"avg_ms": round(avg, 4), "launches": cnt,
                         "alg_GBps": round(alg[name] / (avg * 1e-3) / 1e9, 1) if avg > 0 else None}
    dominant = max(kernels, key=lambda nm: kernels[nm]["avg_ms"])
    return {"ms_per_step": ms_per_step, "ms_per_step_with_events": (t2 - t1) * 1e3 / K, "kernels": kernels,
            "dominant": dominant, "alg": alg, "code_path": path}


def roofline_of(r, tag):
    dom = r["dominant"]
    dom_avg_s = r["kernels"][dom]["avg_ms"] * 1e-3
    achieved = r["alg"][dom] / dom_avg_s / 1e9
    step_alg = sum(r["alg"].values())
    traffic, traffic_src = stored_traffic(tag, dom)
    out = {
        "kernel": dom, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": traffic_src,
        "avg_launch_ms": r["kernels"][dom]["avg_ms"], "alg_bytes_per_launch": r["alg"][dom],
        "step_alg_bytes": step_alg,
        "step_hbm_frac": round(step_alg / (r["ms_per_step"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
    }
    valu_ops = stored_valu(tag, dom)
    if valu_ops:   # the kernel also does plain vector-ALU work: say how close to that peak it runs
        out["valu"] = {"lane_ops_per_launch": valu_ops,
                       "achieved_Tlaneops": round(valu_ops / dom_avg_s / 1e12, 2),
                       "peak_Tlaneops": round(VALU_PEAK_GLANEOPS / 1e3, 2),
                       "frac": round(valu_ops / dom_avg_s / 1e9 / VALU_PEAK_GLANEOPS, 4)}
    return out


def measured_ceilings(api, G, k, d, scratch):
    """What this machine's memory system delivers, timed with HIP events on the current stream: a plain
    copy (1 GiB in, 1 GiB out) and the bare access pattern of the two streaming passes (all of G
    read row by row as the passes read it; the same plus one 96-byte piece per row and wave written
    to the row's own output stream, which is what a 3-bit worker's payload looks like)."""
    import torch
    out = {}

    def timed(fn, reps=5):
        fn()
        torch.cuda.synchronize()
        best = None
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            best = ms if best is None else min(best, ms)
        return best

    nbytes = 1 << 30
    src = scratch[:nbytes // 4]
    dst = scratch[nbytes // 4: nbytes // 2]
    ms = timed(lambda: api.agc_calibration_copy(dst, src, nbytes))
    out["copy_GBps"] = round(2.0 * nbytes / (ms * 1e-3) / 1e9, 1)
    g_bytes = 4.0 * k * (d // 256) * 256
    ms = timed(lambda: api.agc_debug_stream_rows(G, 0, scratch))
    out["pattern_read_ms"] = round(ms, 4)
    out["pattern_read_GBps"] = round(g_bytes / (ms * 1e-3) / 1e9, 1)
    ms = timed(lambda: api.agc_debug_stream_rows(G, 0, scratch, blocks_per_wave=2))
    out["pattern_read_two_block_ms"] = round(ms, 4)
    piece = 96
    w_bytes = float(k) * (d // 256) * piece
    ms = timed(lambda: api.agc_debug_stream_rows(G, piece, scratch, wg_flush=False))
    out["pattern_read_write_per_wave_ms"] = round(ms, 4)
    ms = timed(lambda: api.agc_debug_stream_rows(G, piece, scratch, wg_flush=True))
    out["pattern_read_write_ms"] = round(ms, 4)
    out["pattern_read_write_GBps"] = round((g_bytes + w_bytes) / (ms * 1e-3) / 1e9, 1)
    # the same at the quantize pass's occupancy (four waves per SIMD), bare and with about its arithmetic per row
    ms = timed(lambda: api.agc_debug_stream_rows(G, 0, scratch, waves_per_simd=4))
    out["pattern_read_4waves_ms"] = round(ms, 4)
    ms = timed(lambda: api.agc_debug_stream_rows(G, piece, scratch, wg_flush=True, waves_per_simd=4))
    out["pattern_read_write_4waves_ms"] = round(ms, 4)
    for fma in (40, 100):
        ms = timed(lambda: api.agc_debug_stream_rows(G, piece, scratch, wg_flush=True, waves_per_simd=4, fma_per_row=fma))
        out[f"pattern_read_write_4waves_fma{fma}_ms"] = round(ms, 4)
    out["pattern_note"] = (f"bare row walk over G ({g_bytes / 1e9:.2f} GB), one block per wave or two (the max-abs scale pass's form); with writes: plus {w_bytes / 1e9:.3f} GB "
                           f"in {piece}-byte pieces per block to {k} streams, stored per wave after every row "
                           f"(per_wave) or per workgroup as {4 * piece}-byte lines after a barrier (the quantize pass's form); "
                           f"4waves: the kernel built for four waves per SIMD; fmaN: N dependent multiply-adds per row and lane")
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="resnet50")
    ap.add_argument("--scale", default="maxabs", choices=["maxabs", "l2"])
    ap.add_argument("--code", default="cyclic", choices=["cyclic", "interval"])
    ap.add_argument("--bucket", type=int, default=0, choices=[0, 256],
                    help="256: one scale per 256-coordinate bucket (single pass over G); 0: one per vector")
    ap.add_argument("--layers", type=int, default=0,
                    help="N > 0: layer-wise max-abs scales over N layers of equal size (agc_set_layers)")
    ap.add_argument("--two-pass", "--unfused", dest="two_pass", action="store_true",
                    help="run the step as two passes (stand-alone decode kernel) instead of the fused pass")
    ap.add_argument("--no-variants", action="store_true",
                    help="time only the configuration the flags select (profiling runs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-log2", type=int, default=21,
                    help="the single-thread oracle leg runs on the first 2^this coordinates")
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
    n, k, d = cfg.n, cfg.k, cfg.d
    p, bits, code, w = build_problem(cfg, api, args.code)
    G = I.partial_gradients_torch(cfg, dev)
    assert G.stride(0) % 4 == 0 and G.data_ptr() % 16 == 0
    codes = [torch.empty(api.agc_code_bytes(d, int(b)), dtype=torch.uint8, device=dev) for b in bits]
    ghat = torch.empty(d, dtype=torch.float32, device=dev)
    bufs = (codes, ghat)
    K, W = args.steps, args.warmup
    seed = cfg.philox_seed

    if args.calibrate:   # known traffic: reads 2^30 bytes, writes 2^30 bytes
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        api.agc_calibration_copy(dst, src, 1 << 30)
        torch.cuda.synchronize()
        del src, dst

    main_r = time_variant(api, I, cfg, G, bufs, p, bits, code, w, args.scale, args.bucket, args.two_pass, K, W, seed,
                          layers=args.layers)
    ms_per_step = main_r["ms_per_step"]
    grad_bytes = 4.0 * k * d
    value = grad_bytes / (ms_per_step * 1e-3) / 1e9
    roofline = roofline_of(main_r, tag_of(cfg, args.code, args.scale, args.bucket, args.two_pass, args.layers))

    default_run = (args.workload == "resnet50" and args.scale == "maxabs" and args.code == "cyclic"
                   and not args.bucket and not args.two_pass and not args.layers)
    variants = None
    if default_run and not args.no_variants:
        # the other forms of the step at the same size, same process, same inputs
        Kv = min(K, 20)
        variants = {}
        interval = build_problem(cfg, api, "interval")
        for name, (vcode, vscale, vbucket, vtwo, ckind, vlayers) in {
            "two_pass": (code, "maxabs", 0, True, "cyclic", 0),
            "l2": (code, "l2", 0, False, "cyclic", 0),
            "interval": (interval[2], "maxabs", 0, False, "interval", 0),
            "layers128": (code, "maxabs", 0, False, "cyclic", 128),
            "bucket256": (code, "maxabs", 256, False, "cyclic", 0),
            "bucket256_l2": (code, "l2", 256, False, "cyclic", 0),
            "interval_bucket256": (interval[2], "maxabs", 256, False, "interval", 0),
        }.items():
            vw = interval[3] if ckind == "interval" else w
            r = time_variant(api, I, cfg, G, bufs, p, bits, vcode, vw, vscale, vbucket, vtwo, Kv, 3, seed,
                             layers=vlayers)
            rf = roofline_of(r, tag_of(cfg, ckind, vscale, vbucket, vtwo, vlayers))
            variants[name] = {
                "ms_per_step": round(r["ms_per_step"], 4), "steps": Kv,
                "value_GBps": round(grad_bytes / (r["ms_per_step"] * 1e-3) / 1e9, 1),
                "step_alg_bytes": rf["step_alg_bytes"], "step_hbm_frac": rf["step_hbm_frac"],
                "dominant_kernel": rf["kernel"], "dominant_frac": rf["frac"], "traffic": rf["traffic"],
                "code_path": r["code_path"],
                "kernels_avg_ms": {nm: kv["avg_ms"] for nm, kv in r["kernels"].items()},
            }
        # what the memory system delivers on this machine: copy and the bare access pattern of the passes
        scratch = torch.empty(max(1 << 29, k * (d // 256) * 96 // 4 + 4), dtype=torch.float32, device=dev)
        ceil = measured_ceilings(api, G, k, d, scratch)
        del scratch
        roofline["measured_copy_GBps"] = ceil["copy_GBps"]
        roofline["frac_of_copy"] = round(roofline["achieved"] / ceil["copy_GBps"], 4)
        roofline["measured_pattern"] = ceil
        # the dominant kernel against the bare pattern with the same kind of traffic
        if "pattern_read_write_ms" in ceil and roofline["kernel"] == "quantize":
            roofline["dominant_vs_bare_pattern"] = round(ceil["pattern_read_write_ms"] / roofline["avg_launch_ms"], 4)
            # ... and against the same pattern at the pass's occupancy carrying about the pass's arithmetic per row
            roofline["dominant_vs_pattern_with_arithmetic"] = round(
                ceil["pattern_read_write_4waves_fma100_ms"] / roofline["avg_launch_ms"], 4)

    cpu_baseline = None
    if not args.no_cpu_baseline and not args.layers:   # the layer-wise oracle is a per-layer Python composition: not timed
        from oracle import agc_oracle as O
        csr = O.Csr(code[0], code[1], code[2], k)
        o_mode = O.SCALE_MAXABS if args.scale == "maxabs" else O.SCALE_L2
        o_step = O.step_bucket if args.bucket else O.step
        mask0 = I.arrival_mask(cfg, p, W)
        # (i) all threads, one whole step of the workload (every coordinate)
        Gh = G.cpu().numpy()
        c0 = time.perf_counter()
        o_step(Gh, csr, bits, w, mask0, seed, W, o_mode)
        c1 = time.perf_counter()
        # (ii) one thread, on a bounded sample of the same workload
        ds = min(d, 1 << args.cpu_sample_log2)
        Gs = np.ascontiguousarray(Gh[:, :ds])
        del Gh
        nthreads = O.threads()
        O.set_threads(1)
        s0 = time.perf_counter()
        o_step(Gs, csr, bits, w, mask0, seed, W, o_mode)
        s1 = time.perf_counter()
        O.set_threads(nthreads)
        cpu_baseline = {
            "value": round(4.0 * k * d / (c1 - c0) / 1e9, 4), "unit": "GB/s", "cores": nthreads, "kind": "oracle",
            "sample": f"one whole oracle step of the workload (all {d} coordinates of all {k} partitions, "
                      f"{n * d} coded elements), {c1 - c0:.2f} s wall on {nthreads} threads",
            "single_thread": {"value": round(4.0 * k * ds / (s1 - s0) / 1e9, 4), "unit": "GB/s", "cores": 1,
                              "sample": f"one oracle step on the first {ds} coordinates, {s1 - s0:.2f} s wall"},
        }

    sum_b = float(np.sum(bits))
    out = {
        "metric": "encode+quantize+decode GB/s of gradient traffic",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: n={n} workers, k={k} partitions, s={cfg.s}, d={d}, "
                               f"{cfg.law} gradients, bits sum {int(sum_b)} (mean {sum_b / n:.2f}), "
                               f"{args.code} code, {args.scale} scale"
                               + (f" per {args.bucket}-coordinate bucket" if args.bucket else
                                  f" per layer ({args.layers} layers)" if args.layers else " per vector")
                               + (", two-pass step" if args.two_pass else ", fused step"),
                   "code_path": main_r["code_path"]},
        "coded_elements_per_s": round(n * d / (ms_per_step * 1e-3), 1),
        "timing": {"ms_per_step": "wall clock over the K timed steps, no events between kernels",
                   "ms_per_step_with_events": round(main_r["ms_per_step_with_events"], 4),
                   "kernels": "HIP-event pairs around every kernel over K further steps on the same stream"},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "kernels": main_r["kernels"],
    }
    if variants is not None:
        out["two_pass"] = variants.pop("two_pass")
        out["variants"] = variants
    print(json.dumps(out))


if __name__ == "__main__":
    main()
