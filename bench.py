#!/usr/bin/env python3
"""Benchmark of libsdrop's hot path on one MI355X.

A step is one pass of the whole hot path of arxiv 2411.01238 (Section 3.1 eq. (1)-(3),
Section 3.2) over one batch: draw the block mask, forward GEMM, dX GEMM, dW GEMM.
The workload is the 4096^3 bf16 square case with 128x128 blocks; the headline value is
the effective TFLOP/s (flops of kept blocks only: 3 * 2 * nnz * BM * BK * N per step)
at p = 0.5, and the same is reported for the whole sweep of p together with the
speed-up over this library's own dense run (p = 0, all blocks kept, same kernels).

Prints one JSON line.  One GPU only.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_DENSE_TFLOPS = 2500.0     # MI355X published dense bf16/fp16 MFMA peak
# What the matrix cores of this chip were measured to sustain under its power limit (profiles/probe_clock_mfma_lds_loads.md):
# bf16 MFMAs issued back to back hold 1.56 GHz = 1640 TFLOP/s; with the operand reads from LDS that feed them, 1390
MFMA_ONLY_CEILING_TFLOPS = 1640.0
MFMA_WITH_LDS_READS_CEILING_TFLOPS = 1390.0
# Bytes per launch that crossed L2 -> fabric: rocprofv3 FETCH_SIZE / WRITE_SIZE of an earlier run of this
# benchmark's launches, scaled by a known 1 GiB copy.  Constants from the tracked counter summaries named
# here, NOT measured by this run (counters need the profiler).
TRAFFIC_BYTES = {
    ("square4096", 0.5): {"fwd": 235.6e6, "bwd": 581.2e6, "source": "profiles/bench_square4096_p0.5.md"},
    ("mlp", 0.5): {"fwd": 58.2e6, "bwd": 127.9e6, "source": "profiles/bench_mlp_p0.5.md"},
    ("mlp", 0.1): {"fwd": 85.1e6, "bwd": 135.6e6, "source": "profiles/bench_mlp_p0.1.md"},
    ("ffn_down", 0.1): {"fwd": 372.9e6, "bwd": 671.7e6, "source": "profiles/bench_ffn_down_p0.1.md"},
    ("skinny", 0.3): {"fwd": 1781.5e6, "bwd": 4891.2e6, "source": "profiles/bench_skinny_p0.3.md"},
}


def headline_p(w):
    """The dropout rate the headline is quoted at: 0.5 where the workload is run at it, else the workload's own rate."""
    return 0.5 if 0.5 in w.ps else w.ps[-1]


def _sets(w, n_sets, torch):
    """n_sets independent copies of the inputs and outputs, resident in HBM."""
    from paper_2411_01238_amd.workloads import make_inputs
    X, W, dY = make_inputs(w)
    sets = []
    for _ in range(n_sets):
        s = {"X": X.cuda(), "W": W.cuda(), "dY": dY.cuda()}
        s["Y"] = torch.empty((w.M, w.N), dtype=X.dtype, device="cuda")
        s["dX"] = torch.empty((w.M, w.K), dtype=X.dtype, device="cuda")
        s["dW"] = torch.empty((w.K, w.N), dtype=X.dtype, device="cuda")
        sets.append(s)
    return sets


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="square4096")
    ap.add_argument("--p", type=float, default=None, help="dropout rate of the headline (default: 0.5 where the workload is run at it, else the workload's own)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy, as the known-size reference for HBM byte counters")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (the hot path is a single-GPU kernel path); "
                 "run with --gpus 1")

    import torch
    from paper_2411_01238_amd import sdrop
    from paper_2411_01238_amd.workloads import WORKLOADS

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    sdrop.lib()   # fails loudly if the HIP library is not built
    w = WORKLOADS[args.workload]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    # three buffer sets (576 MiB at 4096^3) rotate so that a step's operands are not left in
    # the 256 MiB Infinity Cache by the step before; a single-set (warm) figure is given too
    sets = _sets(w, 3, torch)
    HEADLINE_P = headline_p(w) if args.p is None else args.p
    mask = sdrop.Mask(w.M, w.K, w.BM, w.BK, HEADLINE_P)
    td = w.torch_dtype
    ws_need = sdrop.workspace_bytes(sdrop.OP_BWD_DW, w.M, w.K, w.N, w.BM, w.BK, td, td)
    ws = torch.empty(max(ws_need, 16), dtype=torch.uint8, device="cuda")

    def step(s, p, seed, events=None):
        if events is not None:
            events[0].record()
        # the mask and eq. (1) in one call: one launch where the block grid is small enough for every
        # workgroup to draw it (the mask object for the backward comes out of the same launch), else two
        sdrop.sdrop_fwd_seeded(s["X"], s["W"], w.BM, w.BK, p, seed, 0, mask=mask, out=s["Y"])
        if events is not None:
            events[1].record()
        # eq. (2) and eq. (3) in one call: one launch where the shapes allow it, else two
        sdrop.sdrop_bwd(s["dY"], s["W"], s["X"], mask, out_dx=s["dX"], out_dw=s["dW"], ws=ws)
        if events is not None:
            events[2].record()

    def nnz_of(p, seed):
        sdrop.sdrop_mask(w.M, w.K, w.BM, w.BK, p, seed, 0, out=mask)
        torch.cuda.synchronize()
        return mask.nnz()

    def timed(p, steps, warmup, n_sets, seed=w.mask_seed):
        for i in range(warmup):
            step(sets[i % n_sets], p, seed)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step(sets[i % n_sets], p, seed)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3     # ms per step

    def per_kernel(p, steps, n_sets, seed=w.mask_seed):
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
        for i in range(steps):
            step(sets[i % n_sets], p, seed, evs[i])
        torch.cuda.synchronize()
        names = ("fwd", "bwd")          # "fwd" is the call that also draws the mask
        return {n: sum(e[k].elapsed_time(e[k + 1]) for e in evs) / steps for k, n in enumerate(names)}

    flops_per_block = 3 * 2.0 * w.BM * w.BK * w.N

    if args.calibrate_copy:
        # reads 1 GiB and writes 1 GiB: what FETCH_SIZE / WRITE_SIZE report for it gives the scale factor
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- headline: p = 0.5, rotating buffer sets ----
    nnz = nnz_of(HEADLINE_P, w.mask_seed)
    # the same measurement straight after start-up, reported beside the headline
    ms_cold = timed(HEADLINE_P, args.steps, args.warmup, 3)
    # settle (untimed, not part of --warmup): the first ~100 steps after start-up run about 10 %
    # slower than the steady state (first touches of the buffers, clocks ramping)
    timed(HEADLINE_P, 150, 0, 3)
    ms = timed(HEADLINE_P, args.steps, args.warmup, 3)
    value = nnz * flops_per_block / (ms * 1e-3) / 1e12
    ms_warm = timed(HEADLINE_P, args.steps, args.warmup, 1)
    kern = per_kernel(HEADLINE_P, args.steps, 3)

    # for reference: eq. (2) and eq. (3) launched on their own (the same kernels, two launches)
    def separate(steps, n_sets):
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
        for i in range(steps):
            s = sets[i % n_sets]
            evs[i][0].record()
            sdrop.sdrop_bwd_dx(s["dY"], s["W"], mask, out=s["dX"])
            evs[i][1].record()
            sdrop.sdrop_bwd_dw(s["X"], s["dY"], mask, out=s["dW"], ws=ws)
            evs[i][2].record()
        torch.cuda.synchronize()
        return {n: sum(e[k].elapsed_time(e[k + 1]) for e in evs) / steps for k, n in enumerate(("dx", "dw"))}
    nnz_of(HEADLINE_P, w.mask_seed)
    kern_sep = separate(args.steps, 3)
    # and the step with the mask as a launch of its own (sdrop_mask, sdrop_fwd, sdrop_bwd)
    sdrop.set_tuning(sdrop.TUNE_FWD_SEEDED, 0)
    ms_mask_launch = timed(HEADLINE_P, args.steps, args.warmup, 3)
    sdrop.set_tuning(sdrop.TUNE_FWD_SEEDED, 1)

    # ---- sweep over p (fewer steps each), speed-up against the library's own dense run ----
    # The points are visited in shuffled order, in several rounds (every round visits every p), and a
    # point's time is the mean over its rounds: drift of the clocks during the sweep then spreads over all
    # points instead of reading as scaling.  p = 0 (the library's own dense run) is always a point.
    sweep = {}
    if not args.no_sweep:
        import random
        rounds = 3
        k_sweep = max(4, args.steps // (2 * rounds))
        points = sorted(set(w.ps) | {0.0})
        acc = {p: [] for p in points}
        rnd = random.Random(20241128)
        for _ in range(rounds):
            order = points[:]
            rnd.shuffle(order)
            for p in order:
                acc[p].append(timed(p, k_sweep, 3, 3))
        ms_dense = sum(acc[0.0]) / rounds
        for p in points:
            n_p = nnz_of(p, w.mask_seed)
            ms_p = sum(acc[p]) / rounds
            sweep["%.1f" % p] = {
                "ms_per_step": round(ms_p, 5), "kept_fraction": round(n_p / (w.MB * w.KB), 5),
                "eff_tflops": round(n_p * flops_per_block / (ms_p * 1e-3) / 1e12, 3),
                "speedup_vs_own_dense": round(ms_dense / ms_p, 4),
                "ideal_speedup": round(w.MB * w.KB / max(n_p, 1), 4),
                "ms_per_round": [round(t, 5) for t in acc[p]],
            }
        sweep_order = "shuffled, %d rounds of %d steps per point, mean over rounds" % (rounds, k_sweep)

    # ---- how linear is t(p) in the kept fraction f?  least squares t = a + b f over the sweep ----
    linearity = None
    if len(sweep) >= 3:
        fs = [v["kept_fraction"] for v in sweep.values()]
        ts = [v["ms_per_step"] for v in sweep.values()]
        n = len(fs)
        mf, mt = sum(fs) / n, sum(ts) / n
        b = sum((f - mf) * (t - mt) for f, t in zip(fs, ts)) / sum((f - mf) ** 2 for f in fs)
        a = mt - b * mf
        ss_res = sum((t - (a + b * f)) ** 2 for f, t in zip(fs, ts))
        ss_tot = sum((t - mt) ** 2 for t in ts)
        linearity = {"fit": "ms_per_step = a + b * kept_fraction", "a_ms": round(a, 5), "b_ms": round(b, 5),
                     "a_over_t_dense": round(a / sweep["0.0"]["ms_per_step"], 4) if "0.0" in sweep else None,
                     "r2": round(1.0 - ss_res / ss_tot, 5)}

    # ---- context only: the vendor's dense GEMMs (torch.matmul) on the same shapes and layouts ----
    vendor = None
    if not args.no_sweep:
        s0 = sets[0]
        def _t(fn, iters=20):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(iters):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / iters
        vendor = {"fwd_X@W": round(_t(lambda: torch.matmul(s0["X"], s0["W"], out=s0["Y"])), 5),
                  "dx_dY@W.T": round(_t(lambda: torch.matmul(s0["dY"], s0["W"].t(), out=s0["dX"])), 5),
                  "dw_X.T@dY": round(_t(lambda: torch.matmul(s0["X"].t(), s0["dY"], out=s0["dW"])), 5)}
        vendor["sum_ms"] = round(sum(vendor.values()), 5)

    # ---- beyond the headline: the block Linear -> ReLU -> SparseDrop -> Linear with all six GEMMs
    #      sparse (producer with bias + ReLU in its tail, eq. (2) with the ReLU gate, eq. (1)/(3) at
    #      scale 1 for the producing layer's gradients); needs N0 = N, true for the square workloads ----
    block = None
    if not args.no_sweep and vendor is not None:
        s0 = sets[0]
        nnz_of(HEADLINE_P, w.mask_seed)
        b0 = torch.zeros(w.K, dtype=torch.float32, device="cuda")
        dz, dh, dw0 = torch.empty_like(s0["dX"]), torch.empty_like(s0["dY"]), torch.empty_like(s0["W"])
        parts = {
            "producer_bias_relu": lambda: sdrop.sdrop_producer(s0["dY"], s0["W"], b0, mask, act=sdrop.ACT_RELU, out=s0["X"]),
            "fwd": lambda: sdrop.sdrop_fwd(s0["X"], s0["W"], mask, out=s0["Y"]),
            "dx_relu_gate": lambda: sdrop.sdrop_bwd_dx_ex(s0["dY"], s0["W"], mask, relu_mask=s0["X"], out=dz),
            "dw": lambda: sdrop.sdrop_bwd_dw(s0["X"], s0["dY"], mask, out=s0["dW"], ws=ws),
            "dh_fwd_scale1": lambda: sdrop.sdrop_fwd_ex(dz, s0["W"], mask, scale_mode=sdrop.SCALE_ONE, out=dh),
            "dw0_dw_scale1": lambda: sdrop.sdrop_bwd_dw_ex(dz, s0["dY"], mask, scale_mode=sdrop.SCALE_ONE, out=dw0, ws=ws),
        }
        gemms = list(parts.values())
        db0 = torch.empty(w.K, dtype=torch.float32, device="cuda")
        ws_bg = torch.empty(max(sdrop.bias_grad_workspace_bytes(w.M, w.K, w.BM, w.BK), 16), dtype=torch.uint8, device="cuda")
        parts["db0_bias_grad"] = lambda: sdrop.sdrop_bias_grad(dz, mask, out=db0, ws=ws_bg)
        def whole():
            for f in gemms:
                f()
        block = {k: round(_t(f), 5) for k, f in parts.items()}
        block["plain_dx"] = round(_t(lambda: sdrop.sdrop_bwd_dx(s0["dY"], s0["W"], mask, out=dz)), 5)
        t_block = _t(whole)
        block["six_gemms_ms"] = round(t_block, 5)
        block["eff_tflops"] = round(6 * 2.0 * nnz * w.BM * w.BK * w.N / (t_block * 1e-3) / 1e12, 3)
        # the same block with a dense producing layer (vendor GEMMs, element-wise passes not counted)
        block["three_sparse_plus_three_vendor_dense_ms"] = round(ms_warm + vendor["sum_ms"], 5)

    # ---- roofline of the dominant kernel (largest average duration among the three GEMMs) ----
    dom = max(("fwd", "bwd"), key=lambda n: kern[n])
    flops_gemm = 2.0 * nnz * w.BM * w.BK * w.N         # algorithmic flops of one of the three products
    flops_launch = flops_gemm * (2 if dom == "bwd" else 1)     # the backward launch holds eq. (2) and eq. (3)
    achieved = flops_launch / (kern[dom] * 1e-3) / 1e12
    traffic = TRAFFIC_BYTES.get((w.name, HEADLINE_P), {})
    roofline = {"bound": "mfma", "kernel": {"fwd": "sdrop_fwd_seeded (mask and eq. 1)", "bwd": "sdrop_bwd (eq. 2 and eq. 3)"}[dom],
                "achieved": round(achieved, 3), "peak": PEAK_BF16_DENSE_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / PEAK_BF16_DENSE_TFLOPS, 5),
                "traffic": traffic.get(dom),
                "traffic_source": ("%s (an earlier profiled run of the same launches, not this run)" % traffic["source"]) if traffic else None,
                "algorithmic_bytes": algorithmic_bytes(w, nnz, dom),
                "traffic_over_algorithmic": round(traffic[dom] / algorithmic_bytes(w, nnz, dom), 3) if traffic.get(dom) else None,
                "duration_is": "HIP events on the launch stream around each launch of the timed steps (includes the dispatch "
                               "latency between dependent launches); profiles/ holds the rocprofv3 kernel trace of the same command",
                "frac_of_measured_mfma_ceiling": {
                    "mfma_only_1640_tflops": round(achieved / MFMA_ONLY_CEILING_TFLOPS, 5),
                    "mfma_with_lds_operand_reads_1390_tflops": round(achieved / MFMA_WITH_LDS_READS_CEILING_TFLOPS, 5),
                    "source": "profiles/probe_clock_mfma_lds_loads.md"},
                "avg_launch_ms": {k: round(v, 5) for k, v in kern.items()},
                "separate_launch_ms": {k: round(v, 5) for k, v in kern_sep.items()}}

    out = {
        "metric": "effective TFLOP/s fwd+bwd (kept blocks) & speedup vs dense GEMM at p in {0.1,0.3,0.5}",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": "%s: M=%d K=%d N=%d %s, block %dx%d, p=%.1f (mask + fwd + dX + dW per step; mask and fwd by one sdrop_fwd_seeded call, dX and dW by one sdrop_bwd call), "
                               "%s outputs, 3 rotating buffer sets" % (w.name, w.M, w.K, w.N, w.dtype, w.BM, w.BK, HEADLINE_P, w.dtype),
                   "kept_blocks": nnz, "blocks": w.MB * w.KB},
        "frac_of_bf16_peak": round(value / PEAK_BF16_DENSE_TFLOPS, 5),
        "ms_per_step_warm_single_set": round(ms_warm, 5),
        "untimed_settle_steps_before_warmup": 150,
        "ms_per_step_before_settle": round(ms_cold, 5),
        "ms_per_step_with_mask_as_its_own_launch": round(ms_mask_launch, 5),
        "sweep": sweep,
        "sweep_order": sweep_order if sweep else None,
        "linearity": linearity,
        "vendor_dense_gemm_ms_single_set": vendor,
        "sparse_relu_block_ms_single_set": block,
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, HEADLINE_P)
    print(json.dumps(out))


def algorithmic_bytes(w, nnz, launch):
    """Minimum HBM bytes of a launch: kept blocks of X, all of W, dY and the outputs, each once."""
    e = 2
    f = nnz / float(w.MB * w.KB)
    fwd = f * w.M * w.K * e + w.K * w.N * e + w.M * w.N * e
    dx = w.M * w.N * e + w.K * w.N * e + w.M * w.K * e
    dw = f * w.M * w.K * e + w.M * w.N * e + w.K * w.N * e
    return fwd if launch == "fwd" else dx + dw


def cpu_baseline(w, p, rows=None):
    """The float64 oracle, as it stands, on the first `rows` rows of the same workload."""
    import numpy as np
    import torch
    from oracle import sdrop_oracle as orc
    from paper_2411_01238_amd.workloads import make_inputs
    rows = w.M if rows is None else rows
    X, W, dY = make_inputs(w, M=rows)
    keep = orc.mask(rows // w.BM, w.KB, p, w.mask_seed, 0)
    Xd, Wd, dYd = (t.to(torch.float64).numpy() for t in (X, W, dY))
    t0 = time.perf_counter()
    orc.fwd(Xd, Wd, keep, w.BM, w.BK, p)
    orc.bwd_dx(dYd, Wd, keep, w.BM, w.BK, p)
    orc.bwd_dw(Xd, dYd, keep, w.BM, w.BK, p)
    dt = time.perf_counter() - t0
    flops = 3 * 2.0 * int(keep.sum()) * w.BM * w.BK * w.N
    return {"value": round(flops / dt / 1e12, 6), "unit": "TFLOP/s", "cores": orc.threads(), "kind": "oracle",
            "sample": "first %d rows of X and dY (M=%d of %d), full K and N, same mask rule, p=%.1f; "
                      "float64 fwd + dX + dW once, %.1f s" % (rows, rows, w.M, p, dt)}


if __name__ == "__main__":
    main()
