"""Benchmark of the pipelined GEMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Workload: the paper's motivating example (Fig. 1(b)): C = A.B with M = N = K = 2048, fp16 inputs
uniform in [-1, 1], fp32 accumulation on the matrix cores, fp16 output.  A "step" is one pass of
the whole hot path: tile decomposition, prologue, the S-stage / 2-level pipelined main loop,
and the epilogue - one alcop_gemm launch with the schedule the model-ranked tuner picked.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = 2516.6      # MI355X dense fp16/bf16 matrix peak: 256 CU x 4096 flop/clk x 2.4 GHz
PEAK_HBM_GBS = 8000.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--quick", action="store_true", help="skip the other shapes and the CPU baseline")
    ap.add_argument("--variants", action="store_true",
                    help="let the tuner also consider the kernels outside the default schedule space "
                         "(k-tile of 128; convolution with the input patch in LDS)")
    ap.add_argument("--workload", default="gemm2048",
                    help="configuration to time (the headline is gemm2048; other names of "
                         "workloads.CONFIGS only together with --sched)")
    ap.add_argument("--tune-report", action="store_true",
                    help="exhaustive search on every configuration and the best-in-top-k curves of the "
                         "two static models (the paper's Sec. 6.4 experiment); prints one JSON object")
    ap.add_argument("--copy-calib", type=int, default=0, metavar="MiB",
                    help="run a plain device-to-device copy of this many MiB --steps times and exit "
                         "(calibrates the FETCH_SIZE / WRITE_SIZE counters under rocprofv3 --pmc)")
    ap.add_argument("--splitk-report", action="store_true",
                    help="time the split-K entry points against the best unsplit schedule on the "
                         "configurations with fewer output tiles than compute units; prints one JSON object")
    ap.add_argument("--conv-patch-report", action="store_true",
                    help="conv56 / conv14: exhaustive search over the default kernels and over the "
                         "LDS-resident-patch variants (schedule variant 1); prints one JSON object")
    ap.add_argument("--ablation-report", action="store_true",
                    help="the headline kernel (and the 8192^3 one) timed with one class of operation left "
                         "out at a time (libalcop_diag.so): what loads, LDS reads, matrix instructions and "
                         "the barrier each cost and how well they overlap; prints one JSON object")
    ap.add_argument("--sched", default=None,
                    help="bm,bn,bk,wm,wn,S,R,F[,raster]: time this schedule only, no tuning (for profiling)")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the path is a single-kernel, single-GPU "
                 "optimisation; no collectives are part of it). Run with --gpus 1.")

    import numpy as np
    import torch

    import paper_2210_16691_amd as al
    import workloads as wl

    dev = "cuda:0"
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()

    if a.copy_calib:
        n = a.copy_calib << 20
        src = torch.empty(n, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(a.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes": n, "steps": a.steps}))
        return

    if a.tune_report:
        print(json.dumps(tune_report(al, wl, torch, dev)))
        return

    if a.splitk_report:
        print(json.dumps(splitk_report(al, wl, torch, dev, stream)))
        return

    if a.ablation_report:
        print(json.dumps(ablation_report(wl, torch, dev)))
        return

    if a.conv_patch_report:
        rep = {}
        for name in ("conv56", "conv14"):
            prob, Ad, Bd, Cd, conv, flops, byts = _setup(al, wl, torch, dev, name)
            base = al.alcop_tune(prob, Ad, Bd, Cd, top_k=0, model=0, iters=30, conv=conv)
            both = al.alcop_tune(prob, Ad, Bd, Cd, top_k=0, model=0, iters=30, conv=conv, variants=True)
            var = [(s, us) for s, _, us in both.log if s.variant == 1]
            best_var = min(var, key=lambda t: t[1]) if var else (None, float("nan"))
            rep[name] = {"default_best_us": round(base.best_us, 2), "default_best": repr(base.best),
                         "variant_best_us": round(best_var[1], 2), "variant_best": repr(best_var[0]),
                         "speedup": round(base.best_us / best_var[1], 3),
                         "tflops_variant": round(flops / best_var[1] / 1e6, 1),
                         "variants": [[repr(s), round(us, 2)] for s, us in sorted(var, key=lambda t: t[1])[:8]]}
        print(json.dumps(rep))
        return

    if a.sched:
        # profiling mode: one fixed schedule of any configuration, no tuning, a minimal JSON line
        s = al.sched(*[int(v) for v in a.sched.split(",")])
        prob, Ad, Bd, Cd, conv, flops, byts = _setup(al, wl, torch, dev, a.workload)
        cfg = wl.CONFIGS[a.workload]

        def launch():
            if cfg["kind"] == "gemm":
                al.alcop_gemm(Ad, Bd, Cd, s, stream=stream)
            elif cfg["kind"] == "bmm":
                al.alcop_bmm(Ad, Bd, Cd, s, transB=cfg["transB"], stream=stream)
            else:
                al.alcop_conv2d_igemm(Ad, Bd, Cd, (1, 1), (1, 1), s, stream=stream)

        for _ in range(a.warmup):
            launch()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(stream)
        for _ in range(a.steps):
            launch()
        e1.record(stream)
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / a.steps
        print(json.dumps({"workload": a.workload, "schedule": repr(s), "kernel_us": round(us, 3),
                          "tflops": round(flops / us / 1e6, 1),
                          "gbs_algorithmic": round(byts / us / 1e3, 1), "steps": a.steps}))
        return

    if a.workload not in ("gemm2048", "gemm4096", "gemm8192", "ffn1", "ffn2"):
        sys.exit("bench.py: the tuned headline run supports the GEMM configurations; use --sched for " + a.workload)
    cfg, A, B = wl.make_inputs(a.workload)
    M, N, K = cfg["M"], cfg["N"], cfg["K"]
    Ad, Bd = A.to(dev), B.to(dev)
    it = al.F16 if cfg["dtype"] == "f16" else al.BF16
    Cd = torch.empty(M, N, dtype=torch.float16 if cfg["out"] == "f16" else torch.bfloat16, device=dev)
    prob = al.problem(al.OP_GEMM, M, N, K, it, it)
    flops = 2.0 * M * N * K

    # ---- tuning: exhaustive (the 100 % reference) and model-ranked top-k ------------------------
    ex = al.alcop_tune(prob, Ad, Bd, Cd, top_k=0, model=0, iters=30, variants=a.variants)
    meas = {s.key(): us for s, _, us in ex.log}
    best_ex = min(meas.values())

    def best_in_top(k, model):
        order = [s for s in al.alcop_sched_ranked(prob, model, a.variants, k) if s.key() in meas]
        return best_ex / min(meas[s.key()] for s in order[:k])

    top10 = al.alcop_tune(prob, Ad, Bd, Cd, top_k=10, model=0, iters=30, variants=a.variants)
    # the tuner's 30-launch trials of the leading schedules lie within their noise: time its three
    # fastest again, 500 launches each, and keep the winner
    finalists = sorted(top10.log, key=lambda t: t[2])[:3]
    retimed = [(al.alcop_time(prob, Ad, Bd, Cd, s, 20, 500), s) for s, _, _ in finalists]
    best = min(retimed, key=lambda t: t[0])[1]
    # the 1-stage (unpipelined) schedule at the same tile
    base = al.sched(best.bm, best.bn, best.bk, best.wm, best.wn, 1, 1, 0, best.raster)
    us_base = al.alcop_time(prob, Ad, Bd, Cd, base, 50, 1000)
    us_best = al.alcop_time(prob, Ad, Bd, Cd, best, 50, 1000)
    # best pipelined vs 1-stage at equal tiles, for every tile of the sweep
    sweep = {}
    for s, _, us in ex.log:
        sweep.setdefault((s.bm, s.bn, s.bk, s.wm, s.wn), {})[(s.stages, s.reg_stages, s.fuse_inner)] = us
    tile_speedups = {"%dx%dx%d/w%dx%d" % t: round(v[(1, 1, 0)] / min(v.values()), 3)
                     for t, v in sweep.items() if (1, 1, 0) in v}
    # ablation in the paper's terms (Sec. 6.1), each the best schedule of its class over all tiles,
    # normalised to the best unpipelined (S=1, R=1) schedule
    def best_of(pred):
        c = [us for s, _, us in ex.log if pred(s)]
        return min(c) if c else float("nan")
    t_unp = best_of(lambda s: s.stages == 1 and s.reg_stages == 1)
    ablation = {
        "unpipelined_us": round(t_unp, 2),
        "double_buffer_only_S2_R1": round(t_unp / best_of(lambda s: s.stages == 2 and s.reg_stages == 1), 3),
        "multi_stage_single_level_R1": round(t_unp / best_of(lambda s: s.reg_stages == 1), 3),
        "multi_level_two_stage_only": round(t_unp / best_of(lambda s: s.stages <= 2), 3),
        "multi_level_unfused": round(t_unp / best_of(lambda s: not s.fuse_inner), 3),
        "multi_stage_multi_level_fused": round(t_unp / best_of(lambda s: True), 3),
    }

    # ---- the timed region --------------------------------------------------------------------
    for _ in range(a.warmup):
        al.alcop_gemm(Ad, Bd, Cd, best)
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(a.steps):
        al.alcop_gemm(Ad, Bd, Cd, best, stream=stream)
    e1.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / a.steps
    kernel_us_region = e0.elapsed_time(e1) * 1e3 / a.steps       # HIP events on the launch stream
    value = flops / (ms_per_step * 1e-3) / 1e12
    # roofline figure: median of 5 repeats, each of enough back-to-back launches for >= 50 ms
    n50 = max(a.steps, int(50e3 / max(kernel_us_region, 1e-3)) + 1)
    reps = []
    for _ in range(5):
        e0.record(stream)
        for _ in range(n50):
            al.alcop_gemm(Ad, Bd, Cd, best, stream=stream)
        e1.record(stream)
        torch.cuda.synchronize()
        reps.append(e0.elapsed_time(e1) * 1e3 / n50)
    kernel_us = sorted(reps)[2]
    achieved = flops / (kernel_us * 1e-6) / 1e12
    # context, not the metric: the same schedule on all-zero operands executes the same instruction
    # stream with less switching in the matrix pipes and data paths; what it gains is clock
    Az, Bz = torch.zeros_like(Ad), torch.zeros_like(Bd)
    for _ in range(200):
        al.alcop_gemm(Az, Bz, Cd, best, stream=stream)
    e0.record(stream)
    for _ in range(n50):
        al.alcop_gemm(Az, Bz, Cd, best, stream=stream)
    e1.record(stream)
    torch.cuda.synchronize()
    zero_us = e0.elapsed_time(e1) * 1e3 / n50
    del Az, Bz

    traffic, traffic_source = None, None
    tf = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tf):
        # HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (see profiles/)
        recs = json.load(open(tf)).get(a.workload) or []
        same_tile = lambda r: r["schedule"].split(" S")[0] == repr(best).split(" S")[0] and \
            r["schedule"].split(" r")[-1].split(" ")[0] == repr(best).split(" r")[-1].split(" ")[0]
        rec = next((r for r in recs if r["schedule"] == repr(best)), None)
        near = rec or next((r for r in recs if same_tile(r)), None)
        if rec:
            traffic = rec["fetch_bytes"] + rec["write_bytes"]
            traffic_source = ("profiles/hbm_traffic.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier "
                              "run of this schedule, scaled by a copy kernel; not measured in this run")
        elif near:
            # the traffic is a property of the tile and the block order: the pipelinings of one tile
            # that were profiled agree within 0.1 %
            traffic = near["fetch_bytes"] + near["write_bytes"]
            traffic_source = ("profiles/hbm_traffic.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of "
                              + near["schedule"] + ", the same tile and block order with another pipelining, "
                              "scaled by a copy kernel; not measured in this run")
        else:
            traffic_source = "none: no schedule with the tuned schedule's tile was profiled (profiles/hbm_traffic.json)"

    out = {
        "metric": "TFLOP/s and % of fp16 MFMA peak per shape; speedup vs 1-stage schedule",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": round(ms_per_step, 6), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": "%s: C=A.B, M=%d N=%d K=%d, %s in, fp32 accumulate, %s out" % (a.workload, M, N, K, cfg["dtype"], cfg["out"]),
                   "schedule": repr(best), "global_batch": 1},
        "pct_of_peak": round(100.0 * value / PEAK_TFLOPS, 2),
        "speedup_vs_1stage_equal_tile": round(us_base / us_best, 3),
        "us_1stage": round(us_base, 2), "us_best": round(us_best, 2),
        "tile_speedups_vs_1stage": tile_speedups,
        "ablation_speedup_vs_unpipelined": ablation,
        "tuner": {"trials": top10.trials, "finalists_retimed_us": [[repr(s), round(us, 2)] for us, s in retimed],
                  "exhaustive_trials": ex.trials,
                  "best_in_top10_pct": round(100 * best_in_top(10, 0), 1),
                  "best_in_top10_pct_bottleneck_model": round(100 * best_in_top(10, 1), 1),
                  "best_in_top5_pct": round(100 * best_in_top(5, 0), 1),
                  "exhaustive_best": repr(ex.best), "exhaustive_best_us": round(ex.best_us, 2)},
        "roofline": {"bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(achieved / PEAK_TFLOPS, 4), "traffic": traffic,
                     "traffic_source": traffic_source,
                     "algorithmic_bytes": 2 * (M * K + K * N) + 2 * M * N,
                     "kernel_us": round(kernel_us, 3),
                     "kernel_us_protocol": "median of 5 repeats of %d back-to-back launches (>= 50 ms each), "
                                           "HIP events on the launch stream" % n50,
                     "kernel_us_repeats": [round(r, 3) for r in reps],
                     "kernel_us_timed_region": round(kernel_us_region, 3),
                     "kernel_us_all_zero_operands": round(zero_us, 3),
                     "frac_all_zero_operands": round(flops / zero_us / 1e6 / PEAK_TFLOPS, 4),
                     "note_all_zero_operands": "context only: the same kernel and launch count on zero-filled A "
                                               "and B; the difference to kernel_us is the clock the power "
                                               "management allows, not the schedule"},
        "paper_context": "A100/TVM: 1.23x mean (0.95-1.73x) single-operator speedup from pipelining; "
                         "another machine, context only",
    }

    if not a.quick:
        out["vendor_library_context"] = vendor_context(wl, torch, dev)
        # the other configurations are tuned over the whole kernel table, including the kernels
        # outside the default schedule space (persistent producer / consumer kernels, k-tile 128,
        # LDS-resident convolution patch)
        out["other_shapes"] = other_shapes(al, wl, torch, dev, True)
        out["cpu_baseline"] = cpu_baseline(wl, A, B, flops)
        if a.workload == "gemm2048":
            # the timed schedule's output against the oracle's (the test suite does this for many
            # schedules; here for the one the headline number belongs to)
            import oracle
            ref = oracle.gemm(wl.bits(A), wl.bits(B), oracle.F16)
            got = Cd.cpu().double().numpy()
            out["headline_output_within_tolerance"] = bool(
                np.all(np.abs(got - ref) <= 1e-2 * (np.abs(ref) + 1.0)))
    print(json.dumps(out))


def ablation_report(wl, torch, dev):
    """Microseconds per launch (back-to-back launches, HIP events) of the same kernel with
    operation classes removed; outputs of the ablated kernels are meaningless."""
    from paper_2210_16691_amd import diag
    names = diag.configs()
    drops = [("full", 0), ("no_dma", diag.NO_DMA), ("no_lds_reads", diag.NO_LDS_READ),
             ("no_mfma", diag.NO_MFMA), ("no_barrier", diag.NO_BARRIER),
             ("no_dma_no_lds_reads", diag.NO_DMA | diag.NO_LDS_READ),
             ("dma_only", diag.NO_LDS_READ | diag.NO_MFMA), ("no_store", diag.NO_STORE),
             ("no_lds_swizzle", diag.NO_SWIZZLE),
             ("launch_prologue_barriers_epilogue", diag.NO_DMA | diag.NO_LDS_READ | diag.NO_MFMA),
             ("the_same_without_stores", diag.NO_DMA | diag.NO_LDS_READ | diag.NO_MFMA | diag.NO_STORE)]
    rep = {"empty_kernel_us": {"%dx%d" % (b, t): round(diag.alcop_diag_launch_floor(b, t, 1000), 2)
                               for b, t in ((1, 64), (256, 256), (256, 512), (1024, 512))}}
    for wname in ("gemm2048", "gemm8192"):
        cfg, A, B = wl.make_inputs(wname)
        Ad, Bd = A.to(dev), B.to(dev)
        Cd = torch.empty(cfg["M"], cfg["N"], dtype=Ad.dtype, device=dev)
        flops = 2.0 * cfg["M"] * cfg["N"] * cfg["K"]
        want = "f16" if cfg["dtype"] == "f16" else "bf16"
        for i, n in enumerate(names):
            if not n.startswith(want + " "):
                continue
            # two passes, second reported: the first absorbs clock ramp-up and order effects
            row = {}
            for _ in range(2):
                for label, d in drops:
                    row[label] = round(diag.alcop_diag_time(i, d, Ad, Bd, Cd, 200 if wname == "gemm2048" else 10), 2)
            # the same kernel (a separately named copy, for the profiler) on all-zero operands: the same
            # instructions and cycles, less switching
            Az, Bz = torch.zeros_like(Ad), torch.zeros_like(Bd)
            n = 200 if wname == "gemm2048" else 10
            diag.alcop_diag_time(i, diag.COPY, Az, Bz, Cd, n)
            row["full_zero_operands"] = round(diag.alcop_diag_time(i, diag.COPY, Az, Bz, Cd, n), 2)
            row["tflops_full"] = round(flops / row["full"] / 1e6, 1)
            rep.setdefault(wname, {})[n] = row
    return rep


def _setup(al, wl, torch, dev, name):
    """Device tensors, problem descriptor and flop / byte counts of a named configuration."""
    cfg, A, B = wl.make_inputs(name)
    Ad, Bd = A.to(dev), B.to(dev)
    it = al.F16 if cfg["dtype"] == "f16" else al.BF16
    tdt = torch.float16 if cfg["out"] == "f16" else torch.bfloat16
    conv = None
    if cfg["kind"] == "gemm":
        M, N, K, b = cfg["M"], cfg["N"], cfg["K"], 1
        prob = al.problem(al.OP_GEMM, M, N, K, it, it)
        Cd = torch.empty(M, N, dtype=tdt, device=dev)
    elif cfg["kind"] == "bmm":
        M, N, K, b = cfg["M"], cfg["N"], cfg["K"], cfg["batch"]
        prob = al.problem(al.OP_BMM, M, N, K, it, it, batch=b, transB=cfg["transB"])
        Cd = torch.empty(b, M, N, dtype=tdt, device=dev)
    else:
        n, H, W, C, Ko, R, S = (cfg[k] for k in ("N", "H", "W", "C", "K", "R", "S"))
        M, N, K, b = n * H * W, Ko, R * S * C, 1
        prob = al.problem(al.OP_CONV2D, M, N, K, it, it, conv_C=C)
        Cd = torch.empty(n, H, W, Ko, dtype=tdt, device=dev)
        conv = (n, H, W, C, Ko, R, S, 1, 1, 1, 1)
    flops = 2.0 * M * N * K * b
    byts = 2.0 * (A.numel() + B.numel() + Cd.numel())
    return prob, Ad, Bd, Cd, conv, flops, byts


def tune_report(al, wl, torch, dev):
    """Exhaustive search per configuration; best-in-top-k of the pipeline-aware model and of the
    bottleneck-only model, normalised to the exhaustive best (paper Sec. 6.4 / 6.5 metrics)."""
    rep = {}
    for name in ("gemm2048", "ffn1", "ffn2", "gemm8192", "bmm_qk", "bmm_pv", "conv56", "conv14",
                 "mm_rn50_fc", "bmm_gpt2_qk"):
        prob, Ad, Bd, Cd, conv, flops, byts = _setup(al, wl, torch, dev, name)
        iters = 5 if name == "gemm8192" else 30
        ex = al.alcop_tune(prob, Ad, Bd, Cd, top_k=0, model=0, iters=iters, conv=conv)
        meas = [(s, us) for s, _, us in ex.log]
        best = min(us for _, us in meas)
        curves = {}
        ks = [k for k in (1, 5, 10, 20, 50) if k <= len(meas)]
        by_key = {s.key(): us for s, us in meas}
        for model, label in ((0, "analytical"), (1, "bottleneck")):
            # the tuner's own order of trials for a budget of k (per-family cap included)
            curves[label] = {}
            for k in ks:
                order = [s for s in al.alcop_sched_ranked(prob, model, False, k) if s.key() in by_key]
                curves[label][str(k)] = round(100.0 * best / min(by_key[s.key()] for s in order[:k]), 1)
        # grid search: schedules in table order
        table = [s.key() for s in al.alcop_sched_space(prob)]
        grid = [by_key[k] for k in table if k in by_key]
        curves["grid"] = {str(k): round(100.0 * best / min(grid[:k]), 1) for k in ks}
        # measurement-corrected model: a real tuning run of 20 trials, best after each prefix
        r2 = al.alcop_tune(prob, Ad, Bd, Cd, top_k=min(20, len(meas)), model=2, iters=iters, conv=conv)
        seq = [us for _, _, us in r2.log]
        curves["analytical_plus_learned"] = {
            str(k): round(100.0 * best / min(seq[:k]), 1) for k in ks if k <= len(seq)}
        top = sorted(meas, key=lambda t: t[1])[:5]
        rep[name] = {"space": ex.space, "exhaustive_best_us": round(best, 2),
                     "tflops": round(flops / best / 1e6, 1), "gbs": round(byts / best / 1e3, 1),
                     "best_in_top_k_pct": curves,
                     "top5": [[repr(s), round(us, 2)] for s, us in top],
                     "all": [[list(s.key()), round(us, 3)] for s, us in meas]}
    return rep


def splitk_report(al, wl, torch, dev, stream):
    """Best unsplit schedule (model's top 10, timed) against split-K (the model's schedule, every
    slice count timed) on the shapes whose tile count leaves compute units idle."""
    rep = {}

    def timed(fn, iters=200):
        for _ in range(10):
            fn()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(stream)
        for _ in range(iters):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / iters

    for name in ("mm_rn50_fc", "conv14", "ffn2"):
        prob, Ad, Bd, Cd, conv, flops, byts = _setup(al, wl, torch, dev, name)
        base = al.alcop_tune(prob, Ad, Bd, Cd, top_k=10, model=0, iters=50, conv=conv)
        M, N = prob.M, prob.N
        s, pick, pred = al.alcop_splitk_auto(prob)
        ws = torch.empty(al.alcop_splitk_workspace_bytes(1, M, N, 32) // 4, dtype=torch.float32, device=dev)
        tuned, tuned_split = al.alcop_tune_splitk(prob, Ad, Bd, Cd, ws, top_k=10, iters=50, conv=conv)
        by_split = {}
        for k in (1, 2, 3, 4, 6, 8, 12, 16, 24, 32):
            if k > (prob.K + s.bk - 1) // s.bk:
                continue
            if conv is None:
                fn = lambda k=k: al.alcop_gemm_splitk(Ad, Bd, Cd, k, ws, s, stream=stream)
            else:
                fn = lambda k=k: al.alcop_conv2d_igemm_splitk(Ad, Bd, Cd, k, ws, (1, 1), (1, 1), s, stream=stream)
            by_split[k] = round(timed(fn), 2)
        best_k = min(by_split, key=by_split.get)
        rep[name] = {"unsplit_best_us": round(base.best_us, 2), "unsplit_schedule": repr(base.best),
                     "splitk_schedule": repr(s), "model_split": pick, "model_predicted_us": round(pred, 2),
                     "tuned_top10": {"schedule": repr(tuned.best), "split": tuned_split,
                                     "us": round(tuned.best_us, 2), "space": tuned.space,
                                     "speedup_vs_unsplit": round(base.best_us / tuned.best_us, 3)},
                     "us_by_split": by_split, "best_split": best_k,
                     "speedup_best_split": round(base.best_us / by_split[best_k], 3),
                     "speedup_model_split": round(base.best_us / by_split.get(pick, float("nan")), 3),
                     "tflops_best_split": round(flops / by_split[best_k] / 1e6, 1)}
    return rep


def _rotating_us(al, torch, stream, cfg, sched, Ad, Bd, Cd, byts, iters):
    """Mean time per launch when consecutive launches use different copies of the operands, enough
    copies (> 320 MB together) that the 256 MB Infinity Cache cannot serve a launch from what the
    previous ones left there.  For the HBM-bound shapes; the operands of one launch fit the cache."""
    nset = max(2, int(320e6 // byts) + 1)
    sets = [(Ad, Bd, Cd)] + [(Ad.clone(), Bd.clone(), torch.empty_like(Cd)) for _ in range(nset - 1)]

    def launch(a, b, c):
        if cfg["kind"] == "bmm":
            al.alcop_bmm(a, b, c, sched, transB=cfg["transB"], stream=stream)
        elif cfg["kind"] == "conv":
            al.alcop_conv2d_igemm(a, b, c, (1, 1), (1, 1), sched, stream=stream)
        else:
            al.alcop_gemm(a, b, c, sched, stream=stream)

    for a, b, c in sets:
        launch(a, b, c)
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record(stream)
    for i in range(iters):
        launch(*sets[i % nset])
    e1.record(stream)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / iters, nset


def other_shapes(al, wl, torch, dev, variants=False):
    """Tuned (top-10 by the model) time of the remaining configurations; context for the headline."""
    res = {}
    stream = torch.cuda.current_stream()
    for name in ("ffn1", "ffn2", "gemm4096", "gemm8192", "bmm_qk", "bmm_pv", "conv56", "conv14", "mm_rn50_fc",
                 "bmm_gpt2_qk"):
        cfg, A, B = wl.make_inputs(name)
        Ad, Bd = A.to(dev), B.to(dev)
        it = al.F16 if cfg["dtype"] == "f16" else al.BF16
        tdt = torch.float16 if cfg["out"] == "f16" else torch.bfloat16
        conv = None
        if cfg["kind"] == "gemm":
            M, N, K, b = cfg["M"], cfg["N"], cfg["K"], 1
            prob = al.problem(al.OP_GEMM, M, N, K, it, it)
            Cd = torch.empty(M, N, dtype=tdt, device=dev)
        elif cfg["kind"] == "bmm":
            M, N, K, b = cfg["M"], cfg["N"], cfg["K"], cfg["batch"]
            prob = al.problem(al.OP_BMM, M, N, K, it, it, batch=b, transB=cfg["transB"])
            Cd = torch.empty(b, M, N, dtype=tdt, device=dev)
        else:
            n, H, W, C, Ko, R, S = (cfg[k] for k in ("N", "H", "W", "C", "K", "R", "S"))
            M, N, K, b = n * H * W, Ko, R * S * C, 1
            prob = al.problem(al.OP_CONV2D, M, N, K, it, it, conv_C=C)
            Cd = torch.empty(n, H, W, Ko, dtype=tdt, device=dev)
            conv = (n, H, W, C, Ko, R, S, 1, 1, 1, 1)
        iters = 10 if name == "gemm8192" else 50
        r = al.alcop_tune(prob, Ad, Bd, Cd, top_k=10, model=0, iters=iters, conv=conv, variants=variants)
        # the unpipelined schedule at the same tile (the tile-at-a-time kernel also for a persistent best)
        base = al.sched(r.best.bm, r.best.bn, r.best.bk, r.best.wm, r.best.wn, 1, 1, 0, r.best.raster,
                        0, 1 if r.best.variant == 1 else 0)
        us1 = al.alcop_time(prob, Ad, Bd, Cd, base, 3, iters, conv=conv)
        fl = 2.0 * M * N * K * b
        byts = 2.0 * (A.numel() + B.numel() + Cd.numel())
        res[name] = {"us": round(r.best_us, 2), "tflops": round(fl / r.best_us / 1e6, 1),
                     "pct_peak": round(100 * fl / r.best_us / 1e6 / PEAK_TFLOPS, 1),
                     "gbs_algorithmic": round(byts / r.best_us / 1e3, 1),
                     "speedup_vs_1stage": round(us1 / r.best_us, 3), "schedule": repr(r.best)}
        if name in ("bmm_qk", "bmm_pv", "bmm_gpt2_qk", "conv56"):
            # HBM-bound: also with the operands rotated out of the Infinity Cache
            try:
                us_rot, nset = _rotating_us(al, torch, stream, cfg, r.best, Ad, Bd, Cd, byts, 4 * iters)
                res[name].update({"us_rotating_buffers": round(us_rot, 2), "buffer_sets": nset,
                                  "gbs_algorithmic_rotating": round(byts / us_rot / 1e3, 1)})
            except Exception as e:      # a context figure must not cost the headline line
                res[name]["us_rotating_buffers"] = "failed: %r" % (e,)
    return res


def vendor_context(wl, torch, dev):
    """torch.matmul (the vendor GEMM library behind it) on the same operands, timed the same way:
    context for the roofline fractions, not a target and not part of the path."""
    res = {}
    for name in ("gemm2048", "ffn1", "ffn2", "gemm4096", "gemm8192", "bmm_qk", "bmm_pv", "mm_rn50_fc"):
        try:
            cfg, A, B = wl.make_inputs(name)
            Ad, Bd = A.to(dev), B.to(dev)
            if cfg["kind"] == "bmm" and cfg["transB"]:
                Bd = Bd.transpose(1, 2)
            iters = 10 if name == "gemm8192" else (50 if name == "gemm4096" else 200)
            for _ in range(5):
                torch.matmul(Ad, Bd)
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            best = None
            for _ in range(3):
                torch.cuda.synchronize()
                e0.record()
                for _ in range(iters):
                    torch.matmul(Ad, Bd)
                e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / iters
                best = us if best is None or us < best else best
            b = cfg.get("batch", 1) if cfg["kind"] == "bmm" else 1
            fl = 2.0 * cfg["M"] * cfg["N"] * cfg["K"] * b
            res[name] = {"torch_matmul_us": round(best, 2), "tflops": round(fl / best / 1e6, 1)}
        except Exception as e:           # a context figure must not cost the headline line
            res[name] = "failed: %r" % (e,)
    # a plain device-to-device copy of 64 MiB: what the memory system gives a trivially
    # bandwidth-bound kernel (read + write counted), for the HBM-bound shapes
    try:
        src = torch.empty(64 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        bufs = [(src, dst)] + [(src.clone(), torch.empty_like(src)) for _ in range(3)]
        for s_, d_ in bufs:
            d_.copy_(s_)
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(200):
            s_, d_ = bufs[i % 4]
            d_.copy_(s_)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / 200
        res["device_copy_64MiB"] = {"us": round(us, 2), "gbs_read_plus_write": round(2 * (64 << 20) / us / 1e3, 1)}
    except Exception as e:
        res["device_copy_64MiB"] = "failed: %r" % (e,)
    return res


def cpu_baseline(wl, A, B, flops):
    """The oracle as it stands, timed on the host cores: the whole 2048^3 problem, repeated until
    about 20 core-seconds of work have passed."""
    import oracle
    ab, bb = wl.bits(A), wl.bits(B)
    oracle.gemm(ab[:64], bb, oracle.F16)                 # page in / spawn threads
    reps, t0 = 0, time.perf_counter()
    while True:
        oracle.gemm(ab, bb, oracle.F16)
        reps += 1
        dt = time.perf_counter() - t0
        if dt * oracle.threads() > 20.0 or reps >= 50:
            break
    return {"value": round(reps * flops / dt / 1e12, 5), "unit": "TFLOP/s", "cores": oracle.threads(),
            "kind": "oracle",
            "sample": "the full 2048^3 GEMM, %d times in %.2f s wall on %d threads (%.0f core-seconds)" % (
                reps, dt, oracle.threads(), dt * oracle.threads())}


if __name__ == "__main__":
    main()
