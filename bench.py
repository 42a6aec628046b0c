#!/usr/bin/env python3
"""Benchmark of the W4A16 GEMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]
                    [--config c4] [--M 1] [--kernel -1] [--split 0] [--warm] [--table] [--fig2] [--ablation]
                    [--split-sweep] [--timeline]

A step is one whole GEMM (Eq. 2: every launch w4a16_gemm enqueues for it) on
seeded synthetic inputs already resident in HBM.  By default consecutive steps
walk over distinct copies of the weights, scales and zero points totalling
more than 640 MB, so that no step finds its weights in the 256 MB last-level
cache ("cold"); --warm reuses one copy and is labelled so.

Prints ONE JSON line on stdout (headline: M=1, K=28672, N=8192).  --table adds
every configuration of the workload list to the line; --out DIR also writes the
tables as JSON files into DIR.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_FP16_PEAK_TFLOPS = 2500.0  # MI355X published dense fp16 MFMA rate
COLD_BYTES = 640 * 1024 * 1024
# HBM bytes per launch of the headline kernel, from the committed rocprofv3 --pmc summaries
# (profiles/hbm_traffic.json: FETCH_SIZE and WRITE_SIZE, scaled by a copy kernel of known size).
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")
KERNEL_NAMES = {0: "wave_split_kernel", 3: "stripe_kernel", 4: "tile_kernel"}


def kernel_name(plan, M, group):
    """The multiply kernel a plan launches (as rocprofv3 names it, without template arguments)."""
    if plan["kernel"] == 3:
        return "stripe_dyn_kernel" if M <= 4 else "stripe_kernel"
    if plan["kernel"] == 4:
        if plan["tile_m"] == 16 and M <= 16:
            return "tile_dyn_kernel"
        if group == 128:
            return "tile_wide_kernel" if plan["waves_k"] == 4 and plan["tile_m"] in (32, 64) else "tile_group_kernel"
    return KERNEL_NAMES.get(plan["kernel"], "?")


def measured_traffic(key):
    try:
        with open(TRAFFIC_FILE) as f:
            return json.load(f).get(key, {}).get("bytes_per_launch")
    except (OSError, ValueError):
        return None


def save(out_dir, name, obj):
    if out_dir:
        os.makedirs(out_dir, exist_ok=True)
        with open(os.path.join(out_dir, name), "w") as f:
            json.dump(obj, f, indent=1)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_gemm(torch, binding, wl, name, M, steps, warmup, kernel=-1, split=0, warm=False, host=None, graph=True,
              replays=5, bf16=False):
    """Returns dict with µs per GEMM: HIP events around `steps` back-to-back GEMMs (one replay of a HIP graph
    that holds them; the median of `replays` replays is the value, the fastest is reported beside it;
    graph=False times the eager Python loop instead).  bf16: the same draw of X as bfloat16, through w4a16_gemm_bf16."""
    cfg = wl.config(name)
    if host is None:
        host = wl.make_config(name)
    Xall, Wp, s, Zp = host
    X = np.ascontiguousarray(Xall[:M])
    wbytes = Wp.nbytes + s.nbytes + Zp.nbytes
    copies = 1 if warm else max(2, -(-COLD_BYTES // wbytes))
    if bf16:
        Xb = wl.make_x_bf16(max(cfg.Ms), cfg.K, cfg.index, cfg.outliers)[:M]
        dX = torch.from_numpy(np.ascontiguousarray(Xb).view(np.int16)).cuda().view(torch.bfloat16)
    else:
        dX = torch.from_numpy(X).cuda()
    base = binding.to_device(X, Wp, s, Zp)[1:]
    sets = [base] + [tuple(t.clone() for t in base) for _ in range(copies - 1)]
    Y = torch.empty((M, cfg.N), dtype=torch.bfloat16 if bf16 else torch.float16, device="cuda")
    stream = torch.cuda.current_stream()
    gemm = binding.gemm_bf16 if bf16 else binding.gemm_ex

    def call(i):
        W_, S_, Z_ = sets[i % copies]
        gemm(dX, W_, S_, Z_, cfg.group, kernel=kernel, split=split, out=Y, stream=torch.cuda.current_stream())

    for i in range(warmup):
        call(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if graph:
        # The K steps are recorded once into a HIP graph (kernel launches only) and replayed: the GPU then
        # runs them back to back, and the Python cost of a call (several us) stays out of the measurement.
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(steps):
                call(warmup + i)
        g.replay()  # untimed: first replay of a new graph
        torch.cuda.synchronize()
        times = []
        for _ in range(replays):
            e0.record(stream)
            g.replay()
            e1.record(stream)
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1) * 1e3 / steps)
        us, us_min = float(np.median(times)), min(times)
    else:
        e0.record(stream)
        for i in range(steps):
            call(warmup + i)
        e1.record(stream)
        torch.cuda.synchronize()
        us = us_min = e0.elapsed_time(e1) * 1e3 / steps
    # Context, never the value: the latency of one call on an idle stream (events around a single eager call), and
    # what the memory system gives a kernel that only reads the same weights, scales and zero points, no arithmetic.
    single = []
    for i in range(15):
        torch.cuda.synchronize()
        e0.record(stream)
        call(warmup + steps + i)
        e1.record(stream)
        torch.cuda.synchronize()
        single.append(e0.elapsed_time(e1) * 1e3)
    probe_us = None
    if graph:
        sink = torch.zeros(4, dtype=torch.int32, device="cuda")
        for i in range(min(warmup, 2 * copies)):
            binding.stream_probe(sets[i % copies], sink)
        torch.cuda.synchronize()
        gp = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gp):
            for i in range(steps):
                binding.stream_probe(sets[i % copies], sink, stream=torch.cuda.current_stream())
        gp.replay()
        torch.cuda.synchronize()
        times = []
        for _ in range(3):
            e0.record(stream)
            gp.replay()
            e1.record(stream)
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1) * 1e3 / steps)
        probe_us = float(np.median(times))
    nbytes = wl.algorithmic_bytes(M, cfg.K, cfg.N, cfg.group)
    flops = 2.0 * M * cfg.K * cfg.N
    plan = binding.query_plan(M, cfg.N, cfg.K, cfg.group, kernel, split)
    res = {
        "config": name, "M": M, "K": cfg.K, "N": cfg.N, "us_per_gemm": us, "us_per_gemm_min": us_min,
        "algorithmic_bytes": nbytes, "GBps": nbytes / us * 1e-3, "hbm_frac": nbytes / us * 1e-3 / HBM_PEAK_GBS,
        "TFLOPs": flops / us * 1e-6, "mfma_frac": flops / us * 1e-6 / MFMA_FP16_PEAK_TFLOPS,
        "cache": "warm (one weight copy, last-level-cache resident)" if warm else "cold (%d weight copies)" % copies,
        "plan": plan,
        "single_call_us": float(np.median(single)),
        "read_only_probe_us": probe_us, "read_only_probe_GBps": (wbytes / probe_us * 1e-3) if probe_us else None,
    }
    return res, Y, (dX, sets[(warmup + steps - 1) % copies])


def cpu_baseline(wl, orc, host, M, cfg):
    """The oracle as it stands, on the host cores, on the same workload."""
    Xall, Wp, s, Zp = host
    X = np.ascontiguousarray(Xall[:M])
    best = None
    t_all = time.time()
    reps = 0
    while reps < 3 or (time.time() - t_all < 6.0 and reps < 10):
        t = time.time()
        ref = orc.gemm(X, Wp, s, Zp, cfg.group)
        dt = time.time() - t
        best = dt if best is None else min(best, dt)
        reps += 1
    return {
        "value": best * 1e6, "unit": "us/GEMM", "cores": orc.threads(), "kind": "oracle",
        "sample": "whole %s GEMM (M=%d, K=%d, N=%d), best of %d passes, fp64 scalar C with OpenMP over columns"
                  % (cfg.name, M, cfg.K, cfg.N, reps),
    }, ref


def fig2(torch, binding, wl, max_steps):
    """Section 4.1's comparison on this GPU: the scheduler's plan (Split-K where it pays) against the
    data-parallel plans, i.e. S = 1 forced on each kernel family that takes the shape: column tiles spread
    over the workgroups, K not split between them.  The baseline is the fastest of those."""
    rows = []
    for name, c in wl.FIG2.items():
        h = wl.make_config(name)
        steps = max(50, min(max_steps, int(2e5 / max(1.0, 1e-6 * c.K * c.N / 16))))
        for M in c.Ms:
            auto, _, _ = time_gemm(torch, binding, wl, name, M, steps, max(10, steps // 10), host=h)
            dp = {}
            for fam, kid in (("wave_split", binding.KERNEL_WAVE_SPLIT), ("stripe", binding.KERNEL_STRIPE),
                             ("tile", binding.KERNEL_TILE)):
                if (kid == binding.KERNEL_WAVE_SPLIT and M > 4) or (kid == binding.KERNEL_STRIPE and M > 16):
                    continue
                if binding.query_plan(M, c.N, c.K, c.group, kid, 1)["split"] != 1:
                    continue  # the family cannot take the whole K in one slice here
                r, _, _ = time_gemm(torch, binding, wl, name, M, steps, max(10, steps // 10), kernel=kid, split=1, host=h)
                dp[fam] = r["us_per_gemm"]
            best = min(dp, key=dp.get)
            row = {"shape": name, "N": c.N, "K": c.K, "M": M, "split_k_us": auto["us_per_gemm"],
                   "split_k_plan": auto["plan"], "data_parallel_us": dp, "data_parallel_best": best,
                   "speedup": dp[best] / auto["us_per_gemm"]}
            log(json.dumps(row))
            rows.append(row)
        del h
    # K << N: the scheduler's plan against forced splits of the same family
    for name, c in wl.WIDE.items():
        h = wl.make_config(name)
        steps = max(50, min(max_steps, int(2e5 / max(1.0, 1e-6 * c.K * c.N / 16))))
        for M in c.Ms:
            auto, _, _ = time_gemm(torch, binding, wl, name, M, steps, max(10, steps // 10), host=h)
            forced = {}
            for S in (1, 2, 4):
                r, _, _ = time_gemm(torch, binding, wl, name, M, steps, max(10, steps // 10), kernel=auto["plan"]["kernel"],
                                    split=S, host=h)
                forced["S=%d" % S] = r["us_per_gemm"]
            row = {"shape": name, "N": c.N, "K": c.K, "M": M, "split_k_us": auto["us_per_gemm"], "split_k_plan": auto["plan"],
                   "forced_us": forced}
            log(json.dumps(row))
            rows.append(row)
        del h
    return rows


def split_sweep(torch, binding, wl, max_steps):
    """The evidence behind the scheduler's split factors (Algorithm 1 takes S as an input and gives no rule):
    us per GEMM against S for both families the scheduler uses, cold weights, on the decode configurations
    and the (N, K) pairs of the paper's Fig. 2."""
    rows = []
    cases = [("c2", (1,)), ("c3", (1, 4, 16)), ("c4", (1, 8)), ("f2a", (1, 16)), ("f2b", (1, 16)), ("f2c", (1, 16)),
             ("f2d", (1, 16)), ("f2e", (1, 16)), ("f2f", (1, 16))]
    for name, Ms in cases:
        c = wl.config(name)
        h = wl.make_config(name)
        G = c.K // c.group
        steps = max(50, min(max_steps, int(1e5 / max(1.0, 1e-6 * c.K * c.N / 16))))
        for M in Ms:
            auto = binding.query_plan(M, c.N, c.K, c.group)
            for fam, kid in (("stripe", binding.KERNEL_STRIPE), ("tile", binding.KERNEL_TILE)):
                if kid == binding.KERNEL_STRIPE and M > 16:
                    continue
                own = binding.query_plan(M, c.N, c.K, c.group, kid, 0)["split"]
                tried = {}
                for S in sorted({1, 2, 3, 4, 6, 7, 8, 12, 14, 16, 24, 28, 32, 48, 56, own}):
                    if S > G:
                        continue
                    plan = binding.query_plan(M, c.N, c.K, c.group, kid, S)
                    if plan["split"] in tried:
                        continue
                    r, _, _ = time_gemm(torch, binding, wl, name, M, steps, 10, kernel=kid, split=S, host=h, replays=3)
                    tried[plan["split"]] = r["us_per_gemm"]
                best = min(tried, key=tried.get)
                row = {"shape": name, "N": c.N, "K": c.K, "M": M, "family": fam, "us_by_split": tried,
                       "family_choice": own, "family_choice_us": tried[own], "best_split": best, "best_us": tried[best],
                       "scheduler_takes_this_family": auto["kernel"] == kid}
                log(json.dumps(row))
                rows.append(row)
        del h
    return rows


def timeline(torch, binding, wl, name, M):
    """Per-phase time stamps of the decode kernel (profiling build of the library, M <= 4 stripe plans): one
    eager launch on cold weights after a few warm-up launches."""
    import ctypes
    cfg = wl.config(name)
    host = wl.make_config(name)
    Xall, Wp, s, Zp = host
    X = np.ascontiguousarray(Xall[:M])
    plan = binding.query_plan(M, cfg.N, cfg.K, cfg.group)
    if plan["kernel"] != binding.KERNEL_STRIPE or M > 4:
        sys.exit("bench.py --timeline: the scheduler's plan for this shape is not the decode kernel")
    base = binding.to_device(X, Wp, s, Zp)
    wbytes = Wp.nbytes + s.nbytes + Zp.nbytes
    copies = max(2, -(-COLD_BYTES // wbytes))
    sets = [base[1:]] + [tuple(t.clone() for t in base[1:]) for _ in range(copies - 1)]
    waves, wgs = plan["waves_k"], plan["workgroups"]
    words = torch.zeros(wgs * 16 * 8, dtype=torch.int64, device="cuda")
    setter = binding.lib().w4a16_timeline_buffer
    setter.argtypes = [ctypes.c_void_p]
    assert setter(words.data_ptr()) == 0
    for i in range(2 * copies + 1):
        binding.gemm(base[0], *sets[i % copies], cfg.group)
    torch.cuda.synchronize()
    setter(None)
    t = words.cpu().numpy().reshape(wgs, 16, 8)[:, :waves, :].astype(np.float64)
    t0 = t[:, :, 0].min()
    us = lambda col: (t[:, :, col] - t0) / 100.0
    phases = {"kernel_entry_last_wave": us(0).max(), "first_unit_in_use_mean": us(1).mean(), "first_unit_in_use_last_wave": us(1).max(),
              "loop_end_first_wave": us(2).min(), "loop_end_mean": us(2).mean(), "loop_end_last_wave": us(2).max(),
              "workgroup_sums_done_last": us(3).max(), "atomic_add_back_last": us(4).max(), "exit_last_wave": us(5).max()}
    return {"config": name, "M": M, "plan": plan, "us_after_first_wave_entry": {k: round(float(v), 2) for k, v in phases.items()}}


def time_calls(torch, fn, steps, warmup, replays=3):
    """us per call of fn(i): HIP events around one replay of a HIP graph holding `steps` calls; the eager
    loop where the calls cannot be captured."""
    stream = torch.cuda.current_stream()
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    try:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(steps):
                fn(warmup + i)
        run = g.replay
    except Exception as e:  # a library call that refuses capture
        log("graph capture refused (%s): timing the eager loop" % e)
        torch.cuda.synchronize()

        def run():
            for i in range(steps):
                fn(warmup + i)
    run()
    torch.cuda.synchronize()
    best = None
    for _ in range(replays):
        e0.record(stream)
        run()
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        best = ms if best is None else min(best, ms)
    return best * 1e3 / steps


def ablation(torch, binding, wl, max_steps):
    """Section 4.2 on this GPU.  Unfused: Phase 1 writes the dequantised FP16 weights to global memory
    (w4a16_dequant), an FP16 GEMM (torch.matmul, i.e. the vendor BLAS) reads them back.  FP16 x FP16: that
    GEMM alone, the weights never quantised.  Fused: w4a16_gemm.  Cold: consecutive steps use different
    copies of the weights (FP16 copies of 100 MB and more are rotated in pairs: one pass already
    exceeds the 256 MB last-level cache together with its successor)."""
    rows = []
    for name, Ms in (("c2", (1,)), ("c3", (1, 16)), ("c4", (1, 8)), ("c5", (32, 128))):
        cfg = wl.config(name)
        host = wl.make_config(name)
        Xall, Wp, s, Zp = host
        dW, dS, dZ = binding.to_device(Xall[:1], Wp, s, Zp)[1:]
        fp16_bytes = 2 * cfg.K * cfg.N
        copies = max(2, -(-COLD_BYTES // fp16_bytes))
        W16 = [binding.dequant(dW, dS, dZ, cfg.group) for _ in range(copies)]
        steps = max(30, min(max_steps, int(5e4 / max(1.0, 1e-6 * cfg.K * cfg.N / 16))))
        t_deq = time_calls(torch, lambda i: binding.dequant(dW, dS, dZ, cfg.group, out=W16[i % copies]), steps, 5)
        for M in Ms:
            dX = torch.from_numpy(np.ascontiguousarray(Xall[:M])).cuda()
            Y = torch.empty((M, cfg.N), dtype=torch.float16, device="cuda")
            t_mm = time_calls(torch, lambda i: torch.matmul(dX, W16[i % copies], out=Y), steps, 5)
            fused, Yf, _ = time_gemm(torch, binding, wl, name, M, steps, 10, host=host)
            d = (Y.float() - Yf.float()).abs().max().item()  # same product up to the FP16 rounding of the weights
            row = {"config": name, "M": M, "K": cfg.K, "N": cfg.N, "fused_us": fused["us_per_gemm"], "dequant_us": t_deq,
                   "fp16_gemm_us": t_mm, "unfused_us": t_deq + t_mm, "unfused_over_fused": (t_deq + t_mm) / fused["us_per_gemm"],
                   "fp16_over_fused": t_mm / fused["us_per_gemm"], "max_abs_diff_unfused_vs_fused": d}
            log(json.dumps(row))
            rows.append(row)
        del W16
        torch.cuda.empty_cache()
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=600)
    ap.add_argument("--warmup", type=int, default=60)
    ap.add_argument("--config", default="c4")
    ap.add_argument("--M", type=int, default=1)
    ap.add_argument("--kernel", type=int, default=-1)
    ap.add_argument("--split", type=int, default=0)
    ap.add_argument("--warm", action="store_true")
    ap.add_argument("--table", action="store_true")
    ap.add_argument("--fig2", action="store_true",
                    help="also time Split-K (the scheduler's plan) against data-parallel plans (S = 1) on the "
                         "(N, K) pairs of the paper's Fig. 2")
    ap.add_argument("--ablation", action="store_true",
                    help="also time the unfused variant (dequantised FP16 weights through HBM + vendor FP16 GEMM) "
                         "and the FP16 x FP16 GEMM alone against the fused path (Section 4.2)")
    ap.add_argument("--split-sweep", action="store_true", help="also time every admissible split factor S of both families "
                    "on the decode shapes (the evidence behind the scheduler's choices)")
    ap.add_argument("--timeline", action="store_true", help="print the decode kernel's per-phase time stamps for --config / --M "
                    "from the profiling build (python -m paper_2601_16536_amd.build --timeline) and exit")
    ap.add_argument("--out", default=None, help="directory for bench_table.json, bench_fig2.json, bench_ablation.json")
    ap.add_argument("--no-cpu", action="store_true", help="skip the host-baseline leg")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the path is a single-device kernel); --gpus %d is not offered"
                 % args.gpus)

    import torch
    from paper_2601_16536_amd import binding, workloads as wl
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    if args.timeline:
        from paper_2601_16536_amd import build as hip_build
        if not os.path.exists(hip_build.TIMELINE_LIB):
            sys.exit("bench.py --timeline: build the profiling library first (python -m paper_2601_16536_amd.build --timeline)")
        binding.use_library(hip_build.TIMELINE_LIB)
    binding.lib()
    torch.cuda.set_device(0)
    if args.timeline:
        print(json.dumps(timeline(torch, binding, wl, args.config, args.M)), flush=True)
        return

    cfg = wl.config(args.config)
    host = wl.make_config(args.config)
    res, Y, _ = time_gemm(torch, binding, wl, args.config, args.M, args.steps, args.warmup, args.kernel, args.split,
                          args.warm, host)
    log("headline:", json.dumps(res))

    from oracle import w4a16_oracle as orc  # host-baseline leg and the parity check of what was timed
    cpu = None
    if not args.no_cpu:
        cpu, ref = cpu_baseline(wl, orc, host, args.M, cfg)
        out = Y.cpu().numpy().astype(np.float64)
        ratio = float(np.max(np.abs(out - ref) / (1e-2 * (1 + np.abs(ref)))))
        log("parity of the timed output vs oracle: err/tol = %.4f" % ratio)
        if ratio > 1.0:
            sys.exit("bench.py: timed output fails parity (err/tol = %.3f)" % ratio)

    line = {
        "metric": "us/GEMM + achieved HBM TB/s (fraction of peak), W4A16 M=1..16, K>>N",
        "value": res["us_per_gemm"], "unit": "us/GEMM", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["us_per_gemm"] * 1e-3, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16 inputs, int4 weights, f32 accumulate", "data": "synthetic",
        "config": {"workload": "%s: M=%d K=%d N=%d group=%d, W4A16, %s" % (args.config, args.M, cfg.K, cfg.N,
                                                                          cfg.group, res["cache"]),
                   "plan": res["plan"]},
        "us_per_gemm_min": res["us_per_gemm_min"], "timing": "median of 5 replays of a HIP graph of %d GEMMs (fastest replay beside it)" % args.steps,
        "achieved_TBps": res["GBps"] * 1e-3, "achieved_TFLOPs": res["TFLOPs"],
        # context, not the metric: one call alone on an idle stream, and a kernel that only reads the same weights
        "context": {"single_call_us": res["single_call_us"], "read_only_probe_us": res["read_only_probe_us"],
                    "read_only_probe_TBps": res["read_only_probe_GBps"] * 1e-3 if res["read_only_probe_GBps"] else None},
        # the roofline that bounds the kernel: HBM below the ridge of 2.5 PFLOP/s over 8 TB/s = 312.5 flop/byte, MFMA above
        "roofline": ({"bound": "hbm", "achieved": res["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": res["hbm_frac"]}
                     if 2.0 * args.M * cfg.K * cfg.N / res["algorithmic_bytes"] < 1e3 * MFMA_FP16_PEAK_TFLOPS / HBM_PEAK_GBS else
                     {"bound": "mfma", "achieved": res["TFLOPs"], "peak": MFMA_FP16_PEAK_TFLOPS, "unit": "TFLOP/s",
                      "frac": res["mfma_frac"]}),
    }
    line["roofline"].update({"traffic": measured_traffic("%s_M%d" % (args.config, args.M)),
                     "launches_per_step": 1 if res["plan"]["split"] == 1 or res["plan"]["workspace_bytes"] ==
                     8 * args.M * cfg.N else 2,
                     "kernel": kernel_name(res["plan"], args.M, cfg.group),
                     "algorithmic_bytes_per_launch": res["algorithmic_bytes"],
                     "algorithmic_flops_per_launch": 2.0 * args.M * cfg.K * cfg.N})
    line["cpu_baseline"] = cpu
    line["environment"] = {"device": torch.cuda.get_device_name(0), "compute_units": torch.cuda.get_device_properties(0).multi_processor_count,
                           "hip": torch.version.hip, "torch": torch.__version__, "host_cpus": os.cpu_count()}

    if args.table:
        rows = []
        for name, c in wl.CONFIGS.items():
            h = host if name == args.config else wl.make_config(name)
            for M in c.Ms:
                steps = max(50, min(args.steps, int(2e5 / max(1.0, 1e-6 * c.K * c.N / 16))))
                r, _, _ = time_gemm(torch, binding, wl, name, M, steps, max(10, steps // 10), host=h)
                r2, _, _ = time_gemm(torch, binding, wl, name, M, steps, max(10, steps // 10), warm=True, host=h)
                r["us_per_gemm_warm"] = r2["us_per_gemm"]
                r3, _, _ = time_gemm(torch, binding, wl, name, M, steps, max(10, steps // 10), host=h, bf16=True)
                r["us_per_gemm_bf16"] = r3["us_per_gemm"]
                log(json.dumps(r))
                rows.append(r)
            del h
        line["table"] = rows
        save(args.out, "bench_table.json", line)
    if args.ablation:
        line["ablation"] = ablation(torch, binding, wl, args.steps)
        save(args.out, "bench_ablation.json", line["ablation"])
    if args.split_sweep:
        line["split_sweep"] = split_sweep(torch, binding, wl, args.steps)
        save(args.out, "bench_split_sweep.json", line["split_sweep"])
    if args.fig2:
        line["fig2"] = fig2(torch, binding, wl, args.steps)
        save(args.out, "bench_fig2.json", line["fig2"])
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
