#!/usr/bin/env python3
"""Side measurements of the TEAL decode path on one MI355X (bench.py holds the headline).

    python bench_extras.py [--workload llama2_7b|llama3_8b|llama_70b] [--format bf16|w8|w4]
                           [--sparsities 0.5,0.4,0] [--layers L] [--steps K] [--warmup W]
                           [--unfused | --stack-launch] [--batch B] [--graph]
                           [--calibration | --swiglu | --rmsnorm]

Without a mode flag: a pass over one decoder block (or a stack with --layers) timed per
sparsity the three ways the library can issue it (one launch per group, per projection, 16
independent groups per launch), every projection and group alone, each projection as one of
16 independent products, and the vendor GEMV for context: the tables of
profiles/bench_results_all_configs.md come from here.  --batch B: the small-batch variant
(Section 5.4.4); --graph: the pass replayed from a captured HIP graph; --calibration: the
threshold calibration pass (Section 4.2); --swiglu / --rmsnorm: the products with their input
formed in the kernel against the two-launch path (Appendix A.3).  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

import teal_inputs as ti
from bench_lib import (BITS, CACHE_DEFEAT_BYTES, HBM_PEAK_GBS, KERNEL, FusedGroup, Projection,  # noqa: F401
                       Replica, StackCall, algorithmic_bytes, build_stack, cpu_baseline,
                       cpu_baseline_one_core, deep_layer_check, fuse, gpu_clocks, measured_traffic,
                       one_step, pct, read_ceiling, survivor_counts_match, time_projection,
                       time_projection_spread, time_steps, time_steps_graph, time_torch_matmul)


CALIBRATION_LEVELS = [0.25, 0.4, 0.5, 0.65, 0.9]


def run_calibration(T, torch, args) -> int:
    """Threshold calibration (Section 4.2) for one decoder block: a histogram pass over a
    sample of `tokens` hidden states for each of the block's four distinct projection inputs
    (attention input, attention output, MLP input: width d; MLP intermediate: width d_ff),
    then the thresholds for the levels of Section 5 read off each histogram."""
    import numpy as np
    shapes = ti.LAYER_SHAPES[args.workload]
    d, d_ff = shapes["q"][1], shapes["down"][1]
    tokens = args.calibration_tokens
    sites = [("attn_in", d, "gaussian"), ("attn_out", d, "laplace"),
             ("mlp_in", d, "gaussian"), ("mlp_mid", d_ff, "laplace")]
    samples, hists, ts = [], [], []
    for k, (_, width, dist) in enumerate(sites):
        # one seeded row block of 64 tokens, tiled: the kernel's work does not depend on repeats
        base = ti.make_x(64 * width, 7000 + k, dist)
        xd = torch.from_numpy(base.view(np.int16)).cuda().repeat(tokens // 64)
        samples.append(xd)
        hists.append(torch.zeros(T.TEAL_HIST_BINS, dtype=torch.int64, device="cuda"))
        ts.append(torch.zeros(len(CALIBRATION_LEVELS), dtype=torch.float32, device="cuda"))
    counts = [x.numel() for x in samples]

    def step():
        for x, h, t in zip(samples, hists, ts):
            T.check(T.teal_abs_histogram(x, x.numel(), h))
            T.check(T.teal_histogram_thresholds(h, CALIBRATION_LEVELS, t))

    def timed(fn, reps):
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record()
        for _ in range(reps):
            fn()
        stop.record()
        torch.cuda.synchronize()
        return start.elapsed_time(stop) * 1e-3 / reps

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    sec = timed(step, args.steps)
    # the histogram kernel alone, per site (the dominant kernel)
    per_site, hist_sec = {}, 0.0
    for (name, width, dist), x, h in zip(sites, samples, hists):
        s1 = timed(lambda: T.check(T.teal_abs_histogram(x, x.numel(), h)), args.steps)
        hist_sec += s1
        per_site[name] = {"values": x.numel(), "width": width, "dist": dist, "us": s1 * 1e6,
                          "GBps": 2 * x.numel() / s1 / 1e9}
    # the same kernel over growing prefixes of the widest sample: the counting phase streams at
    # the HBM rate, the per-block flush of LDS counters (global atomics) is a fixed cost
    sweep = {}
    x, h = samples[3], hists[3]
    for frac in (1 / 16, 1 / 4, 1):
        cnt = int(x.numel() * frac)
        s1 = timed(lambda: T.check(T.teal_abs_histogram(x, cnt, h)), args.steps)
        sweep[f"{2 * cnt / 1e6:.0f}MB"] = {"us": s1 * 1e6, "GBps": 2 * cnt / s1 / 1e9}
    total_bytes = 2 * sum(counts)
    achieved = total_bytes / hist_sec / 1e9
    out = {
        "metric": "threshold calibration: fp16 activation sample scanned, GB/s (histogram of "
                  "|x| + thresholds at 5 levels, 4 projection inputs of one decoder block)",
        "value": total_bytes / sec / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": sec * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u16/u64", "data": "synthetic",
        "config": {"workload": f"{args.workload} calibration sample, {tokens} tokens: 3 x "
                               f"[{tokens} x {d}] + [{tokens} x {d_ff}] fp16",
                   "levels": CALIBRATION_LEVELS},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "kernel": "abs_histogram_kernel (4 launches per step)",
                     "bytes_per_launch_avg": total_bytes / 4, "kernel_avg_us": hist_sec * 1e6 / 4},
        "per_site": per_site,
        "size_sweep_mlp_mid": sweep,
    }
    if not args.no_cpu_baseline:
        from oracle import teal_oracle as orc
        x = np.tile(ti.make_x(64 * d, 7000, "gaussian"), 64)        # 4096 tokens: ~15-20 s of sorting
        t0 = time.perf_counter()
        want = [orc.quantile_threshold(x, p) for p in CALIBRATION_LEVELS]
        cpu = time.perf_counter() - t0
        h = torch.zeros(T.TEAL_HIST_BINS, dtype=torch.int64, device="cuda")
        t = torch.zeros(len(CALIBRATION_LEVELS), dtype=torch.float32, device="cuda")
        xd = torch.from_numpy(x.view(np.int16)).cuda()
        T.check(T.teal_abs_histogram(xd, x.size, h))
        T.check(T.teal_histogram_thresholds(h, CALIBRATION_LEVELS, t))
        torch.cuda.synchronize()
        out["cpu_baseline"] = {
            "value": 2 * x.size / cpu / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"{x.size} values ({x.size // d} tokens x {d}), one sort per level, "
                      f"{cpu:.1f} s", "matches_gpu": [float(v) for v in t.cpu()] == want}
    print(json.dumps(out))
    return 0


def run_swiglu(T, torch, args) -> int:
    """The W_down step including the formation of its input h = SiLU(gate) * up
    (Appendix A.3), two ways: the element-wise producer kernel followed by the sparse
    GEMV (two launches, h written to and read back from HBM), and the fused call."""
    n, m = ti.LAYER_SHAPES[args.workload]["down"]
    cfg = ti.CONFIG_INDEX[args.workload]
    gate, up = ti.mlp_gate_up(m, ti.x_seed(cfg, 0, "down"))
    w = ti.weights_bf16(n, m, ti.weight_seed(cfg, 0, "down"))
    copies = max(2, -(-CACHE_DEFEAT_BYTES // (n * m * 2)))
    wd = torch.from_numpy(w.view(np.int16)).cuda()
    wt0 = torch.empty((m, n), dtype=torch.int16, device="cuda")
    T.check(T.teal_pack_bf16(wd, wt0, m, n))
    wts = [wt0] + [wt0.clone() for _ in range(copies - 1)]
    gd, ud = torch.from_numpy(gate).cuda(), torch.from_numpy(up).cuda()
    hd = torch.empty(m, dtype=torch.int16, device="cuda")
    y = torch.empty(n, dtype=torch.float32, device="cuda")
    ws = torch.zeros(T.teal_workspace_bytes(m, n), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    # the intermediate as the library forms it, copied back only to pick the thresholds
    T.check(T.teal_swiglu_f16(gd, ud, hd, m))
    torch.cuda.synchronize()
    h = hd.cpu().numpy().view(np.float16)
    wp = [t.data_ptr() for t in wts]
    gp, up_, hp, yp, wsp, wsb = gd.data_ptr(), ud.data_ptr(), hd.data_ptr(), y.data_ptr(), ws.data_ptr(), ws.numel()

    def two_launch(k, t):
        T.teal_swiglu_f16(gp, up_, hp, m, stream)
        T.check(T.teal_sparse_gemv_bf16(wp[k % copies], hp, t, yp, m, n, wsp, wsb, stream))

    def fused(k, t):
        T.check(T.teal_sparse_gemv_bf16_swiglu(wp[k % copies], gp, up_, t, yp, m, n, wsp, wsb, stream))

    def timed(fn, t):
        for k in range(args.warmup):
            fn(k, t)
        torch.cuda.synchronize()
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record()
        for k in range(args.steps):
            fn(k, t)
        stop.record()
        torch.cuda.synchronize()
        return start.elapsed_time(stop) * 1e-3 / args.steps

    sparsities = [float(v) for v in args.sparsities.split(",")]
    if 0.0 not in sparsities:
        sparsities.append(0.0)
    head = sparsities[0]
    detail, sec_f = {}, {}
    for p in sparsities:
        t = ti.quantile_threshold(h, p)
        nnz = int(np.count_nonzero(np.abs(h.astype(np.float32)) > np.float32(t)))
        sf, s2 = timed(fused, t), timed(two_launch, t)
        sec_f[p] = sf
        b = nnz * n * 2 + 8 * m + 4 * n              # surviving rows + gate + up (fp32) + y
        detail[pct(p)] = {"nnz": nnz, "fused_us": sf * 1e6, "two_launch_us": s2 * 1e6,
                          "saved_us": (s2 - sf) * 1e6, "effective_bytes": b,
                          "effective_GBps": b / sf / 1e9,
                          "frac_of_hbm_peak": b / sf / 1e9 / HBM_PEAK_GBS}
    for p in sparsities:
        detail[pct(p)]["speedup_vs_dense"] = sec_f[0.0] / sec_f[p]
    d = detail[pct(head)]
    out = {
        "metric": f"W_down step with its input formed in the kernel, effective HBM GB/s at "
                  f"{pct(head)} sparsity of the MLP intermediate",
        "value": d["effective_GBps"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": d["fused_us"] * 1e-3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}-shaped W_down ({n} x {m}, bf16), input "
                               f"h = fp16(SiLU(gate) * up) from fp32 gate ~ N(0,1.5^2), up ~ N(0,1); "
                               f"t at the {pct(head)} quantile of |h|",
                   "weight_copies_walked": copies},
        "roofline": {"bound": "hbm", "achieved": d["effective_GBps"], "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": d["frac_of_hbm_peak"], "traffic": None,
                     "kernel": "sparse_gemv_swiglu_kernel<FmtBF16> (1 launch per step)",
                     "bytes_per_launch_avg": d["effective_bytes"], "kernel_avg_us": d["fused_us"]},
        "detail": detail,
    }
    if not args.no_cpu_baseline:
        # the oracle on the same call, timed on the host cores; its output checks the fused one
        from oracle import teal_oracle as orc
        t = ti.quantile_threshold(h, head)
        fused(0, t)
        torch.cuda.synchronize()
        got = y.cpu().numpy().astype(np.float64)
        passes, spent, want = 0, 0.0, None
        while spent < 5.0 and passes < 200:
            t0 = time.perf_counter()
            want = orc.sparse_gemv_bf16_swiglu(w, gate, up, t)
            spent += time.perf_counter() - t0
            passes += 1
        sec = spent / passes
        out["cpu_baseline"] = {
            "value": d["effective_bytes"] / sec / 1e9, "unit": "GB/s", "cores": orc.num_threads(),
            "kind": "oracle",
            "sample": f"{passes} passes of the same call at {pct(head)} (intermediate in binary32, "
                      f"fp64 dense loop over the zeroed state), {sec * 1e3:.1f} ms per pass",
            "rel_l2_gpu_vs_oracle": float(np.linalg.norm(got - want) / np.linalg.norm(want)),
            "intermediate_bits_equal": bool(np.array_equal(orc.swiglu_f16(gate, up).view(np.uint16),
                                                           h.view(np.uint16))),
        }
    print(json.dumps(out))
    return 0


def run_rmsnorm(T, torch, args) -> int:
    """The two grouped calls that read a normalised hidden state (q+k+v and gate+up,
    Appendix A.3) including the normalisation, two ways: the normalisation kernel followed
    by the grouped sparse GEMV (two launches, x written to and read back from memory), and
    the fused call."""
    shapes = ti.LAYER_SHAPES[args.workload]
    cfg = ti.CONFIG_INDEX[args.workload]
    eps = float(np.float32(1e-5))
    stream = torch.cuda.current_stream().cuda_stream
    sparsities = [float(v) for v in args.sparsities.split(",")]
    if 0.0 not in sparsities:
        sparsities.append(0.0)
    head = sparsities[0]
    out_groups, rel_worst, bits_equal, cpu_sec, cpu_bytes, cpu_passes = {}, 0.0, True, 0.0, 0, 0
    for gname, projs in (("q+k+v", ("q", "k", "v")), ("gate+up", ("gate", "up"))):
        m = shapes[projs[0]][1]
        ns = [shapes[pj][0] for pj in projs]
        h, gamma = ti.norm_inputs(m, ti.x_seed(cfg, 0, projs[0]))
        ws_host = [ti.weights_bf16(n, m, ti.weight_seed(cfg, 0, pj)) for n, pj in zip(ns, projs)]
        group_bytes = sum(ns) * m * 2
        copies = max(2, -(-CACHE_DEFEAT_BYTES // group_bytes))
        packed = []
        for w, n in zip(ws_host, ns):
            wd = torch.from_numpy(w.view(np.int16)).cuda()
            wt0 = torch.empty((m, n), dtype=torch.int16, device="cuda")
            T.check(T.teal_pack_bf16(wd, wt0, m, n))
            packed.append([wt0] + [wt0.clone() for _ in range(copies - 1)])
        hd, gd = torch.from_numpy(h).cuda(), torch.from_numpy(gamma).cuda()
        xd = torch.empty(m, dtype=torch.int16, device="cuda")
        # the normalised state as the library forms it, copied back only to pick the thresholds
        T.check(T.teal_rmsnorm_f16(hd, gd, eps, xd, m))
        torch.cuda.synchronize()
        x = xd.cpu().numpy().view(np.float16)
        ys = [torch.empty(n, dtype=torch.float32, device="cuda") for n in ns]
        ws = torch.zeros(T.teal_workspace_bytes(m, sum(ns)), dtype=torch.uint8, device="cuda")
        wlists = [[packed[j][c] for j in range(len(ns))] for c in range(copies)]

        def two_launch(k, ts):
            T.teal_rmsnorm_f16(hd, gd, eps, xd, m, stream)
            T.check(T.teal_sparse_gemv_bf16_multi(wlists[k % copies], ts, ys, ns, xd, m, ws,
                                                  stream=stream))

        def fused(k, ts):
            T.check(T.teal_sparse_gemv_bf16_rmsnorm_multi(wlists[k % copies], ts, ys, ns, hd, gd,
                                                          eps, m, ws, stream=stream))

        def timed(fn, ts):
            for k in range(args.warmup):
                fn(k, ts)
            torch.cuda.synchronize()
            start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            start.record()
            for k in range(args.steps):
                fn(k, ts)
            stop.record()
            torch.cuda.synchronize()
            return start.elapsed_time(stop) * 1e-3 / args.steps

        detail, sec_f = {}, {}
        for p in sparsities:
            t = ti.quantile_threshold(x, p)
            ts = [t] * len(ns)
            nnz = int(np.count_nonzero(np.abs(x.astype(np.float32)) > np.float32(t)))
            sf, s2 = timed(fused, ts), timed(two_launch, ts)
            sec_f[p] = sf
            b = nnz * sum(ns) * 2 + 8 * m + 4 * sum(ns)     # surviving rows + h + gamma (fp32) + y
            detail[pct(p)] = {"nnz": nnz, "fused_us": sf * 1e6, "two_launch_us": s2 * 1e6,
                              "saved_us": (s2 - sf) * 1e6, "effective_bytes": b,
                              "effective_GBps": b / sf / 1e9,
                              "frac_of_hbm_peak": b / sf / 1e9 / HBM_PEAK_GBS}
        for p in sparsities:
            detail[pct(p)]["speedup_vs_dense"] = sec_f[0.0] / sec_f[p]
        if not args.no_cpu_baseline:
            # the oracle on the same calls, timed on the host cores; its outputs check the fused ones
            from oracle import teal_oracle as orc
            t = ti.quantile_threshold(x, head)
            fused(0, [t] * len(ns))
            torch.cuda.synchronize()
            bits_equal = bits_equal and bool(np.array_equal(
                orc.rmsnorm_f16(h, gamma, eps).view(np.uint16), x.view(np.uint16)))
            for w, y in zip(ws_host, ys):
                t0 = time.perf_counter()
                want = orc.sparse_gemv_bf16_rmsnorm(w, h, gamma, eps, t)
                cpu_sec += time.perf_counter() - t0
                rel = float(np.linalg.norm(y.cpu().numpy().astype(np.float64) - want) / np.linalg.norm(want))
                rel_worst = max(rel_worst, rel)
            cpu_bytes += detail[pct(head)]["effective_bytes"]
            cpu_passes += 1
        out_groups[gname] = {"n": ns, "m": m, "weight_copies_walked": copies, **detail}
        del packed, wlists
        torch.cuda.empty_cache()
    us = sum(g[pct(head)]["fused_us"] for g in out_groups.values())
    us2 = sum(g[pct(head)]["two_launch_us"] for g in out_groups.values())
    b = sum(g[pct(head)]["effective_bytes"] for g in out_groups.values())
    gbps = b / us / 1e3
    out = {
        "metric": f"q+k+v and gate+up steps with the normalisation of their input formed in the "
                  f"kernel, effective HBM GB/s at {pct(head)} sparsity",
        "value": gbps, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": us * 1e-3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}-shaped q+k+v and gate+up groups (bf16), input "
                               f"x = fp16(gamma * h * rsqrt(mean(h^2) + 1e-5)) from fp32 h ~ "
                               f"N(0, 2.5^2) with 1 in 512 channels x 40, gamma ~ 0.5 + 0.1 N(0,1); "
                               f"t at the {pct(head)} quantile of |x|"},
        "roofline": {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": gbps / HBM_PEAK_GBS, "traffic": None,
                     "kernel": "sparse_gemv_rmsnorm_multi_kernel<FmtBF16> (2 launches per step)",
                     "bytes_per_launch_avg": b / 2, "kernel_avg_us": us / 2},
        "two_launch_us_per_step": us2, "saved_us_per_step": us2 - us,
        "detail": out_groups,
    }
    if not args.no_cpu_baseline:
        from oracle import teal_oracle as orc
        out["cpu_baseline"] = {
            "value": cpu_bytes / cpu_sec / 1e9, "unit": "GB/s", "cores": orc.num_threads(),
            "kind": "oracle",
            "sample": f"one pass over both groups at {pct(head)} (normalised state in the stated "
                      f"arithmetic, fp64 dense loop over the zeroed state), {cpu_sec * 1e3:.1f} ms",
            "rel_l2_gpu_vs_oracle_worst": rel_worst,
            "normalised_state_bits_equal": bits_equal,
        }
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="llama2_7b", choices=sorted(ti.LAYER_SHAPES))
    ap.add_argument("--format", default="bf16", choices=sorted(BITS))
    ap.add_argument("--sparsities", default="0.5,0.4,0",
                    help="comma-separated; the first is the headline, 0 (dense) is always included")
    ap.add_argument("--layers", type=int, default=1, help="blocks per step (a stack when > 1)")
    ap.add_argument("--copies", type=int, default=0, help="weight copies to walk (0 = auto)")
    ap.add_argument("--fused", action="store_true",
                    help="(default for bf16 at batch 1) one launch per group of projections that "
                         "read the same hidden state: q+k+v, o, gate+up, down")
    ap.add_argument("--unfused", action="store_true",
                    help="one launch per projection (7 per block) as the headline")
    ap.add_argument("--stack-launch", action="store_true",
                    help="headline = the groups of the pass as independent work in one launch per "
                         "16 groups (teal_sparse_gemv_bf16_stack): a bare stack of projections, "
                         "not a decoder's dependent sequence")
    ap.add_argument("--batch", type=int, default=0,
                    help="B >= 1: a small batch of B hidden states per projection with the batch-wide "
                         "mask of the averaged magnitude (Section 5.4.4); bf16 only. 0 = one state")
    ap.add_argument("--graph", action="store_true",
                    help="also time the headline pass replayed from a captured HIP graph")
    ap.add_argument("--rmsnorm", action="store_true",
                    help="time the q+k+v and gate+up steps with the normalisation of their input "
                         "formed in the kernel against the two-launch path (Appendix A.3)")
    ap.add_argument("--swiglu", action="store_true",
                    help="time the W_down step with its input formed from gate and up in the kernel "
                         "against the two-launch path (Appendix A.3)")
    ap.add_argument("--calibration", action="store_true",
                    help="time threshold calibration (histogram + thresholds) instead of the GEMV path")
    ap.add_argument("--calibration-tokens", type=int, default=16384)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--rows", default="packed", choices=("packed", "padded"),
                    help="padded: W_q, W_k, W_v, W_gate, W_up stored with rows 256 bytes further apart "
                         "(bf16 / int8, batch 1; the stack launch needs packed rows and is skipped)")
    ap.add_argument("--no-per-projection", action="store_true")
    ap.add_argument("--no-other-mode", action="store_true",
                    help="skip timing the pass in the launch mode that is not the headline")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench_extras.py: this build runs on ONE GPU only; --gpus must be 1", file=sys.stderr)
        return 2

    clocks = gpu_clocks()
    import torch
    import paper_2408_14690_amd as T
    if not torch.cuda.is_available():
        print("bench_extras.py: no GPU visible", file=sys.stderr)
        return 2
    if not os.path.exists(T.library_path()):
        from paper_2408_14690_amd import build
        build.build(verbose=False)
    T.load_library()
    if args.swiglu:
        return run_swiglu(T, torch, args)
    if args.rmsnorm:
        return run_rmsnorm(T, torch, args)
    if args.calibration:
        if args.calibration_tokens % 64 or args.calibration_tokens <= 0:
            print("bench_extras.py: --calibration-tokens must be a positive multiple of 64", file=sys.stderr)
            return 2
        return run_calibration(T, torch, args)

    sparsities = [float(s) for s in args.sparsities.split(",")]
    if 0.0 not in sparsities:
        sparsities.append(0.0)
    head = sparsities[0]
    fmt = args.format
    fused = not args.unfused
    shapes = ti.LAYER_SHAPES[args.workload]
    block_bytes = sum(n * m * BITS[fmt] // 8 for n, m in shapes.values())
    if args.layers > 1:
        copies = args.copies or 1
    else:
        copies = args.copies or max(2, -(-CACHE_DEFEAT_BYTES // block_bytes))
    if args.batch and (fmt != "bf16" or not 1 <= args.batch <= T.TEAL_MAX_BATCH):
        print("bench_extras.py: --batch needs bf16 and 1 <= B <= 8", file=sys.stderr)
        return 2
    row_pad = {}
    if args.rows == "padded":
        if args.batch or fmt == "w4" or args.stack_launch:
            print("bench_extras.py: --rows padded needs bf16 or int8, batch 1, no --stack-launch",
                  file=sys.stderr)
            return 2
        row_pad = {name: 256 * 8 // BITS[fmt] for name in ("q", "k", "v", "gate", "up")}
    projections = build_stack(T, torch, args.workload, fmt, sparsities, args.layers, copies,
                              args.batch, row_pad=row_pad)
    block0 = projections[:7]
    groups = fuse(T, torch, projections)
    stack_calls = None
    if not args.batch and not row_pad and (args.stack_launch or not args.no_other_mode):
        stack_calls = [StackCall(T, torch, groups[i:i + 16]) for i in range(0, len(groups), 16)]
    if args.stack_launch:
        if stack_calls is None or args.unfused:
            print("bench_extras.py: --stack-launch needs batch 1 and grouped launches", file=sys.stderr)
            return 2
        stack = stack_calls
    else:
        stack = groups if fused else projections
    launches_per_step = len(stack)

    def timed_passes(calls):
        sec = {p: time_steps(T, torch, calls, p, args.steps, args.warmup) for p in sparsities}
        out = {}
        for p in sparsities:
            eff = sum(C.bytes(p) for C in calls)
            out[pct(p)] = {
                "us_per_step": sec[p] * 1e6, "launches_per_step": len(calls),
                "effective_bytes": eff,
                "effective_GBps": eff / sec[p] / 1e9,
                "frac_of_hbm_peak": eff / sec[p] / 1e9 / HBM_PEAK_GBS,
                "speedup_vs_dense": sec[0.0] / sec[p],
            }
        return sec, out

    seconds, detail = timed_passes(stack)
    detail[pct(head)]["host_issue_us_per_step"] = time_steps.host_issue_us

    # Dominant kernel: the sparse GEMV kernel, the only kernel of a call.  Its average launch
    # duration is the timed region of the headline pass divided by the launches in it.
    head_bytes = sum(C.bytes(head) for C in stack)
    achieved = head_bytes / seconds[head] / 1e9

    # The same pass launched the other way: one launch per projection when the headline
    # groups the projections that share their input (q+k+v, o, gate+up, down: Appendix A.3,
    # teal_sparse_gemv_bf16_multi), or the grouped launches when the headline does not.
    other_detail = {}
    if groups is not None and not args.no_other_mode:
        _, other_detail = timed_passes(projections if fused and not args.stack_launch else groups)

    # The whole pass as a bare stack: the groups do not depend on each other here (every group
    # has its own synthetic input), so up to 16 of them go out as one launch and the ends of
    # one group's work lie under the next group's row stream.  Reported beside the headline,
    # never as it: inside a decoder the groups depend on each other and are separate launches.
    stack_detail = {}
    if stack_calls is not None and not args.no_other_mode and not args.stack_launch:
        _, stack_detail = timed_passes(stack_calls)
        one_step(T, stack_calls, head, 0)
        torch.cuda.synchronize()
        checks = [C.survivors_match(T, torch, head) for C in stack_calls]
        # the outputs of that launch against those of the grouped launches of the same inputs
        ys_stack = [P.y.clone() for P in block0]
        one_step(T, groups[:4], head, 0)
        torch.cuda.synchronize()
        stack_detail["block0_outputs_bitwise_equal_grouped_launches"] = all(
            bool(torch.equal(a.view(torch.int32), P.y.view(torch.int32)))
            for a, P in zip(ys_stack, block0))
        stack_detail["survivor_counts_equal_host_counts"] = all(ok for ok, _ in checks)
        stack_detail["matrices_checked"] = sum(c for _, c in checks)

    def alone(calls):
        table = {}
        for C in calls:
            us = time_projection(T, torch, C, head, 300) * 1e6
            us_dense = time_projection(T, torch, C, 0.0, 300) * 1e6
            b = C.bytes(head)
            table[C.name] = {
                "n": C.ns if hasattr(C, "ns") else C.n, "m": C.m, "us": us, "us_dense": us_dense,
                "effective_GBps": b / us / 1e3, "frac_of_hbm_peak": b / us / 1e3 / HBM_PEAK_GBS,
                "speedup_vs_dense": us_dense / us,
            }
            table[C.name].update(time_projection_spread(T, torch, C, head))
        return table

    graph_detail = {}
    if args.graph:
        for p in (head, 0.0):
            gsec = time_steps_graph(T, torch, stack, p, args.steps, copies)
            graph_detail[pct(p)] = {"us_per_step": gsec * 1e6,
                                    "vs_direct_launches": seconds[p] / gsec}
        graph_detail[pct(head)]["speedup_vs_dense"] = (graph_detail[pct(0.0)]["us_per_step"]
                                                       / graph_detail[pct(head)]["us_per_step"])

    per_proj, per_group = {}, {}
    if not args.no_per_projection:
        per_proj = alone(block0)
        for P in block0:
            if args.batch:
                per_proj[P.name]["launch"] = "chosen inside teal_sparse_gemv_bf16_batch"
            else:
                per_proj[P.name]["launch"] = T.teal_gemv_plan(BITS[fmt], P.m, P.n)[1]
            per_proj[P.name]["nnz"] = P.nnz[head]
            if fmt == "bf16" and not args.batch:
                # context only: a failure of the vendor path must not cost the run its result
                try:
                    per_proj[P.name]["us_dense_torch_matmul_same_layout"] = \
                        time_torch_matmul(torch, P, False) * 1e6
                    if args.layers == 1:
                        per_proj[P.name]["us_dense_torch_matmul_canonical_layout"] = \
                            time_torch_matmul(torch, P, True) * 1e6
                except RuntimeError as e:
                    per_proj[P.name]["us_dense_torch_matmul_error"] = str(e)[:200]
        if groups is not None:
            per_group = alone(groups[:4])

    # Each projection as one of 16 independent products of its own shape in one launch: its
    # time when the serial ends of a call lie under other products' row streams.
    per_proj_stack = {}
    if stack_calls is not None and not args.no_per_projection:
        for P in block0:
            if len(P.wp) < 2:
                continue
            call = StackCall(T, torch, [Replica(torch, P, j) for j in range(16)])
            us = time_projection(T, torch, call, head, 100) * 1e6 / 16
            us_dense = time_projection(T, torch, call, 0.0, 100) * 1e6 / 16
            b = P.bytes(head)
            per_proj_stack[P.name] = {
                "n": P.n, "m": P.m, "us_per_projection": us, "us_per_projection_dense": us_dense,
                "effective_GBps": b / us / 1e3, "frac_of_hbm_peak": b / us / 1e3 / HBM_PEAK_GBS,
                "speedup_vs_dense": us_dense / us,
                # bytes read before a weight copy comes round again; the last-level cache holds 256 MB
                "weight_bytes_walked": len(P.wp) * P.nnz[head] * P.n * BITS[fmt] // 8,
            }
            del call

    multi_kernel = {"bf16": "sparse_gemv_multi_kernel<FmtBF16>", "w8": "sparse_gemv_multi_kernel<FmtW8>",
                    "w4": "sparse_gemv_w4_multi_kernel"}[fmt]
    if args.batch:
        kernel = "sparse_gemv_batch_multi_kernel" if fused else "sparse_gemv_batch_kernel"
    else:
        kernel = multi_kernel if fused else KERNEL[fmt]
    if args.stack_launch:
        kernel = {"bf16": "sparse_gemv_stack_kernel<FmtBF16>", "w8": "sparse_gemv_stack_kernel<FmtW8>",
                  "w4": "sparse_gemv_w4_stack_kernel"}[fmt]
    out = {
        "metric": f"sparse GEMV effective HBM GB/s at {pct(head)} sparsity (one decoder-block "
                  f"pass); us and speedup vs dense per sparsity in detail",
        "value": detail[pct(head)]["effective_GBps"],
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": seconds[head] * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": f"{args.workload}-shaped decoder block x {args.layers}, 7 projections "
                        f"each, batch {max(args.batch, 1)}, {fmt} W from N(0,0.02^2), fp16 x (Gaussian / "
                        f"Laplace by role), t at the {pct(head)} quantile of "
                        f"{'the batch-averaged |x|' if args.batch else '|x|'} per projection",
            "weight_format": fmt,
            "weight_rows": args.rows,
            "weight_bytes_per_block": block_bytes,
            "blocks_per_step": args.layers,
            "launches": "one per 16 groups (q+k+v, o, gate+up, down of 4 blocks), the groups taken "
                        "as independent work: a bare stack of projections, not a decoder's "
                        "dependent sequence" if args.stack_launch else
                        "one per group of projections that read the same hidden state (q+k+v, o, "
                        "gate+up, down), each projection with its own threshold" if fused
                        else "one per projection",
            "weight_copies_walked": copies,
        },
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": measured_traffic(args.workload, fmt, head, args.layers,
                                        "stack" if args.stack_launch else "grouped" if fused
                                        else "per_projection", T.teal_version())[0],
            "kernel": f"{kernel} ({launches_per_step} launches per step, {pct(head)})",
            "bytes_per_launch_avg": head_bytes / launches_per_step,
            "kernel_avg_us": seconds[head] * 1e6 / launches_per_step,
        },
        "detail": detail,
        ("detail_one_launch_per_projection" if fused and not args.stack_launch
         else "detail_grouped_launches"): other_detail,
        "detail_independent_groups_in_one_launch": stack_detail,
        "detail_hip_graph_replay": graph_detail,
        f"per_projection_alone_{pct(head)}": per_proj,
        f"per_group_alone_{pct(head)}": per_group,
        f"per_projection_in_a_launch_of_16_independent_{pct(head)}": per_proj_stack,
    }
    if not args.no_other_mode:
        # the practical ceiling beside the published peak: a plain read of one launch's bytes
        # (back to back, like the timed launches) and of 1 GiB
        per_launch = int(head_bytes / launches_per_step)
        ceil = read_ceiling(T, torch, [per_launch, 1 << 30])
        out["roofline"]["plain_read_of_the_same_bytes"] = ceil[0]
        out["roofline"]["plain_read_of_1GiB"] = ceil[1]
        out["roofline"]["achieved_over_plain_read_of_the_same_bytes"] = achieved / ceil[0]["GBps"]
    # the same reading while the headline pass keeps the GPU busy (about a second of steps)
    import threading
    busy = {}
    th = threading.Thread(target=lambda: busy.update(clocks=gpu_clocks()))
    th.start()
    k = 0
    while th.is_alive():
        for _ in range(max(1, 200 // args.layers)):
            one_step(T, stack, head, k)
            k += 1
        torch.cuda.synchronize()
    th.join()
    out["gpu_clocks"] = {"idle_before_the_run": clocks, "under_the_headline_pass": busy.get("clocks")}
    ok, compared = survivor_counts_match(T, torch, stack, head)
    out["parity_in_this_run"] = {"survivor_counts_equal_host_counts": ok, "matrices": compared}
    if not args.no_cpu_baseline:
        sec, passes, threads, want = cpu_baseline(block0, head)
        # the pass above left block 0's outputs of the timed launch configuration on the device
        worst = 0.0
        for P, w in zip(block0, want):
            got = P.y.cpu().numpy().astype(np.float64).reshape(np.shape(w))
            worst = max(worst, float(np.linalg.norm(got - w) / np.linalg.norm(w)))
        out["parity_in_this_run"]["block0_rel_l2_vs_oracle_worst"] = worst
        block_head_bytes = sum(P.bytes(head) for P in block0)
        out["cpu_baseline"] = {
            "value": block_head_bytes / sec / 1e9,
            "unit": "GB/s",
            "cores": threads,
            "kind": "oracle",
            "sample": f"{passes} whole passes over block 0 at {pct(head)} (fp64 dense loop over "
                      f"the zeroed x), {sec * 1e3:.1f} ms per pass",
            "ms_per_step": sec * 1e3 * args.layers,
            "one_core_ms_per_pass": cpu_baseline_one_core(block0, head) * 1e3,
        }
        if args.layers > 2 and fmt == "bf16" and not args.batch:
            deep = sorted({(args.layers - 1) // 2, args.layers - 1})
            worst, checked = deep_layer_check(T, torch, projections, deep, head)
            out["parity_in_this_run"]["deep_blocks_all_outputs"] = {
                "blocks": deep, "outputs_checked": checked, "rel_l2_vs_oracle_worst": worst}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
