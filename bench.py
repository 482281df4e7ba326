#!/usr/bin/env python3
"""Benchmark of the TEAL decode hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama2_7b]

A step is one pass of the whole hot path over one synthetic decoder block at
batch 1: for each of the seven projections, threshold the hidden state, compact
the survivors and stream only the surviving weight rows (one C-ABI call per
projection).  The headline value is the effective HBM bandwidth of that pass at
50% sparsity (algorithmic bytes / time); the same pass at 40% and at 0% (t = 0,
the same kernels run dense) gives the speed-up over dense.  Weights, states and
the workspace are resident in HBM before the timed region.  Consecutive steps
walk over several copies of the weights so that no step finds its rows in the
256 MB last-level cache.

Prints ONE JSON line.  More than one GPU is not supported.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

import teal_inputs as ti

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
CACHE_DEFEAT_BYTES = 3 << 30    # distinct weight bytes walked before a copy is reused
SPARSITIES = (0.5, 0.4, 0.0)    # headline first
# HBM bytes per launch of sparse_gemv_kernel at 50% (average over the 7 launches of a step),
# from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script, scaled by the factors a
# plain copy of known size gives on the same box (2.0 and 1.0):
# profiles/sparse_gemv_kernel_llama2_7b_hbm_traffic.txt.
MEASURED_TRAFFIC_BYTES = {"llama2_7b": (200310.07 + 1555.31) * 1024 / 7}


def algorithmic_bytes(nnz: int, m: int, n: int) -> int:
    """Bytes the method must move for one projection: surviving bf16 rows + x + y."""
    return nnz * n * 2 + 2 * m + 4 * n


def build_layer(T, torch, model: str, copies: int):
    """Seeded block on the host -> device, laid out input-channel-major by the library."""
    layer = []
    for proj, n, m, w, x in ti.layer_inputs(model):
        wd = torch.from_numpy(w.view(np.int16)).cuda()
        wts = []
        for c in range(copies):
            wt = torch.empty((m, n), dtype=torch.int16, device="cuda")
            if c == 0:
                T.check(T.teal_pack_bf16(wd, wt, m, n))
            else:
                wt.copy_(wts[0])
            wts.append(wt)
        del wd
        thresholds, nnz = {}, {}
        for p in SPARSITIES:
            t = ti.quantile_threshold(x, p)
            thresholds[p] = t
            nnz[p] = int(np.count_nonzero(np.abs(x.astype(np.float32)) > np.float32(t)))
        layer.append(dict(
            proj=proj, n=n, m=m, w_host=w, x_host=x, wt=wts,
            x=torch.from_numpy(x.view(np.int16)).cuda(),
            y=torch.empty(n, dtype=torch.float32, device="cuda"),
            ws=torch.zeros(T.teal_workspace_bytes(m, n), dtype=torch.uint8, device="cuda"),
            t=thresholds, nnz=nnz))
    torch.cuda.synchronize()
    return layer


def one_step(T, layer, p: float, copy: int) -> None:
    for L in layer:
        st = T.teal_sparse_gemv_bf16(L["wt"][copy], L["x"], L["t"][p], L["y"], L["m"], L["n"],
                                     L["ws"])
        if st != 0:
            T.check(st)


def time_steps(T, torch, layer, p: float, steps: int, warmup: int, copies: int) -> float:
    """Seconds for `steps` back-to-back passes (HIP events on the launch stream)."""
    for k in range(warmup):
        one_step(T, layer, p, k % copies)
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for k in range(steps):
        one_step(T, layer, p, k % copies)
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) * 1e-3


def time_projection(T, torch, L, p: float, launches: int, copies: int) -> float:
    """Seconds per call for one projection launched back to back (one kernel per call),
    walking the weight copies; HIP events on the launch stream around the whole batch."""
    def run(k):
        st = T.teal_sparse_gemv_bf16(L["wt"][k % copies], L["x"], L["t"][p], L["y"], L["m"],
                                     L["n"], L["ws"])
        if st != 0:
            T.check(st)
    for k in range(20):
        run(k)
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for k in range(launches):
        run(k)
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) * 1e-3 / launches


def cpu_baseline(layer, p: float, budget_s: float = 12.0):
    """The fp64 oracle, as it stands, on the host cores: whole passes over the
    same block until about `budget_s` seconds of CPU work have been spent."""
    from oracle import teal_oracle as orc
    threads = orc.num_threads()
    for L in layer[:1]:
        orc.sparse_gemv_bf16(L["w_host"], L["x_host"], L["t"][p])      # warm-up
    passes, spent = 0, 0.0
    while spent < budget_s and passes < 1000:
        t0 = time.perf_counter()
        for L in layer:
            orc.sparse_gemv_bf16(L["w_host"], L["x_host"], L["t"][p])
        spent += time.perf_counter() - t0
        passes += 1
    return spent / passes, passes, threads


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="llama2_7b", choices=sorted(ti.LAYER_SHAPES))
    ap.add_argument("--copies", type=int, default=0, help="weight copies to walk (0 = auto)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only; --gpus must be 1", file=sys.stderr)
        return 2

    import torch
    import paper_2408_14690_amd as T
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    if not os.path.exists(T.library_path()):
        from paper_2408_14690_amd import build
        build.build(verbose=False)
    T.load_library()

    shapes = ti.LAYER_SHAPES[args.workload]
    dense_bytes = sum(n * m * 2 for n, m in shapes.values())
    copies = args.copies or max(2, -(-CACHE_DEFEAT_BYTES // dense_bytes))
    layer = build_layer(T, torch, args.workload, copies)

    detail, seconds = {}, {}
    for p in SPARSITIES:
        sec = time_steps(T, torch, layer, p, args.steps, args.warmup, copies)
        seconds[p] = sec / args.steps
        eff = sum(algorithmic_bytes(L["nnz"][p], L["m"], L["n"]) for L in layer)
        detail[f"{int(round(p * 100))}%"] = {
            "us_per_step": seconds[p] * 1e6,
            "effective_bytes": eff,
            "effective_GBps": eff / seconds[p] / 1e9,
            "frac_of_hbm_peak": eff / seconds[p] / 1e9 / HBM_PEAK_GBS,
        }
    for p in SPARSITIES:
        detail[f"{int(round(p * 100))}%"]["speedup_vs_dense"] = seconds[0.0] / seconds[p]

    # Dominant kernel: sparse_gemv_kernel, the only kernel of a call (one launch per
    # projection).  Its average launch duration is the timed region of the 50% pass
    # divided by the launches in it; the algorithmic bytes are those of the 7 calls.
    calls_bytes = sum(algorithmic_bytes(L["nnz"][0.5], L["m"], L["n"]) for L in layer)
    launches_per_step = len(layer)
    kernel_avg_us = seconds[0.5] * 1e6 / launches_per_step
    achieved = calls_bytes / seconds[0.5] / 1e9
    per_proj = {}
    for L in layer:
        b = algorithmic_bytes(L["nnz"][0.5], L["m"], L["n"])
        us = time_projection(T, torch, L, 0.5, 300, copies) * 1e6
        us_dense = time_projection(T, torch, L, 0.0, 300, copies) * 1e6
        _, plan = T.teal_gemv_plan(16, L["m"], L["n"])
        per_proj[L["proj"]] = {
            "n": L["n"], "m": L["m"], "nnz": L["nnz"][0.5], "us": us, "us_dense": us_dense,
            "effective_GBps": b / us / 1e3, "frac_of_hbm_peak": b / us / 1e3 / HBM_PEAK_GBS,
            "speedup_vs_dense": us_dense / us, "launch": plan,
        }

    out = {
        "metric": "sparse GEMV effective HBM GB/s at 50% sparsity (one decoder-block pass); "
                  "us and speedup vs dense at 0/40/50% in detail",
        "value": detail["50%"]["effective_GBps"],
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": seconds[0.5] * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": f"{args.workload}-shaped decoder block, 7 projections, batch 1, bf16 W "
                        f"(N(0,0.02^2)), fp16 x (Gaussian / Laplace by role), t at the 50% "
                        f"quantile of |x| per projection",
            "dense_weight_bytes": dense_bytes,
            "weight_copies_walked": copies,
        },
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": MEASURED_TRAFFIC_BYTES.get(args.workload),
            "kernel": "sparse_gemv_kernel (one launch per projection; 7 launches per step, 50%)",
            "bytes_per_launch_avg": calls_bytes / launches_per_step,
            "kernel_avg_us": kernel_avg_us,
        },
        "detail": detail,
        "per_projection_50%": per_proj,
    }
    if not args.no_cpu_baseline:
        sec, passes, threads = cpu_baseline(layer, 0.5)
        out["cpu_baseline"] = {
            "value": calls_bytes / sec / 1e9,
            "unit": "GB/s",
            "cores": threads,
            "kind": "oracle",
            "sample": f"{passes} whole passes over the same block at 50% (fp64 dense loop over "
                      f"the zeroed x), {sec * 1e3:.1f} ms per pass",
            "ms_per_step": sec * 1e3,
        }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
