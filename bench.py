#!/usr/bin/env python3
"""Benchmark of the TEAL decode hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--repeats R]
                    [--workload llama_70b|llama3_8b|llama2_7b] [--layers L]
                    [--format bf16|w8|w4] [--sparsities 0.5,0]
                    [--unfused | --stack-launch] [--rows padded|packed] [--no-detail]
                    [--no-cpu-baseline]

A step is one pass of the whole hot path over a synthetic stack of decoder blocks at batch
1: for each of the seven projections of every block, threshold the hidden state, compact the
survivors and stream only the surviving weight rows.  The default workload is the largest
single-GPU configuration: an 80-block Llama-70B-shaped stack, 137 GB of bf16 weights resident
in HBM, one fresh seeded input per projection, thresholds at the 50 % quantile.  The
projections that read the same hidden state -- q+k+v, o, gate+up, down, each projection with
its own threshold -- go out as one C-ABI call = one kernel launch per group, the way a
decoder would issue them (320 launches per step); --unfused launches every projection on its
own, --stack-launch issues 16 groups per launch as independent work (a bare stack, not a
decoder's dependent sequence).  The headline value is the effective HBM bandwidth of that
pass at the first listed sparsity: algorithmic bytes / time, the time being the median over
R repetitions of a region of exactly K back-to-back steps.  The same pass at t = 0 (the same
kernels run dense) gives the speed-up over dense.  The matrices of the grouped launches (q,
k, v, gate, up) are stored with rows 256 bytes further apart (the library's own layout step,
teal_pack_bf16_pitch; --rows packed for packed rows): a narrow tile then meets every quarter
of the address space over its rows and the gate + up pair runs without split-K.

Beside the headline, `llama3_8b_block` carries the 4096 x 14336-class figures: every
projection and every group of a Llama-3-8B-shaped block timed alone (packed and padded rows),
the block pass, and the MLP on its own data flow in one, two and three launches; it is timed
before the stack is laid out.  Side measurements (calibration,
producer fusion, small batches, graph replay, the sparsity sweep) live in bench_extras.py.

Prints ONE JSON line.  More than one GPU is not supported.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import threading
import time

import numpy as np

import teal_inputs as ti
from bench_lib import (BITS, CACHE_DEFEAT_BYTES, HBM_PEAK_GBS, FusedGroup, MlpCall, Projection,  # noqa: F401
                       StackCall,
                       algorithmic_bytes, build_stack, cpu_baseline, cpu_baseline_one_core,
                       deep_layer_check, fuse, gpu_clocks, measured_traffic, one_step, pct,
                       read_ceiling, survivor_counts_match, time_projection)

DEFAULT_LAYERS = {"llama_70b": 80, "llama3_8b": 1, "llama2_7b": 1}


def time_region(T, torch, calls, p, steps: int, first_copy: int) -> float:
    """THE timed region: exactly `steps` back-to-back passes over `calls` at sparsity p, between
    two HIP events on the launch stream, with a device synchronisation on both sides.  Seconds."""
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for k in range(steps):
        one_step(T, calls, p, first_copy + k)
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) * 1e-3


def time_pass(T, torch, calls, p, steps: int, warmup: int, repeats: int):
    """`warmup` untimed passes, then `repeats` timed regions of `steps` passes each.  Returns the
    seconds per step of every region, in the order taken."""
    for k in range(warmup):
        one_step(T, calls, p, k)
    return [time_region(T, torch, calls, p, steps, warmup + r * steps) / steps for r in range(repeats)]


def median(v):
    s = sorted(v)
    return s[len(s) // 2] if len(s) % 2 else 0.5 * (s[len(s) // 2 - 1] + s[len(s) // 2])


def pass_figures(calls, p, per_step, dense_per_step=None):
    eff = sum(C.bytes(p) for C in calls)
    sec = median(per_step)
    out = {"us_per_step": sec * 1e6, "us_per_step_min": min(per_step) * 1e6,
           "us_per_step_max": max(per_step) * 1e6, "regions": len(per_step),
           "launches_per_step": len(calls), "effective_bytes": eff,
           "effective_GBps": eff / sec / 1e9, "frac_of_hbm_peak": eff / sec / 1e9 / HBM_PEAK_GBS}
    if dense_per_step is not None:
        out["speedup_vs_dense"] = median(dense_per_step) / sec
    return out


def call_us(T, torch, C, p, launches=200, regions=5):
    """Microseconds per call of one call launched back to back: the median over `regions`
    timed regions of `launches` launches each (the first region after a change of call or
    sparsity was measured 1-3 % slower than the following ones: clocks and first touches)."""
    return median([time_projection(T, torch, C, p, launches) for _ in range(regions)]) * 1e6


def alone(T, torch, C, p_head):
    """One call launched back to back on its own at the headline sparsity and dense, walking
    enough weight copies that no launch finds its rows in the last-level cache."""
    members = getattr(C, "members", [C])
    for P in members:
        P.ensure_walk(p_head)
    C.prepared = {}
    us = call_us(T, torch, C, p_head)
    us_dense = call_us(T, torch, C, 0.0)
    b = C.bytes(p_head)
    return {"n": [P.n for P in members] if len(members) > 1 else members[0].n, "m": C.m,
            "us": us, "us_dense": us_dense, "effective_bytes": b,
            "effective_GBps": b / us / 1e3, "frac_of_hbm_peak": b / us / 1e3 / HBM_PEAK_GBS,
            "speedup_vs_dense": us_dense / us,
            "weight_bytes_walked": min(P.walked_bytes(p_head) for P in members)}


def padded_rows_detail(T, torch, by_name, groups, fmt, sparsities, p_head, packed_per_step):
    """The matrices of the grouped launches (W_q, W_k, W_v; W_gate, W_up) stored with rows 256
    bytes further apart (the library's _pitch entry points; the same weights and inputs): each
    group in one launch, one gate alone, and the block pass with the two launches replaced.
    With such rows the gate + up pair runs in tiles of 256 bytes of a row without split-K."""
    pad = 256 * 8 // BITS[fmt]
    wide = {name: Projection(T, torch, name, by_name[name].n, by_name[name].m, fmt, by_name[name].x_host,
                             sparsities, len(by_name[name].weights), w_host=by_name[name].w_host,
                             row_pad=pad) for name in ("q", "k", "v", "gate", "up")}
    new_groups = {"q+k+v": FusedGroup(T, torch, [wide["q"], wide["k"], wide["v"]]),
                  "gate+up": FusedGroup(T, torch, [wide["gate"], wide["up"]])}
    out = {"row_pad_elements": pad}
    # same sums as the packed calls, possibly in another order: compared by value
    worst = 0.0
    for name, group in new_groups.items():
        packed = next(g for g in groups if g.name == name)
        T.check(packed.enqueue(T, 0, p_head))
        T.check(group.enqueue(T, 0, p_head))
        torch.cuda.synchronize()
        for a, b in zip(packed.members, group.members):
            ya, yb = a.y.double(), b.y.double()
            worst = max(worst, float((ya - yb).norm() / ya.norm()))
    out["rel_l2_vs_packed_rows"] = worst
    for name, group in new_groups.items():
        out[name] = alone(T, torch, group, p_head)
        out[name]["launch"] = T.teal_gemv_plan_multi_pitch(BITS[fmt], group.m, group.ns,
                                                           [P.pitch for P in group.members])[1]
    out["gate"] = alone(T, torch, wide["gate"], p_head)
    out["gate"]["launch"] = T.teal_gemv_plan_multi_pitch(BITS[fmt], wide["gate"].m, [wide["gate"].n],
                                                         [wide["gate"].pitch])[1]
    swapped = [new_groups.get(g.name, g) for g in groups]
    per_step = time_pass(T, torch, swapped, p_head, 200, 50, 5)
    dense = time_pass(T, torch, swapped, 0.0, 200, 50, 5)
    out["block_pass_one_launch_per_group"] = pass_figures(swapped, p_head, per_step, dense)
    return out


def llama3_8b_block_detail(T, torch, fmt: str, p_head: float):
    """The 4096 x 14336-class shapes (both orientations) in a driver-run record: a
    Llama-3-8B-shaped block, bf16 unless another format was asked for, 50 % and dense."""
    sparsities = [p_head, 0.0]
    shapes = ti.LAYER_SHAPES["llama3_8b"]
    block_bytes = sum(n * m * BITS[fmt] // 8 for n, m in shapes.values())
    copies = max(2, -(-CACHE_DEFEAT_BYTES // block_bytes))
    block = build_stack(T, torch, "llama3_8b", fmt, sparsities, 1, copies)
    groups = fuse(T, torch, block)
    out = {"weight_format": fmt, "weight_copies_walked": copies}
    per_step = {p: time_pass(T, torch, groups, p, 200, 50, 5) for p in sparsities}
    out["block_pass_one_launch_per_group"] = pass_figures(groups, p_head, per_step[p_head], per_step[0.0])
    by_name = {P.name: P for P in block}
    mlp = MlpCall(T, torch, by_name["gate"], by_name["up"], by_name["down"], sparsities)
    mlp_out = {"note": "gate and up read x, W_down reads h = SiLU(gate) * up formed from their "
                       "outputs (Appendix A.3): the dependent sequence a decoder runs",
               "effective_bytes": mlp.bytes(p_head)}
    modes = ("one_launch", "two_launches", "three_launches") + \
        (("one_launch_padded_rows",) if fmt in ("bf16", "w8") else ())
    for mode in modes:
        mlp.mode = mode
        us = call_us(T, torch, mlp, p_head)
        us_dense = call_us(T, torch, mlp, 0.0)
        b = mlp.bytes(p_head)
        mlp_out[mode] = {"us": us, "us_dense": us_dense, "effective_GBps": b / us / 1e3,
                         "frac_of_hbm_peak": b / us / 1e3 / HBM_PEAK_GBS,
                         "speedup_vs_dense": us_dense / us}
    if fmt in ("bf16", "w8"):
        st, sh = T.teal_mlp_plan(BITS[fmt], mlp.m, mlp.f, mlp.d)
        mlp_out["one_launch"]["shape"] = sh.as_dict()
        mlp_out["one_launch_padded_rows"]["shape"] = mlp.padded_shape.as_dict()
        mlp_out["one_launch_padded_rows"]["note"] = (
            "the same matrices stored with rows 256 bytes further apart, in the shape teal_mlp_plan "
            "gives for those pitches: every block's reads then spread evenly over the memory channels")
        # the padded layout must not change a bit of the result where the shape stays the same;
        # another shape adds the same terms in another order
        outs = {}
        for mode in ("one_launch", "one_launch_padded_rows"):
            mlp.mode = mode
            T.check(mlp._enqueue(T, 0, p_head))
            torch.cuda.synchronize()
            outs[mode] = (mlp.g.clone(), mlp.u.clone(), mlp.y.clone())
        mlp_out["one_launch_padded_rows"]["bitwise_equal_to_one_launch"] = all(
            torch.equal(a.view(torch.int32), b.view(torch.int32))
            for a, b in zip(outs["one_launch"], outs["one_launch_padded_rows"]))
        mlp_out["one_launch_padded_rows"]["rel_l2_vs_one_launch"] = max(
            float(((a.double() - b.double()).norm() / b.double().norm()).item())
            for a, b in zip(outs["one_launch_padded_rows"], outs["one_launch"]))
    mlp.mode = "one_launch"
    one_step(T, [mlp], p_head, 0)
    torch.cuda.synchronize()
    off = T.teal_mlp_status_offset(mlp.m, mlp.f, mlp.d)
    mlp_out["status_word_after_the_run"] = int(mlp.ws[off:off + 4].view(torch.int32).item())
    out["mlp"] = mlp_out
    out["per_group_alone"] = {G.name: alone(T, torch, G, p_head) for G in groups}
    out["per_projection_alone"] = {}
    for P in block:
        if P.name in ("k", "up"):                  # same shape as v / gate
            continue
        out["per_projection_alone"][P.name] = alone(T, torch, P, p_head)
        out["per_projection_alone"][P.name]["launch"] = T.teal_gemv_plan(BITS[fmt], P.m, P.n)[1]
    if fmt in ("bf16", "w8"):
        out["padded_rows"] = padded_rows_detail(T, torch, by_name, groups, fmt, sparsities, p_head,
                                                per_step)
    del mlp, groups, block
    torch.cuda.empty_cache()
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--repeats", type=int, default=10,
                    help="timed regions of --steps steps each; the headline is their median")
    ap.add_argument("--workload", default="llama_70b", choices=sorted(ti.LAYER_SHAPES))
    ap.add_argument("--layers", type=int, default=0, help="blocks per step; 0 = 80 for llama_70b, else 1")
    ap.add_argument("--format", default="bf16", choices=sorted(BITS))
    ap.add_argument("--sparsities", default="0.5,0",
                    help="comma-separated; the first is the headline, 0 (dense) is always included")
    ap.add_argument("--copies", type=int, default=0, help="weight copies to walk (0 = auto)")
    ap.add_argument("--unfused", action="store_true", help="one launch per projection (7 per block)")
    ap.add_argument("--stack-launch", action="store_true",
                    help="16 groups per launch as independent work (a bare stack of projections)")
    ap.add_argument("--rows", default="padded", choices=("padded", "packed"),
                    help="padded: W_gate and W_up stored with rows 256 bytes further apart where that "
                         "lets the pair run without split-K (bf16 / int8, one launch per group)")
    ap.add_argument("--no-detail", action="store_true",
                    help="skip the Llama-3-8B-shaped block detail and the plain-read ceiling")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only; --gpus must be 1", file=sys.stderr)
        return 2
    if args.steps < 1 or args.warmup < 0 or args.repeats < 1:
        print("bench.py: --steps and --repeats must be at least 1", file=sys.stderr)
        return 2

    clocks = gpu_clocks()
    import torch
    import paper_2408_14690_amd as T
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    if not os.path.exists(T.library_path()):
        from paper_2408_14690_amd import build
        build.build(verbose=False)
    T.load_library()

    sparsities = [float(s) for s in args.sparsities.split(",")]
    if 0.0 not in sparsities:
        sparsities.append(0.0)
    head, fmt = sparsities[0], args.format
    layers = args.layers or DEFAULT_LAYERS[args.workload]
    if fmt != "bf16" and layers > 1:
        print("bench.py: the quantised formats are benchmarked on one block (host quantiser)", file=sys.stderr)
        return 2
    shapes = ti.LAYER_SHAPES[args.workload]
    block_bytes = sum(n * m * BITS[fmt] // 8 for n, m in shapes.values())
    # consecutive steps walk several copies of a small workload's weights; a stack beyond the
    # last-level cache many times over needs none
    copies = args.copies or max(1, -(-CACHE_DEFEAT_BYTES // (block_bytes * layers)))
    # Layout of the matrices of the grouped launches (W_q, W_k, W_v and W_gate, W_up): rows 256
    # bytes further apart, so that a narrow tile meets all four 256-byte quarters of a KiB over
    # its rows; the gate + up pair then runs without split-K where the library's rule allows
    # (teal_gemv_plan_multi_pitch).  The layout is the library's own step (teal_pack_bf16_pitch),
    # the bytes read are the same.
    row_pad, rows = {}, "packed"
    if args.rows == "padded" and fmt in ("bf16", "w8") and not args.stack_launch and not args.unfused:
        pad = 256 * 8 // BITS[fmt]
        row_pad, rows = {name: pad for name in ("q", "k", "v", "gate", "up")}, "padded"
    # The block detail is timed first.  Once a 137 GB stack has been allocated and freed, later
    # allocations on the box (of this process and of the next ones) were measured to give
    # 3-5 % slower small launches, while the long headline pass is the same either way: 11.52
    # and 11.54 ms with the detail first, 11.49 and 11.55 ms with it last.
    detail_block = None if args.no_detail else llama3_8b_block_detail(T, torch, fmt, head)
    t_build = time.perf_counter()
    projections = build_stack(T, torch, args.workload, fmt, sparsities, layers, copies, row_pad=row_pad)
    block0 = projections[:7]
    groups = fuse(T, torch, projections)
    if args.stack_launch:
        calls = [StackCall(T, torch, groups[i:i + 16]) for i in range(0, len(groups), 16)]
        mode = "stack"
    elif args.unfused:
        calls, mode = projections, "per_projection"
    else:
        calls, mode = groups, "grouped"
    build_s = time.perf_counter() - t_build

    # ---- the timed region of the headline: see time_region ----
    per_step = {p: time_pass(T, torch, calls, p, args.steps, args.warmup, args.repeats)
                for p in sparsities}
    detail = {pct(p): pass_figures(calls, p, per_step[p], per_step[0.0]) for p in sparsities}
    sec_head = median(per_step[head])
    head_bytes = sum(C.bytes(head) for C in calls)
    achieved = head_bytes / sec_head / 1e9
    launches_per_step = len(calls)

    kernel = {("bf16", "grouped"): "sparse_gemv_multi_kernel<FmtBF16>",
              ("bf16", "per_projection"): "sparse_gemv_kernel<FmtBF16>",
              ("bf16", "stack"): "sparse_gemv_stack_kernel<FmtBF16>",
              ("w8", "grouped"): "sparse_gemv_multi_kernel<FmtW8>",
              ("w8", "per_projection"): "sparse_gemv_kernel<FmtW8>",
              ("w8", "stack"): "sparse_gemv_stack_kernel<FmtW8>",
              ("w4", "grouped"): "sparse_gemv_w4_multi_kernel",
              ("w4", "per_projection"): "sparse_gemv_w4_kernel",
              ("w4", "stack"): "sparse_gemv_w4_stack_kernel"}[(fmt, mode)]
    traffic, traffic_source = measured_traffic(args.workload, fmt, head, layers, mode, T.teal_version(),
                                               rows=rows)
    launches_text = {"grouped": "one per group of projections that read the same hidden state (q+k+v, o, "
                                "gate+up, down), each projection with its own threshold: the calls a "
                                "decoder would make",
                     "per_projection": "one per projection",
                     "stack": "one per 16 groups taken as independent work: a bare stack of projections, "
                              "not a decoder's dependent sequence"}[mode]
    out = {
        "metric": f"sparse GEMV effective HBM GB/s at {pct(head)} sparsity (one pass over the stack of "
                  f"decoder blocks); us and speedup vs dense per sparsity in detail",
        "value": achieved,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": sec_head * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": f"{args.workload}-shaped stack of {layers} decoder block(s), 7 projections each, "
                        f"batch 1, {fmt} W from N(0,0.02^2) ({block_bytes * layers / 1e9:.1f} GB resident), "
                        f"one fresh seeded fp16 x per projection input (Gaussian / Laplace by role), t at "
                        f"the {pct(head)} quantile of |x| per projection",
            "weight_format": fmt,
            "weight_rows": ("W_q, W_k, W_v, W_gate and W_up stored with rows 256 bytes further apart "
                            "(teal_pack_bf16_pitch), W_o and W_down packed" if rows == "padded" else "packed"),
            "weight_bytes_per_block": block_bytes,
            "blocks_per_step": layers,
            "launches": launches_text,
            "launches_per_step": launches_per_step,
            "weight_copies_walked": copies,
            "timing": f"median over {args.repeats} regions of {args.steps} back-to-back steps each, "
                      f"HIP events on the launch stream, after {args.warmup} warm-up steps",
            "library_version": T.teal_version(),
        },
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": traffic,
            "traffic_source": traffic_source,
            "kernel": f"{kernel} ({launches_per_step} launches per step, {pct(head)})",
            "bytes_per_launch_avg": head_bytes / launches_per_step,
            "kernel_avg_us": sec_head * 1e6 / launches_per_step,
        },
        "detail": detail,
        "ms_per_step_each_region": [s * 1e3 for s in per_step[head]],
        "build_seconds": build_s,
    }

    # the same reading of the clocks while the headline pass keeps the GPU busy
    busy = {}
    th = threading.Thread(target=lambda: busy.update(clocks=gpu_clocks()))
    th.start()
    k = 0
    while th.is_alive():
        one_step(T, calls, head, k)
        k += 1
        torch.cuda.synchronize()
    th.join()
    out["gpu_clocks"] = {"idle_before_the_run": clocks, "under_the_headline_pass": busy.get("clocks")}

    ok, compared = survivor_counts_match(T, torch, calls, head)
    out["parity_in_this_run"] = {"survivor_counts_equal_host_counts": ok, "matrices": compared}
    if not args.no_cpu_baseline:
        sec, passes, threads, want = cpu_baseline(block0, head)
        worst = 0.0
        for P, w in zip(block0, want):       # the pass above left block 0's outputs on the device
            got = P.y.cpu().numpy().astype(np.float64)
            worst = max(worst, float(np.linalg.norm(got - w) / np.linalg.norm(w)))
        out["parity_in_this_run"]["block0_rel_l2_vs_oracle_worst"] = worst
        block_head_bytes = sum(P.bytes(head) for P in block0)
        out["cpu_baseline"] = {
            "value": block_head_bytes / sec / 1e9,
            "unit": "GB/s",
            "cores": threads,
            "kind": "oracle",
            "sample": f"{passes} whole passes over block 0 of the stack at {pct(head)} (fp64 dense loop "
                      f"over the zeroed x), {sec * 1e3:.1f} ms per pass; the stack is {layers} such blocks",
            "ms_per_step": sec * 1e3 * layers,
            "one_core_ms_per_pass": cpu_baseline_one_core(block0, head) * 1e3,
        }
        if layers > 2 and fmt == "bf16":
            deep = sorted({(layers - 1) // 2, layers - 1})
            worst, checked = deep_layer_check(T, torch, projections, deep, head)
            out["parity_in_this_run"]["deep_blocks_all_outputs"] = {
                "blocks": deep, "outputs_checked": checked, "rel_l2_vs_oracle_worst": worst}

    if not args.no_detail:
        # free the stack first: the plain-read probe needs its 3 GiB buffer
        per_launch = int(head_bytes / launches_per_step)
        del calls, groups, projections, block0
        torch.cuda.empty_cache()
        ceil = read_ceiling(T, torch, [per_launch, 1 << 30])
        out["roofline"]["plain_read_of_the_same_bytes"] = ceil[0]
        out["roofline"]["plain_read_of_1GiB"] = ceil[1]
        out["roofline"]["achieved_over_plain_read_of_the_same_bytes"] = achieved / ceil[0]["GBps"]
        out["llama3_8b_block"] = detail_block
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
