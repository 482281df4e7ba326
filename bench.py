#!/usr/bin/env python3
"""Benchmark of the TEAL decode hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]
                    [--workload llama2_7b|llama3_8b|llama_70b] [--format bf16|w8|w4]
                    [--sparsities 0.5,0.4,0] [--layers L] [--unfused] [--batch B]
                    [--calibration] [--swiglu] [--rmsnorm] [--graph]

A step is one pass of the whole hot path over a synthetic decoder block at
batch 1: for each of the seven projections, threshold the hidden state, compact
the survivors and stream only the surviving weight rows.  By default (bf16) the
projections that read the same hidden state -- q+k+v, o, gate+up, down, each
projection with its own threshold -- go out as one C-ABI call = one kernel
launch per group, 4 launches per block; --unfused launches every projection
on its own (7 per block), and both are timed and reported.  The headline value
is the effective HBM bandwidth of that pass at the first listed sparsity (50%
by default): algorithmic bytes / time.  The same pass at the other sparsities,
and at 0% (t = 0, the same kernels run dense), gives the speed-up over dense.
Weights, states and the workspace are resident in HBM before the timed region.
Consecutive steps walk over several copies of the weights so that no step
finds its rows in the 256 MB last-level cache.  With --layers L > 1 a step is
a stack of L blocks with their own weights and states (the 80-block
70B-shaped stack is 137 GB resident), and no copies are needed.  --batch B
runs the small-batch variant (one mask per batch from the averaged magnitude),
--calibration the threshold calibration pass, --swiglu the W_down step with its
input formed in the kernel, --rmsnorm the q+k+v and gate+up steps with the
normalisation of their input formed in the kernel.

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
BITS = {"bf16": 16, "w8": 8, "w4": 4}
KERNEL = {"bf16": "sparse_gemv_kernel<FmtBF16>", "w8": "sparse_gemv_kernel<FmtW8>",
          "w4": "sparse_gemv_w4_kernel"}
# HBM bytes per launch at 50% (average over the launches of a step), from rocprofv3 --pmc
# FETCH_SIZE / WRITE_SIZE runs of this script, scaled by the factors a plain copy of known
# size gives on the same box (2.0 and 1.0).  Keyed by (workload, format, sparsity, layers,
# grouped launches | "stack"): profiles/sparse_gemv_multi_kernel_llama2_7b_hbm_traffic.txt,
# profiles/sparse_gemv_kernel_llama2_7b_hbm_traffic.txt and
# profiles/sparse_gemv_stack_kernel_llama2_7b_kernel_trace_hbm_traffic.txt.
MEASURED_TRAFFIC_BYTES = {
    ("llama2_7b", "bf16", 0.5, 1, True): (199469.51 + 1129.88) * 1024 / 4,
    ("llama2_7b", "bf16", 0.5, 1, False): (200469.62 + 1557.28) * 1024 / 7,
    ("llama2_7b", "bf16", 0.5, 1, "stack"): (199512.0 + 1129.88) * 1024,
}


def algorithmic_bytes(fmt: str, nnz: int, m: int, n: int, batch: int = 1) -> int:
    """Bytes the method must move for one projection: surviving rows (once, whatever the
    batch) + x + y per batch row + scales."""
    scales = {"bf16": 0, "w8": 2 * n, "w4": 2 * n * (m // 128)}[fmt]
    return nnz * n * BITS[fmt] // 8 + batch * (2 * m + 4 * n) + scales


class Projection:
    """One weight matrix resident on the device in the format under test."""

    def __init__(self, T, torch, name, n, m, fmt, x_host, sparsities, copies, w_host=None,
                 device_seed=None, batch=0):
        """batch = 0: one hidden state x_host[m] (Definition 1); batch >= 1: x_host is
        [batch][m] and the batch-wide criterion of Section 5.4.4 applies."""
        self.name, self.n, self.m, self.fmt, self.batch = name, n, m, fmt, batch
        self.x_host, self.w_host = x_host, w_host
        self.host_q = None
        if w_host is None:
            # weights drawn on the device (harness only), canonical layout, then laid out by the library
            g = torch.Generator(device="cuda")
            g.manual_seed(int(device_seed))
            wd = (torch.randn((n, m), generator=g, device="cuda", dtype=torch.float32) * 0.02) \
                .to(torch.bfloat16).view(torch.int16)
        else:
            wd = torch.from_numpy(w_host.view(np.int16)).cuda()
        if fmt == "bf16":
            wt = torch.empty((m, n), dtype=torch.int16, device="cuda")
            T.check(T.teal_pack_bf16(wd, wt, m, n))
            first = (wt,)
        else:
            if w_host is None:
                raise ValueError("quantised formats need host weights")
            if fmt == "w8":
                q, scale = ti.quantize_w8(w_host)
            else:
                q, scale = ti.quantize_w4(w_host, 128)
            self.host_q = (q, scale)
            first = (torch.from_numpy(q).cuda(), torch.from_numpy(scale.view(np.int16)).cuda())
        del wd
        self.weights = [first] + [tuple(t.clone() for t in first) for _ in range(copies - 1)]
        self.x = torch.from_numpy(x_host.view(np.int16)).cuda()
        self.y = torch.empty(max(batch, 1) * n, dtype=torch.float32, device="cuda")
        ws_bytes = T.teal_workspace_bytes_batch(m, n, batch) if batch else T.teal_workspace_bytes(m, n)
        self.ws = torch.zeros(ws_bytes, dtype=torch.uint8, device="cuda")
        self.t, self.nnz = {}, {}
        for p in sparsities:
            if batch:
                t = ti.batch_quantile_threshold(x_host, p)
                total = np.abs(x_host.astype(np.float64)).sum(axis=0)
                self.nnz[p] = int(np.count_nonzero(total > batch * float(np.float32(t))))
            else:
                t = ti.quantile_threshold(x_host, p)
                self.nnz[p] = int(np.count_nonzero(np.abs(x_host.astype(np.float32)) > np.float32(t)))
            self.t[p] = t
        # raw device addresses, so that the timed loop spends its host time in the library call
        self.wp = [tuple(t.data_ptr() for t in w) for w in self.weights]
        self.xp, self.yp, self.wsp = self.x.data_ptr(), self.y.data_ptr(), self.ws.data_ptr()
        self.ws_bytes = self.ws.numel()
        self.stream = torch.cuda.current_stream().cuda_stream
        self.prepared = {}

    def launch(self, T, copy: int, p: float) -> int:
        """The call, marshalled once per (weight copy, sparsity, stream) and re-issued."""
        key = (copy % len(self.wp), p, self.stream)
        call = self.prepared.get(key)
        if call is None:
            call = self.prepared[key] = T.prepare(lambda: self.enqueue(T, copy, p))
        return call()

    def enqueue(self, T, copy: int, p: float) -> int:
        w = self.wp[copy % len(self.wp)]
        if self.batch:
            return T.teal_sparse_gemv_bf16_batch(w[0], self.xp, self.batch, self.t[p], self.yp,
                                                 self.m, self.n, self.wsp, self.ws_bytes,
                                                 self.stream)
        if self.fmt == "bf16":
            return T.teal_sparse_gemv_bf16(w[0], self.xp, self.t[p], self.yp, self.m, self.n,
                                           self.wsp, self.ws_bytes, self.stream)
        if self.fmt == "w8":
            return T.teal_sparse_gemv_w8(w[0], w[1], self.xp, self.t[p], self.yp, self.m, self.n,
                                         self.wsp, self.ws_bytes, self.stream)
        return T.teal_sparse_gemv_w4(w[0], w[1], 128, self.xp, self.t[p], self.yp, self.m, self.n,
                                     self.wsp, self.ws_bytes, self.stream)

    def bytes(self, p: float) -> int:
        return algorithmic_bytes(self.fmt, self.nnz[p], self.m, self.n, max(self.batch, 1))

    def oracle(self, orc, p: float):
        if self.batch:
            return orc.sparse_gemv_bf16_batch(self.w_host, self.x_host, self.t[p])
        if self.fmt == "bf16":
            return orc.sparse_gemv_bf16(self.w_host, self.x_host, self.t[p])
        if self.fmt == "w8":
            return orc.sparse_gemv_w8(self.host_q[0], self.host_q[1], self.x_host, self.t[p])
        return orc.sparse_gemv_w4(self.host_q[0], self.host_q[1], 128, self.x_host, self.t[p])


class FusedGroup:
    """Projections that read the same hidden state, launched as one kernel."""

    def __init__(self, T, torch, members):
        self.members = members
        self.name = "+".join(P.name for P in members)
        self.m = members[0].m
        self.ns = [P.n for P in members]
        self.ys = [P.yp for P in members]
        self.batch = members[0].batch
        nbytes = (T.teal_workspace_bytes_batch(self.m, sum(self.ns), self.batch) if self.batch
                  else T.teal_workspace_bytes(self.m, sum(self.ns)))
        self.ws = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
        self.wsp, self.ws_bytes = self.ws.data_ptr(), self.ws.numel()
        self.stream = members[0].stream
        self.prepared = {}

    def launch(self, T, copy: int, p: float) -> int:
        """The call, marshalled once per (weight copy, sparsity, stream) and re-issued."""
        key = (copy % len(self.members[0].wp), p, self.stream)
        call = self.prepared.get(key)
        if call is None:
            call = self.prepared[key] = T.prepare(lambda: self.enqueue(T, copy, p))
        return call()

    def enqueue(self, T, copy: int, p: float) -> int:
        if self.batch:
            wts = [P.wp[copy % len(P.wp)][0] for P in self.members]
            return T.teal_sparse_gemv_bf16_batch_multi(wts, [P.t[p] for P in self.members],
                                                       self.ys, self.ns, self.members[0].xp,
                                                       self.batch, self.m, self.wsp,
                                                       self.ws_bytes, self.stream)
        if self.members[0].fmt == "w4":
            ws = [P.wp[copy % len(P.wp)] for P in self.members]
            return T.teal_sparse_gemv_w4_multi([w[0] for w in ws], [w[1] for w in ws], 128,
                                               [P.t[p] for P in self.members], self.ys, self.ns,
                                               self.members[0].xp, self.m, self.wsp,
                                               self.ws_bytes, self.stream)
        if self.members[0].fmt == "w8":
            ws = [P.wp[copy % len(P.wp)] for P in self.members]
            return T.teal_sparse_gemv_w8_multi([w[0] for w in ws], [w[1] for w in ws],
                                               [P.t[p] for P in self.members], self.ys, self.ns,
                                               self.members[0].xp, self.m, self.wsp,
                                               self.ws_bytes, self.stream)
        wts = [P.wp[copy % len(P.wp)][0] for P in self.members]
        return T.teal_sparse_gemv_bf16_multi(wts, [P.t[p] for P in self.members], self.ys, self.ns,
                                             self.members[0].xp, self.m, self.wsp, self.ws_bytes,
                                             self.stream)

    def bytes(self, p: float) -> int:
        # x is read once for the group
        return (sum(P.bytes(p) for P in self.members)
                - 2 * self.m * max(self.batch, 1) * (len(self.members) - 1))


class StackCall:
    """Up to 16 groups that do not depend on each other, issued as ONE launch
    (teal_sparse_gemv_bf16_stack): a bare stack of projections, each group with its own
    input, nothing between the products."""

    def __init__(self, T, torch, groups):
        self.groups = groups
        self.name = " | ".join(G.name for G in groups)
        self.counts = [len(G.members) for G in groups]
        self.ns = [n for G in groups for n in G.ns]
        self.ys = [y for G in groups for y in G.ys]
        self.ms = [G.m for G in groups]
        self.xs = [G.members[0].xp for G in groups]
        self.ws = torch.zeros(T.teal_workspace_bytes_stack(self.counts, self.ns, self.ms),
                              dtype=torch.uint8, device="cuda")
        self.region = [0]
        for G in groups:
            self.region.append(self.region[-1] + T.teal_workspace_bytes(G.m, sum(G.ns)))
        self.wsp, self.ws_bytes = self.ws.data_ptr(), self.ws.numel()
        self.stream = groups[0].stream
        self.prepared = {}

    def launch(self, T, copy: int, p: float) -> int:
        key = (copy % len(self.groups[0].members[0].wp), p, self.stream)
        call = self.prepared.get(key)
        if call is None:
            call = self.prepared[key] = T.prepare(lambda: self.enqueue(T, copy, p))
        return call()

    def enqueue(self, T, copy: int, p: float) -> int:
        members = [P for G in self.groups for P in G.members]
        ws = [P.wp[copy % len(P.wp)] for P in members]
        ts = [P.t[p] for P in members]
        fmt = members[0].fmt
        if fmt == "w8":
            return T.teal_sparse_gemv_w8_stack(self.counts, [w[0] for w in ws], [w[1] for w in ws], ts,
                                               self.ys, self.ns, self.xs, self.ms, self.wsp,
                                               self.ws_bytes, self.stream)
        if fmt == "w4":
            return T.teal_sparse_gemv_w4_stack(self.counts, [w[0] for w in ws], [w[1] for w in ws], 128,
                                               ts, self.ys, self.ns, self.xs, self.ms, self.wsp,
                                               self.ws_bytes, self.stream)
        return T.teal_sparse_gemv_bf16_stack(self.counts, [w[0] for w in ws], ts, self.ys, self.ns,
                                             self.xs, self.ms, self.wsp, self.ws_bytes, self.stream)

    def bytes(self, p: float) -> int:
        return sum(G.bytes(p) for G in self.groups)

    def survivors_match(self, T, torch, p: float):
        """The counts the last call left in the groups' regions against the host counts."""
        off = T.teal_survivors_offset()
        ok, compared = True, 0
        for G, at in zip(self.groups, self.region):
            got = self.ws[at + off:at + off + 4 * len(G.members)].view(torch.int32).cpu().tolist()
            ok = ok and got == [P.nnz[p] for P in G.members]
            compared += len(G.members)
        return ok, compared


class Replica:
    """A projection as one of several independent products in a stack launch: the same
    x and thresholds, its own output, and the weight copies walked from its own offset (so
    that the replicas of one launch read different memory)."""

    def __init__(self, torch, P, j: int):
        self.name, self.m, self.ns, self.stream = P.name, P.m, [P.n], P.stream
        self.y = torch.empty(P.n, dtype=torch.float32, device="cuda")
        self.ys = [self.y.data_ptr()]
        j %= len(P.wp)
        self.wp, self.t, self.nnz, self.xp, self.fmt = P.wp[j:] + P.wp[:j], P.t, P.nnz, P.xp, P.fmt
        self.members = [self]
        self._bytes = P.bytes

    def bytes(self, p: float) -> int:
        return self._bytes(p)


def fuse(T, torch, stack):
    """Group consecutive projections of each block that share their input (Appendix A.3)."""
    out, i = [], 0
    while i < len(stack):
        j = i + 1
        while (j < len(stack) and stack[j].m == stack[i].m
               and ti.PROJ_XGROUP[stack[j].name] == ti.PROJ_XGROUP[stack[i].name]
               and ti.PROJ_ORDER.index(stack[j].name) > ti.PROJ_ORDER.index(stack[j - 1].name)):
            j += 1
        out.append(FusedGroup(T, torch, stack[i:j]))
        i = j
    return out


def build_stack(T, torch, model, fmt, sparsities, layers, copies, batch=0):
    """`layers` synthetic blocks.  Block 0 comes from the seeded host recipe (so the CPU
    baseline sees the same numbers); further blocks of a bf16 stack draw their weights on
    the device."""
    cfg = ti.CONFIG_INDEX[model]
    stack = []
    for layer in range(layers):
        host = layer == 0 or fmt != "bf16"
        for proj in ti.PROJ_ORDER:
            n, m = ti.LAYER_SHAPES[model][proj]
            if batch:
                x = ti.make_X(batch, m, ti.x_seed(cfg, layer, proj), ti.PROJ_DIST[proj])
            else:
                x = ti.make_x(m, ti.x_seed(cfg, layer, proj), ti.PROJ_DIST[proj])
            w = ti.weights_bf16(n, m, ti.weight_seed(cfg, layer, proj)) if host else None
            stack.append(Projection(T, torch, proj, n, m, fmt, x, sparsities, copies, w_host=w,
                                    device_seed=ti.weight_seed(cfg, layer, proj), batch=batch))
            if layer > 0:
                stack[-1].w_host = None          # keep host memory flat for deep stacks
                stack[-1].host_q = None
    torch.cuda.synchronize()
    return stack


def one_step(T, stack, p: float, copy: int) -> None:
    for P in stack:
        st = P.launch(T, copy, p)
        if st != 0:
            T.check(st)


def time_steps(T, torch, stack, p, steps, warmup) -> float:
    """Seconds per step over `steps` back-to-back passes (HIP events on the launch stream)."""
    for k in range(warmup):
        one_step(T, stack, p, k)
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    start.record()
    for k in range(steps):
        one_step(T, stack, p, k)
    stop.record()
    issue = time.perf_counter() - t0
    torch.cuda.synchronize()
    time_steps.host_issue_us = issue * 1e6 / steps      # host time to enqueue one step
    return start.elapsed_time(stop) * 1e-3 / steps


def time_steps_graph(T, torch, stack, p, steps, copies) -> float:
    """Seconds per step when the launches of `copies` consecutive steps (one walk over the
    weight copies) are captured once into a HIP graph and the graph is replayed."""
    side = torch.cuda.Stream()
    calls = set()
    for C in stack:
        calls.add(C)
        calls.update(getattr(C, "members", ()))
    saved = {C: C.stream for C in calls}
    side.wait_stream(torch.cuda.current_stream())
    try:
        for C in calls:
            C.stream = side.cuda_stream
        with torch.cuda.stream(side):
            for k in range(copies):
                one_step(T, stack, p, k)                     # warm the capture stream
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for k in range(copies):
                one_step(T, stack, p, k)
        replays = max(1, steps // copies)
        with torch.cuda.stream(side):
            graph.replay()
            side.synchronize()
            start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            start.record(side)
            for _ in range(replays):
                graph.replay()
            stop.record(side)
        side.synchronize()
        sec = start.elapsed_time(stop) * 1e-3 / (replays * copies)
        del graph
    finally:
        for C, st in saved.items():
            C.stream = st
    torch.cuda.current_stream().wait_stream(side)
    return sec


def time_projection(T, torch, P, p, launches) -> float:
    """Seconds per call for one projection launched back to back, walking its weight copies."""
    for k in range(20):
        P.launch(T, k, p)
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for k in range(launches):
        P.launch(T, k, p)
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) * 1e-3 / launches


def time_torch_matmul(torch, P, canonical: bool, launches=300) -> float:
    """Context only: the dense product through torch.matmul (the vendor BLAS) in bf16, walking
    as many weight copies as the timed calls do; seconds per call.  canonical: W[n][m] times
    x (the layout a model keeps its weights in); else x times the input-channel-major
    Wt[m][n] the library reads."""
    xb = P.x.view(torch.float16).to(torch.bfloat16)
    if canonical:
        ws = [w[0].view(torch.bfloat16).t().contiguous() for w in P.weights]
        out = torch.empty(P.n, dtype=torch.bfloat16, device="cuda")
        run = lambda k: torch.mv(ws[k % len(ws)], xb, out=out)
    else:
        ws = [w[0].view(torch.bfloat16) for w in P.weights]
        xrow = xb.unsqueeze(0)
        out = torch.empty((1, P.n), dtype=torch.bfloat16, device="cuda")
        run = lambda k: torch.matmul(xrow, ws[k % len(ws)], out=out)
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


def time_projection_spread(T, torch, P, p, batches=10, launches=100, singles=20):
    """The same call timed in `batches` separate batches of back-to-back launches (us per
    call: median and minimum over the batches) and as single launches, each bracketed by
    its own pair of events on an idle stream (median; includes the start-up of a kernel on
    an idle GPU, which back-to-back launches hide)."""
    per_batch = sorted(time_projection(T, torch, P, p, launches) * 1e6 for _ in range(batches))
    single = []
    for k in range(singles):
        torch.cuda.synchronize()
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record()
        P.launch(T, k, p)
        stop.record()
        torch.cuda.synchronize()
        single.append(start.elapsed_time(stop) * 1e3)
    single.sort()
    return {"us_median_of_batches": per_batch[len(per_batch) // 2], "us_min_of_batches": per_batch[0],
            "us_single_launch_median": single[len(single) // 2]}


def read_ceiling(T, torch, sizes, launches=200):
    """What a kernel that only reads reaches on this machine (teal_stream_read_probe: the row
    stream's 16-byte non-temporal loads, no other work) for launches of the given sizes,
    back to back, each launch on a different part of a 3 GiB buffer so that nothing comes
    from a cache; the best over a few grid sizes."""
    total = CACHE_DEFEAT_BYTES
    buf = torch.empty(total // 4, dtype=torch.int32, device="cuda").random_()
    sink = torch.zeros(8192, dtype=torch.int32, device="cuda")
    base, stream = buf.data_ptr(), torch.cuda.current_stream().cuda_stream
    out = []
    for size in sizes:
        size = min(int(size), total // 2) // 256 * 256
        slots = (total - size) // 256
        step = max(1, (size + 255) // 256)
        best = None
        for blocks in (256, 512, 1024, 2048, 4096, 8192):
            calls = [T.prepare(lambda k=k: T.teal_stream_read_probe(
                base + 256 * ((k * step) % slots), size, blocks, 0xFFFFFFFF, sink, stream))
                for k in range(max(2, total // size))]
            for k in range(20):
                T.check(calls[k % len(calls)]())
            torch.cuda.synchronize()
            start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            start.record()
            for k in range(launches):
                calls[k % len(calls)]()
            stop.record()
            torch.cuda.synchronize()
            us = start.elapsed_time(stop) * 1e3 / launches
            if best is None or us < best["us_per_launch"]:
                best = {"bytes_per_launch": size, "us_per_launch": us, "GBps": size / us / 1e3,
                        "frac_of_hbm_peak": size / us / 1e3 / HBM_PEAK_GBS, "blocks": blocks}
        out.append(best)
    del buf
    return out


def cpu_baseline(block, p: float, budget_s: float = 12.0):
    """The fp64 oracle, as it stands, on the host cores: whole passes over block 0 until
    about `budget_s` seconds of CPU work have been spent."""
    from oracle import teal_oracle as orc
    threads = orc.num_threads()
    block[0].oracle(orc, p)                                   # warm-up
    passes, spent, outputs = 0, 0.0, None
    while spent < budget_s and passes < 1000:
        t0 = time.perf_counter()
        ys = [P.oracle(orc, p) for P in block]
        spent += time.perf_counter() - t0
        passes += 1
        outputs = outputs or ys
    return spent / passes, passes, threads, outputs


def cpu_baseline_one_core(block, p: float) -> float:
    """Seconds for one pass of the oracle over block 0 on a single host core."""
    from oracle import teal_oracle as orc
    threads = orc.num_threads()
    orc.set_num_threads(1)
    try:
        t0 = time.perf_counter()
        for P in block:
            P.oracle(orc, p)
        return time.perf_counter() - t0
    finally:
        orc.set_num_threads(threads)


def deep_layer_check(T, torch, projections, layers, p: float):
    """Blocks past the first draw their weights on the device; for the given blocks, every
    output of every projection (what the last pass left on the device) against the oracle
    run on the weights copied back, one matrix at a time.  Worst relative L2 over the
    matrices, and the number of outputs compared."""
    from oracle import teal_oracle as orc
    worst, checked = 0.0, 0
    for layer in layers:
        for P in projections[7 * layer:7 * layer + 7]:
            wt = P.weights[0][0]                                        # [m][n] bf16 bits
            w = wt.t().contiguous().cpu().numpy().view(np.uint16)       # canonical [n][m]
            want = orc.sparse_gemv_bf16(w, P.x_host, P.t[p])
            del w
            got = P.y.cpu().numpy().astype(np.float64)
            worst = max(worst, float(np.linalg.norm(got - want) / np.linalg.norm(want)))
            checked += P.n
    return worst, checked


def survivor_counts_match(T, torch, stack, p: float):
    """After one more pass at sparsity p: the count of surviving channels each call left in
    its workspace against the count taken on the host from the same x and t.  Returns
    (all equal, number of matrices compared)."""
    one_step(T, stack, p, 0)
    torch.cuda.synchronize()
    off = T.teal_survivors_offset()
    ok, compared = True, 0
    for C in stack:
        if hasattr(C, "survivors_match"):
            one_ok, count = C.survivors_match(T, torch, p)
            ok, compared = ok and one_ok, compared + count
            continue
        members = getattr(C, "members", [C])
        got = C.ws[off:off + 4 * len(members)].view(torch.int32).cpu().tolist()
        ok = ok and got == [P.nnz[p] for P in members]
        compared += len(members)
    return ok, compared


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


def gpu_clocks():
    """Current core and memory clock levels of the first GPU as the driver shows them in
    sysfs (whatever the box gives; nothing is changed here).  Plain file reads: no other
    program is started.  None where the files are absent."""
    import glob
    out = {}
    for name in ("sclk", "mclk"):
        for path in sorted(glob.glob(f"/sys/class/drm/card*/device/pp_dpm_{name}")):
            try:
                lines = open(path).read().split("\n")
            except OSError:
                continue
            current = [ln.split(":", 1)[1].replace("*", "").strip() for ln in lines if ln.rstrip().endswith("*")]
            if current:
                out[name] = current[0]
                break
    return out or None


def pct(p: float) -> str:
    return f"{int(round(p * 100))}%"


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
    ap.add_argument("--no-per-projection", action="store_true")
    ap.add_argument("--no-other-mode", action="store_true",
                    help="skip timing the pass in the launch mode that is not the headline")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only; --gpus must be 1", file=sys.stderr)
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
    if args.swiglu:
        return run_swiglu(T, torch, args)
    if args.rmsnorm:
        return run_rmsnorm(T, torch, args)
    if args.calibration:
        if args.calibration_tokens % 64 or args.calibration_tokens <= 0:
            print("bench.py: --calibration-tokens must be a positive multiple of 64", file=sys.stderr)
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
        print("bench.py: --batch needs bf16 and 1 <= B <= 8", file=sys.stderr)
        return 2
    projections = build_stack(T, torch, args.workload, fmt, sparsities, args.layers, copies,
                              args.batch)
    block0 = projections[:7]
    groups = fuse(T, torch, projections)
    stack_calls = None
    if not args.batch and (args.stack_launch or not args.no_other_mode):
        stack_calls = [StackCall(T, torch, groups[i:i + 16]) for i in range(0, len(groups), 16)]
    if args.stack_launch:
        if stack_calls is None or args.unfused:
            print("bench.py: --stack-launch needs batch 1 and grouped launches", file=sys.stderr)
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
            "traffic": MEASURED_TRAFFIC_BYTES.get(
                (args.workload, fmt, head, args.layers, "stack" if args.stack_launch else fused)),
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
