"""Shared pieces of the benchmarks (bench.py: the headline path; bench_extras.py: the side
measurements): the synthetic decoder-block workload resident on the device, the calls that
make up a pass over it, timing helpers, the CPU-oracle baseline, the plain-read ceiling and
the lookup of measured HBM traffic in profiles/."""
from __future__ import annotations

import json
import os
import re
import time

import numpy as np

import teal_inputs as ti

ROOT = os.path.dirname(os.path.abspath(__file__))

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
CACHE_DEFEAT_BYTES = 3 << 30    # distinct weight bytes walked before a copy is reused
WALK_BYTES_ALONE = 600 << 20    # the same for one call timed alone (the last-level cache holds 256 MB)
BITS = {"bf16": 16, "w8": 8, "w4": 4}
KERNEL = {"bf16": "sparse_gemv_kernel<FmtBF16>", "w8": "sparse_gemv_kernel<FmtW8>",
          "w4": "sparse_gemv_w4_kernel"}


def algorithmic_bytes(fmt: str, nnz: int, m: int, n: int, batch: int = 1) -> int:
    """Bytes the method must move for one projection: surviving rows (once, whatever the
    batch) + x + y per batch row + scales."""
    scales = {"bf16": 0, "w8": 2 * n, "w4": 2 * n * (m // 128)}[fmt]
    return nnz * n * BITS[fmt] // 8 + batch * (2 * m + 4 * n) + scales


class Projection:
    """One weight matrix resident on the device in the format under test."""

    def __init__(self, T, torch, name, n, m, fmt, x_host, sparsities, copies, w_host=None,
                 device_seed=None, batch=0, row_pad=0):
        """batch = 0: one hidden state x_host[m] (Definition 1); batch >= 1: x_host is
        [batch][m] and the batch-wide criterion of Section 5.4.4 applies.  row_pad > 0 (bf16,
        int8, batch 0): the matrix is stored with rows n + row_pad elements apart and the
        calls are the library's _pitch entry points."""
        self.name, self.n, self.m, self.fmt, self.batch = name, n, m, fmt, batch
        self.pitch = n + row_pad
        if row_pad and (batch or fmt == "w4"):
            raise ValueError("padded rows: bf16 and int8, batch 1")
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
            wt = torch.zeros((m, self.pitch), dtype=torch.int16, device="cuda")
            T.check(T.teal_pack_bf16_pitch(wd, wt, m, n, self.pitch) if row_pad
                    else T.teal_pack_bf16(wd, wt, m, n))
            first = (wt,)
        else:
            if w_host is None:
                raise ValueError("quantised formats need host weights")
            if fmt == "w8":
                q, scale = ti.quantize_w8(w_host)
            else:
                q, scale = ti.quantize_w4(w_host, 128)
            self.host_q = (q, scale)
            qd = torch.from_numpy(q).cuda()
            if row_pad:
                wide = torch.zeros((m, self.pitch), dtype=torch.int8, device="cuda")
                wide[:, :n] = qd
                qd = wide
            first = (qd, torch.from_numpy(scale.view(np.int16)).cuda())
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
        if self.pitch != self.n:
            if self.fmt == "bf16":
                return T.teal_sparse_gemv_bf16_multi_pitch([w[0]], [self.pitch], [self.t[p]], [self.yp],
                                                           [self.n], self.xp, self.m, self.wsp,
                                                           self.ws_bytes, self.stream)
            return T.teal_sparse_gemv_w8_multi_pitch([w[0]], [self.pitch], [w[1]], [self.t[p]],
                                                     [self.yp], [self.n], self.xp, self.m, self.wsp,
                                                     self.ws_bytes, self.stream)
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

    def walked_bytes(self, p: float) -> int:
        """Weight bytes read before a weight copy comes round again when this projection is
        launched back to back on its own."""
        return len(self.wp) * self.nnz[p] * self.n * BITS[self.fmt] // 8

    def ensure_walk(self, p: float, need: int = WALK_BYTES_ALONE) -> None:
        """More copies of the weights until a back-to-back run at sparsity p walks at least
        `need` distinct bytes (about twice the 256 MB last-level cache): the block-sized copy
        count is too small for a narrow projection timed alone."""
        per_copy = max(1, self.nnz[p] * self.n * BITS[self.fmt] // 8)
        while len(self.weights) * per_copy < need:
            self.weights.append(tuple(t.clone() for t in self.weights[0]))
        self.wp = [tuple(t.data_ptr() for t in w) for w in self.weights]

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
        padded = any(P.pitch != P.n for P in self.members)
        if self.members[0].fmt == "w8" and padded:
            ws = [P.wp[copy % len(P.wp)] for P in self.members]
            return T.teal_sparse_gemv_w8_multi_pitch([w[0] for w in ws], [P.pitch for P in self.members],
                                                     [w[1] for w in ws], [P.t[p] for P in self.members],
                                                     self.ys, self.ns, self.members[0].xp, self.m,
                                                     self.wsp, self.ws_bytes, self.stream)
        if self.members[0].fmt == "w8":
            ws = [P.wp[copy % len(P.wp)] for P in self.members]
            return T.teal_sparse_gemv_w8_multi([w[0] for w in ws], [w[1] for w in ws],
                                               [P.t[p] for P in self.members], self.ys, self.ns,
                                               self.members[0].xp, self.m, self.wsp,
                                               self.ws_bytes, self.stream)
        wts = [P.wp[copy % len(P.wp)][0] for P in self.members]
        if padded:
            return T.teal_sparse_gemv_bf16_multi_pitch(wts, [P.pitch for P in self.members],
                                                       [P.t[p] for P in self.members], self.ys,
                                                       self.ns, self.members[0].xp, self.m, self.wsp,
                                                       self.ws_bytes, self.stream)
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


def build_stack(T, torch, model, fmt, sparsities, layers, copies, batch=0, row_pad=None):
    """`layers` synthetic blocks.  Block 0 comes from the seeded host recipe (so the CPU
    baseline sees the same numbers); further blocks of a bf16 stack draw their weights on
    the device.  row_pad: {projection name: elements added to its row pitch}."""
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
                                    device_seed=ti.weight_seed(cfg, layer, proj), batch=batch,
                                    row_pad=(row_pad or {}).get(proj, 0)))
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
            wt = P.weights[0][0][:, :P.n]                               # [m][n] bf16 bits
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


class MlpCall:
    """The MLP of one block on its own data flow (Appendix A.3): gate and up read x, W_down
    reads h = SiLU(gate) * up formed from their outputs, so the three products depend on each
    other as in a decoder.  Issued three ways: one launch (teal_sparse_mlp_*), two (the
    grouped gate + up call, then W_down with its input formed in the kernel), or three (gate,
    up, W_down each on its own).  The threshold of W_down is the quantile of |h| for the h
    the library's own producer forms from the gate / up outputs at that sparsity.
    "one_launch_padded_rows" (bf16, int8) is the one launch on copies of the same matrices
    stored with rows 256 bytes further apart (teal_mlp_shape's row pitches; same bytes read),
    in the shape teal_mlp_plan picks for that layout."""

    PAD_BYTES = 256      # added to a row's pitch: rows then lie an odd multiple of 256 bytes apart

    def __init__(self, T, torch, gate, up, down, sparsities):
        self.gate, self.up, self.down = gate, up, down
        self.name = "mlp(gate+up->down)"
        self.m, self.f, self.d, self.fmt = gate.m, gate.n, down.n, gate.fmt
        self.stream = gate.stream
        self.g = torch.empty(self.f, dtype=torch.float32, device="cuda")
        self.u = torch.empty(self.f, dtype=torch.float32, device="cuda")
        self.y = torch.empty(self.d, dtype=torch.float32, device="cuda")
        self.ws = torch.zeros(T.teal_workspace_bytes_mlp(self.m, self.f, self.d), dtype=torch.uint8,
                              device="cuda")
        self.ws_gu = torch.zeros(T.teal_workspace_bytes(self.m, 2 * self.f), dtype=torch.uint8,
                                 device="cuda")
        self.mode = "one_launch"
        self.torch = torch
        self.padded, self.padded_shape = None, None
        self.t_down, self.nnz_h, self.prepared = {}, {}, {}
        h = torch.empty(self.f, dtype=torch.int16, device="cuda")
        for p in sparsities:
            T.check(self._enqueue(T, 0, p, t_down=0.0))
            T.check(T.teal_swiglu_f16(self.g, self.u, h, self.f))
            torch.cuda.synchronize()
            hh = h.cpu().numpy().view(np.float16)
            self.t_down[p] = ti.quantile_threshold(hh, p)
            self.nnz_h[p] = int(np.count_nonzero(np.abs(hh.astype(np.float32)) > np.float32(self.t_down[p])))

    def _pad_weights(self, T):
        """Padded-row copies of the matrices (bf16, int8), one per weight copy, and the shape
        the library plans for their pitches."""
        torch = self.torch
        pad_elems = self.PAD_BYTES * 8 // BITS[self.fmt]

        def pad(w, pitch):
            out = torch.zeros((w.shape[0], pitch), dtype=w.dtype, device="cuda")
            out[:, :w.shape[1]] = w
            return out

        pg, pd = self.f + pad_elems, self.d + pad_elems
        G, U, D = self.gate, self.up, self.down
        self.padded = [(pad(G.weights[c][0], pg), pad(U.weights[c % len(U.weights)][0], pg),
                        pad(D.weights[c % len(D.weights)][0], pd)) for c in range(len(G.weights))]
        st, sh = T.teal_mlp_plan(BITS[self.fmt], self.m, self.f, self.d, pg, pd)
        T.check(st)
        self.padded_shape = sh

    def _enqueue(self, T, copy, p, t_down=None):
        G, U, D = self.gate, self.up, self.down
        wg, wu, wd = G.wp[copy % len(G.wp)], U.wp[copy % len(U.wp)], D.wp[copy % len(D.wp)]
        td = self.t_down[p] if t_down is None else t_down
        gp, up_, yp = self.g.data_ptr(), self.u.data_ptr(), self.y.data_ptr()
        m, f, d, st = self.m, self.f, self.d, self.stream
        if self.mode == "one_launch_padded_rows":
            if self.fmt not in ("bf16", "w8"):
                raise ValueError("padded rows are timed for bf16 and int8")
            if self.padded is None:
                self._pad_weights(T)
            w = self.padded[copy % len(self.padded)]
            if self.fmt == "w8":
                return T.teal_sparse_mlp_w8(w[0].data_ptr(), w[1].data_ptr(), w[2].data_ptr(), wg[1],
                                            wu[1], wd[1], G.xp, G.t[p], U.t[p], td, gp, up_, yp, m, f, d,
                                            self.ws.data_ptr(), self.ws.numel(), st,
                                            shape=self.padded_shape)
            return T.teal_sparse_mlp_bf16(w[0].data_ptr(), w[1].data_ptr(), w[2].data_ptr(), G.xp,
                                          G.t[p], U.t[p], td, gp, up_, yp, m, f, d,
                                          self.ws.data_ptr(), self.ws.numel(), st,
                                          shape=self.padded_shape)
        if self.mode == "one_launch":
            wsp, wsb = self.ws.data_ptr(), self.ws.numel()
            if self.fmt == "bf16":
                return T.teal_sparse_mlp_bf16(wg[0], wu[0], wd[0], G.xp, G.t[p], U.t[p], td, gp, up_, yp,
                                              m, f, d, wsp, wsb, st)
            if self.fmt == "w8":
                return T.teal_sparse_mlp_w8(wg[0], wu[0], wd[0], wg[1], wu[1], wd[1], G.xp, G.t[p], U.t[p],
                                            td, gp, up_, yp, m, f, d, wsp, wsb, st)
            return T.teal_sparse_mlp_w4(wg[0], wu[0], wd[0], wg[1], wu[1], wd[1], 128, G.xp, G.t[p],
                                        U.t[p], td, gp, up_, yp, m, f, d, wsp, wsb, st)
        wsp, wsb = self.ws_gu.data_ptr(), self.ws_gu.numel()
        if self.mode == "two_launches":
            if self.fmt == "bf16":
                s1 = T.teal_sparse_gemv_bf16_multi([wg[0], wu[0]], [G.t[p], U.t[p]], [gp, up_], [f, f],
                                                   G.xp, m, wsp, wsb, st)
                s2 = T.teal_sparse_gemv_bf16_swiglu(wd[0], gp, up_, td, yp, f, d, D.wsp, D.ws_bytes, st)
            elif self.fmt == "w8":
                s1 = T.teal_sparse_gemv_w8_multi([wg[0], wu[0]], [wg[1], wu[1]], [G.t[p], U.t[p]],
                                                 [gp, up_], [f, f], G.xp, m, wsp, wsb, st)
                s2 = T.teal_sparse_gemv_w8_swiglu(wd[0], wd[1], gp, up_, td, yp, f, d, D.wsp, D.ws_bytes, st)
            else:
                s1 = T.teal_sparse_gemv_w4_multi([wg[0], wu[0]], [wg[1], wu[1]], 128, [G.t[p], U.t[p]],
                                                 [gp, up_], [f, f], G.xp, m, wsp, wsb, st)
                s2 = T.teal_sparse_gemv_w4_swiglu(wd[0], wd[1], 128, gp, up_, td, yp, f, d, D.wsp,
                                                  D.ws_bytes, st)
            return s1 or s2
        # three launches
        if self.fmt == "bf16":
            s1 = T.teal_sparse_gemv_bf16(wg[0], G.xp, G.t[p], gp, m, f, G.wsp, G.ws_bytes, st)
            s2 = T.teal_sparse_gemv_bf16(wu[0], U.xp, U.t[p], up_, m, f, U.wsp, U.ws_bytes, st)
            s3 = T.teal_sparse_gemv_bf16_swiglu(wd[0], gp, up_, td, yp, f, d, D.wsp, D.ws_bytes, st)
        elif self.fmt == "w8":
            s1 = T.teal_sparse_gemv_w8(wg[0], wg[1], G.xp, G.t[p], gp, m, f, G.wsp, G.ws_bytes, st)
            s2 = T.teal_sparse_gemv_w8(wu[0], wu[1], U.xp, U.t[p], up_, m, f, U.wsp, U.ws_bytes, st)
            s3 = T.teal_sparse_gemv_w8_swiglu(wd[0], wd[1], gp, up_, td, yp, f, d, D.wsp, D.ws_bytes, st)
        else:
            s1 = T.teal_sparse_gemv_w4(wg[0], wg[1], 128, G.xp, G.t[p], gp, m, f, G.wsp, G.ws_bytes, st)
            s2 = T.teal_sparse_gemv_w4(wu[0], wu[1], 128, U.xp, U.t[p], up_, m, f, U.wsp, U.ws_bytes, st)
            s3 = T.teal_sparse_gemv_w4_swiglu(wd[0], wd[1], 128, gp, up_, td, yp, f, d, D.wsp,
                                              D.ws_bytes, st)
        return s1 or s2 or s3

    def launch(self, T, copy: int, p: float) -> int:
        key = (self.mode, copy % len(self.gate.wp), p, self.stream)
        call = self.prepared.get(key)
        if call is None:
            call = self.prepared[key] = T.prepare(lambda: self._enqueue(T, copy, p))
        return call()

    def bytes(self, p: float) -> int:
        """Surviving rows of the three matrices, x, y, and gate / up written and read once."""
        b = BITS[self.fmt]
        rows = (self.gate.nnz[p] + self.up.nnz[p]) * self.f * b // 8 + self.nnz_h[p] * self.d * b // 8
        scales = {"bf16": 0, "w8": 4 * self.f + 2 * self.d,
                  "w4": 2 * (2 * self.f * (self.m // 128) + self.d * (self.f // 128))}[self.fmt]
        return rows + 2 * self.m + 4 * self.d + 16 * self.f + scales


def measured_traffic(workload: str, fmt: str, sparsity: float, layers: int, launches: str,
                     library_version: int, folder: str = "", rows: str = "packed"):
    """HBM bytes per launch (fetched + written) of the dominant kernel, as measured with
    rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and written down in a summary under profiles/.
    A summary carries one line per measured case,
        TRAFFIC workload=... format=... sparsity=... layers=... launches=... library_version=...
                fetch_bytes_per_launch=... write_bytes_per_launch=... (counter values already
                scaled by the factors a plain copy of known size gives; stated in the file)
    and only a line whose key fields all match this run counts: a summary taken with other
    kernels (another library version) is not this run's traffic.  Returns (bytes or None, the
    file the figure comes from or the reason there is none)."""
    want = {"workload": workload, "format": fmt, "sparsity": f"{sparsity:g}", "layers": str(layers),
            "launches": launches, "library_version": str(library_version), "rows": rows}
    folder = folder or os.path.join(ROOT, "profiles")
    stale = None
    for name in sorted(os.listdir(folder)) if os.path.isdir(folder) else []:
        if not name.endswith((".txt", ".md")):
            continue
        for line in open(os.path.join(folder, name), errors="replace"):
            if not line.startswith("TRAFFIC "):
                continue
            kv = dict(tok.split("=", 1) for tok in line.split()[1:] if "=" in tok)
            kv.setdefault("rows", "packed")
            if all(kv.get(k) == v for k, v in want.items() if k != "library_version"):
                if kv.get("library_version") == want["library_version"]:
                    return (float(kv["fetch_bytes_per_launch"]) + float(kv["write_bytes_per_launch"]),
                            f"profiles/{name}")
                stale = f"profiles/{name} was taken with library version {kv.get('library_version')}, this is {library_version}"
    return None, stale or "no rocprofv3 counter summary under profiles/ for this workload, format, sparsity and launch mode"


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
