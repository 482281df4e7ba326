"""GPU parity of teal_sparse_gemv_bf16_stack: several independent grouped calls in one
launch.  Each group must give, bit for bit, what its own teal_sparse_gemv_bf16_multi call
gives, agree with the CPU oracle (relative L2 <= 2e-3), and leave its exact survivor
counts in its region of the workspace."""
import numpy as np
import pytest

import teal_inputs as ti
from oracle import teal_oracle as orc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-3
TIGHT = 2e-5


@pytest.fixture(scope="module")
def T():
    import paper_2408_14690_amd as T
    assert torch.cuda.is_available(), "these tests need the GPU"
    T.load_library()          # raises if the HIP library is not built: no fallback
    return T


def dev(a: np.ndarray):
    a = np.ascontiguousarray(a)
    if a.dtype in (np.uint16, np.float16):
        return torch.from_numpy(a.view(np.int16)).cuda()
    return torch.from_numpy(a).cuda()


def rel_l2(got, want):
    den = np.linalg.norm(want)
    if den == 0.0:
        return 0.0 if not np.any(got) else np.inf
    return float(np.linalg.norm(got.astype(np.float64) - want) / den)


class Stack:
    """Seeded groups: group g has len(ns[g]) matrices of widths ns[g] reading one x of length ms[g]."""

    def __init__(self, T, ms, ns, ps, seed, dists=None):
        self.T, self.ms, self.ns = T, ms, ns
        self.counts = [len(g) for g in ns]
        self.flat_n = [n for g in ns for n in g]
        self.x, self.w, self.t = [], [], []
        for g, (m, group) in enumerate(zip(ms, ns)):
            dist = dists[g] if dists else ("gaussian", "laplace")[g % 2]
            x = ti.make_x(m, seed + 100 * g, dist)
            self.x.append(x)
            for k, n in enumerate(group):
                self.w.append(ti.weights_bf16(n, m, seed=seed + 100 * g + k + 1))
                self.t.append(ti.quantile_threshold(x, ps[g][k]))
        self.xd = [dev(x) for x in self.x]
        self.wd = [dev(ti.to_input_channel_major(w)) for w in self.w]
        self.group_of = [g for g, c in enumerate(self.counts) for _ in range(c)]
        self.ws_bytes = T.teal_workspace_bytes_stack(self.counts, self.flat_n, ms)
        assert self.ws_bytes > 0
        self.ws = torch.zeros(self.ws_bytes, dtype=torch.uint8, device="cuda")
        self.region = np.cumsum([0] + [T.teal_workspace_bytes(m, sum(g)) for m, g in zip(ms, ns)])
        assert self.region[-1] == self.ws_bytes

    def run(self, t=None):
        T = self.T
        ys = [torch.full((n,), float("nan"), dtype=torch.float32, device="cuda") for n in self.flat_n]
        T.check(T.teal_sparse_gemv_bf16_stack(self.counts, self.wd, t or self.t, ys, self.flat_n,
                                              self.xd, self.ms, self.ws))
        torch.cuda.synchronize()
        return [y.cpu().numpy() for y in ys]

    def run_separately(self, t=None):
        """The groups' own grouped calls, one after the other."""
        T, t = self.T, t or self.t
        out, first = [], 0
        for g, c in enumerate(self.counts):
            sl = slice(first, first + c)
            n_total = sum(self.flat_n[sl])
            ws = torch.zeros(T.teal_workspace_bytes(self.ms[g], n_total), dtype=torch.uint8, device="cuda")
            ys = [torch.full((n,), float("nan"), dtype=torch.float32, device="cuda") for n in self.flat_n[sl]]
            T.check(T.teal_sparse_gemv_bf16_multi(self.wd[sl], t[sl], ys, self.flat_n[sl], self.xd[g],
                                                  self.ms[g], ws))
            torch.cuda.synchronize()
            out += [y.cpu().numpy() for y in ys]
            first += c
        return out

    def survivors(self):
        off = self.T.teal_survivors_offset()
        got, host = [], self.ws.cpu().numpy()
        for g, c in enumerate(self.counts):
            at = int(self.region[g]) + off
            got += host[at:at + 4 * c].view(np.int32).tolist()
        return got

    def oracle_counts(self, t=None):
        t = t or self.t
        return [orc.sparsify(self.x[g], tk)[3] for g, tk in zip(self.group_of, t)]

    def check_against_oracle(self, ys, t=None, tol=TIGHT):
        t = t or self.t
        for k, (g, y) in enumerate(zip(self.group_of, ys)):
            want = orc.sparse_gemv_bf16(self.w[k], self.x[g], t[k])
            assert rel_l2(y, want) <= tol, (k, g)
            assert tol <= TOL_BF16


def test_mixed_groups_against_oracle_and_separate_calls(T):
    """Groups of 1 to 4 matrices, different input lengths and widths (ragged right edges, a
    ragged last slice), different thresholds per matrix."""
    ms = [1000, 4096, 264, 2048]
    ns = [[520, 72], [1024], [4096, 1024, 1024, 72], [8, 2056]]
    ps = [[0.5, 0.25], [0.4], [0.5, 0.4, 0.25, 0.9], [0.65, 0.5]]
    s = Stack(T, ms, ns, ps, seed=4100)
    ys = s.run()
    s.check_against_oracle(ys)
    assert s.survivors() == s.oracle_counts()
    for k, (a, b) in enumerate(zip(ys, s.run_separately())):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), k


def test_sixteen_groups_and_every_row_width(T):
    """The most groups a call takes; widths chosen so that launches with 16, 32 and 64 lanes
    per weight row all occur in the one launch."""
    ms = [512 + 64 * g for g in range(16)]
    widths = [128, 4096, 8192, 16384]
    ns = [[widths[g % 4]] if g % 3 else [widths[g % 4], 256] for g in range(16)]
    ps = [[0.5] * len(g) for g in ns]
    plans = {T.teal_gemv_plan_multi(16, m, g)[1]["lanes_per_row"] if len(g) > 1
             else T.teal_gemv_plan(16, m, g[0])[1]["lanes_per_row"] for m, g in zip(ms, ns)}
    assert plans == {16, 32, 64}, plans
    s = Stack(T, ms, ns, ps, seed=4200)
    ys = s.run()
    s.check_against_oracle(ys)
    assert s.survivors() == s.oracle_counts()
    for k, (a, b) in enumerate(zip(ys, s.run_separately())):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), k


def test_degenerate_groups_and_repeated_calls(T):
    """A group in which nothing survives (y all zeros), a dense group (t = 0), a tie at the
    threshold; then a second call on the same workspace with other thresholds."""
    ms = [640, 640, 1536]
    ns = [[264], [264, 520], [1032]]
    ps = [[0.5], [0.0, 0.5], [0.4]]
    s = Stack(T, ms, ns, ps, seed=4300)
    t = list(s.t)
    t[0] = 1.0e4                                   # above every |x|
    t[3] = float(np.abs(s.x[2].astype(np.float32))[17])   # equals an entry: dropped (strict >)
    ys = s.run(t)
    assert not np.any(ys[0])
    s.check_against_oracle(ys, t)
    counts = s.oracle_counts(t)
    assert counts[0] == 0 and counts[1] == int(np.count_nonzero(s.x[1]))
    assert s.survivors() == counts
    t2 = [ti.quantile_threshold(s.x[g], p) for g, p in zip(s.group_of, (0.25, 0.8, 0.65, 0.9))]
    ys2 = s.run(t2)
    s.check_against_oracle(ys2, t2)
    assert s.survivors() == s.oracle_counts(t2)


def test_llama2_7b_block_in_one_launch(T):
    """The four groups of a Llama-2-7B-shaped block (Appendix A.3) at 50 %: bitwise the
    separate grouped calls, exact survivor counts, sampled outputs against the oracle."""
    shapes = ti.LAYER_SHAPES["llama2_7b"]
    groups = [("q", "k", "v"), ("o",), ("gate", "up"), ("down",)]
    ms = [shapes[g[0]][1] for g in groups]
    ns = [[shapes[p][0] for p in g] for g in groups]
    ps = [[0.5] * len(g) for g in groups]
    s = Stack(T, ms, ns, ps, seed=4400, dists=["gaussian", "laplace", "gaussian", "laplace"])
    ys = s.run()
    assert s.survivors() == s.oracle_counts()
    for k, (a, b) in enumerate(zip(ys, s.run_separately())):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), k
    rng = np.random.default_rng(44)
    for k, (g, y) in enumerate(zip(s.group_of, ys)):
        rows = np.sort(rng.choice(s.flat_n[k], size=96, replace=False))
        want = orc.sparse_gemv_bf16_rows(s.w[k], s.x[g], s.t[k], rows)
        assert rel_l2(y[rows], want) <= TIGHT, k


def test_argument_errors_leave_outputs_alone(T):
    ms, ns = [512, 512], [[128], [128]]
    s = Stack(T, ms, ns, [[0.5], [0.5]], seed=4500)
    ys = [torch.full((128,), 3.0, dtype=torch.float32, device="cuda") for _ in range(2)]
    small = s.ws[:s.ws_bytes - 256]
    assert T.teal_sparse_gemv_bf16_stack(s.counts, s.wd, s.t, ys, s.flat_n, s.xd, ms, small) \
        == T.TEAL_ERR_WORKSPACE
    assert T.teal_sparse_gemv_bf16_stack(s.counts, s.wd, [0.1, -1.0], ys, s.flat_n, s.xd, ms, s.ws) \
        == T.TEAL_ERR_THRESHOLD
    torch.cuda.synchronize()
    assert all(bool((y == 3.0).all()) for y in ys)


@pytest.mark.parametrize("fmt", ["w8", "w4"])
def test_quantised_stacks(T, fmt):
    """int8 / int4 groups in one launch: bitwise the groups' own grouped calls, within
    tolerance of the oracle on the same (q, scale), exact survivor counts; two calls in a
    row on one workspace."""
    ms = [1024, 4096, 640, 2048]
    ns = [[544, 96], [1024], [4096, 1024, 1024, 96], [32, 2080]]
    ps = [[0.5, 0.25], [0.4], [0.5, 0.4, 0.25, 0.9], [0.65, 0.0]]
    counts = [len(g) for g in ns]
    flat_n = [n for g in ns for n in g]
    group_of = [g for g, c in enumerate(counts) for _ in range(c)]
    xs = [ti.make_x(m, 4600 + g, ("gaussian", "laplace")[g % 2]) for g, m in enumerate(ms)]
    qs, scs, ts = [], [], []
    for k, (g, n) in enumerate(zip(group_of, flat_n)):
        w = ti.weights_bf16(n, ms[g], seed=4700 + k)
        qs.append(ti.quantize_w8(w) if fmt == "w8" else ti.quantize_w4(w, 128))
        ts.append(ti.quantile_threshold(xs[g], ps[g][k - sum(counts[:g])]))
    qd = [dev(q) for q, _ in qs]
    sd = [dev(sc) for _, sc in qs]
    xd = [dev(x) for x in xs]
    ws = torch.zeros(T.teal_workspace_bytes_stack(counts, flat_n, ms), dtype=torch.uint8, device="cuda")
    region = np.cumsum([0] + [T.teal_workspace_bytes(m, sum(g)) for m, g in zip(ms, ns)])

    def stack(t):
        ys = [torch.full((n,), float("nan"), dtype=torch.float32, device="cuda") for n in flat_n]
        if fmt == "w8":
            T.check(T.teal_sparse_gemv_w8_stack(counts, qd, sd, t, ys, flat_n, xd, ms, ws))
        else:
            T.check(T.teal_sparse_gemv_w4_stack(counts, qd, sd, 128, t, ys, flat_n, xd, ms, ws))
        torch.cuda.synchronize()
        host = ws.cpu().numpy()
        off = T.teal_survivors_offset()
        got = []
        for g, c in enumerate(counts):
            at = int(region[g]) + off
            got += host[at:at + 4 * c].view(np.int32).tolist()
        return [y.cpu().numpy() for y in ys], got

    def separately(t):
        out, first = [], 0
        for g, c in enumerate(counts):
            sl = slice(first, first + c)
            w1 = torch.zeros(T.teal_workspace_bytes(ms[g], sum(flat_n[sl])), dtype=torch.uint8, device="cuda")
            ys = [torch.full((n,), float("nan"), dtype=torch.float32, device="cuda") for n in flat_n[sl]]
            if fmt == "w8":
                T.check(T.teal_sparse_gemv_w8_multi(qd[sl], sd[sl], t[sl], ys, flat_n[sl], xd[g], ms[g], w1))
            else:
                T.check(T.teal_sparse_gemv_w4_multi(qd[sl], sd[sl], 128, t[sl], ys, flat_n[sl], xd[g],
                                                    ms[g], w1))
            torch.cuda.synchronize()
            out += [y.cpu().numpy() for y in ys]
            first += c
        return out

    for t in (ts, [ti.quantile_threshold(xs[g], 0.8) for g in group_of]):
        ys, counts_got = stack(t)
        assert counts_got == [orc.sparsify(xs[g], tk)[3] for g, tk in zip(group_of, t)]
        for k, (a, b) in enumerate(zip(ys, separately(t))):
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), k
        for k, (g, y) in enumerate(zip(group_of, ys)):
            q, sc = qs[k]
            want = (orc.sparse_gemv_w8(q, sc, xs[g], t[k]) if fmt == "w8"
                    else orc.sparse_gemv_w4(q, sc, 128, xs[g], t[k]))
            assert rel_l2(y, want) <= TIGHT, (k, g)


def test_quantised_stack_argument_errors(T):
    m, n = 512, 128
    x = dev(ti.gaussian_x(m, 4800))
    q8, s8 = ti.quantize_w8(ti.weights_bf16(n, m, seed=4801))
    q4, s4 = ti.quantize_w4(ti.weights_bf16(n, m, seed=4802), 128)
    y = torch.full((n,), 3.0, dtype=torch.float32, device="cuda")
    ws = torch.zeros(T.teal_workspace_bytes_stack([1], [n], [m]), dtype=torch.uint8, device="cuda")
    assert T.teal_sparse_gemv_w4_stack([1], [dev(q4)], [dev(s4)], 64, [0.1], [y], [n], [x], [m], ws) \
        == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_sparse_gemv_w8_stack([1], [dev(q8)], [dev(s8)], [float("inf")], [y], [n], [x], [m], ws) \
        == T.TEAL_ERR_THRESHOLD
    assert T.teal_sparse_gemv_w8_stack([1], [dev(q8)], [dev(s8)], [0.1], [y], [n], [x], [m], ws[:4096]) \
        == T.TEAL_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((y == 3.0).all())


@pytest.mark.parametrize("seed", range(6))
def test_random_stacks(T, seed):
    """Random numbers of groups and matrices, input lengths (ragged), widths and sparsity
    levels (including nothing dropped and everything dropped)."""
    rng = np.random.Generator(np.random.PCG64(5000 + seed))
    groups = int(rng.integers(1, 17))
    ms, ns, ps = [], [], []
    for _ in range(groups):
        m = int(rng.integers(1, 24)) * 128 + (int(rng.integers(1, 128)) if rng.random() < 0.5 else 0)
        count = int(rng.integers(1, 5))
        ms.append(m)
        ns.append([int(rng.integers(1, 160)) * 8 for _ in range(count)])
        ps.append([float(rng.choice([0.0, 0.1, 0.5, 0.77, 0.95, 1.0])) for _ in range(count)])
    s = Stack(T, ms, ns, ps, seed=5100 + 1000 * seed)
    ys = s.run()
    s.check_against_oracle(ys)
    assert s.survivors() == s.oracle_counts()
    for k, (a, b) in enumerate(zip(ys, s.run_separately())):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), k
