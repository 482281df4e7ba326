"""GPU parity of the MLP of a block in one launch (Appendix A.3) through the C ABI.

What is unique is compared exactly: gate, up and y bit for bit against the library's own
separate calls with the same launch shapes (the grouped gate + up product, the producer of
h = fp16(SiLU(gate) * up), the W_down product), the three survivor counts against the
oracle's masks.  Against the fp64 oracle: gate and up within the parity bar of the plain
product; y within the bar of the oracle's W_down step applied to the gate / up values the
GPU produced (h decides an integer mask, so both sides form it from the same binary32
inputs in the same stated arithmetic)."""
import numpy as np
import pytest

import teal_inputs as ti
from oracle import teal_oracle as orc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-3
TOL_WQ = 5e-3
TIGHT = 2e-5
TIGHT_WQ = 1e-4


@pytest.fixture(scope="module")
def T():
    import paper_2408_14690_amd as T
    assert torch.cuda.is_available(), "these tests need the GPU"
    T.load_library()
    return T


def dev(a):
    a = np.ascontiguousarray(a)
    if a.dtype in (np.uint16, np.float16):
        return torch.from_numpy(a.view(np.int16)).cuda()
    return torch.from_numpy(a).cuda()


def rel_l2(got, want):
    den = np.linalg.norm(want)
    if den == 0.0:
        return 0.0 if not np.any(got) else np.inf
    return float(np.linalg.norm(got.astype(np.float64) - want) / den)


def bits_equal(a, b):
    return bool(torch.equal(a.view(torch.int32), b.view(torch.int32)))


class Mlp:
    """Seeded weights and input of one synthetic MLP, resident on the device (bf16)."""

    def __init__(self, T, m, f, d, seed, p_gate=0.5, p_up=0.5, p_down=0.5, x_scale=1.0):
        self.m, self.f, self.d = m, f, d
        self.w = [ti.weights_bf16(f, m, seed), ti.weights_bf16(f, m, seed + 1),
                  ti.weights_bf16(d, f, seed + 2, std=0.02)]
        self.x = ti.gaussian_x(m, seed + 3)
        self.t_gate = ti.quantile_threshold(self.x, p_gate)
        self.t_up = ti.quantile_threshold(self.x, p_up)
        self.p_down = p_down
        self.wt = []
        for w, (n, k) in zip(self.w, ((f, m), (f, m), (d, f))):
            wd = dev(w)
            wt = torch.empty((k, n), dtype=torch.int16, device="cuda")
            T.check(T.teal_pack_bf16(wd, wt, k, n))
            self.wt.append(wt)
        self.xd = dev(self.x)
        torch.cuda.synchronize()

    def t_down_from(self, gate, up):
        """The threshold of W_down: the p_down quantile of |h| for the h these gate / up give
        (h from the oracle's producer; any non-negative finite t would do for parity)."""
        h = orc.swiglu_f16(gate, up)
        return ti.quantile_threshold(h, self.p_down)


def run_mlp(T, M, t_down, ws, shape=None):
    gate = torch.full((M.f,), float("nan"), dtype=torch.float32, device="cuda")
    up = torch.full((M.f,), float("nan"), dtype=torch.float32, device="cuda")
    y = torch.full((M.d,), float("nan"), dtype=torch.float32, device="cuda")
    T.check(T.teal_sparse_mlp_bf16(M.wt[0], M.wt[1], M.wt[2], M.xd, M.t_gate, M.t_up, t_down, gate,
                                   up, y, M.m, M.f, M.d, ws, shape=shape))
    torch.cuda.synchronize()
    return gate, up, y


def status_word(T, M, ws):
    off = T.teal_mlp_status_offset(M.m, M.f, M.d)
    return int(ws[off:off + 4].view(torch.int32).item())


def survivor_counts(T, M, ws):
    off = T.teal_survivors_offset()
    g, u = ws[off:off + 8].view(torch.int32).cpu().tolist()
    at = T.teal_mlp_down_region_offset(M.m, M.f) + off
    return g, u, int(ws[at:at + 4].view(torch.int32).item())


def separate_calls(T, M, t_down, sh):
    """The same three products as separate launches with the shapes `sh` names."""
    f, m, d = M.f, M.m, M.d
    outs = []
    for k, t in ((0, M.t_gate), (1, M.t_up)):
        yk = torch.full((f,), float("nan"), dtype=torch.float32, device="cuda")
        ws = torch.zeros(T.teal_workspace_bytes(m, f), dtype=torch.uint8, device="cuda")
        T.check(T.teal_sparse_gemv_bf16_ex(M.wt[k], M.xd, t, yk, m, f, ws,
                                           lanes_per_row=sh.gu_lanes_per_row,
                                           tile_cols=sh.gu_tile_cols, splits=sh.gu_splits,
                                           waves=8, unroll=4))
        outs.append(yk)
    h = torch.empty(f, dtype=torch.int16, device="cuda")
    T.check(T.teal_swiglu_f16(outs[0], outs[1], h, f))
    y = torch.full((d,), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.zeros(T.teal_workspace_bytes(f, d), dtype=torch.uint8, device="cuda")
    T.check(T.teal_sparse_gemv_bf16_ex(M.wt[2], h, t_down, y, f, d, ws,
                                       lanes_per_row=sh.down_lanes_per_row,
                                       tile_cols=sh.down_tile_cols, splits=sh.down_splits,
                                       waves=8, unroll=4))
    torch.cuda.synchronize()
    return outs[0], outs[1], y


def check_against_oracle(T, M, gate, up, y, t_down, ws, rows=None):
    g_np, u_np = gate.cpu().numpy(), up.cpu().numpy()
    if rows is None:
        assert rel_l2(g_np, orc.sparse_gemv_bf16(M.w[0], M.x, M.t_gate)) <= TIGHT
        assert rel_l2(u_np, orc.sparse_gemv_bf16(M.w[1], M.x, M.t_up)) <= TIGHT
    else:
        assert rel_l2(g_np[rows], orc.sparse_gemv_bf16_rows(M.w[0], M.x, M.t_gate, rows)) <= TIGHT
        assert rel_l2(u_np[rows], orc.sparse_gemv_bf16_rows(M.w[1], M.x, M.t_up, rows)) <= TIGHT
    want = orc.sparse_gemv_bf16_swiglu(M.w[2], g_np, u_np, t_down)
    err = rel_l2(y.cpu().numpy(), want)
    assert err <= TIGHT and err <= TOL_BF16
    h = orc.swiglu_f16(g_np, u_np)
    counts = (orc.sparsify(M.x, M.t_gate)[3], orc.sparsify(M.x, M.t_up)[3], orc.sparsify(h, t_down)[3])
    assert survivor_counts(T, M, ws) == counts
    assert status_word(T, M, ws) == 0


SMALL = [
    # m, f, d, shape overrides: several tiles, ragged right edges, ragged last K-slice and phase
    (520, 1224, 264, dict(gu_lanes_per_row=16, gu_tile_cols=120, gu_splits=3, gu_phase_tiles=2,
                          down_lanes_per_row=16, down_tile_cols=72, down_splits=5)),
    (1000, 2048, 1032, dict(gu_lanes_per_row=32, gu_tile_cols=256, gu_splits=1, gu_phase_tiles=3,
                            down_lanes_per_row=64, down_tile_cols=512, down_splits=7)),
    (1024, 1536, 512, dict(gu_lanes_per_row=64, gu_tile_cols=512, gu_splits=4, gu_phase_tiles=1,
                           down_lanes_per_row=16, down_tile_cols=128, down_splits=1)),
    (777, 840, 8, dict(gu_lanes_per_row=16, gu_tile_cols=8, gu_splits=2, gu_phase_tiles=50,
                       down_lanes_per_row=16, down_tile_cols=8, down_splits=3)),
    (2048, 4096, 2048, {}),
]


@pytest.mark.parametrize("m,f,d,over", SMALL)
def test_mlp_matches_separate_calls_and_the_oracle(T, m, f, d, over):
    M = Mlp(T, m, f, d, seed=31000 + m, p_gate=0.5, p_up=0.4, p_down=0.6)
    st, sh = T.teal_mlp_plan(16, m, f, d)
    T.check(st)
    for k, v in over.items():
        setattr(sh, k, v)
    ws = torch.zeros(T.teal_workspace_bytes_mlp(m, f, d), dtype=torch.uint8, device="cuda")
    # a first pass gives gate / up, from which the threshold of W_down is taken
    g0, u0, _ = run_mlp(T, M, 0.0, ws, sh)
    t_down = M.t_down_from(g0.cpu().numpy(), u0.cpu().numpy())
    gate, up, y = run_mlp(T, M, t_down, ws, sh)              # the same workspace again
    rg, ru, ry = separate_calls(T, M, t_down, sh)
    assert bits_equal(gate, rg) and bits_equal(up, ru) and bits_equal(y, ry)
    check_against_oracle(T, M, gate, up, y, t_down, ws)
    # dense W_down (t = 0) from the first pass, against the oracle as well
    _, _, y0 = run_mlp(T, M, 0.0, ws, sh)
    want0 = orc.sparse_gemv_bf16_swiglu(M.w[2], gate.cpu().numpy(), up.cpu().numpy(), 0.0)
    assert rel_l2(y0.cpu().numpy(), want0) <= TIGHT


@pytest.mark.parametrize("m,f,d", [(4096, 14336, 4096), (4096, 11008, 4096)])
def test_library_shape_is_bitwise_the_separate_calls(T, m, f, d):
    """shape = NULL: the launch shape teal_mlp_plan reports; bitwise the separate calls with it."""
    M = Mlp(T, m, f, d, seed=32000 + f)
    st, sh = T.teal_mlp_plan(16, m, f, d)
    T.check(st)
    ws = torch.zeros(T.teal_workspace_bytes_mlp(m, f, d), dtype=torch.uint8, device="cuda")
    g0, u0, _ = run_mlp(T, M, 0.0, ws)
    t_down = M.t_down_from(g0.cpu().numpy(), u0.cpu().numpy())
    gate, up, y = run_mlp(T, M, t_down, ws)
    rg, ru, ry = separate_calls(T, M, t_down, sh)
    assert bits_equal(gate, rg) and bits_equal(up, ru) and bits_equal(y, ry)
    rows = np.unique(np.concatenate([np.arange(0, f, 97), [f - 1]])).astype(np.int32)
    check_against_oracle(T, M, gate, up, y, t_down, ws, rows=rows)


def test_shapes_of_the_grouped_calls_are_bitwise_those_calls(T):
    """With the launch shapes the grouped gate + up call and the fused W_down call pick
    themselves, the one-launch MLP is bitwise those two calls."""
    m, f, d = 4096, 14336, 4096
    M = Mlp(T, m, f, d, seed=32000)
    st, sh = T.teal_mlp_plan(16, m, f, d)
    st, gu = T.teal_gemv_plan_multi(16, m, [f, f])
    sh.gu_lanes_per_row, sh.gu_tile_cols, sh.gu_splits = gu["lanes_per_row"], gu["tile_cols"], gu["splits"]
    ws = torch.zeros(T.teal_workspace_bytes_mlp(m, f, d), dtype=torch.uint8, device="cuda")
    g0, u0, _ = run_mlp(T, M, 0.0, ws, sh)
    t_down = M.t_down_from(g0.cpu().numpy(), u0.cpu().numpy())
    gate, up, y = run_mlp(T, M, t_down, ws, sh)
    rg = torch.empty(f, dtype=torch.float32, device="cuda")
    ru = torch.empty(f, dtype=torch.float32, device="cuda")
    ws2 = torch.zeros(T.teal_workspace_bytes(m, 2 * f), dtype=torch.uint8, device="cuda")
    T.check(T.teal_sparse_gemv_bf16_multi([M.wt[0], M.wt[1]], [M.t_gate, M.t_up], [rg, ru], [f, f],
                                          M.xd, m, ws2))
    ry = torch.empty(d, dtype=torch.float32, device="cuda")
    ws3 = torch.zeros(T.teal_workspace_bytes(f, d), dtype=torch.uint8, device="cuda")
    T.check(T.teal_sparse_gemv_bf16_swiglu(M.wt[2], rg, ru, t_down, ry, f, d, ws3))
    torch.cuda.synchronize()
    assert bits_equal(gate, rg) and bits_equal(up, ru) and bits_equal(y, ry)


@pytest.mark.parametrize("over", [
    dict(gu_phase_tiles=4),
    dict(gu_lanes_per_row=16, gu_tile_cols=128, gu_splits=4, gu_phase_tiles=14,
         down_lanes_per_row=32, down_tile_cols=256, down_splits=16),
    dict(gu_lanes_per_row=32, gu_tile_cols=256, gu_splits=2, gu_phase_tiles=7, extra_lds_bytes=40960),
])
def test_full_size_mlp_in_phases(T, over):
    """Llama-3-8B-sized MLP with more blocks than fit the chip at once, the gate / up blocks in
    phases: the W_down blocks are dispatched as earlier blocks retire and wait for their tiles."""
    m, f, d = 4096, 14336, 4096
    M = Mlp(T, m, f, d, seed=32000)
    st, sh = T.teal_mlp_plan(16, m, f, d)
    for k, v in over.items():
        setattr(sh, k, v)
    ws = torch.zeros(T.teal_workspace_bytes_mlp(m, f, d), dtype=torch.uint8, device="cuda")
    g0, u0, _ = run_mlp(T, M, 0.0, ws, sh)
    t_down = M.t_down_from(g0.cpu().numpy(), u0.cpu().numpy())
    for _ in range(3):                                       # back to back on one workspace
        gate, up, y = run_mlp(T, M, t_down, ws, sh)
    rg, ru, ry = separate_calls(T, M, t_down, sh)
    assert bits_equal(gate, rg) and bits_equal(up, ru) and bits_equal(y, ry)
    rows = np.unique(np.concatenate([np.arange(0, f, 211), [f - 1]])).astype(np.int32)
    check_against_oracle(T, M, gate, up, y, t_down, ws, rows=rows)


def test_70b_sized_mlp(T):
    """The MLP of the 70B-shaped block (8192 -> 28672 -> 8192) in one launch, the library's
    shape: bitwise the separate calls, sampled gate / up outputs and all of y against the
    oracle, survivor counts exact."""
    m, f, d = 8192, 28672, 8192
    M = Mlp(T, m, f, d, seed=35000)
    st, sh = T.teal_mlp_plan(16, m, f, d)
    T.check(st)
    ws = torch.zeros(T.teal_workspace_bytes_mlp(m, f, d), dtype=torch.uint8, device="cuda")
    g0, u0, _ = run_mlp(T, M, 0.0, ws)
    t_down = M.t_down_from(g0.cpu().numpy(), u0.cpu().numpy())
    gate, up, y = run_mlp(T, M, t_down, ws)
    rg, ru, ry = separate_calls(T, M, t_down, sh)
    assert bits_equal(gate, rg) and bits_equal(up, ru) and bits_equal(y, ry)
    rows = np.unique(np.concatenate([np.arange(0, f, 401), [f - 1]])).astype(np.int32)
    check_against_oracle(T, M, gate, up, y, t_down, ws, rows=rows)


def test_nothing_survives_and_everything_survives(T):
    m, f, d = 1024, 2048, 512
    M = Mlp(T, m, f, d, seed=33000)
    ws = torch.zeros(T.teal_workspace_bytes_mlp(m, f, d), dtype=torch.uint8, device="cuda")
    # a threshold above every |x|: gate = up = 0, h = 0, y = 0
    M.t_gate = M.t_up = 60000.0
    gate, up, y = run_mlp(T, M, 0.5, ws)
    assert not gate.any() and not up.any() and not y.any()
    assert survivor_counts(T, M, ws) == (0, 0, 0)
    # dense everywhere
    M.t_gate = M.t_up = 0.0
    gate, up, y = run_mlp(T, M, 0.0, ws)
    check_against_oracle(T, M, gate, up, y, 0.0, ws)


def test_a_wait_that_expires_ends_the_kernel_and_sets_the_status_word(T):
    """The bounded wait, forced from the host: with a limit of zero polls a block of W_down
    that does not find its inputs finished when it starts gives up at once.  Every block
    still runs to its end; the status word tells the caller, who zero-fills the workspace
    before the next call."""
    m, f, d = 4096, 14336, 4096
    M = Mlp(T, m, f, d, seed=32000)
    st, sh = T.teal_mlp_plan(16, m, f, d)
    ws = torch.zeros(T.teal_workspace_bytes_mlp(m, f, d), dtype=torch.uint8, device="cuda")
    gate, up, y_good = run_mlp(T, M, 0.1, ws, sh)
    assert status_word(T, M, ws) == 0
    sh.spin_limit = 0
    run_mlp(T, M, 0.1, ws, sh)         # all blocks resident at once: W_down's start before gate / up end
    assert status_word(T, M, ws) == 1
    ws.zero_()
    sh.spin_limit = 1 << 20
    gate2, up2, y2 = run_mlp(T, M, 0.1, ws, sh)
    assert status_word(T, M, ws) == 0
    assert bits_equal(gate, gate2) and bits_equal(up, up2) and bits_equal(y_good, y2)


def quantised(T, fmt, m, f, d, seed):
    ws_ = [ti.weights_bf16(f, m, seed), ti.weights_bf16(f, m, seed + 1), ti.weights_bf16(d, f, seed + 2)]
    q = [ti.quantize_w8(w) if fmt == "w8" else ti.quantize_w4(w, 128) for w in ws_]
    x = ti.gaussian_x(m, seed + 3)
    return q, x


@pytest.mark.parametrize("fmt", ["w8", "w4"])
@pytest.mark.parametrize("m,f,d,over", [
    (1024, 2048, 1024, {}),
    (1024, 3072, 512, dict(gu_phase_tiles=2, gu_splits=2, down_splits=6)),
    (4096, 14336, 4096, dict(gu_phase_tiles=3)),
])
def test_quantised_mlp(T, fmt, m, f, d, over):
    bits = 8 if fmt == "w8" else 4
    q, x = quantised(T, fmt, m, f, d, 34000 + m + f)
    t_gate, t_up = ti.quantile_threshold(x, 0.5), ti.quantile_threshold(x, 0.4)
    st, sh = T.teal_mlp_plan(bits, m, f, d)
    T.check(st)
    for k, v in over.items():
        setattr(sh, k, v)
    qd = [dev(a) for a, _ in q]
    sd = [dev(s) for _, s in q]
    xd = dev(x)
    ws = torch.zeros(T.teal_workspace_bytes_mlp(m, f, d), dtype=torch.uint8, device="cuda")

    def run(t_down):
        gate = torch.full((f,), float("nan"), dtype=torch.float32, device="cuda")
        up = torch.full((f,), float("nan"), dtype=torch.float32, device="cuda")
        y = torch.full((d,), float("nan"), dtype=torch.float32, device="cuda")
        if fmt == "w8":
            T.check(T.teal_sparse_mlp_w8(qd[0], qd[1], qd[2], sd[0], sd[1], sd[2], xd, t_gate, t_up,
                                         t_down, gate, up, y, m, f, d, ws, shape=sh))
        else:
            T.check(T.teal_sparse_mlp_w4(qd[0], qd[1], qd[2], sd[0], sd[1], sd[2], 128, xd, t_gate,
                                         t_up, t_down, gate, up, y, m, f, d, ws, shape=sh))
        torch.cuda.synchronize()
        return gate, up, y

    g0, u0, _ = run(0.0)
    h = orc.swiglu_f16(g0.cpu().numpy(), u0.cpu().numpy())
    t_down = ti.quantile_threshold(h, 0.5)
    gate, up, y = run(t_down)
    gate, up, y = run(t_down)
    off = T.teal_mlp_status_offset(m, f, d)
    assert int(ws[off:off + 4].view(torch.int32).item()) == 0
    g_np, u_np = gate.cpu().numpy(), up.cpu().numpy()
    if fmt == "w8":
        want_g = orc.sparse_gemv_w8(q[0][0], q[0][1], x, t_gate)
        want_u = orc.sparse_gemv_w8(q[1][0], q[1][1], x, t_up)
    else:
        want_g = orc.sparse_gemv_w4(q[0][0], q[0][1], 128, x, t_gate)
        want_u = orc.sparse_gemv_w4(q[1][0], q[1][1], 128, x, t_up)
    assert rel_l2(g_np, want_g) <= TIGHT_WQ and rel_l2(u_np, want_u) <= TIGHT_WQ
    h = orc.swiglu_f16(g_np, u_np)
    if fmt == "w8":
        want_y = orc.sparse_gemv_w8(q[2][0], q[2][1], h, t_down)
    else:
        want_y = orc.sparse_gemv_w4(q[2][0], q[2][1], 128, h, t_down)
    err = rel_l2(y.cpu().numpy(), want_y)
    assert err <= TIGHT_WQ and err <= TOL_WQ
    # bitwise the format's own separate calls when the shapes are the library's
    if not over:
        rg = torch.empty(f, dtype=torch.float32, device="cuda")
        ru = torch.empty(f, dtype=torch.float32, device="cuda")
        ry = torch.empty(d, dtype=torch.float32, device="cuda")
        ws2 = torch.zeros(T.teal_workspace_bytes(m, 2 * f), dtype=torch.uint8, device="cuda")
        ws3 = torch.zeros(T.teal_workspace_bytes(f, d), dtype=torch.uint8, device="cuda")
        if fmt == "w8":
            T.check(T.teal_sparse_gemv_w8_multi([qd[0], qd[1]], [sd[0], sd[1]], [t_gate, t_up],
                                                [rg, ru], [f, f], xd, m, ws2))
            T.check(T.teal_sparse_gemv_w8_swiglu(qd[2], sd[2], rg, ru, t_down, ry, f, d, ws3))
        else:
            T.check(T.teal_sparse_gemv_w4_multi([qd[0], qd[1]], [sd[0], sd[1]], 128, [t_gate, t_up],
                                                [rg, ru], [f, f], xd, m, ws2))
            T.check(T.teal_sparse_gemv_w4_swiglu(qd[2], sd[2], 128, rg, ru, t_down, ry, f, d, ws3))
        torch.cuda.synchronize()
        assert bits_equal(gate, rg) and bits_equal(up, ru) and bits_equal(y, ry)
    counts = (orc.sparsify(x, t_gate)[3], orc.sparsify(x, t_up)[3], orc.sparsify(h, t_down)[3])
    o = T.teal_survivors_offset()
    at = T.teal_mlp_down_region_offset(m, f) + o
    got = tuple(ws[o:o + 8].view(torch.int32).cpu().tolist()) + (int(ws[at:at + 4].view(torch.int32).item()),)
    assert got == counts


def padded(T, wt, pitch):
    """The same matrix stored with rows `pitch` elements apart, the padding holding bf16 NaNs
    (0x7FC0): a kernel that read it into a sum would show it."""
    k, n = wt.shape
    out = torch.full((k, pitch), 0x7FC0, dtype=torch.int16, device="cuda")
    out[:, :n] = wt
    return out


@pytest.mark.parametrize("m,f,d,pg,pd,over", [
    (520, 1224, 264, 1224 + 8, 264 + 40, dict(gu_lanes_per_row=16, gu_tile_cols=120, gu_splits=3,
                                             down_lanes_per_row=16, down_tile_cols=72, down_splits=5)),
    (1024, 1536, 512, 1536 + 128, 0, dict(gu_lanes_per_row=64, gu_tile_cols=512, gu_splits=4,
                                         down_lanes_per_row=16, down_tile_cols=128, down_splits=1)),
    (4096, 14336, 4096, 14336 + 128, 4096 + 128, {}),
    # 70B-sized: gate / up without split-K, a block compacting all 8192 channels
    (8192, 28672, 8192, 28672 + 128, 8192 + 128, dict(gu_lanes_per_row=32, gu_tile_cols=256, gu_splits=1)),
])
def test_padded_rows_give_the_same_bits(T, m, f, d, pg, pd, over):
    """Row pitches above the row length (teal_mlp_shape): gate, up and y are bit for bit those
    of the packed layout, the padding is never read into a result, and teal_pack_bf16_pitch
    writes that layout."""
    M = Mlp(T, m, f, d, seed=36000 + m)
    st, sh = T.teal_mlp_plan(16, m, f, d)
    T.check(st)
    assert sh.gu_row_pitch == 0 and sh.down_row_pitch == 0
    for k, v in over.items():
        setattr(sh, k, v)
    ws = torch.zeros(T.teal_workspace_bytes_mlp(m, f, d), dtype=torch.uint8, device="cuda")
    g0, u0, _ = run_mlp(T, M, 0.0, ws, sh)
    t_down = M.t_down_from(g0.cpu().numpy(), u0.cpu().numpy())
    gate, up, y = run_mlp(T, M, t_down, ws, sh)
    check_against_oracle(T, M, gate, up, y, t_down, ws,
                         rows=None if f <= 4096 else np.arange(0, f, 193).astype(np.int32))
    rg, ru, ry = separate_calls(T, M, t_down, sh)
    assert bits_equal(gate, rg) and bits_equal(up, ru) and bits_equal(y, ry)
    packed = M.wt
    M.wt = [padded(T, packed[0], pg), padded(T, packed[1], pg),
            padded(T, packed[2], pd) if pd else packed[2]]
    sh.gu_row_pitch, sh.down_row_pitch = pg, pd
    gate2, up2, y2 = run_mlp(T, M, t_down, ws, sh)
    assert bits_equal(gate, gate2) and bits_equal(up, up2) and bits_equal(y, y2)
    assert status_word(T, M, ws) == 0
    # the pack step writes this layout and leaves the padding alone
    wt = torch.full((m, pg), 0x1234, dtype=torch.int16, device="cuda")
    T.check(T.teal_pack_bf16_pitch(dev(M.w[0]), wt, m, f, pg))
    torch.cuda.synchronize()
    assert torch.equal(wt[:, :f], packed[0]) and bool((wt[:, f:] == 0x1234).all())


def test_padded_rows_int8(T):
    m, f, d = 1024, 2048, 1024
    q, x = quantised(T, "w8", m, f, d, 36500)
    t = ti.quantile_threshold(x, 0.5)
    st, sh = T.teal_mlp_plan(8, m, f, d)
    T.check(st)
    qd = [dev(a) for a, _ in q]
    sd = [dev(s_) for _, s_ in q]
    xd = dev(x)
    ws = torch.zeros(T.teal_workspace_bytes_mlp(m, f, d), dtype=torch.uint8, device="cuda")

    def run(mats):
        outs = [torch.full((n,), float("nan"), dtype=torch.float32, device="cuda") for n in (f, f, d)]
        T.check(T.teal_sparse_mlp_w8(mats[0], mats[1], mats[2], sd[0], sd[1], sd[2], xd, t, t, 0.05,
                                     outs[0], outs[1], outs[2], m, f, d, ws, shape=sh))
        torch.cuda.synchronize()
        return outs

    want = run(qd)
    pg, pd = f + 256, d + 16

    def pad(a, pitch):
        out = torch.full((a.shape[0], pitch), 127, dtype=torch.int8, device="cuda")
        out[:, :a.shape[1]] = a
        return out

    sh.gu_row_pitch, sh.down_row_pitch = pg, pd
    got = run([pad(qd[0], pg), pad(qd[1], pg), pad(qd[2], pd)])
    assert all(bits_equal(a, b) for a, b in zip(want, got))


@pytest.mark.parametrize("fmt,m,f,d,want_gu", [
    ("w8", 4096, 14336, 4096, (8, 128, 1)),
    ("bf16", 8192, 28672, 8192, (32, 256, 1)),
])
def test_planned_shape_for_padded_rows(T, fmt, m, f, d, want_gu):
    """teal_mlp_plan told the row pitches picks narrow gate / up tiles without split-K; the
    launch in that shape matches the oracle, and gate / up are bit for bit those of the grouped
    call on the same padded rows (which plans the same shape)."""
    bits = 8 if fmt == "w8" else 16
    pad = 256 * 8 // bits
    pg, pd = f + pad, d + pad
    st, sh = T.teal_mlp_plan(bits, m, f, d, pg, pd)
    T.check(st)
    assert (sh.gu_lanes_per_row, sh.gu_tile_cols, sh.gu_splits) == want_gu
    assert (sh.gu_row_pitch, sh.down_row_pitch) == (pg, pd)
    grouped = T.teal_gemv_plan_multi_pitch(bits, m, [f, f], [pg, pg])[1]
    assert (grouped["lanes_per_row"], grouped["tile_cols"], grouped["splits"]) == want_gu
    ws = torch.zeros(T.teal_workspace_bytes_mlp(m, f, d), dtype=torch.uint8, device="cuda")
    ws2 = torch.zeros(T.teal_workspace_bytes(m, 2 * f), dtype=torch.uint8, device="cuda")
    outs = [torch.full((n,), float("nan"), dtype=torch.float32, device="cuda") for n in (f, f, d)]
    rg, ru = (torch.full((f,), float("nan"), dtype=torch.float32, device="cuda") for _ in range(2))
    rows = np.arange(0, f, 97).astype(np.int32)
    if fmt == "w8":
        q, x = quantised(T, "w8", m, f, d, 36700)
        t = ti.quantile_threshold(x, 0.5)

        def pad8(a, pitch):
            out = torch.full((a.shape[0], pitch), 127, dtype=torch.int8, device="cuda")
            out[:, :a.shape[1]] = dev(a)
            return out

        mats = [pad8(q[0][0], pg), pad8(q[1][0], pg), pad8(q[2][0], pd)]
        sd = [dev(s_) for _, s_ in q]
        xd = dev(x)

        def run(t_down):
            T.check(T.teal_sparse_mlp_w8(mats[0], mats[1], mats[2], sd[0], sd[1], sd[2], xd, t, t,
                                         t_down, outs[0], outs[1], outs[2], m, f, d, ws, shape=sh))
            torch.cuda.synchronize()

        run(0.0)
        h = orc.swiglu_f16(outs[0].cpu().numpy(), outs[1].cpu().numpy())
        t_down = ti.quantile_threshold(h, 0.5)
        run(t_down)
        T.check(T.teal_sparse_gemv_w8_multi_pitch(mats[:2], [pg, pg], sd[:2], [t, t], [rg, ru], [f, f],
                                                  xd, m, ws2))
        torch.cuda.synchronize()
        g_np, u_np = outs[0].cpu().numpy(), outs[1].cpu().numpy()
        assert rel_l2(g_np, orc.sparse_gemv_w8(q[0][0], q[0][1], x, t)) <= TIGHT_WQ
        assert rel_l2(u_np, orc.sparse_gemv_w8(q[1][0], q[1][1], x, t)) <= TIGHT_WQ
        h = orc.swiglu_f16(g_np, u_np)
        assert rel_l2(outs[2].cpu().numpy(), orc.sparse_gemv_w8(q[2][0], q[2][1], h, t_down)) <= TIGHT_WQ
    else:
        M = Mlp(T, m, f, d, seed=36800)
        M.wt = [padded(T, M.wt[0], pg), padded(T, M.wt[1], pg), padded(T, M.wt[2], pd)]
        g0, u0, _ = run_mlp(T, M, 0.0, ws, sh)
        t_down = M.t_down_from(g0.cpu().numpy(), u0.cpu().numpy())
        outs = list(run_mlp(T, M, t_down, ws, sh))
        check_against_oracle(T, M, outs[0], outs[1], outs[2], t_down, ws, rows=rows)
        T.check(T.teal_sparse_gemv_bf16_multi_pitch(M.wt[:2], [pg, pg], [M.t_gate, M.t_up], [rg, ru],
                                                    [f, f], M.xd, m, ws2))
        torch.cuda.synchronize()
    assert bits_equal(outs[0], rg) and bits_equal(outs[1], ru)
    off = T.teal_mlp_status_offset(m, f, d)
    assert int(ws[off:off + 4].view(torch.int32).item()) == 0
