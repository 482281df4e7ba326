"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs.  Masks, index lists and counts must be bit-exact;
y must agree to relative L2 <= 2e-3 (bf16 W) / 5e-3 (quantised W)."""
import numpy as np
import pytest

import teal_inputs as ti
from oracle import teal_oracle as orc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-3
TOL_WQ = 5e-3
# What fp32 accumulation of exact products should achieve; looser bars above are
# the contract, this one catches a wrong-but-close kernel (e.g. a dropped row).
TIGHT = 2e-5


@pytest.fixture(scope="module")
def T():
    import paper_2408_14690_amd as T
    assert torch.cuda.is_available(), "these tests need the GPU"
    T.load_library()          # raises if the HIP library is not built: no fallback
    return T


def dev(a: np.ndarray):
    """numpy -> device tensor of the same bytes (16-bit types travel as int16)."""
    a = np.ascontiguousarray(a)
    if a.dtype in (np.uint16, np.float16):
        return torch.from_numpy(a.view(np.int16)).cuda()
    return torch.from_numpy(a).cuda()


def rel_l2(got, want):
    den = np.linalg.norm(want)
    if den == 0.0:
        return 0.0 if not np.any(got) else np.inf
    return float(np.linalg.norm(got.astype(np.float64) - want) / den)


def workspace(T, m, n):
    # zero-filled once; every successful call leaves it ready for the next
    return torch.zeros(T.teal_workspace_bytes(m, n), dtype=torch.uint8, device="cuda")


def survivors(T, ws, count=1):
    """The survivor counts a completed call left in its workspace."""
    off = T.teal_survivors_offset()
    return ws[off:off + 4 * count].view(torch.int32).cpu().tolist()


def run_bf16(T, wt_dev, x_dev, t, m, n, ws, **shape):
    # poison y: the call must overwrite every element
    y = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    if shape:
        T.check(T.teal_sparse_gemv_bf16_ex(wt_dev, x_dev, t, y, m, n, ws, **shape))
    else:
        T.check(T.teal_sparse_gemv_bf16(wt_dev, x_dev, t, y, m, n, ws))
    torch.cuda.synchronize()
    return y.cpu().numpy()


# ---------------------------------------------------------------------------
# teal_sparsify
# ---------------------------------------------------------------------------

def gpu_sparsify(T, x, t):
    m = x.size
    xd = dev(x) if m else torch.empty(1, dtype=torch.int16, device="cuda")
    mask = torch.full((max(m, 1),), 7, dtype=torch.uint8, device="cuda")
    idx = torch.full((max(m, 1),), -1, dtype=torch.int32, device="cuda")
    count = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    T.check(T.teal_sparsify(xd, m, t, mask, idx, count))
    torch.cuda.synchronize()
    c = int(count.item())
    return mask.cpu().numpy()[:m], idx.cpu().numpy(), c


@pytest.mark.parametrize("m", [1, 63, 64, 65, 1000, 1024, 1025, 4096, 11008, 14336, 28672])
@pytest.mark.parametrize("dist", ["gaussian", "laplace"])
def test_sparsify_bit_exact(T, m, dist):
    x = ti.make_x(m, 7000 + m, dist)
    for p in (0.0, 0.25, 0.4, 0.5, 0.65, 0.9, 1.0):
        t = ti.quantile_threshold(x, p)
        _, mask_o, idx_o, count_o = orc.sparsify(x, t)
        mask, idx, count = gpu_sparsify(T, x, t)
        assert count == count_o
        assert np.array_equal(mask, mask_o)
        assert np.array_equal(idx[:count], idx_o)
        assert np.all(idx[count:] == -1)              # capacity beyond count untouched


@pytest.mark.parametrize("m", [7, 8, 9, 4097, 8191, 8193, 32768, 32775, 100003])
@pytest.mark.parametrize("x_off,mask_off", [(0, 0), (0, 3), (1, 0), (4, 1)])
def test_sparsify_every_alignment_and_long_vectors(T, m, x_off, mask_off):
    """x on and off a 16-byte boundary (eight channels per thread, or one), the mask on and
    off an 8-byte boundary, lengths around the vector width and beyond one group of passes."""
    x = ti.make_x(m, 7100 + m, "laplace")
    buf = torch.zeros(m + 8, dtype=torch.int16, device="cuda")
    buf[x_off:x_off + m] = torch.from_numpy(x.view(np.int16)).cuda()
    xd = buf[x_off:x_off + m]
    assert xd.data_ptr() % 16 == (2 * x_off) % 16
    for p in (0.0, 0.5, 0.97):
        t = ti.quantile_threshold(x, p)
        _, mask_o, idx_o, count_o = orc.sparsify(x, t)
        mbuf = torch.full((m + 8,), 7, dtype=torch.uint8, device="cuda")
        mask = mbuf[mask_off:mask_off + m]
        idx = torch.full((m,), -1, dtype=torch.int32, device="cuda")
        count = torch.full((1,), -1, dtype=torch.int32, device="cuda")
        T.check(T.teal_sparsify(xd, m, t, mask, idx, count))
        torch.cuda.synchronize()
        assert int(count.item()) == count_o
        assert np.array_equal(mask.cpu().numpy(), mask_o)
        got = idx.cpu().numpy()
        assert np.array_equal(got[:count_o], idx_o) and np.all(got[count_o:] == -1)
        outside = mbuf.cpu().numpy()
        assert np.all(outside[:mask_off] == 7) and np.all(outside[mask_off + m:] == 7)


def test_sparsify_ties_special_values_and_empty(T):
    x = np.array([1.0, -1.0, 1.0009765625, 0.0, -0.0, np.nan, np.inf, -np.inf, 6e-8, -65504.0] * 13,
                 dtype=np.float16)
    for t in (0.0, 1.0, 6e-8, 65504.0):
        t = float(np.float32(t))
        _, mask_o, idx_o, count_o = orc.sparsify(x, t)
        mask, idx, count = gpu_sparsify(T, x, t)
        assert count == count_o and np.array_equal(mask, mask_o)
        assert np.array_equal(idx[:count], idx_o)
    mask, idx, count = gpu_sparsify(T, np.zeros(0, np.float16), 0.5)
    assert count == 0 and mask.size == 0
    # outputs are optional
    xd = dev(x)
    count_only = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    T.check(T.teal_sparsify(xd, x.size, 1.0, None, None, count_only))
    torch.cuda.synchronize()
    assert int(count_only.item()) == orc.sparsify(x, 1.0)[3]


# ---------------------------------------------------------------------------
# teal_pack_bf16
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("n,m", [(1, 1), (8, 5), (64, 64), (65, 63), (200, 333), (1024, 4096)])
def test_pack_is_the_transpose(T, n, m):
    w = ti.weights_bf16(n, m, seed=n * 31 + m)
    wd = dev(w)
    wt = torch.zeros((m, n), dtype=torch.int16, device="cuda")
    T.check(T.teal_pack_bf16(wd, wt, m, n))
    torch.cuda.synchronize()
    assert np.array_equal(wt.cpu().numpy().view(np.uint16), ti.to_input_channel_major(w))


# ---------------------------------------------------------------------------
# teal_sparse_gemv_bf16: small and ragged shapes, every kernel variant
# ---------------------------------------------------------------------------

SMALL = [(8, 1), (8, 64), (24, 40), (136, 65), (520, 333), (1032, 2049), (2056, 4100), (4096, 4096)]


@pytest.mark.parametrize("n,m", SMALL)
def test_gemv_bf16_small_shapes_default_launch(T, n, m):
    w = ti.weights_bf16(n, m, seed=11 * n + m)
    wt = dev(ti.to_input_channel_major(w))
    ws = workspace(T, m, n)
    for dist in ("gaussian", "laplace"):
        x = ti.make_x(m, 77 + m, dist)
        xd = dev(x)
        for p in (0.0, 0.4, 0.5, 0.9):
            t = ti.quantile_threshold(x, p)
            want = orc.sparse_gemv_bf16(w, x, t)
            got = run_bf16(T, wt, xd, t, m, n, ws)
            assert rel_l2(got, want) <= TIGHT, (n, m, dist, p)
            assert rel_l2(got, want) <= TOL_BF16


@pytest.mark.parametrize("lanes", [64, 32, 16, 8])
@pytest.mark.parametrize("waves,unroll", [(4, 4), (4, 8), (8, 4), (8, 8), (16, 4)])
def test_gemv_bf16_every_variant(T, lanes, waves, unroll):
    for (n, m) in [(520, 333), (1032, 2049), (4096, 4096)]:
        w = ti.weights_bf16(n, m, seed=3 * n + m)
        wt = dev(ti.to_input_channel_major(w))
        x = ti.laplace_x(m, 5 + m)
        xd = dev(x)
        ws = workspace(T, m, n)
        for p in (0.0, 0.5):
            t = ti.quantile_threshold(x, p)
            want = orc.sparse_gemv_bf16(w, x, t)
            for splits in (1, 3, 16, 128):
                # full-width tiles, and narrower ones that leave lanes idle and a ragged last tile
                for tile_cols in (0, lanes * 8 - 8, 24):
                    got = run_bf16(T, wt, xd, t, m, n, ws, lanes_per_row=lanes, splits=splits,
                                   waves=waves, unroll=unroll, tile_cols=tile_cols)
                    assert rel_l2(got, want) <= TIGHT, (n, m, p, lanes, waves, unroll, splits,
                                                        tile_cols)


def test_gemv_bf16_degenerate_sparsity(T):
    n, m = 1032, 2049
    w = ti.weights_bf16(n, m, seed=9)
    wt = dev(ti.to_input_channel_major(w))
    x = ti.gaussian_x(m, 10)
    xd = dev(x)
    ws = workspace(T, m, n)
    tmax = float(np.abs(x.astype(np.float32)).max())
    got = run_bf16(T, wt, xd, tmax, m, n, ws)          # nothing survives
    assert np.all(got == 0.0) and not np.any(np.signbit(got))
    # exactly one survivor: y is that one weight row times x_i, exactly
    second = float(np.sort(np.abs(x.astype(np.float32)))[-2])
    got = run_bf16(T, wt, xd, second, m, n, ws)
    want = orc.sparse_gemv_bf16(w, x, second)
    assert np.array_equal(got.astype(np.float64), want)
    # a state of zeros at t = 0: |0| > 0 is false, nothing is read
    zd = dev(np.zeros(m, np.float16))
    assert np.all(run_bf16(T, wt, zd, 0.0, m, n, ws) == 0.0)


def test_gemv_bf16_ties_at_threshold_are_dropped(T):
    n, m = 256, 512
    w = ti.weights_bf16(n, m, seed=21)
    wt = dev(ti.to_input_channel_major(w))
    x = (np.arange(m) % 5 - 2).astype(np.float16)     # magnitudes 0, 1, 2 with many ties
    ws = workspace(T, m, n)
    for t in (0.0, 1.0, 2.0):
        got = run_bf16(T, wt, dev(x), t, m, n, ws)
        want = orc.sparse_gemv_bf16(w, x, t)
        assert rel_l2(got, want) <= TIGHT


def test_gemv_bf16_is_bitwise_reproducible(T):
    n, m = 4096, 4096
    w = ti.weights_bf16(n, m, seed=33)
    wt = dev(ti.to_input_channel_major(w))
    x = ti.gaussian_x(m, 34)
    xd = dev(x)
    t = ti.quantile_threshold(x, 0.5)
    ws = workspace(T, m, n)
    first = run_bf16(T, wt, xd, t, m, n, ws)
    for _ in range(5):
        assert np.array_equal(run_bf16(T, wt, xd, t, m, n, ws), first)
    assert np.array_equal(run_bf16(T, wt, xd, t, m, n, workspace(T, m, n)), first)
    for shape in (dict(lanes_per_row=16, splits=16), dict(lanes_per_row=64, splits=128, waves=8, tile_cols=448)):
        a = run_bf16(T, wt, xd, t, m, n, ws, **shape)
        for _ in range(3):
            assert np.array_equal(run_bf16(T, wt, xd, t, m, n, ws, **shape), a)


def test_one_workspace_serves_calls_of_different_shapes(T):
    """A workspace sized for the largest call is reused, without re-zeroing, by
    calls of other shapes and launch shapes, back to back on one stream."""
    shapes = [(4096, 4096), (1032, 2049), (520, 333), (14336, 4096), (4096, 14336), (1024, 4096)]
    ws = workspace(T, max(m for _, m in shapes), max(n for n, _ in shapes))
    cases = []
    for (n, m) in shapes:
        w = ti.weights_bf16(n, m, seed=n + 3 * m)
        x = ti.gaussian_x(m, seed=n + 5 * m)
        t = ti.quantile_threshold(x, 0.5)
        cases.append((n, m, dev(ti.to_input_channel_major(w)), dev(x), t,
                      orc.sparse_gemv_bf16(w, x, t)))
    ys = []
    for rep in range(3):
        for (n, m, wt, xd, t, want) in cases:
            y = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
            if rep == 1:
                T.check(T.teal_sparse_gemv_bf16_ex(wt, xd, t, y, m, n, ws, lanes_per_row=16,
                                                   splits=7))
            else:
                T.check(T.teal_sparse_gemv_bf16(wt, xd, t, y, m, n, ws))
            ys.append((y, want))
    torch.cuda.synchronize()
    for y, want in ys:
        assert rel_l2(y.cpu().numpy(), want) <= TIGHT


# ---------------------------------------------------------------------------
# full-size projections in the launch configuration the benchmark times
# ---------------------------------------------------------------------------

FULL = [("llama2_7b", p) for p in ("q", "gate", "down")] + \
       [("llama3_8b", p) for p in ("k", "up", "down")]


@pytest.mark.parametrize("model,proj", FULL)
def test_gemv_bf16_full_size(T, model, proj):
    n, m = ti.LAYER_SHAPES[model][proj]
    cfg = ti.CONFIG_INDEX[model]
    w = ti.weights_bf16(n, m, ti.weight_seed(cfg, 0, proj))
    x = ti.make_x(m, ti.x_seed(cfg, 0, proj), ti.PROJ_DIST[proj])
    # upload canonical W and lay it out on the device, as the benchmark does
    wd = dev(w)
    wt = torch.empty((m, n), dtype=torch.int16, device="cuda")
    T.check(T.teal_pack_bf16(wd, wt, m, n))
    del wd
    xd = dev(x)
    ws = workspace(T, m, n)
    for p in (0.0, 0.4, 0.5, 0.9):
        t = ti.quantile_threshold(x, p)
        want = orc.sparse_gemv_bf16(w, x, t)
        got = run_bf16(T, wt, xd, t, m, n, ws)
        assert rel_l2(got, want) <= TIGHT, (model, proj, p)
        mask, idx, count = gpu_sparsify(T, x, t)
        _, mask_o, idx_o, count_o = orc.sparsify(x, t)
        assert count == count_o and np.array_equal(mask, mask_o)
        assert np.array_equal(idx[:count], idx_o)


def test_relative_error_follows_theorem_a1_at_full_size(T, golden_dir):
    """A property that holds at any size (Theorem A.1): for Gaussian x and Gaussian W the
    error of the sparsified product relative to the dense one is sqrt(p - 2 t_p phi(t_p)).
    Checked on the GPU's own dense (t = 0) and sparse outputs at 14336 x 4096, 4 draws of x."""
    import os
    rows = []
    with open(os.path.join(golden_dir, "thm_a1_relative_error.txt")) as f:
        for line in f:
            if not line.startswith("#"):
                rows.append(tuple(float(v) for v in line.split()))
    n, m = 14336, 4096
    g = torch.Generator(device="cuda")
    g.manual_seed(99)
    w = (torch.randn((n, m), generator=g, device="cuda") * 0.02).to(torch.bfloat16).view(torch.int16)
    wt = torch.empty((m, n), dtype=torch.int16, device="cuda")
    T.check(T.teal_pack_bf16(w, wt, m, n))
    ws = workspace(T, m, n)
    xs = [ti.gaussian_x(m, 8000 + k) for k in range(4)]
    dense = [run_bf16(T, wt, dev(x), 0.0, m, n, ws).astype(np.float64) for x in xs]
    for p, _, err in rows:
        num = den = 0.0
        for x, yd in zip(xs, dense):
            t = ti.quantile_threshold(x, p)
            ys = run_bf16(T, wt, dev(x), t, m, n, ws).astype(np.float64)
            assert survivors(T, ws) == [int(np.count_nonzero(np.abs(x.astype(np.float32)) > np.float32(t)))]
            num += np.linalg.norm(yd - ys)
            den += np.linalg.norm(yd)
        assert abs(num / den - err) <= 0.05 * err, (p, num / den, err)


def test_gemv_bf16_70b_shape_sampled_rows(T):
    """28672 x 8192 (gate/up of the 70B-shaped block): sampled outputs one by one."""
    n, m = ti.LAYER_SHAPES["llama_70b"]["gate"]
    w = ti.weights_bf16(n, m, ti.weight_seed(4, 0, "gate"))
    x = ti.gaussian_x(m, ti.x_seed(4, 0, "gate"))
    wd = dev(w)
    wt = torch.empty((m, n), dtype=torch.int16, device="cuda")
    T.check(T.teal_pack_bf16(wd, wt, m, n))
    del wd
    ws = workspace(T, m, n)
    t = ti.quantile_threshold(x, 0.5)
    got = run_bf16(T, wt, dev(x), t, m, n, ws)
    rows = np.unique(np.concatenate([np.arange(0, n, 97), [n - 1, n - 8, 511, 512]])).astype(np.int32)
    want = orc.sparse_gemv_bf16_rows(w, x, t, rows)
    assert rel_l2(got[rows], want) <= TIGHT
    assert np.all(np.isfinite(got))


def test_gemv_bf16_70b_shape_grouped_sampled_rows(T):
    """The largest launch the benchmark times: gate + up of the 70B-shaped block in one
    call (2 x 28672 x 8192, own thresholds), sampled outputs one by one and the survivor
    counts."""
    n, m = ti.LAYER_SHAPES["llama_70b"]["gate"]
    x = ti.gaussian_x(m, ti.x_seed(4, 0, "gate"))
    xd = dev(x)
    ws_host, wts = [], []
    for proj in ("gate", "up"):
        w = ti.weights_bf16(n, m, ti.weight_seed(4, 0, proj))
        wd = dev(w)
        wt = torch.empty((m, n), dtype=torch.int16, device="cuda")
        T.check(T.teal_pack_bf16(wd, wt, m, n))
        del wd
        ws_host.append(w)
        wts.append(wt)
    ts = [ti.quantile_threshold(x, 0.5), ti.quantile_threshold(x, 0.4)]
    ys = [torch.full((n,), float("nan"), dtype=torch.float32, device="cuda") for _ in range(2)]
    ws = workspace(T, m, 2 * n)
    T.check(T.teal_sparse_gemv_bf16_multi(wts, ts, ys, [n, n], xd, m, ws))
    torch.cuda.synchronize()
    assert survivors(T, ws, 2) == [orc.sparsify(x, t)[3] for t in ts]
    rows = np.unique(np.concatenate([np.arange(0, n, 89), [n - 1, n - 8, 447, 448]])).astype(np.int32)
    for k in range(2):
        got = ys[k].cpu().numpy()
        assert np.all(np.isfinite(got))
        assert rel_l2(got[rows], orc.sparse_gemv_bf16_rows(ws_host[k], x, ts[k], rows)) <= TIGHT, k


def max_abs_err_scaled(got, want):
    """Largest element-wise error relative to the vector's RMS: a single wrong output shows
    here even where a norm over many outputs would hide it."""
    rms = np.sqrt(np.mean(want ** 2))
    return float(np.max(np.abs(got.astype(np.float64) - want)) / rms) if rms > 0 else float(np.any(got))


@pytest.mark.parametrize("proj", ["q", "k", "down"])
def test_gemv_bf16_remaining_70b_shapes_sampled_rows(T, proj):
    """8192 x 8192 (q / o), 1024 x 8192 (k / v) and 8192 x 28672 (down) of the 70B-shaped
    block at full size, the launch shape the benchmark times: survivor count exact, sampled
    outputs one by one against the oracle (norm and element-wise), every output finite."""
    n, m = ti.LAYER_SHAPES["llama_70b"][proj]
    w = ti.weights_bf16(n, m, ti.weight_seed(4, 0, proj))
    x = ti.make_x(m, ti.x_seed(4, 0, proj), ti.PROJ_DIST[proj])
    wd = dev(w)
    wt = torch.empty((m, n), dtype=torch.int16, device="cuda")
    T.check(T.teal_pack_bf16(wd, wt, m, n))
    del wd
    ws = workspace(T, m, n)
    xd = dev(x)
    for p in (0.5, 0.0):
        t = ti.quantile_threshold(x, p)
        got = run_bf16(T, wt, xd, t, m, n, ws)
        assert survivors(T, ws) == [orc.sparsify(x, t)[3]]
        rows = np.unique(np.concatenate([np.arange(0, n, 61), [n - 1, n - 8, 127, 128, 255, 256]])).astype(np.int32)
        want = orc.sparse_gemv_bf16_rows(w, x, t, rows)
        assert rel_l2(got[rows], want) <= TIGHT, (proj, p)
        assert max_abs_err_scaled(got[rows], want) <= 1e-4, (proj, p)
        assert np.all(np.isfinite(got))


def test_gemv_bf16_70b_qkv_group_sampled_rows(T):
    """q + k + v of the 70B-shaped block in one call (8192, 1024, 1024 columns of an 8192-wide
    state, own thresholds): the other grouped launch of the headline benchmark."""
    m = 8192
    x = ti.gaussian_x(m, ti.x_seed(4, 0, "q"))
    xd = dev(x)
    hosts, wts, ns = [], [], []
    for proj in ("q", "k", "v"):
        n, _ = ti.LAYER_SHAPES["llama_70b"][proj]
        w = ti.weights_bf16(n, m, ti.weight_seed(4, 0, proj))
        wt = torch.empty((m, n), dtype=torch.int16, device="cuda")
        T.check(T.teal_pack_bf16(dev(w), wt, m, n))
        hosts.append(w)
        wts.append(wt)
        ns.append(n)
    ts = [ti.quantile_threshold(x, p) for p in (0.5, 0.4, 0.65)]
    ys = [torch.full((n,), float("nan"), dtype=torch.float32, device="cuda") for n in ns]
    ws = workspace(T, m, sum(ns))
    T.check(T.teal_sparse_gemv_bf16_multi(wts, ts, ys, ns, xd, m, ws))
    torch.cuda.synchronize()
    assert survivors(T, ws, 3) == [orc.sparsify(x, t)[3] for t in ts]
    for k in range(3):
        got = ys[k].cpu().numpy()
        rows = np.unique(np.concatenate([np.arange(0, ns[k], 53), [ns[k] - 1]])).astype(np.int32)
        want = orc.sparse_gemv_bf16_rows(hosts[k], x, ts[k], rows)
        assert np.all(np.isfinite(got))
        assert rel_l2(got[rows], want) <= TIGHT and max_abs_err_scaled(got[rows], want) <= 1e-4, k


@pytest.mark.parametrize("group,ps", [(("gate", "up"), (0.5, 0.4)), (("q", "k", "v"), (0.5, 0.4, 0.65))],
                         ids=["gate+up", "q+k+v"])
def test_gemv_bf16_70b_groups_with_padded_rows(T, group, ps):
    """The grouped launches of the 70B-shaped block on matrices stored with rows 256 bytes
    further apart (teal_pack_bf16_pitch): the gate + up pair without split-K, a block
    compacting all 8192 channels (a list of 64 KiB in LDS); q + k + v with the shape of the
    packed call.  Survivor counts exact, sampled outputs one by one against
    the oracle, and bit for bit the packed matrix under the same launch shape."""
    m = 8192
    x = ti.gaussian_x(m, ti.x_seed(4, 0, group[0]))
    xd = dev(x)
    hosts, wide, ns, pitches = [], [], [], []
    for proj in group:
        n, _ = ti.LAYER_SHAPES["llama_70b"][proj]
        w = ti.weights_bf16(n, m, ti.weight_seed(4, 0, proj))
        wt = torch.full((m, n + 128), 0x7FC0, dtype=torch.int16, device="cuda")
        T.check(T.teal_pack_bf16_pitch(dev(w), wt, m, n, n + 128))
        hosts.append(w)
        wide.append(wt)
        ns.append(n)
        pitches.append(n + 128)
    st, plan = T.teal_gemv_plan_multi_pitch(16, m, ns, pitches)
    assert st == 0 and (plan["splits"] == 1) == (len(group) == 2)
    ts = [ti.quantile_threshold(x, p) for p in ps]
    ys = [torch.full((n,), float("nan"), dtype=torch.float32, device="cuda") for n in ns]
    ws = workspace(T, m, sum(ns))
    for _ in range(2):                                       # twice on one workspace
        T.check(T.teal_sparse_gemv_bf16_multi_pitch(wide, pitches, ts, ys, ns, xd, m, ws))
    torch.cuda.synchronize()
    assert survivors(T, ws, len(ns)) == [orc.sparsify(x, t)[3] for t in ts]
    ws1 = workspace(T, m, max(ns))
    for k, n in enumerate(ns):
        got = ys[k].cpu().numpy()
        rows = np.unique(np.concatenate([np.arange(0, n, 59), [n - 1, n - 8, 255, 256]])).astype(np.int32)
        want = orc.sparse_gemv_bf16_rows(hosts[k], x, ts[k], rows)
        assert np.all(np.isfinite(got))
        assert rel_l2(got[rows], want) <= TIGHT and max_abs_err_scaled(got[rows], want) <= 1e-4, k
        packed = wide[k][:, :n].contiguous()
        assert np.array_equal(got, run_bf16(T, packed, xd, ts[k], m, n, ws1, **plan)), k


# ---------------------------------------------------------------------------
# several matrices sharing one hidden state in one launch
# ---------------------------------------------------------------------------

MULTI = [
    ("llama3 q,k,v", [4096, 1024, 1024], 4096, [0.5, 0.4, 0.25]),
    ("llama2 gate,up", [11008, 11008], 4096, [0.5, 0.5]),
    ("llama3 gate,up", [14336, 14336], 4096, [0.4, 0.5]),
    ("ragged", [520, 24, 136, 8], 333, [0.0, 0.5, 0.9, 1.0]),
    ("single", [1032], 2049, [0.5]),
]


@pytest.mark.parametrize("name,ns,m,ps", MULTI, ids=[c[0] for c in MULTI])
def test_gemv_bf16_multi(T, name, ns, m, ps):
    x = ti.gaussian_x(m, 900 + m)
    xd = dev(x)
    ws = workspace(T, m, sum(ns))
    ws1 = workspace(T, m, max(ns))
    ws_host, wts, ts, ys = [], [], [], []
    for k, (n, p) in enumerate(zip(ns, ps)):
        w = ti.weights_bf16(n, m, seed=1000 * k + n + m)
        ws_host.append(w)
        wts.append(dev(ti.to_input_channel_major(w)))
        ts.append(ti.quantile_threshold(x, p))
        ys.append(torch.full((n,), float("nan"), dtype=torch.float32, device="cuda"))
    T.check(T.teal_sparse_gemv_bf16_multi(wts, ts, ys, ns, xd, m, ws))
    torch.cuda.synchronize()
    st, plan = T.teal_gemv_plan_multi(16, m, ns)
    assert st == 0
    for k, n in enumerate(ns):
        got = ys[k].cpu().numpy()
        want = orc.sparse_gemv_bf16(ws_host[k], x, ts[k])
        assert rel_l2(got, want) <= TIGHT, (name, k)
        # bitwise the separate call with the same launch shape
        alone = run_bf16(T, wts[k], xd, ts[k], m, n, ws1, **plan)
        assert np.array_equal(got, alone), (name, k)
    # the shared workspace is left ready: a second fused call gives the same bits
    ys2 = [torch.full((n,), float("nan"), dtype=torch.float32, device="cuda") for n in ns]
    T.check(T.teal_sparse_gemv_bf16_multi(wts, ts, ys2, ns, xd, m, ws))
    torch.cuda.synchronize()
    for a, b in zip(ys, ys2):
        assert torch.equal(a, b)


MULTI_PITCH = [
    # name, widths, row pitches (elements), m, sparsity levels
    ("llama3 gate,up rotating", [14336, 14336], [14336 + 128, 14336 + 384], 4096, [0.5, 0.4]),
    ("llama2 gate,up rotating", [11008, 11008], [11008 + 128, 11008 + 128], 4096, [0.5, 0.5]),
    ("llama3 q,k,v padded", [4096, 1024, 1024], [4096 + 128, 1024 + 8, 1024], 4096, [0.5, 0.4, 0.25]),
    ("ragged", [520, 24, 136, 8], [520 + 8, 24 + 104, 136, 8 + 128], 333, [0.0, 0.5, 0.9, 1.0]),
    ("single", [1032], [1032 + 128], 2049, [0.5]),
    ("llama3 gate alone rotating", [14336], [14336 + 128], 4096, [0.5]),
]


def padded_rows(wt_dev, pitch, fill):
    """The matrix stored with rows `pitch` elements apart; the padding holds `fill`."""
    k, n = wt_dev.shape
    out = torch.full((k, pitch), fill, dtype=wt_dev.dtype, device="cuda")
    out[:, :n] = wt_dev
    return out


@pytest.mark.parametrize("name,ns,pitches,m,ps", MULTI_PITCH, ids=[c[0] for c in MULTI_PITCH])
def test_gemv_bf16_multi_pitch(T, name, ns, pitches, m, ps):
    """Padded rows: the oracle's result, bit for bit the packed matrix under the launch shape
    the padded call reports, and the padding (bf16 NaNs here) never enters a sum."""
    x = ti.gaussian_x(m, 910 + m)
    xd = dev(x)
    ws = workspace(T, m, sum(ns))
    ws1 = workspace(T, m, max(ns))
    hosts, packed, padded, ts, ys = [], [], [], [], []
    for k, (n, p) in enumerate(zip(ns, ps)):
        w = ti.weights_bf16(n, m, seed=1100 * k + n + m)
        hosts.append(w)
        packed.append(dev(ti.to_input_channel_major(w)))
        padded.append(padded_rows(packed[-1], pitches[k], 0x7FC0))
        ts.append(ti.quantile_threshold(x, p))
        ys.append(torch.full((n,), float("nan"), dtype=torch.float32, device="cuda"))
    T.check(T.teal_sparse_gemv_bf16_multi_pitch(padded, pitches, ts, ys, ns, xd, m, ws))
    torch.cuda.synchronize()
    st, plan = T.teal_gemv_plan_multi_pitch(16, m, ns, pitches)
    assert st == 0
    if "rotating" in name:
        assert plan["splits"] == 1 and plan["tile_cols"] == (128 if len(ns) > 1 else 64)
    for k, n in enumerate(ns):
        got = ys[k].cpu().numpy()
        assert rel_l2(got, orc.sparse_gemv_bf16(hosts[k], x, ts[k])) <= TIGHT, (name, k)
        alone = run_bf16(T, packed[k], xd, ts[k], m, n, ws1, **plan)
        assert np.array_equal(got, alone), (name, k)
    assert survivors(T, ws, len(ns)) == [orc.sparsify(x, t)[3] for t in ts]
    # the workspace is left ready; the packed call on the same workspace still works
    ys2 = [torch.full((n,), float("nan"), dtype=torch.float32, device="cuda") for n in ns]
    T.check(T.teal_sparse_gemv_bf16_multi(packed, ts, ys2, ns, xd, m, ws))
    T.check(T.teal_sparse_gemv_bf16_multi_pitch(padded, pitches, ts, ys2, ns, xd, m, ws))
    torch.cuda.synchronize()
    for a, b in zip(ys, ys2):
        assert torch.equal(a, b)


def test_multi_pitch_edge_cases(T):
    """Padded rows at the edges: nothing / everything survives and ties at the threshold on the
    shape without split-K; one matrix of the group on rotating rows and one not (the packed
    call's shape on padded rows); a pitch far above the row; four matrices; run-to-run and
    workspace-to-workspace reproducibility."""
    m = 4096
    ns = [14336, 14336]
    x = ti.gaussian_x(m, 930)
    x[100:164] = np.float16(0.5)                       # a run of ties at the threshold below
    x[200:232] = np.float16(-0.5)
    xd = dev(x)
    hosts = [ti.weights_bf16(n, m, seed=1200 + k) for k, n in enumerate(ns)]
    packed = [dev(ti.to_input_channel_major(w)) for w in hosts]

    def run(pitches, ts, ws):
        wide = [padded_rows(p, pitch, 0x7FC0) for p, pitch in zip(packed, pitches)]
        ys = [torch.full((n,), float("nan"), dtype=torch.float32, device="cuda") for n in ns]
        T.check(T.teal_sparse_gemv_bf16_multi_pitch(wide, pitches, ts, ys, ns, xd, m, ws))
        torch.cuda.synchronize()
        return [y.cpu().numpy() for y in ys]

    ws = workspace(T, m, sum(ns))
    rot = [n + 128 for n in ns]
    rows = np.arange(0, ns[0], 131).astype(np.int32)
    # ties: |x| == t is dropped (Definition 1), also without split-K
    got = run(rot, [0.5, 0.5], ws)
    assert survivors(T, ws, 2) == [orc.sparsify(x, 0.5)[3]] * 2
    for k in range(2):
        assert rel_l2(got[k][rows], orc.sparse_gemv_bf16_rows(hosts[k], x, 0.5, rows)) <= TIGHT
    # nothing survives / everything survives
    got = run(rot, [70000.0, 0.0], ws)
    assert not got[0].any() and survivors(T, ws, 2) == [0, orc.sparsify(x, 0.0)[3]]
    assert rel_l2(got[1][rows], orc.sparse_gemv_bf16_rows(hosts[1], x, 0.0, rows)) <= TIGHT
    # run to run, and on another workspace: the same bits
    a = run(rot, [0.25, 0.625], ws)
    b = run(rot, [0.25, 0.625], workspace(T, m, sum(ns)))
    assert all(np.array_equal(u, v) for u, v in zip(a, b))
    # only one matrix on rotating rows, and a pitch far above the row: the packed call's shape
    for pitches in ([ns[0] + 128, ns[1]], [ns[0] + 4096 + 8, ns[1] + 40]):
        st, plan = T.teal_gemv_plan_multi_pitch(16, m, ns, pitches)
        assert st == 0 and plan == T.teal_gemv_plan_multi(16, m, ns)[1]
        c = run(pitches, [0.25, 0.625], ws)
        for k in range(2):
            assert rel_l2(c[k], a[k].astype(np.float64)) <= TIGHT
            assert rel_l2(c[k][rows], orc.sparse_gemv_bf16_rows(hosts[k], x, [0.25, 0.625][k], rows)) <= TIGHT
    # four matrices that share x, rotating rows: 4 x 5120 columns = 160 tiles of 256 bytes
    ns4 = [5120] * 4
    hosts4 = [ti.weights_bf16(n, m, seed=1300 + k) for k, n in enumerate(ns4)]
    wide4 = [padded_rows(dev(ti.to_input_channel_major(w)), n + 384, 0x7FC0) for w, n in zip(hosts4, ns4)]
    ts4 = [ti.quantile_threshold(x, p) for p in (0.25, 0.5, 0.65, 0.9)]
    ys4 = [torch.full((n,), float("nan"), dtype=torch.float32, device="cuda") for n in ns4]
    st, plan = T.teal_gemv_plan_multi_pitch(16, m, ns4, [n + 384 for n in ns4])
    assert st == 0 and (plan["tile_cols"], plan["splits"]) == (128, 1)
    T.check(T.teal_sparse_gemv_bf16_multi_pitch(wide4, [n + 384 for n in ns4], ts4, ys4, ns4, xd, m, ws))
    torch.cuda.synchronize()
    assert survivors(T, ws, 4) == [orc.sparsify(x, t)[3] for t in ts4]
    for k in range(4):
        assert rel_l2(ys4[k].cpu().numpy(), orc.sparse_gemv_bf16(hosts4[k], x, ts4[k])) <= TIGHT, k


def test_gemv_w8_multi_pitch(T):
    ns, m = [14336 * 2, 14336 * 2], 4096
    pitches = [n + 256 for n in ns]
    x = ti.laplace_x(m, 720)
    xd = dev(x)
    ws = workspace(T, m, sum(ns))
    hosts, packed, padded, scs, ts, ys = [], [], [], [], [], []
    for k, n in enumerate(ns):
        q, scale = ti.quantize_w8(ti.weights_bf16(n, m, seed=2100 * k + n))
        hosts.append((q, scale))
        packed.append(dev(q))
        padded.append(padded_rows(packed[-1], pitches[k], 127))
        scs.append(dev(scale))
        ts.append(ti.quantile_threshold(x, 0.5 - 0.1 * k))
        ys.append(torch.full((n,), float("nan"), dtype=torch.float32, device="cuda"))
    st, plan = T.teal_gemv_plan_multi_pitch(8, m, ns, pitches)
    assert st == 0 and plan["splits"] == 1
    T.check(T.teal_sparse_gemv_w8_multi_pitch(padded, pitches, scs, ts, ys, ns, xd, m, ws))
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([np.arange(0, ns[0], 61), [ns[0] - 1]])).astype(np.int32)
    for k, n in enumerate(ns):
        got = ys[k].cpu().numpy()
        q, scale = hosts[k]
        want = orc.sparse_gemv_w8(np.ascontiguousarray(q[:, rows]), np.ascontiguousarray(scale[rows]), x, ts[k])
        assert np.all(np.isfinite(got))
        assert rel_l2(got[rows], want) <= TIGHT, k
    # the packed call computes the same sums (another launch shape: tolerance, not bits)
    ys2 = [torch.full((n,), float("nan"), dtype=torch.float32, device="cuda") for n in ns]
    T.check(T.teal_sparse_gemv_w8_multi(packed, scs, ts, ys2, ns, xd, m, ws))
    torch.cuda.synchronize()
    for a, b in zip(ys, ys2):
        assert rel_l2(a.cpu().numpy(), b.cpu().numpy().astype(np.float64)) <= TIGHT


# ---------------------------------------------------------------------------
# weight-quantised variants
# ---------------------------------------------------------------------------

def run_w8(T, q_dev, s_dev, x_dev, t, m, n, ws):
    y = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    T.check(T.teal_sparse_gemv_w8(q_dev, s_dev, x_dev, t, y, m, n, ws))
    torch.cuda.synchronize()
    return y.cpu().numpy()


def run_w4(T, q_dev, s_dev, x_dev, t, m, n, ws):
    y = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    T.check(T.teal_sparse_gemv_w4(q_dev, s_dev, 128, x_dev, t, y, m, n, ws))
    torch.cuda.synchronize()
    return y.cpu().numpy()


@pytest.mark.parametrize("n,m", [(16, 1), (48, 100), (528, 333), (1040, 2049), (4096, 4096),
                                 (1024, 4096), (14336, 4096), (4096, 14336)])
def test_gemv_w8(T, n, m):
    w = ti.weights_bf16(n, m, seed=7 * n + m)
    q, scale = ti.quantize_w8(w)
    qd, sd = dev(q), dev(scale)
    ws = workspace(T, m, n)
    dist = "laplace" if m > n else "gaussian"
    x = ti.make_x(m, 13 + m, dist)
    xd = dev(x)
    for p in (0.0, 0.4, 0.5, 1.0):
        t = ti.quantile_threshold(x, p)
        want = orc.sparse_gemv_w8(q, scale, x, t)
        got = run_w8(T, qd, sd, xd, t, m, n, ws)
        assert rel_l2(got, want) <= TIGHT, (n, m, p)
        assert rel_l2(got, want) <= TOL_WQ


@pytest.mark.parametrize("name,ns,m,ps", [
    ("llama3 q,k,v", [4096, 1024, 1024], 4096, [0.5, 0.4, 0.25]),
    ("llama3 gate,up", [14336, 14336], 4096, [0.4, 0.5]),
    ("ragged", [528, 32, 144, 16], 333, [0.0, 0.5, 0.9, 1.0]),
    ("single", [1040], 2049, [0.5]),
], ids=["qkv", "gate_up", "ragged", "single"])
def test_gemv_w8_multi(T, name, ns, m, ps):
    x = ti.laplace_x(m, 700 + m)
    xd = dev(x)
    ws = workspace(T, m, sum(ns))
    ws1 = workspace(T, m, max(ns))
    qs_host, qs, scs, ts, ys = [], [], [], [], []
    for k, (n, p) in enumerate(zip(ns, ps)):
        q, scale = ti.quantize_w8(ti.weights_bf16(n, m, seed=2000 * k + n + m))
        qs_host.append((q, scale))
        qs.append(dev(q))
        scs.append(dev(scale))
        ts.append(ti.quantile_threshold(x, p))
        ys.append(torch.full((n,), float("nan"), dtype=torch.float32, device="cuda"))
    T.check(T.teal_sparse_gemv_w8_multi(qs, scs, ts, ys, ns, xd, m, ws))
    torch.cuda.synchronize()
    for k, n in enumerate(ns):
        got = ys[k].cpu().numpy()
        want = orc.sparse_gemv_w8(qs_host[k][0], qs_host[k][1], x, ts[k])
        assert rel_l2(got, want) <= TIGHT, (name, k)
        assert rel_l2(got, want) <= TOL_WQ
        # the separate call computes the same sums (its launch shape may differ)
        alone = run_w8(T, qs[k], scs[k], xd, ts[k], m, n, ws1)
        assert rel_l2(got, alone.astype(np.float64)) <= TIGHT
    ys2 = [torch.full((n,), float("nan"), dtype=torch.float32, device="cuda") for n in ns]
    T.check(T.teal_sparse_gemv_w8_multi(qs, scs, ts, ys2, ns, xd, m, ws))
    torch.cuda.synchronize()
    for a, b in zip(ys, ys2):
        assert torch.equal(a, b)


@pytest.mark.parametrize("n,m", [(32, 128), (96, 384), (544, 256), (1056, 2176), (4096, 4096),
                                 (1024, 4096), (14336, 4096), (4096, 14336)])
def test_gemv_w4(T, n, m):
    w = ti.weights_bf16(n, m, seed=5 * n + m)
    packed, scale = ti.quantize_w4(w, 128)
    qd, sd = dev(packed), dev(scale)
    ws = workspace(T, m, n)
    dist = "laplace" if m > n else "gaussian"
    x = ti.make_x(m, 17 + m, dist)
    xd = dev(x)
    for p in (0.0, 0.4, 0.5, 1.0):
        t = ti.quantile_threshold(x, p)
        want = orc.sparse_gemv_w4(packed, scale, 128, x, t)
        got = run_w4(T, qd, sd, xd, t, m, n, ws)
        assert rel_l2(got, want) <= TIGHT, (n, m, p)
        assert rel_l2(got, want) <= TOL_WQ


@pytest.mark.parametrize("name,ns,m,ps", [
    ("llama3 q,k,v", [4096, 1024, 1024], 4096, [0.5, 0.4, 0.25]),
    ("llama3 gate,up", [14336, 14336], 4096, [0.4, 0.5]),
    ("ragged", [544, 32, 160, 64], 384, [0.0, 0.5, 0.9, 1.0]),
    ("single", [1056], 2176, [0.5]),
], ids=["qkv", "gate_up", "ragged", "single"])
def test_gemv_w4_multi(T, name, ns, m, ps):
    x = ti.gaussian_x(m, 800 + m)
    xd = dev(x)
    ws = workspace(T, m, sum(ns))
    ws1 = workspace(T, m, max(ns))
    qs_host, qs, scs, ts, ys = [], [], [], [], []
    for k, (n, p) in enumerate(zip(ns, ps)):
        q, scale = ti.quantize_w4(ti.weights_bf16(n, m, seed=3000 * k + n + m), 128)
        qs_host.append((q, scale))
        qs.append(dev(q))
        scs.append(dev(scale))
        ts.append(ti.quantile_threshold(x, p))
        ys.append(torch.full((n,), float("nan"), dtype=torch.float32, device="cuda"))
    T.check(T.teal_sparse_gemv_w4_multi(qs, scs, 128, ts, ys, ns, xd, m, ws))
    torch.cuda.synchronize()
    for k, n in enumerate(ns):
        got = ys[k].cpu().numpy()
        want = orc.sparse_gemv_w4(qs_host[k][0], qs_host[k][1], 128, x, ts[k])
        assert rel_l2(got, want) <= TOL_WQ, (name, k)
        assert rel_l2(got, want) <= 1e-4, (name, k)
        alone = run_w4(T, qs[k], scs[k], xd, ts[k], m, n, ws1)
        assert rel_l2(got, alone.astype(np.float64)) <= 1e-4
    ys2 = [torch.full((n,), float("nan"), dtype=torch.float32, device="cuda") for n in ns]
    T.check(T.teal_sparse_gemv_w4_multi(qs, scs, 128, ts, ys2, ns, xd, m, ws))
    torch.cuda.synchronize()
    for a, b in zip(ys, ys2):
        assert torch.equal(a, b)

# ---------------------------------------------------------------------------
# the survivor count every call leaves in its workspace
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("n,m", [(16, 1), (144, 65), (528, 333), (1040, 2049), (4096, 4096),
                                 (1024, 14336)])
def test_survivor_count_one_matrix(T, n, m):
    n4, m4 = (n + 31) // 32 * 32, (m + 127) // 128 * 128      # a shape the int4 format takes
    w = ti.weights_bf16(n, m, seed=5 * n + m)
    wt = dev(ti.to_input_channel_major(w))
    q8, s8 = ti.quantize_w8(w)
    q4, s4 = ti.quantize_w4(ti.weights_bf16(n4, m4, seed=6 * n + m))
    q8d, s8d, q4d, s4d = dev(q8), dev(s8), dev(q4), dev(s4)
    ws = workspace(T, m4, n4)
    ws.fill_(0x5A)                     # the report area needs no initial value ...
    ws[:T.teal_survivors_offset()].zero_()      # ... the arrival counters do
    x4 = ti.make_x(m4, 31 + m, "laplace")
    x = x4[:m].copy()
    xd, x4d = dev(x), dev(x4)
    for p in (0.0, 0.3, 0.5, 0.97, 1.0):
        t = ti.quantile_threshold(x, p)
        want = orc.sparsify(x, t)[3]
        run_bf16(T, wt, xd, t, m, n, ws)
        assert survivors(T, ws) == [want], (n, m, p)
        run_w8(T, q8d, s8d, xd, t, m, n, ws)
        assert survivors(T, ws) == [want], (n, m, p)
        t4 = ti.quantile_threshold(x4, p)
        run_w4(T, q4d, s4d, x4d, t4, m4, n4, ws)
        assert survivors(T, ws) == [orc.sparsify(x4, t4)[3]], (n, m, p)
    # every launch shape reports the same count
    t = ti.quantile_threshold(x, 0.5)
    want = orc.sparsify(x, t)[3]
    for splits in (1, 2, 3, 7, 16, 128):
        if (m + splits - 1) // splits > 4096:
            continue
        run_bf16(T, wt, xd, t, m, n, ws, splits=splits)
        assert survivors(T, ws) == [want], splits


def test_survivor_counts_grouped_calls(T):
    m, ns, ps = 4096, [4096, 1024, 1024, 72], [0.5, 0.4, 0.25, 0.9]
    x = ti.gaussian_x(m, 808)
    xd = dev(x)
    ws = workspace(T, m, sum(ns))
    ts = [ti.quantile_threshold(x, p) for p in ps]
    want = [orc.sparsify(x, t)[3] for t in ts]
    wts = [dev(ti.to_input_channel_major(ti.weights_bf16(n, m, seed=90 + k))) for k, n in enumerate(ns)]
    ys = [torch.empty(n, dtype=torch.float32, device="cuda") for n in ns]
    T.check(T.teal_sparse_gemv_bf16_multi(wts, ts, ys, ns, xd, m, ws))
    torch.cuda.synchronize()
    assert survivors(T, ws, 4) == want
    # fewer matrices, other thresholds, same workspace: slots of this call only
    T.check(T.teal_sparse_gemv_bf16_multi(wts[2:0:-1], ts[2:0:-1], ys[2:0:-1], ns[2:0:-1], xd, m, ws))
    torch.cuda.synchronize()
    assert survivors(T, ws, 2) == want[2:0:-1]
    ns16 = [4096, 1024, 1024]
    qs, scs = [], []
    for k, n in enumerate(ns16):
        q, scale = ti.quantize_w8(ti.weights_bf16(n, m, seed=190 + k))
        qs.append(dev(q))
        scs.append(dev(scale))
    T.check(T.teal_sparse_gemv_w8_multi(qs, scs, ts[:3], ys[:3], ns16, xd, m, ws))
    torch.cuda.synchronize()
    assert survivors(T, ws, 3) == want[:3]
    qs, scs = [], []
    for k, n in enumerate(ns16):
        q, scale = ti.quantize_w4(ti.weights_bf16(n, m, seed=290 + k))
        qs.append(dev(q))
        scs.append(dev(scale))
    # the same three matrices in reverse order (every per-matrix list reversed alike)
    T.check(T.teal_sparse_gemv_w4_multi(qs[::-1], scs[::-1], 128, ts[2::-1], ys[2::-1], ns16[::-1],
                                        xd, m, ws))
    torch.cuda.synchronize()
    assert survivors(T, ws, 3) == want[2::-1]



def test_very_wide_output(T):
    """A million output columns from a handful of input channels: thousands of tiles, one
    arrival counter each, more blocks than the chip holds at once."""
    m, n = 130, (1 << 20) + 16
    w = ti.weights_bf16(n, m, seed=777)
    wt = dev(ti.to_input_channel_major(w))
    x = ti.gaussian_x(m, 778)
    xd = dev(x)
    ws = workspace(T, m, n)
    for p in (0.5, 0.0):
        t = ti.quantile_threshold(x, p)
        got = run_bf16(T, wt, xd, t, m, n, ws)
        assert rel_l2(got, orc.sparse_gemv_bf16(w, x, t)) <= TIGHT, p
        assert survivors(T, ws) == [orc.sparsify(x, t)[3]]
    # with split-K forced on: 2049 tiles x 2 splits
    t = ti.quantile_threshold(x, 0.5)
    got = run_bf16(T, wt, xd, t, m, n, ws, splits=2)
    assert rel_l2(got, orc.sparse_gemv_bf16(w, x, t)) <= TIGHT
    q, scale = ti.quantize_w8(w)
    got = run_w8(T, dev(q), dev(scale), xd, t, m, n, ws)
    assert rel_l2(got, orc.sparse_gemv_w8(q, scale, x, t)) <= TIGHT


# An input longer than 128 x 4096 channels: a block compacts at most 4096 channels, so
# the call runs with more split-K blocks than a caller may ask for, and the workspace
# holds one partial row for each of them.
LONG_M = 128 * 4096 + 640


def test_very_long_input_every_format(T):
    m, n = LONG_M, 32
    w = ti.weights_bf16(n, m, seed=424242)
    x = ti.laplace_x(m, 4242)
    xd = dev(x)
    t = ti.quantile_threshold(x, 0.5)
    ws = workspace(T, m, 3 * n)
    assert T.teal_workspace_bytes(m, n) >= (m + 4095) // 4096 * n * 4

    want = orc.sparse_gemv_bf16(w, x, t)
    wt = dev(ti.to_input_channel_major(w))
    got = run_bf16(T, wt, xd, t, m, n, ws)
    assert rel_l2(got, want) <= TIGHT
    kept = orc.sparsify(x, t)[3]
    assert survivors(T, ws) == [kept]
    # a block takes at most 8192 channels: asking for fewer splits than that needs gives the
    # call with slices of 8192
    few = run_bf16(T, wt, xd, t, m, n, ws, splits=1)
    assert rel_l2(few, want) <= TIGHT
    assert np.array_equal(few, run_bf16(T, wt, xd, t, m, n, ws, splits=2))   # both: slices of 8192
    assert survivors(T, ws) == [kept]
    ys = [torch.full((k,), float("nan"), dtype=torch.float32, device="cuda") for k in (n, n)]
    t2 = ti.quantile_threshold(x, 0.9)
    T.check(T.teal_sparse_gemv_bf16_multi([wt, wt], [t, t2], ys, [n, n], xd, m, ws))
    torch.cuda.synchronize()
    assert rel_l2(ys[0].cpu().numpy(), want) <= TIGHT
    assert rel_l2(ys[1].cpu().numpy(), orc.sparse_gemv_bf16(w, x, t2)) <= TIGHT
    assert survivors(T, ws, 2) == [kept, orc.sparsify(x, t2)[3]]

    q, scale = ti.quantize_w8(w)
    got = run_w8(T, dev(q), dev(scale), xd, t, m, n, ws)
    assert rel_l2(got, orc.sparse_gemv_w8(q, scale, x, t)) <= TIGHT

    q4, scale4 = ti.quantize_w4(w)
    got = run_w4(T, dev(q4), dev(scale4), xd, t, m, n, ws)
    assert rel_l2(got, orc.sparse_gemv_w4(q4, scale4, 128, x, t)) <= TIGHT
    assert survivors(T, ws) == [kept]



# ---------------------------------------------------------------------------
# captured into a HIP graph
# ---------------------------------------------------------------------------

def test_prepared_calls_give_the_same_bits(T):
    """A call recorded once with prepare() and re-issued equals the direct call."""
    m, ns = 4096, [1032, 264]
    x = ti.gaussian_x(m, 61)
    xd = dev(x)
    ts = [ti.quantile_threshold(x, 0.5), ti.quantile_threshold(x, 0.25)]
    ws_host = [ti.weights_bf16(n, m, seed=62 + n) for n in ns]
    wts = [dev(ti.to_input_channel_major(w)) for w in ws_host]
    ws = workspace(T, m, sum(ns))
    ys = [torch.full((n,), float("nan"), dtype=torch.float32, device="cuda") for n in ns]
    T.check(T.teal_sparse_gemv_bf16_multi(wts, ts, ys, ns, xd, m, ws))
    torch.cuda.synchronize()
    direct = [y.clone() for y in ys]
    run = T.prepare(lambda: T.teal_sparse_gemv_bf16_multi(wts, ts, ys, ns, xd, m, ws))
    for _ in range(3):
        for y in ys:
            y.fill_(float("nan"))
        T.check(run())
        torch.cuda.synchronize()
        for a, b in zip(direct, ys):
            assert torch.equal(a, b)
    assert rel_l2(ys[0].cpu().numpy(), orc.sparse_gemv_bf16(ws_host[0], x, ts[0])) <= TIGHT


def test_calls_replay_from_a_hip_graph(T):
    """The calls only enqueue kernels on the given stream (no allocation, no host
    synchronisation, no memset), so a sequence of them can be captured once and replayed.
    Every replay must give the bits of the eager calls, with eager work in between."""
    m, n = 4096, 1032
    w = ti.weights_bf16(n, m, 41)
    wt = dev(ti.to_input_channel_major(w))
    q, scale = ti.quantize_w8(ti.weights_bf16(1040, m, 42))
    qd, sd = dev(q), dev(scale)
    x = ti.gaussian_x(m, 43)
    X = ti.make_X(4, m, 44, "laplace")
    xd, Xd = dev(x), dev(X)
    t = ti.quantile_threshold(x, 0.5)
    tb = ti.batch_quantile_threshold(X, 0.5)
    ws = workspace(T, m, 2 * n + 1040)
    wsb = torch.zeros(T.teal_workspace_bytes_batch(m, n, 4), dtype=torch.uint8, device="cuda")
    outs = [torch.zeros(n, dtype=torch.float32, device="cuda") for _ in range(9)]
    y8 = torch.zeros(1040, dtype=torch.float32, device="cuda")
    Yb = torch.zeros((4, n), dtype=torch.float32, device="cuda")
    gate, up = ti.mlp_gate_up(m, 45)
    h, gamma = ti.norm_inputs(m, 46)
    gated, upd, hd, gammad = dev(gate), dev(up), dev(h), dev(gamma)
    eps = float(np.float32(1e-5))
    th = ti.quantile_threshold(orc.swiglu_f16(gate, up), 0.5)
    tn = ti.quantile_threshold(orc.rmsnorm_f16(h, gamma, eps), 0.4)
    ws2 = workspace(T, m, 2 * n)           # kept apart: its survivor counts are read below
    x1 = np.ascontiguousarray(X[1])
    x1d = dev(x1)
    t1 = ti.quantile_threshold(x1, 0.65)
    ws3 = torch.zeros(T.teal_workspace_bytes_stack([2, 1], [n, n, n], [m, m]), dtype=torch.uint8,
                      device="cuda")

    def enqueue(stream):
        T.check(T.teal_sparse_gemv_bf16(wt, xd, t, outs[0], m, n, ws, stream=stream))
        T.check(T.teal_sparse_gemv_bf16_multi([wt, wt], [t, 0.0], [outs[1], outs[2]], [n, n], xd, m,
                                              ws, stream=stream))
        T.check(T.teal_sparse_gemv_w8(qd, sd, xd, t, y8, m, 1040, ws, stream=stream))
        T.check(T.teal_sparse_gemv_bf16_batch(wt, Xd, 4, tb, Yb, m, n, wsb, stream=stream))
        T.check(T.teal_sparse_gemv_bf16_swiglu(wt, gated, upd, th, outs[3], m, n, ws, stream=stream))
        T.check(T.teal_sparse_gemv_bf16_rmsnorm_multi([wt, wt], [tn, 0.0], [outs[4], outs[5]],
                                                      [n, n], hd, gammad, eps, m, ws2, stream=stream))
        T.check(T.teal_sparse_gemv_bf16_stack([2, 1], [wt, wt, wt], [t, 0.0, t1], outs[6:9], [n, n, n],
                                              [xd, x1d], [m, m], ws3, stream=stream))

    def snapshot():
        torch.cuda.synchronize()
        return [o.clone() for o in outs] + [y8.clone(), Yb.clone(),
                                            torch.tensor(survivors(T, ws2, 2))]

    def poison():
        for o in outs + [y8, Yb]:
            o.fill_(float("nan"))

    enqueue(torch.cuda.current_stream())
    eager = snapshot()
    assert rel_l2(eager[0].cpu().numpy(), orc.sparse_gemv_bf16(w, x, t)) <= TIGHT
    assert rel_l2(eager[3].cpu().numpy(), orc.sparse_gemv_bf16_swiglu(w, gate, up, th)) <= TIGHT
    assert rel_l2(eager[4].cpu().numpy(), orc.sparse_gemv_bf16_rmsnorm(w, h, gamma, eps, tn)) <= TIGHT
    assert torch.equal(eager[6], eager[1]) and torch.equal(eager[7], eager[2])
    assert rel_l2(eager[8].cpu().numpy(), orc.sparse_gemv_bf16(w, x1, t1)) <= TIGHT
    xn = orc.rmsnorm_f16(h, gamma, eps)
    assert eager[-1].tolist() == [orc.sparsify(xn, tn)[3], orc.sparsify(xn, 0.0)[3]]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        enqueue(side)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        enqueue(side)
    for replay in range(4):
        poison()
        ws2[T.teal_survivors_offset():T.teal_survivors_offset() + 8].zero_()
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for a, b in zip(eager, got):
            assert torch.equal(a, b), replay
        # eager work of the program itself between replays, on the same workspaces
        poison()
        enqueue(torch.cuda.current_stream())
        for a, b in zip(eager, snapshot()):
            assert torch.equal(a, b), replay


def test_long_slices_replay_from_a_hip_graph(T):
    """A block that takes more than 4096 channels needs more dynamic LDS than the default
    limit; the limit is raised at the first (eager) launch of that kernel, so the same call
    recorded into a graph afterwards replays with the bits of the eager call."""
    m, n = 8192, 264
    w = ti.weights_bf16(n, m, 51)
    wt = dev(ti.to_input_channel_major(w))
    x = ti.gaussian_x(m, 52)
    xd = dev(x)
    t = ti.quantile_threshold(x, 0.5)
    ws = workspace(T, m, 2 * n)
    wide = padded_rows(wt, n + 128, 0x7FC0)
    ys = [torch.zeros(n, dtype=torch.float32, device="cuda") for _ in range(3)]

    def enqueue(stream):
        T.check(T.teal_sparse_gemv_bf16_ex(wt, xd, t, ys[0], m, n, ws, stream=stream, lanes_per_row=16,
                                           tile_cols=128, splits=1, waves=8, unroll=4))
        T.check(T.teal_sparse_gemv_bf16_multi_pitch([wide, wide], [n + 128] * 2, [t, 0.0], ys[1:], [n, n],
                                                    xd, m, ws, stream=stream))

    enqueue(torch.cuda.current_stream())
    torch.cuda.synchronize()
    eager = [y.clone() for y in ys]
    assert rel_l2(eager[0].cpu().numpy(), orc.sparse_gemv_bf16(w, x, t)) <= TIGHT
    assert rel_l2(eager[1].cpu().numpy(), orc.sparse_gemv_bf16(w, x, t)) <= TIGHT
    assert rel_l2(eager[2].cpu().numpy(), orc.sparse_gemv_bf16(w, x, 0.0)) <= TIGHT
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        enqueue(side)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        enqueue(side)
    for replay in range(3):
        for y in ys:
            y.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(eager, ys):
            assert torch.equal(a, b), replay
        enqueue(torch.cuda.current_stream())
        torch.cuda.synchronize()
        for a, b in zip(eager, ys):
            assert torch.equal(a, b), replay


# ---------------------------------------------------------------------------
# seeded random shapes through the default launch of every format
# ---------------------------------------------------------------------------

def _random_cases(count, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    cases = []
    for _ in range(count):
        n = int(rng.integers(1, 70)) * 32                     # multiple of 32: valid for every format
        m = int(rng.integers(1, 40)) * 128                    # multiple of 128: valid for int4 groups
        if rng.random() < 0.5:
            m += int(rng.integers(1, 128))                    # ragged for bf16 / int8
        p = float(rng.choice([0.0, 0.1, 0.5, 0.77, 0.95, 1.0]))
        dist = "laplace" if rng.random() < 0.5 else "gaussian"
        cases.append((n, m, p, dist))
    return cases


@pytest.mark.parametrize("chunk", range(4))
def test_random_shapes_every_format(T, chunk):
    for n, m, p, dist in _random_cases(10, 1234 + chunk):
        w = ti.weights_bf16(n, m, seed=n * 7 + m)
        x = ti.make_x(m, n + m + 1, dist)
        t = ti.quantile_threshold(x, p)
        xd = dev(x)
        ws = workspace(T, m, n)
        tag = (n, m, p, dist)
        got = run_bf16(T, dev(ti.to_input_channel_major(w)), xd, t, m, n, ws)
        assert rel_l2(got, orc.sparse_gemv_bf16(w, x, t)) <= TIGHT, ("bf16",) + tag
        q, scale = ti.quantize_w8(w)
        got = run_w8(T, dev(q), dev(scale), xd, t, m, n, ws)
        assert rel_l2(got, orc.sparse_gemv_w8(q, scale, x, t)) <= TIGHT, ("w8",) + tag
        if m % 128 == 0:
            q4, s4 = ti.quantize_w4(w, 128)
            got = run_w4(T, dev(q4), dev(s4), xd, t, m, n, ws)
            assert rel_l2(got, orc.sparse_gemv_w4(q4, s4, 128, x, t)) <= 1e-4, ("w4",) + tag


def test_concurrent_streams_and_host_threads(T):
    """The library keeps no state between calls: calls on different streams with different
    workspaces, issued from different host threads at the same time, give the bits of the same
    calls issued one after the other."""
    import threading
    m, ns = 4096, [1032, 4096, 520]
    x = ti.laplace_x(m, 907)
    xd = dev(x)
    t = ti.quantile_threshold(x, 0.5)
    wts = [dev(ti.to_input_channel_major(ti.weights_bf16(n, m, seed=910 + k))) for k, n in enumerate(ns)]
    q, scale = ti.quantize_w8(ti.weights_bf16(1040, m, 915))
    qd, sd = dev(q), dev(scale)

    def sequence(stream, ws, ws8, outs, y8, rounds):
        for _ in range(rounds):
            for wt, n, y in zip(wts, ns, outs):
                T.check(T.teal_sparse_gemv_bf16(wt, xd, t, y, m, n, ws, stream=stream))
            T.check(T.teal_sparse_gemv_bf16_multi(wts[:2], [t, 0.0], outs[3:5], ns[:2], xd, m, ws, stream=stream))
            T.check(T.teal_sparse_gemv_w8(qd, sd, xd, t, y8, m, 1040, ws8, stream=stream))

    def buffers():
        outs = [torch.full((n,), float("nan"), dtype=torch.float32, device="cuda") for n in ns + ns[:2]]
        return (workspace(T, m, sum(ns)), workspace(T, m, 1040), outs,
                torch.full((1040,), float("nan"), dtype=torch.float32, device="cuda"))

    ws, ws8, outs, y8 = buffers()
    sequence(torch.cuda.current_stream().cuda_stream, ws, ws8, outs, y8, 1)
    torch.cuda.synchronize()
    want = [o.clone() for o in outs] + [y8.clone()]
    assert rel_l2(want[1].cpu().numpy(), orc.sparse_gemv_bf16(
        ti.weights_bf16(ns[1], m, seed=911), x, t)) <= TIGHT

    lanes = []
    for _ in range(3):
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        lanes.append((s, buffers()))
    errors = []

    def work(s, bufs):
        try:
            sequence(s.cuda_stream, *bufs, 25)
        except Exception as e:                     # noqa: BLE001 - reported below
            errors.append(e)

    threads = [threading.Thread(target=work, args=lane) for lane in lanes]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for _, (_, _, got, got8) in lanes:
        for a, b in zip(want, got + [got8]):
            assert torch.equal(a, b)


def test_stream_read_probe_reads_every_vector(T):
    """The measurement aid reads all of its range: a single non-zero word anywhere in it is
    found by exactly the block whose thread reads that vector."""
    blocks = 24
    threads = blocks * 512
    for vecs in (1, 511, threads * 8 + 37, threads * 19 + 5):
        buf = torch.zeros(vecs * 4, dtype=torch.int32, device="cuda")
        for v in sorted({0, vecs // 2, vecs - 1}):
            buf.zero_()
            buf[4 * v + 3] = 5
            sink = torch.full((blocks,), 7, dtype=torch.int32, device="cuda")
            T.check(T.teal_stream_read_probe(buf, 16 * vecs, blocks, 5, sink))
            torch.cuda.synchronize()
            want = [7] * blocks
            want[(v % threads) // 512] = 5
            assert sink.cpu().tolist() == want, (vecs, v)
        sink = torch.full((blocks,), 7, dtype=torch.int32, device="cuda")
        T.check(T.teal_stream_read_probe(buf, 16 * vecs, blocks, 9, sink))
        torch.cuda.synchronize()
        assert sink.cpu().tolist() == [7] * blocks
    assert T.teal_stream_read_probe(buf, 24, blocks, 0, sink) == T.TEAL_ERR_SHAPE
    assert T.teal_stream_read_probe(buf, 16, 0, 0, sink) == T.TEAL_ERR_SHAPE
