"""GPU parity of the small-batch variant (Section 5.4.4) against the CPU oracle:
one mask per batch from the batch-averaged magnitude (bit-exact), every row of
the batch times W^T over the kept channels (relative L2 <= 2e-3, bf16 W)."""
import numpy as np
import pytest

import teal_inputs as ti
from oracle import teal_oracle as orc

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-3
TIGHT = 2e-5      # what fp32 accumulation of exact products achieves; catches a dropped row


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


def gpu_sparsify_batch(T, X, t):
    batch, m = X.shape
    mask = torch.full((max(m, 1),), 7, dtype=torch.uint8, device="cuda")
    idx = torch.full((max(m, 1),), -1, dtype=torch.int32, device="cuda")
    count = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    T.check(T.teal_sparsify_batch(dev(X), batch, m, t, mask, idx, count))
    torch.cuda.synchronize()
    return mask.cpu().numpy()[:m], idx.cpu().numpy(), int(count.item())


def run_batch(T, wt_dev, X, t, m, n, ws=None, **shape):
    batch = X.shape[0]
    if ws is None:
        ws = torch.zeros(T.teal_workspace_bytes_batch(m, n, batch), dtype=torch.uint8, device="cuda")
    Y = torch.full((batch, n), float("nan"), dtype=torch.float32, device="cuda")
    if shape:
        T.check(T.teal_sparse_gemv_bf16_batch_ex(wt_dev, dev(X), batch, t, Y, m, n, ws, **shape))
    else:
        T.check(T.teal_sparse_gemv_bf16_batch(wt_dev, dev(X), batch, t, Y, m, n, ws))
    torch.cuda.synchronize()
    return Y.cpu().numpy()


@pytest.mark.parametrize("batch", [1, 3, 8])
@pytest.mark.parametrize("m", [8, 1000, 8192, 8200, 28672, 70000])
@pytest.mark.parametrize("x_off,mask_off", [(0, 0), (0, 5), (4, 0)])
def test_sparsify_batch_every_alignment_and_long_vectors(T, batch, m, x_off, mask_off):
    """X on and off a 16-byte boundary (eight channels per thread, or one), the mask on and
    off an 8-byte boundary, lengths from one vector to several passes of the block."""
    X = ti.make_X(batch, m, 41 * batch + m, "laplace")
    buf = torch.zeros(batch * m + 8, dtype=torch.int16, device="cuda")
    buf[x_off:x_off + batch * m] = torch.from_numpy(X.view(np.int16).reshape(-1)).cuda()
    Xd = buf[x_off:x_off + batch * m]
    for p in (0.0, 0.5, 0.97):
        t = ti.batch_quantile_threshold(X, p)
        _, mask_o, idx_o, count_o = orc.sparsify_batch(X, t)
        mbuf = torch.full((m + 8,), 7, dtype=torch.uint8, device="cuda")
        mask = mbuf[mask_off:mask_off + m]
        idx = torch.full((m,), -1, dtype=torch.int32, device="cuda")
        count = torch.full((1,), -1, dtype=torch.int32, device="cuda")
        T.check(T.teal_sparsify_batch(Xd, batch, m, t, mask, idx, count))
        torch.cuda.synchronize()
        assert int(count.item()) == count_o
        assert np.array_equal(mask.cpu().numpy(), mask_o)
        got = idx.cpu().numpy()
        assert np.array_equal(got[:count_o], idx_o) and np.all(got[count_o:] == -1)
        outside = mbuf.cpu().numpy()
        assert np.all(outside[:mask_off] == 7) and np.all(outside[mask_off + m:] == 7)


@pytest.mark.parametrize("batch", [1, 2, 3, 4, 5, 8])
@pytest.mark.parametrize("m", [1, 64, 65, 1000, 4096, 14336])
def test_sparsify_batch_bit_exact(T, batch, m):
    X = ti.make_X(batch, m, 31 * batch + m, "laplace" if m % 2 else "gaussian")
    for p in (0.0, 0.4, 0.5, 0.9, 1.0):
        t = ti.batch_quantile_threshold(X, p)
        _, mask_o, idx_o, count_o = orc.sparsify_batch(X, t)
        mask, idx, count = gpu_sparsify_batch(T, X, t)
        assert count == count_o
        assert np.array_equal(mask, mask_o)
        assert np.array_equal(idx[:count], idx_o)


def test_sparsify_batch_ties_nan_inf(T):
    X = np.array([[1.0, 1.0, 3.0, 6.0, np.nan, np.inf, 0.0],
                  [-2.0, 2.0, -3.0, 0.0, 100.0, 0.0, -0.0],
                  [3.0, 3.002, 0.0, 0.0, 1.0, 1.0, 0.0]], np.float16)
    for t in (2.0, float(np.nextafter(np.float32(2.0), np.float32(0))), 0.0, 1e4):
        _, mask_o, idx_o, count_o = orc.sparsify_batch(X, t)
        mask, idx, count = gpu_sparsify_batch(T, X, t)
        assert count == count_o and np.array_equal(mask, mask_o) and np.array_equal(idx[:count], idx_o)
    # a mean that only division rounding would put on the wrong side
    Z = np.array([[0.5], [0.25], [0.25]], np.float16)
    for t in (float(np.float32(1.0 / 3.0)), float(np.nextafter(np.float32(1.0 / 3.0), np.float32(0)))):
        assert gpu_sparsify_batch(T, Z, t)[0].tolist() == orc.sparsify_batch(Z, t)[1].tolist()


SMALL = [(8, 1), (16, 63), (72, 200), (264, 1000), (1032, 2049), (520, 4096)]


@pytest.mark.parametrize("batch", [1, 2, 3, 4, 7, 8])
@pytest.mark.parametrize("n,m", SMALL)
def test_gemv_batch_small_shapes(T, batch, n, m):
    w = ti.weights_bf16(n, m, 100 + n + m)
    wt = dev(ti.to_input_channel_major(w))
    X = ti.make_X(batch, m, 7 * batch + n, "gaussian")
    ws = torch.zeros(T.teal_workspace_bytes_batch(m, n, batch), dtype=torch.uint8, device="cuda")
    off = T.teal_survivors_offset()
    for p in (0.0, 0.5, 0.9):
        t = ti.batch_quantile_threshold(X, p)
        want = orc.sparse_gemv_bf16_batch(w, X, t)
        got = run_batch(T, wt, X, t, m, n, ws)
        assert not np.isnan(got).any()
        for b in range(batch):
            assert rel_l2(got[b], want[b]) <= TIGHT, (b, p)
        # the survivor count the call leaves in its workspace
        assert ws[off:off + 4].view(torch.int32).item() == orc.sparsify_batch(X, t)[3], p


@pytest.mark.parametrize("batch,lanes", [(2, 64), (2, 32), (2, 16), (4, 64), (4, 32), (4, 16),
                                         (8, 32), (8, 16), (3, 64), (6, 32)])
def test_gemv_batch_every_variant(T, batch, lanes):
    n, m = 1544, 3000                      # ragged right edge, ragged last slice
    w = ti.weights_bf16(n, m, 5)
    wt = dev(ti.to_input_channel_major(w))
    X = ti.make_X(batch, m, 6 + batch, "laplace")
    t = ti.batch_quantile_threshold(X, 0.5)
    want = orc.sparse_gemv_bf16_batch(w, X, t)
    for splits, tile_cols in ((2, 0), (5, 8 * lanes - 64), (16, 0)):
        got = run_batch(T, wt, X, t, m, n, lanes_per_row=lanes, splits=splits, tile_cols=tile_cols)
        assert rel_l2(got, want) <= TIGHT, (splits, tile_cols)
    assert rel_l2(got, want) <= TOL_BF16


def test_gemv_batch_degenerate_and_reproducible(T):
    n, m = 1024, 4096
    w = ti.weights_bf16(n, m, 9)
    wt = dev(ti.to_input_channel_major(w))
    X = ti.make_X(4, m, 10, "gaussian")
    ws = torch.zeros(T.teal_workspace_bytes_batch(m, n, 4), dtype=torch.uint8, device="cuda")
    # nothing survives: all zeros; the workspace stays usable
    got = run_batch(T, wt, X, 1000.0, m, n, ws)
    assert not got.any()
    # everything survives: the dense product
    W64 = ti.bf16_bits_to_f32(w).astype(np.float64)
    dense = X.astype(np.float64) @ W64.T
    got = run_batch(T, wt, X, 0.0, m, n, ws)
    assert rel_l2(got, dense) <= TIGHT
    # same call twice: bitwise equal (fixed summation order)
    t = ti.batch_quantile_threshold(X, 0.5)
    a = run_batch(T, wt, X, t, m, n, ws)
    b = run_batch(T, wt, X, t, m, n, ws)
    assert np.array_equal(a, b)
    # a batch of one goes through the same kernel and matches Definition 1's product
    x = X[:1]
    t1 = ti.quantile_threshold(x[0], 0.5)
    want = orc.sparse_gemv_bf16(w, x[0], t1)
    assert rel_l2(run_batch(T, wt, x, t1, m, n)[0], want) <= TIGHT


@pytest.mark.parametrize("batch", [2, 4, 8])
@pytest.mark.parametrize("proj", ["gate", "down"])
def test_gemv_batch_full_size(T, batch, proj):
    """Llama-3-8B gate (14336 x 4096) and down (4096 x 14336) in the default launch."""
    n, m = ti.LAYER_SHAPES["llama3_8b"][proj]
    w = ti.weights_bf16(n, m, ti.weight_seed(3, 0, proj))
    wt = dev(ti.to_input_channel_major(w))
    X = ti.make_X(batch, m, 900 + batch, ti.PROJ_DIST[proj])
    t = ti.batch_quantile_threshold(X, 0.5)
    want = orc.sparse_gemv_bf16_batch(w, X, t)
    got = run_batch(T, wt, X, t, m, n)
    for b in range(batch):
        assert rel_l2(got[b], want[b]) <= TIGHT
    mask, _, count = gpu_sparsify_batch(T, X, t)
    assert np.array_equal(mask, orc.sparsify_batch(X, t)[1])
    assert abs(count - m / 2) <= 2


@pytest.mark.parametrize("name,ns,m,ps,batch", [
    ("llama3 q,k,v", [4096, 1024, 1024], 4096, [0.5, 0.4, 0.25], 4),
    ("llama3 gate,up", [14336, 14336], 4096, [0.4, 0.5], 8),
    ("ragged", [520, 24, 136, 8], 333, [0.0, 0.5, 0.9, 1.0], 3),
    ("single", [1032], 2049, [0.5], 2),
    ("one row", [264, 72], 1000, [0.5, 0.5], 1),
], ids=["qkv_b4", "gate_up_b8", "ragged_b3", "single_b2", "pair_b1"])
def test_gemv_batch_multi(T, name, ns, m, ps, batch):
    X = ti.make_X(batch, m, 900 + m + batch, "gaussian")
    Xd = dev(X)
    ws = torch.zeros(T.teal_workspace_bytes_batch(m, sum(ns), batch), dtype=torch.uint8, device="cuda")
    ws_host, wts, ts, Ys = [], [], [], []
    for k, (n, p) in enumerate(zip(ns, ps)):
        w = ti.weights_bf16(n, m, seed=1000 * k + n + m)
        ws_host.append(w)
        wts.append(dev(ti.to_input_channel_major(w)))
        ts.append(ti.batch_quantile_threshold(X, p))
        Ys.append(torch.full((batch, n), float("nan"), dtype=torch.float32, device="cuda"))
    T.check(T.teal_sparse_gemv_bf16_batch_multi(wts, ts, Ys, ns, Xd, batch, m, ws))
    torch.cuda.synchronize()
    off = T.teal_survivors_offset()
    kept = ws[off:off + 4 * len(ns)].view(torch.int32).cpu().tolist()
    assert kept == [orc.sparsify_batch(X, t)[3] for t in ts]
    for k, n in enumerate(ns):
        got = Ys[k].cpu().numpy()
        want = orc.sparse_gemv_bf16_batch(ws_host[k], X, ts[k])
        assert not np.isnan(got).any()
        for b in range(batch):
            assert rel_l2(got[b], want[b]) <= TIGHT, (name, k, b)
    # the shared workspace is left ready: a second call gives the same bits
    Ys2 = [torch.full((batch, n), float("nan"), dtype=torch.float32, device="cuda") for n in ns]
    T.check(T.teal_sparse_gemv_bf16_batch_multi(wts, ts, Ys2, ns, Xd, batch, m, ws))
    torch.cuda.synchronize()
    for a, b in zip(Ys, Ys2):
        assert torch.equal(a, b)


def test_very_long_input(T):
    """More than 128 x 2048 input channels: a block compacts at most 2048 channels of a
    batch, so the call runs with more split-K blocks than the usual 16 partial rows."""
    m, n, batch = 128 * 2048 + 704, 32, 3
    w = ti.weights_bf16(n, m, seed=515151)
    wt = dev(ti.to_input_channel_major(w))
    X = ti.make_X(batch, m, 5151, "laplace")
    t = ti.batch_quantile_threshold(X, 0.5)
    want = orc.sparse_gemv_bf16_batch(w, X, t)
    ws = torch.zeros(T.teal_workspace_bytes_batch(m, 2 * n, batch), dtype=torch.uint8, device="cuda")
    got = run_batch(T, wt, X, t, m, n, ws)
    for b in range(batch):
        assert rel_l2(got[b], want[b]) <= TIGHT, b
    off = T.teal_survivors_offset()
    assert ws[off:off + 4].view(torch.int32).item() == orc.sparsify_batch(X, t)[3]
    Ys = [torch.full((batch, n), float("nan"), dtype=torch.float32, device="cuda") for _ in range(2)]
    t2 = ti.batch_quantile_threshold(X, 0.25)
    T.check(T.teal_sparse_gemv_bf16_batch_multi([wt, wt], [t, t2], Ys, [n, n], dev(X), batch, m, ws))
    torch.cuda.synchronize()
    want2 = orc.sparse_gemv_bf16_batch(w, X, t2)
    for b in range(batch):
        assert rel_l2(Ys[0].cpu().numpy()[b], want[b]) <= TIGHT, b
        assert rel_l2(Ys[1].cpu().numpy()[b], want2[b]) <= TIGHT, b
