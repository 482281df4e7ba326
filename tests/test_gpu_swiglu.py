"""GPU parity of the W_down step with its input formed in the kernel (Appendix A.3):
the intermediate h = fp16(SiLU(gate) * up) must equal the oracle's bit for bit (it decides
the mask), the mask of h likewise, and y must agree to relative L2 <= 2e-3."""
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


def gpu_h(T, g, u):
    m = g.size
    h = torch.full((max(m, 1),), 0x7E00, dtype=torch.int16, device="cuda")
    T.check(T.teal_swiglu_f16(dev(g), dev(u), h, m))
    torch.cuda.synchronize()
    return h.cpu().numpy()[:m].view(np.uint16)


def special_inputs():
    g = np.array([0.0, -0.0, 1.0, -1.0, 20.0, -20.0, 79.9, -79.9, 80.0, -80.0, 88.0, -88.0, 100.0,
                  -100.0, 1e-30, -1e-30, 1e-40, 3e38, -3e38, np.inf, -np.inf, np.nan, 1.0, 2.5,
                  -1.2784645, 0.34657359, -0.34657359, 0.69314718, 11.09, 65504.0], np.float32)
    u = np.array([1.0, 1.0, 1.0, 1.0, 1.0, 1.0, 1.0, 1.0, 1.0, 1.0, 1.0, 1.0, 1.0,
                  6e4, 1.0, 1.0, 1.0, 1.0, 1.0, 2.0, 2.0, 1.0, np.nan, np.inf,
                  1.0, 1e-5, 6e4, -3.0, 5907.0, 1.0], np.float32)
    return g, u


def test_intermediate_bit_exact_on_special_values(T):
    g, u = special_inputs()
    want = orc.swiglu_f16(g, u).view(np.uint16)
    got = gpu_h(T, g, u)
    nan = (want & 0x7FFF) > 0x7C00
    assert np.array_equal((got & 0x7FFF) > 0x7C00, nan)
    assert np.array_equal(got[~nan], want[~nan])


@pytest.mark.parametrize("m", [1, 255, 256, 257, 4096, 14336, 28672])
def test_intermediate_bit_exact(T, m):
    g, u = ti.mlp_gate_up(m, 40 + m)
    assert np.array_equal(gpu_h(T, g, u), orc.swiglu_f16(g, u).view(np.uint16))
    # wide ranges: large gates (sigma saturates), tiny and huge products (fp16 subnormals, overflow)
    rng = np.random.Generator(np.random.PCG64(m))
    g2 = (rng.standard_normal(m) * np.exp(rng.uniform(-8, 5, m))).astype(np.float32)
    u2 = (rng.standard_normal(m) * np.exp(rng.uniform(-12, 9, m))).astype(np.float32)
    assert np.array_equal(gpu_h(T, g2, u2), orc.swiglu_f16(g2, u2).view(np.uint16))


def test_rounding_of_the_product_is_two_step(T):
    """Entries whose exact product lies within half an fp32 ulp of an fp16 rounding tie:
    rounding once and rounding twice differ there; both sides must round twice."""
    rng = np.random.Generator(np.random.PCG64(77))
    m = 1 << 20
    g = (rng.standard_normal(m) * 1.5).astype(np.float32)
    u = rng.standard_normal(m).astype(np.float32)
    want = orc.swiglu_f16(g, u).view(np.uint16)
    assert np.array_equal(gpu_h(T, g, u), want)


def run_fused(T, wt, g, u, t, m, n, ws):
    y = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    T.check(T.teal_sparse_gemv_bf16_swiglu(wt, dev(g), dev(u), t, y, m, n, ws))
    torch.cuda.synchronize()
    return y.cpu().numpy()


@pytest.mark.parametrize("n,m", [(8, 1), (72, 200), (1032, 2049), (520, 4096), (4096, 14336),
                                 (4096, 11008)])
def test_fused_product_against_oracle_and_unfused(T, n, m):
    w = ti.weights_bf16(n, m, 300 + n + m)
    wt = dev(ti.to_input_channel_major(w))
    g, u = ti.mlp_gate_up(m, 7 + m)
    h = orc.swiglu_f16(g, u)
    ws = torch.zeros(T.teal_workspace_bytes(m, n), dtype=torch.uint8, device="cuda")
    hd = torch.empty(m, dtype=torch.int16, device="cuda")
    T.check(T.teal_swiglu_f16(dev(g), dev(u), hd, m))
    for p in (0.0, 0.5, 0.9, 1.0):
        t = ti.quantile_threshold(h, p)
        want = orc.sparse_gemv_bf16_swiglu(w, g, u, t)
        got = run_fused(T, wt, g, u, t, m, n, ws)
        assert rel_l2(got, want) <= TIGHT, p
        assert rel_l2(got, want) <= TOL_BF16
        # the count of surviving channels the fused call leaves in its workspace
        off = T.teal_survivors_offset()
        assert ws[off:off + 4].view(torch.int32).item() == orc.sparsify(h, t)[3], p
        # bitwise the two-launch path: producer kernel, then the plain call
        y2 = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
        T.check(T.teal_sparse_gemv_bf16(wt, hd, t, y2, m, n, ws))
        torch.cuda.synchronize()
        assert np.array_equal(got, y2.cpu().numpy()), p
        # mask of the intermediate, bit-exact
        mask = torch.empty(m, dtype=torch.uint8, device="cuda")
        count = torch.empty(1, dtype=torch.int32, device="cuda")
        T.check(T.teal_sparsify(hd, m, t, mask, None, count))
        torch.cuda.synchronize()
        _, mask_o, _, count_o = orc.sparsify(h, t)
        assert int(count.item()) == count_o and np.array_equal(mask.cpu().numpy(), mask_o)


def test_fused_product_with_nan_and_saturated_gates(T):
    n, m = 264, 1000
    w = ti.weights_bf16(n, m, 5)
    wt = dev(ti.to_input_channel_major(w))
    g, u = ti.mlp_gate_up(m, 6)
    g[3] = np.nan
    u[10] = np.nan
    g[20], g[21] = 500.0, -500.0
    h = orc.swiglu_f16(g, u)
    t = ti.quantile_threshold(np.nan_to_num(h, nan=0.0).astype(np.float16), 0.5)
    ws = torch.zeros(T.teal_workspace_bytes(m, n), dtype=torch.uint8, device="cuda")
    want = orc.sparse_gemv_bf16_swiglu(w, g, u, t)
    got = run_fused(T, wt, g, u, t, m, n, ws)
    assert np.isfinite(got).all() and rel_l2(got, want) <= TIGHT


@pytest.mark.parametrize("n,m", [(16, 1), (80, 200), (1040, 2049), (528, 4096), (4096, 14336)])
def test_fused_product_int8_weights(T, n, m):
    """teal_sparse_gemv_w8_swiglu: the oracle's int8 product on the oracle's intermediate,
    bitwise the producer kernel followed by teal_sparse_gemv_w8, exact survivor count."""
    q, scale = ti.quantize_w8(ti.weights_bf16(n, m, 900 + n + m))
    qd, sd = dev(q), dev(scale)
    g, u = ti.mlp_gate_up(m, 17 + m)
    h = orc.swiglu_f16(g, u)
    gd, ud = dev(g), dev(u)
    ws = torch.zeros(T.teal_workspace_bytes(m, n), dtype=torch.uint8, device="cuda")
    hd = torch.empty(m, dtype=torch.int16, device="cuda")
    T.check(T.teal_swiglu_f16(gd, ud, hd, m))
    for p in (0.0, 0.5, 0.9, 1.0):
        t = ti.quantile_threshold(h, p)
        y = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
        T.check(T.teal_sparse_gemv_w8_swiglu(qd, sd, gd, ud, t, y, m, n, ws))
        torch.cuda.synchronize()
        got = y.cpu().numpy()
        assert rel_l2(got, orc.sparse_gemv_w8(q, scale, h, t)) <= TIGHT, p
        off = T.teal_survivors_offset()
        assert ws[off:off + 4].view(torch.int32).item() == orc.sparsify(h, t)[3], p
        y2 = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
        T.check(T.teal_sparse_gemv_w8(qd, sd, hd, t, y2, m, n, ws))
        torch.cuda.synchronize()
        assert np.array_equal(got, y2.cpu().numpy()), p


@pytest.mark.parametrize("n,m", [(32, 128), (96, 256), (1056, 2048), (544, 4096), (4096, 14336)])
def test_fused_product_int4_weights(T, n, m):
    """teal_sparse_gemv_w4_swiglu: the oracle's int4 product on the oracle's intermediate,
    bitwise the producer kernel followed by teal_sparse_gemv_w4, exact survivor count."""
    q, scale = ti.quantize_w4(ti.weights_bf16(n, m, 950 + n + m), 128)
    qd, sd = dev(q), dev(scale)
    g, u = ti.mlp_gate_up(m, 19 + m)
    h = orc.swiglu_f16(g, u)
    gd, ud = dev(g), dev(u)
    ws = torch.zeros(T.teal_workspace_bytes(m, n), dtype=torch.uint8, device="cuda")
    hd = torch.empty(m, dtype=torch.int16, device="cuda")
    T.check(T.teal_swiglu_f16(gd, ud, hd, m))
    for p in (0.0, 0.5, 0.9, 1.0):
        t = ti.quantile_threshold(h, p)
        y = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
        T.check(T.teal_sparse_gemv_w4_swiglu(qd, sd, 128, gd, ud, t, y, m, n, ws))
        torch.cuda.synchronize()
        got = y.cpu().numpy()
        assert rel_l2(got, orc.sparse_gemv_w4(q, scale, 128, h, t)) <= TIGHT, p
        off = T.teal_survivors_offset()
        assert ws[off:off + 4].view(torch.int32).item() == orc.sparsify(h, t)[3], p
        y2 = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
        T.check(T.teal_sparse_gemv_w4(qd, sd, 128, hd, t, y2, m, n, ws))
        torch.cuda.synchronize()
        assert np.array_equal(got, y2.cpu().numpy()), p
    assert T.teal_sparse_gemv_w4_swiglu(qd, sd, 64, gd, ud, 0.1, y, m, n, ws) == T.TEAL_ERR_UNSUPPORTED
