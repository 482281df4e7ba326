"""Pins for the CPU oracle: each test checks it against something other than
itself -- the bit-level format definitions as numpy/torch implement them, the
hand-worked example, brute-force enumeration, exact rational arithmetic, a
dense library product, the order statistic behind the threshold, and the
closed-form error of Theorem A.1.  CPU only."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import teal_inputs as ti
from oracle import teal_oracle as orc


# ---------------------------------------------------------------------------
# storage-format decoders, all 65536 patterns each
# ---------------------------------------------------------------------------

def test_f16_decoder_matches_numpy_on_every_pattern():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([orc.f16_bits_to_f64(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_bf16_decoder_matches_torch_on_every_pattern():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    tt = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16)
    want = tt.to(torch.float64).numpy()
    got = np.array([orc.bf16_bits_to_f64(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


# ---------------------------------------------------------------------------
# hand-worked example (tests/golden/def1_worked_example.txt)
# ---------------------------------------------------------------------------

def _read_example(golden_dir):
    d = {}
    with open(os.path.join(golden_dir, "def1_worked_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            d[k] = [float(s) for s in v]
    m, n = int(d["m"][0]), int(d["n"][0])
    w = np.array([d[f"W{j}"] for j in range(n)], dtype=np.float32)
    assert w.shape == (n, m)
    return d, ti.f32_to_bf16_bits(w), np.array(d["x"], dtype=np.float16)


def test_worked_example_mask_and_output(golden_dir):
    d, w_bits, x = _read_example(golden_dir)
    xs, mask, idx, count = orc.sparsify(x, d["t"][0])
    assert mask.tolist() == [int(v) for v in d["mask"]]
    assert idx.tolist() == [int(v) for v in d["idx"]]
    assert count == int(d["count"][0])
    assert xs.tolist() == [0.0, -2.0, 0.0, 1.5, 0.0, 0.0]
    y = orc.sparse_gemv_bf16(w_bits, x, d["t"][0])
    assert y.tolist() == d["y"]                      # short dyadic sums: exact
    assert orc.sparse_gemv_bf16(w_bits, x, 0.0).tolist() == d["y_dense"]
    rows = orc.sparse_gemv_bf16_rows(w_bits, x, d["t"][0], [2, 0])
    assert rows.tolist() == [d["y"][2], d["y"][0]]


# ---------------------------------------------------------------------------
# Definition 1 by brute-force enumeration, ties included
# ---------------------------------------------------------------------------

def _brute_mask(x_f16, t):
    """Definition 1 spelled out in exact rational arithmetic."""
    keep = []
    for v in x_f16.tolist():
        if math.isnan(v):
            keep.append(0)
        elif math.isinf(v):
            keep.append(1)
        else:
            keep.append(1 if abs(Fraction(v)) > Fraction(t) else 0)
    return keep


def test_mask_bruteforce_every_threshold_on_tiny_vectors():
    rng = np.random.default_rng(7)
    for trial in range(40):
        m = int(rng.integers(1, 17))
        # coarse grid so that equal magnitudes (ties, +/- pairs, zeros) are common
        x = (rng.integers(-6, 7, m) / 4.0).astype(np.float16)
        mags = sorted(set(np.abs(x.astype(np.float64)).tolist()))
        mids = [(a + b) / 2 for a, b in zip(mags, mags[1:])]
        for t in [0.0] + mags + mids + [mags[-1] + 1.0]:
            xs, mask, idx, count = orc.sparsify(x, t)
            want = _brute_mask(x, t)
            assert mask.tolist() == want
            assert idx.tolist() == [i for i, k in enumerate(want) if k]
            assert count == sum(want)
            assert np.all(np.diff(idx) > 0)
            xf = x.astype(np.float64)
            assert xs.tolist() == [xf[i] if want[i] else 0.0 for i in range(m)]


def test_tie_at_threshold_is_zeroed_and_special_values():
    x = np.array([1.0, -1.0, 1.0009765625, 0.0, -0.0, np.nan, np.inf, -np.inf,
                  6e-8, -65504.0], dtype=np.float16)
    xs, mask, idx, count = orc.sparsify(x, 1.0)
    #            1  -1  1+ulp 0  -0  nan inf -inf tiny -max
    assert mask.tolist() == [0, 0, 1, 0, 0, 0, 1, 1, 0, 1]
    assert count == 4 and idx.tolist() == [2, 6, 7, 9]
    assert xs[5] == 0.0 and xs[6] == np.inf and xs[7] == -np.inf
    # t = 0 drops only the zeros (and NaN); the smallest subnormal survives
    _, mask0, _, count0 = orc.sparsify(x, 0.0)
    assert mask0.tolist() == [1, 1, 1, 0, 0, 0, 1, 1, 1, 1] and count0 == 7
    # empty input
    _, mask_e, idx_e, count_e = orc.sparsify(np.zeros(0, np.float16), 0.5)
    assert mask_e.size == 0 and idx_e.size == 0 and count_e == 0


# ---------------------------------------------------------------------------
# y against exact rational arithmetic on tiny shapes
# ---------------------------------------------------------------------------

def _exact_y(w_bits, x_f16, t):
    w = ti.bf16_bits_to_f32(w_bits).astype(np.float64)
    n, m = w.shape
    keep = _brute_mask(x_f16, t)
    out = []
    for j in range(n):
        acc = Fraction(0)
        for i in range(m):
            if keep[i]:
                acc += Fraction(float(x_f16[i])) * Fraction(float(w[j, i]))
        out.append(acc)
    return out


def test_output_matches_exact_rationals_on_tiny_shapes():
    rng = np.random.default_rng(11)
    for trial in range(30):
        m = int(rng.integers(1, 9))
        n = int(rng.integers(1, 5))
        x = rng.standard_normal(m).astype(np.float16)
        w_bits = ti.f32_to_bf16_bits((0.02 * rng.standard_normal((n, m))).astype(np.float32))
        for p in (0.0, 0.3, 0.5, 0.9, 1.0):
            t = ti.quantile_threshold(x, p)
            y = orc.sparse_gemv_bf16(w_bits, x, t)
            exact = _exact_y(w_bits, x, t)
            for got, want in zip(y.tolist(), exact):
                scale = max(abs(float(want)), 1e-300)
                assert abs(Fraction(got) - want) <= Fraction(1e-15) * Fraction(scale) + Fraction(1, 10**300)


# ---------------------------------------------------------------------------
# y against a dense library product
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("n,m", [(24, 40), (130, 67), (512, 768)])
def test_t0_equals_dense_library_gemv(n, m):
    w_bits = ti.weights_bf16(n, m, seed=100 + n)
    x = ti.gaussian_x(m, seed=200 + m)
    y = orc.sparse_gemv_bf16(w_bits, x, 0.0)
    dense = ti.bf16_bits_to_f32(w_bits).astype(np.float64) @ x.astype(np.float64)
    assert np.linalg.norm(y - dense) <= 1e-13 * np.linalg.norm(dense)


@pytest.mark.parametrize("n,m,dist", [(24, 40, "gaussian"), (130, 67, "laplace"),
                                      (512, 768, "gaussian")])
@pytest.mark.parametrize("p", [0.25, 0.5, 0.9, 1.0])
def test_equals_dense_product_on_explicitly_zeroed_x(n, m, dist, p):
    w_bits = ti.weights_bf16(n, m, seed=300 + n)
    x = ti.make_x(m, 400 + m, dist)
    t = ti.quantile_threshold(x, p)
    y = orc.sparse_gemv_bf16(w_bits, x, t)
    xd = x.astype(np.float64)
    xz = np.where(np.abs(xd) > t, xd, 0.0)          # (x . s), s = [|x| > t]
    dense = ti.bf16_bits_to_f32(w_bits).astype(np.float64) @ xz
    if p == 1.0:
        assert np.all(y == 0.0) and np.all(dense == 0.0)
    else:
        assert np.linalg.norm(y - dense) <= 1e-13 * np.linalg.norm(dense)
    # kept part + dropped part = the dense product (s_t(x) + (x - s_t(x)) = x)
    full = orc.sparse_gemv_bf16(w_bits, x, 0.0)
    xdrop = np.where(np.abs(xd) > t, 0.0, xd)
    rest = ti.bf16_bits_to_f32(w_bits).astype(np.float64) @ xdrop
    assert np.linalg.norm(y + rest - full) <= 1e-12 * max(np.linalg.norm(full), 1e-300)


def test_selected_rows_agree_with_full_output():
    w_bits = ti.weights_bf16(96, 160, seed=5)
    x = ti.laplace_x(160, seed=6)
    t = ti.quantile_threshold(x, 0.5)
    y = orc.sparse_gemv_bf16(w_bits, x, t)
    rows = np.array([95, 0, 17, 17, 64], np.int32)
    assert np.array_equal(orc.sparse_gemv_bf16_rows(w_bits, x, t, rows), y[rows])


def test_single_entry_probes_orientation():
    """W[j][i] = 1 at one place: y must light up at j for input i, not the transpose."""
    n, m = 5, 9
    for (j, i) in [(0, 8), (4, 0), (2, 5)]:
        w = np.zeros((n, m), np.float32)
        w[j, i] = 1.0
        x = np.arange(1, m + 1).astype(np.float16)
        y = orc.sparse_gemv_bf16(ti.f32_to_bf16_bits(w), x, 0.0)
        want = np.zeros(n)
        want[j] = float(i + 1)
        assert np.array_equal(y, want)


# ---------------------------------------------------------------------------
# sparsity vs the order statistic that chose t
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("dist", ["gaussian", "laplace"])
@pytest.mark.parametrize("m", [4096, 11008, 14336])
@pytest.mark.parametrize("p", [0.0, 0.25, 0.4, 0.5, 0.65, 0.8, 0.9])
def test_measured_sparsity_matches_quantile_threshold(dist, m, p):
    x = ti.make_x(m, 900 + m, dist)
    t = ti.quantile_threshold(x, p)
    _, mask, idx, count = orc.sparsify(x, t)
    zeros = m - count                                # entries with |x_i| <= t
    k = ti.quantile_rank(m, p)
    mags = np.abs(x.astype(np.float64))
    if p == 0.0:
        assert t == 0.0 and zeros == int(np.sum(mags == 0.0))
        return
    ties = int(np.sum(mags == t))
    assert ties >= 1
    assert k <= zeros <= k + ties - 1
    assert abs(zeros / m - p) <= (1 + ties) / m
    assert count + zeros == m and int(mask.sum()) == count and idx.size == count


# ---------------------------------------------------------------------------
# Theorem A.1
# ---------------------------------------------------------------------------

def _read_thm(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "thm_a1_relative_error.txt")) as f:
        for line in f:
            if not line.startswith("#"):
                rows.append(tuple(float(s) for s in line.split()))
    return rows


def test_theorem_a1_table_matches_the_integral(golden_dir):
    """Var of the dropped part is the integral of x^2 phi(x) over [-t, t]."""
    from scipy.integrate import quad
    from scipy.stats import norm
    for p, t, err in _read_thm(golden_dir):
        assert abs((2 * norm.cdf(t) - 1) - p) < 1e-5
        var, _ = quad(lambda u: u * u * norm.pdf(u), -t, t)
        assert abs(math.sqrt(var) - err) < 2e-5


def test_oracle_reproduces_theorem_a1(golden_dir):
    """Gaussian x, Gaussian W: ||Y - Yhat|| / ||Y|| ~ sqrt(p - 2 t phi(t)).

    The theorem is a ratio of expectations; averaged over 8 draws of x at
    m = 4096, n = 512 the empirical ratio sits within 5% of it."""
    n, m = 512, 4096
    w_bits = ti.weights_bf16(n, m, seed=1234)
    xs = [ti.gaussian_x(m, seed=5000 + k) for k in range(8)]
    dense = [orc.sparse_gemv_bf16(w_bits, x, 0.0) for x in xs]
    for p, _, err in _read_thm(golden_dir):
        num = den = 0.0
        for x, yd in zip(xs, dense):
            t = ti.quantile_threshold(x, p)
            ys = orc.sparse_gemv_bf16(w_bits, x, t)
            num += np.linalg.norm(yd - ys)
            den += np.linalg.norm(yd)
        assert abs(num / den - err) <= 0.05 * err, (p, num / den, err)


# ---------------------------------------------------------------------------
# weight-quantised variants
# ---------------------------------------------------------------------------

def _unpack_w4(packed, n):
    lo = (packed & 0x0F).astype(np.int16)
    hi = (packed >> 4).astype(np.int16)
    q = np.empty((packed.shape[0], n), np.int16)
    q[:, 0::2] = lo
    q[:, 1::2] = hi
    return np.where(q >= 8, q - 16, q).astype(np.float64)


@pytest.mark.parametrize("p", [0.0, 0.4, 0.5])
def test_w8_equals_dequantise_then_dense(p):
    n, m = 96, 256
    w_bits = ti.weights_bf16(n, m, seed=31)
    q, scale = ti.quantize_w8(w_bits)
    assert q.shape == (m, n) and scale.shape == (n,)
    x = ti.gaussian_x(m, seed=32)
    t = ti.quantile_threshold(x, p)
    y = orc.sparse_gemv_w8(q, scale, x, t)
    wd = (q.astype(np.float64) * scale.astype(np.float64)[None, :]).T     # [n][m]
    xd = x.astype(np.float64)
    want = wd @ np.where(np.abs(xd) > t, xd, 0.0)
    assert np.linalg.norm(y - want) <= 1e-13 * np.linalg.norm(want)
    # the quantised weights are close to the originals (8-bit RTN: <= scale/2)
    w = ti.bf16_bits_to_f32(w_bits).astype(np.float64)
    assert np.all(np.abs(wd - w) <= 0.5 * scale.astype(np.float64)[:, None] * (1 + 1e-9))


@pytest.mark.parametrize("p", [0.0, 0.4, 0.5])
def test_w4_equals_dequantise_then_dense(p):
    n, m, group = 64, 384, 128
    w_bits = ti.weights_bf16(n, m, seed=41)
    packed, scale = ti.quantize_w4(w_bits, group)
    assert packed.shape == (m, n // 2) and scale.shape == (m // group, n)
    x = ti.laplace_x(m, seed=42)
    t = ti.quantile_threshold(x, p)
    y = orc.sparse_gemv_w4(packed, scale, group, x, t)
    qv = _unpack_w4(packed, n)                                            # [m][n]
    sc = np.repeat(scale.astype(np.float64), group, axis=0)               # [m][n]
    wd = (qv * sc).T
    xd = x.astype(np.float64)
    want = wd @ np.where(np.abs(xd) > t, xd, 0.0)
    assert np.linalg.norm(y - want) <= 1e-13 * np.linalg.norm(want)
    w = ti.bf16_bits_to_f32(w_bits).astype(np.float64)
    assert np.all(np.abs(wd - w) <= 0.5 * sc.T * (1 + 1e-9))


def test_w4_nibble_order_and_scale_indexing_by_hand():
    """One non-zero nibble at a time; expected values written out by hand."""
    m, n, group = 256, 4, 128
    x = np.zeros(m, np.float16)
    x[3] = 2.0          # group 0
    x[200] = -1.0       # group 1
    scale = np.ones((2, n), np.float16)
    scale[0] = [1.0, 2.0, 4.0, 8.0]
    scale[1] = [0.5, 0.25, 0.125, 16.0]
    # low nibble of byte 0 is output 0, high nibble is output 1, byte 1: outputs 2, 3
    for (i, byte_col, byte, want) in [
        (3, 0, 0x05, [2.0 * 5 * 1.0, 0, 0, 0]),            # low nibble +5 -> j = 0
        (3, 0, 0x50, [0, 2.0 * 5 * 2.0, 0, 0]),            # high nibble +5 -> j = 1
        (3, 1, 0x0F, [0, 0, 2.0 * -1 * 4.0, 0]),           # 0xF = -1 -> j = 2
        (200, 1, 0x90, [0, 0, 0, -1.0 * -7 * 16.0]),       # 0x9 = -7 -> j = 3, group 1
        (200, 0, 0x37, [-1.0 * 7 * 0.5, -1.0 * 3 * 0.25, 0, 0]),
    ]:
        packed = np.zeros((m, n // 2), np.uint8)
        packed[i, byte_col] = byte
        y = orc.sparse_gemv_w4(packed, scale, group, x, 0.0)
        assert y.tolist() == [float(v) for v in want]


def test_w8_layout_by_hand():
    m, n = 3, 2
    q = np.array([[1, -2], [3, 4], [-127, 0]], np.int8)     # q[i][j]
    scale = np.array([0.5, 2.0], np.float16)
    x = np.array([1.0, 10.0, 0.25], np.float16)
    # t = 0.25 drops i = 2 (tie): y0 = (1*1 + 10*3)*0.5 = 15.5, y1 = (-2 + 40)*2 = 76
    assert orc.sparse_gemv_w8(q, scale, x, 0.25).tolist() == [15.5, 76.0]
    # t = 0: y0 = 15.5 + 0.25*(-127)*0.5 = -0.375
    assert orc.sparse_gemv_w8(q, scale, x, 0.0).tolist() == [-0.375, 76.0]
