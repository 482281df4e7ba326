"""Pins for the oracle's batched sparsification (Section 5.4.4): one mask for a
small batch, from the magnitude averaged over the batch dimension, then every
row times W^T over the kept channels.  CPU only."""
from fractions import Fraction

import numpy as np
import pytest

import teal_inputs as ti
from oracle import teal_oracle as orc


def frac16(v) -> Fraction:
    return Fraction(float(np.float16(v)))


def brute_mask(X, t):
    """mean_b |X[b][i]| > t in exact rational arithmetic."""
    batch, m = X.shape
    tq = Fraction(float(np.float32(t)))
    out = []
    for i in range(m):
        vals = [X[b, i] for b in range(batch)]
        if any(np.isnan(v) for v in vals):
            out.append(0)
            continue
        if any(np.isinf(v) for v in vals):
            out.append(1)
            continue
        mean = sum(abs(frac16(v)) for v in vals) / batch
        out.append(1 if mean > tq else 0)
    return np.array(out, np.uint8)


def test_batch_of_one_is_definition_1():
    for seed in range(5):
        x = ti.gaussian_x(300, seed)
        for p in (0.0, 0.3, 0.5, 0.9):
            t = ti.quantile_threshold(x, p)
            _, mask1, idx1, c1 = orc.sparsify(x, t)
            mean, maskb, idxb, cb = orc.sparsify_batch(x[None, :], t)
            assert np.array_equal(mask1, maskb) and np.array_equal(idx1, idxb) and c1 == cb
            assert np.array_equal(mean, np.abs(x.astype(np.float64)))
    w = ti.weights_bf16(24, 300, 7)
    y1 = orc.sparse_gemv_bf16(w, x, t)
    yb = orc.sparse_gemv_bf16_batch(w, x[None, :], t)
    assert yb.shape == (1, 24) and np.array_equal(y1, yb[0])


@pytest.mark.parametrize("batch", [2, 3, 5, 8])
def test_mask_against_exact_rational_mean(batch):
    rng = np.random.Generator(np.random.PCG64(100 + batch))
    m = 12
    for trial in range(40):
        X = rng.standard_normal((batch, m)).astype(np.float16)
        X[:, 0] = np.float16(0.0)
        means = np.abs(X.astype(np.float64)).mean(axis=0)
        cands = [0.0, float(np.float32(means.max() * 2))]
        for v in means:
            f = np.float32(v)
            cands += [float(f), float(np.nextafter(f, np.float32(0))), float(np.nextafter(f, np.float32(9)))]
        for t in cands:
            _, mask, idx, count = orc.sparsify_batch(X, t)
            want = brute_mask(X, t)
            assert np.array_equal(mask, want), (trial, t)
            assert count == int(want.sum()) and np.array_equal(idx, np.flatnonzero(want))


def test_exact_ties_of_the_mean_are_dropped_and_signs_do_not_cancel():
    # channel 0: magnitudes 1, 2, 3 -> mean exactly 2; channel 1: a hair above;
    # channel 2: +3 and -3 and 0 (mean of |x| is 2, the plain mean is 0);
    # channel 3: one large entry among zeros (max 6, mean 2)
    X = np.array([[1.0, 1.0, 3.0, 6.0],
                  [-2.0, 2.0, -3.0, 0.0],
                  [3.0, 3.002, 0.0, 0.0]], np.float16)
    _, mask, _, count = orc.sparsify_batch(X, 2.0)
    assert mask.tolist() == [0, 1, 0, 0] and count == 1
    _, mask, _, _ = orc.sparsify_batch(X, float(np.nextafter(np.float32(2.0), np.float32(0))))
    assert mask.tolist() == [1, 1, 1, 1]
    # a threshold that 1/3 of the sum only reaches after rounding: t = fp32(1/3), sum = 1
    Y = np.array([[0.5], [0.25], [0.25]], np.float16)
    t = float(np.float32(1.0 / 3.0))          # slightly above 1/3
    assert Fraction(t) > Fraction(1, 3)
    assert orc.sparsify_batch(Y, t)[1].tolist() == [0]
    t_lo = float(np.nextafter(np.float32(1.0 / 3.0), np.float32(0)))
    assert orc.sparsify_batch(Y, t_lo)[1].tolist() == [1]


def test_nan_drops_the_channel_and_inf_keeps_it():
    X = np.array([[1.0, np.nan, np.inf, 5.0],
                  [1.0, 100.0, 0.0, -np.inf]], np.float16)
    _, mask, idx, count = orc.sparsify_batch(X, 0.5)
    assert mask.tolist() == [1, 0, 1, 1] and count == 3 and idx.tolist() == [0, 2, 3]
    assert np.array_equal(mask, brute_mask(X, 0.5))


@pytest.mark.parametrize("batch,n,m,dist", [(2, 40, 333, "gaussian"), (4, 64, 512, "laplace"),
                                             (8, 17, 1000, "gaussian"), (3, 33, 257, "laplace")])
def test_product_equals_dense_numpy_on_masked_rows(batch, n, m, dist):
    w = ti.weights_bf16(n, m, 11 * batch)
    X = ti.make_X(batch, m, 5 + batch, dist)
    W64 = ti.bf16_bits_to_f32(w).astype(np.float64)
    X64 = X.astype(np.float64)
    for p in (0.0, 0.4, 0.5, 0.9, 1.0):
        t = ti.batch_quantile_threshold(X, p)
        _, mask, _, count = orc.sparsify_batch(X, t)
        keep = np.abs(X64).sum(axis=0) > batch * float(np.float32(t))
        assert np.array_equal(mask.astype(bool), keep)
        want = (X64 * keep[None, :]) @ W64.T
        got = orc.sparse_gemv_bf16_batch(w, X, t)
        scale = np.linalg.norm(want) + 1e-300
        assert np.linalg.norm(got - want) / scale < 1e-13
        if p == 0.0:
            assert np.linalg.norm(got - X64 @ W64.T) / np.linalg.norm(X64 @ W64.T) < 1e-13
        if p == 1.0:
            assert count == 0 and not got.any()


def test_identical_rows_reduce_to_the_single_vector_case():
    x = ti.laplace_x(400, 3)
    w = ti.weights_bf16(16, 400, 4)
    t = ti.quantile_threshold(x, 0.5)
    for batch in (2, 3, 7):
        X = np.repeat(x[None, :], batch, axis=0)
        _, mask, _, count = orc.sparsify_batch(X, t)
        _, mask1, _, count1 = orc.sparsify(x, t)
        assert np.array_equal(mask, mask1) and count == count1
        Y = orc.sparse_gemv_bf16_batch(w, X, t)
        y1 = orc.sparse_gemv_bf16(w, x, t)
        for b in range(batch):
            assert np.array_equal(Y[b], y1)


def test_order_of_the_batch_does_not_matter():
    X = ti.make_X(5, 200, 9, "gaussian")
    w = ti.weights_bf16(8, 200, 10)
    t = ti.batch_quantile_threshold(X, 0.5)
    perm = np.array([3, 0, 4, 1, 2])
    _, mask, _, _ = orc.sparsify_batch(X, t)
    _, mask_p, _, _ = orc.sparsify_batch(X[perm], t)
    assert np.array_equal(mask, mask_p)
    Y = orc.sparse_gemv_bf16_batch(w, X, t)
    Yp = orc.sparse_gemv_bf16_batch(w, X[perm], t)
    assert np.array_equal(Y[perm], Yp)


@pytest.mark.parametrize("batch", [2, 4, 8])
def test_measured_sparsity_matches_the_quantile_of_the_mean(batch):
    m = 4096
    X = ti.make_X(batch, m, 77, "gaussian")
    mean = np.abs(X.astype(np.float64)).sum(axis=0) / batch
    for p in (0.25, 0.5, 0.65, 0.9):
        k = ti.quantile_rank(m, p)
        t = ti.batch_quantile_threshold(X, p)
        _, _, _, count = orc.sparsify_batch(X, t)
        dropped = m - count
        assert dropped >= k
        assert dropped == int((mean <= float(np.float32(t))).sum())   # batch is a power of two: mean is exact
        assert dropped <= k + 2


def test_a_common_mask_differs_from_each_rows_own_choice():
    """Section 5.4.4: different inputs prefer different sparsity patterns.  For
    independent rows the batch-wide mask at 50% agrees with each row's own 50%
    mask on clearly more than half of the channels, and on clearly fewer than all."""
    m = 8192
    X = ti.make_X(4, m, 5, "gaussian")
    t = ti.batch_quantile_threshold(X, 0.5)
    _, mask, _, _ = orc.sparsify_batch(X, t)
    rows = [orc.sparsify(X[b], ti.quantile_threshold(X[b], 0.5))[1] for b in range(4)]
    agree = np.mean([np.mean(mask == r) for r in rows])
    assert 0.55 < agree < 0.9
