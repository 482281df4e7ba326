"""Pins for the oracle's normalised hidden state x = gamma * h / sqrt(mean(h^2) + eps)
(the input of W_q/W_k/W_v and W_gate/W_up, Appendix A.3), which a kernel fused with those
products forms itself.  The scale is checked against closed forms and exact rational
arithmetic, the summation tree against a hand-worked case, the binary16 result against
the exact value within the rounding bound, and the product against the composition with
Definition 1's oracle.  CPU only."""
from decimal import Decimal, getcontext
from fractions import Fraction

import numpy as np
import pytest

import teal_inputs as ti
from oracle import teal_oracle as orc

EPS = float(np.float32(1e-5))


def ulp32(v):
    return float(np.spacing(np.float32(abs(v))))


def exact_scale(h, eps):
    """1 / sqrt(mean(h^2) + eps) from exact rational sums, to 50 digits."""
    getcontext().prec = 60
    ss = sum(Fraction(float(a)) ** 2 for a in h)
    v = ss / len(h) + Fraction(eps)
    return 1 / (Decimal(v.numerator) / Decimal(v.denominator)).sqrt()


def test_scale_closed_forms():
    # |h_j| = 2^k everywhere, eps = 0: mean square 4^k, scale 2^-k exactly, any length
    for k in (-6, 0, 5):
        for m in (1, 2, 7, 64, 1000, 4096):
            h = np.full(m, 2.0 ** k, np.float32)
            h[::3] *= -1
            assert orc.rms_scale(h, 0.0) == 2.0 ** -k, (k, m)
    # the mean divides by m, not by the padded length of the summation tree
    assert orc.rms_scale(np.full(1000, 3.0, np.float32), 0.0) == float(np.float32(1.0 / 3.0))
    # eps sits inside the square root, added to the mean
    assert orc.rms_scale(np.zeros(100, np.float32), 2.0 ** -20) == 1024.0
    assert orc.rms_scale(np.full(100, 2.0 ** -10, np.float32), 3 * 2.0 ** -20) == 512.0
    # one large channel among zeros: mean = c^2 / m
    h = np.zeros(256, np.float32)
    h[77] = -48.0
    assert orc.rms_scale(h, 0.0) == float(np.float32(1.0 / 3.0))


def test_summation_tree_on_a_hand_worked_case():
    # squares 2^54, 1, 1, 1, 4, 1, 1, 1 (one unit in the last place at 2^54 is 4).
    # Adjacent pairs: 2^54 + 1 -> 2^54;  1 + 1 = 2;  4 + 1 = 5;  1 + 1 = 2.
    # Pairs of those: 2^54 + 2 is a tie -> even -> 2^54;  5 + 2 = 7.
    # Halves: 2^54 + 7 -> 2^54 + 8.   (Left to right the sum ends at 2^54 + 4, a tree that
    # pairs j with j + 4 first at 2^54 + 12; the exact sum is 2^54 + 10.)
    h = np.array([2.0 ** 27, 1, 1, 1, 2, 1, 1, 1], np.float32)
    assert orc.sum_of_squares(h) == 2.0 ** 54 + 8
    # seven entries: the eighth leaf is a zero.  2^54, 2, 5, 1 -> 2^54, 6 -> tie -> 2^54 + 8
    assert orc.sum_of_squares(h[:7]) == 2.0 ** 54 + 8
    # three entries pad to four: (2^54 + 1 -> 2^54) + (1 + 0)  -> 2^54
    assert orc.sum_of_squares(h[:3]) == 2.0 ** 54
    assert orc.sum_of_squares(np.array([3.0], np.float32)) == 9.0
    assert orc.sum_of_squares(np.array([], np.float32)) == 0.0


def test_sum_of_squares_within_the_pairwise_bound_of_the_exact_sum():
    for seed, m in ((1, 1), (2, 100), (3, 777), (4, 4096), (5, 5000)):
        h, _ = ti.norm_inputs(m, seed)
        exact = sum(Fraction(float(a)) ** 2 for a in h)
        got = Fraction(orc.sum_of_squares(h))
        # pairwise summation of non-negative terms: relative error <= ceil(log2 m) * 2^-53
        levels = max(int(np.ceil(np.log2(m))), 1)
        assert abs(got - exact) <= exact * levels * Fraction(1, 2 ** 53)


def test_scale_is_the_correctly_rounded_exact_value():
    for seed, m in ((11, 5), (12, 333), (13, 4096), (14, 8192)):
        h, _ = ti.norm_inputs(m, seed)
        for eps in (0.0, EPS, float(np.float32(1e-6))):
            r = orc.rms_scale(h, eps)
            true = exact_scale(h, eps)
            assert abs(Decimal(r) - true) <= Decimal(ulp32(r)) * Decimal("0.5000001")


def test_normalised_state_within_rounding_of_the_exact_value():
    for seed, m in ((21, 64), (22, 1000), (23, 4096)):
        h, gamma = ti.norm_inputs(m, seed)
        x = orc.rmsnorm_f16(h, gamma, EPS)
        true_r = float(exact_scale(h, EPS))
        exact = h.astype(np.float64) * true_r * gamma.astype(np.float64)
        # three binary32 roundings (scale, two products), then one to binary16
        half_ulp16 = np.spacing(np.abs(x).astype(np.float16)).astype(np.float64) / 2
        slack = np.abs(exact) * 3 * 2.0 ** -24
        assert np.all(np.abs(x.astype(np.float64) - exact) <= half_ulp16 + slack)
        # and nearly always the correctly rounded value itself
        assert np.mean(x == exact.astype(np.float16)) > 0.995
        # unit-order Gaussian-shaped output (the input recipe's claim)
        assert 0.3 < np.std(x.astype(np.float64)) < 0.8


def test_normalised_state_exact_cases_pin_indices_and_signs():
    # |h_j| = 4, eps = 0: scale 1/4, x_j = sign(h_j) * gamma_j exactly (gamma fp16-exact)
    m = 300
    rng = np.random.Generator(np.random.PCG64(31))
    sign = np.where(rng.random(m) < 0.5, -1.0, 1.0)
    gamma = rng.standard_normal(m).astype(np.float16).astype(np.float32)
    x = orc.rmsnorm_f16((4.0 * sign).astype(np.float32), gamma, 0.0)
    assert np.array_equal(x.astype(np.float32), (sign * gamma).astype(np.float32))
    # scaling h by a power of two changes nothing when eps = 0
    h, gamma = ti.norm_inputs(1000, 32)
    a = orc.rmsnorm_f16(h, gamma, 0.0)
    b = orc.rmsnorm_f16(h * np.float32(2.0 ** 9), gamma, 0.0)
    c = orc.rmsnorm_f16(h * np.float32(2.0 ** -7), gamma, 0.0)
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))
    assert np.array_equal(a.view(np.uint16), c.view(np.uint16))
    # a NaN anywhere in h makes the scale, hence every x, NaN (all dropped by Definition 1)
    h2 = h.copy()
    h2[5] = np.nan
    assert np.all(np.isnan(orc.rmsnorm_f16(h2, gamma, EPS)))
    # a NaN in gamma stays local
    g2 = gamma.copy()
    g2[5] = np.nan
    xg = orc.rmsnorm_f16(h, g2, EPS)
    assert np.isnan(xg[5]) and not np.isnan(np.delete(xg, 5)).any()


def test_two_roundings_of_the_product():
    # m = 1, eps = 0, h = 1: scale 1, a = h; b = a * gamma rounds to binary32 first.
    # gamma = 1 + 2^-11 + 2^-30 lies above the tie between 1 and 1 + 2^-10 in binary16, but
    # binary32 cannot hold it: it is stored as 1 + 2^-11, the tie, which goes to even.
    gamma = np.array([1.0 + 2.0 ** -11 + 2.0 ** -30], np.float32)
    assert float(gamma[0]) == 1.0 + 2.0 ** -11
    x = orc.rmsnorm_f16(np.array([1.0], np.float32), gamma, 0.0)
    assert float(x[0]) == 1.0
    # h * r is rounded before gamma multiplies: h = 3, r = binary32(1/3), a = 1 (rounded
    # from 1 + 2^-25...), so x = gamma exactly; unrounded, a * gamma would differ from gamma
    gamma = np.array([1.0 + 2.0 ** -10], np.float32)
    x = orc.rmsnorm_f16(np.array([3.0], np.float32), gamma, 0.0)
    assert float(x[0]) == 1.0 + 2.0 ** -10
    # The order (h * r) * gamma and the rounding of h * r both matter here: h = 7,
    # r = binary32(1/7) = (1 + 2^-25.4..)/7, so h * r = 1 + 4.5e-8 rounds to 1 and b = gamma.
    # gamma = 1580.5 / 1024 is a binary16 tie, which goes to the even 1580 / 1024.  Any
    # variant that keeps the excess of h * r over 1 ((h * gamma) * r, or one rounding of
    # the exact product) lands above the tie and gives 1581 / 1024.
    gamma = np.array([1580.5 / 1024.0], np.float32)
    assert float(gamma[0]) == 1580.5 / 1024.0
    x = orc.rmsnorm_f16(np.array([7.0], np.float32), gamma, 0.0)
    assert float(x[0]) == 1580.0 / 1024.0
    x = orc.rmsnorm_f16(np.array([-7.0], np.float32), gamma, 0.0)
    assert float(x[0]) == -1580.0 / 1024.0


@pytest.mark.parametrize("n,m", [(8, 1), (24, 40), (136, 333), (264, 1000)])
def test_product_is_the_composition_with_definition_1(n, m):
    w = ti.weights_bf16(n, m, seed=40 + n + m)
    h, gamma = ti.norm_inputs(m, 41 + m)
    x = orc.rmsnorm_f16(h, gamma, EPS)
    for p in (0.0, 0.5, 0.9, 1.0):
        t = ti.quantile_threshold(x, p)
        y = orc.sparse_gemv_bf16_rmsnorm(w, h, gamma, EPS, t)
        assert np.array_equal(y, orc.sparse_gemv_bf16(w, x, t))
    # independent dense fp64 product on the zeroed x
    t = ti.quantile_threshold(x, 0.5)
    xs = np.where(np.abs(x.astype(np.float64)) > t, x.astype(np.float64), 0.0)
    want = ti.bf16_bits_to_f32(w).astype(np.float64) @ xs
    got = orc.sparse_gemv_bf16_rmsnorm(w, h, gamma, EPS, t)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-14)
