"""Pins for the oracle's threshold calibration (Section 4.2): the k-th smallest
|x| over a sample, against numpy's selection, a brute-force reading of the
definition, and the histogram route (counting sort) as a cross-check."""
import numpy as np
import pytest

import teal_inputs as ti
from oracle import teal_oracle as orc

LEVELS = [0.0, 0.1, 0.25, 0.3, 0.4, 0.5, 0.65, 0.8, 0.9, 0.999, 1.0]


def _brute(x, p):
    """Smallest sample magnitude t with #{|x| <= t} >= p N (0 when p N rounds to 0)."""
    mags = np.abs(x[~np.isnan(x)].astype(np.float64))
    n = mags.size
    if n == 0 or p * n <= 1e-9:
        return 0.0
    for t in np.unique(mags):
        if np.count_nonzero(mags <= t) >= p * n - 1e-9:
            return float(t)
    raise AssertionError


@pytest.mark.parametrize("dist", ["gaussian", "laplace"])
@pytest.mark.parametrize("m", [1, 10, 4096, 14336])
def test_threshold_matches_numpy_selection(dist, m):
    x = ti.make_x(m, 31 + m, dist)
    for p in LEVELS:
        assert orc.quantile_threshold(x, p) == ti.quantile_threshold(x, p), (m, p)


def test_threshold_is_the_definition_on_small_samples():
    rng = np.random.default_rng(3)
    for trial in range(60):
        m = int(rng.integers(1, 40))
        x = (rng.integers(-8, 9, m) / 4.0).astype(np.float16)      # many ties and zeros
        if trial % 5 == 0:
            x[rng.integers(0, m)] = np.nan
        if trial % 7 == 0:
            x[rng.integers(0, m)] = np.inf
        for p in LEVELS:
            assert orc.quantile_threshold(x, p) == _brute(x, p), (x, p)


def test_rank_guards_binary_roundoff_and_clamps():
    assert orc.quantile_rank(10, 0.3) == 3
    assert orc.quantile_rank(4096, 0.4) == 1639
    assert orc.quantile_rank(4096, 0.5) == 2048
    assert orc.quantile_rank(7, 1.0) == 7
    assert orc.quantile_rank(7, 0.0) == 0
    assert orc.quantile_rank(0, 0.5) == 0


def test_special_values_and_empty():
    x = np.array([np.nan, -np.inf, 0.0, -0.0, 6e-8, -65504.0, np.nan], np.float16)
    # valid sample: inf, 0, 0, 6e-8, 65504  (N = 5)
    assert orc.quantile_threshold(x, 0.2) == 0.0
    assert orc.quantile_threshold(x, 0.4) == 0.0
    assert orc.quantile_threshold(x, 0.6) == float(np.float16(6e-8))
    assert orc.quantile_threshold(x, 0.8) == 65504.0
    assert orc.quantile_threshold(x, 1.0) == np.inf
    assert orc.quantile_threshold(np.zeros(0, np.float16), 0.5) == 0.0
    assert orc.quantile_threshold(np.full(3, np.nan, np.float16), 0.5) == 0.0


def test_histogram_counts_every_pattern_and_selects_the_same_threshold():
    x = np.concatenate([ti.gaussian_x(50_000, 1), ti.laplace_x(50_000, 2),
                        np.array([np.nan, np.inf, -np.inf, 0.0, -0.0], np.float16)])
    hist = orc.abs_histogram(x)
    bits = x.view(np.uint16) & 0x7FFF
    want = np.bincount(bits[bits <= 0x7C00], minlength=32768).astype(np.uint64)
    assert np.array_equal(hist, want)
    assert int(hist.sum()) == x.size - 1
    # accumulation
    h2 = orc.abs_histogram(x[:1000])
    orc.abs_histogram(x[1000:], h2)
    assert np.array_equal(h2, hist)
    # counting-sort selection from the histogram equals the sort-based threshold
    cum = np.cumsum(hist)
    for p in LEVELS:
        k = orc.quantile_rank(int(cum[-1]), p)
        t = 0.0 if k == 0 else float(np.array([np.searchsorted(cum, k)], np.uint16).view(np.float16)[0])
        assert t == orc.quantile_threshold(x, p), p


def test_threshold_approaches_the_closed_form_quantiles():
    """|N(0,1)| has quantile sqrt(2) erfinv(p); |Laplace(0,1)| is Exp(1): -ln(1 - p)."""
    from scipy.special import erfinv
    n = 400_000
    g, l = ti.gaussian_x(n, 77), ti.laplace_x(n, 78)
    for p in (0.25, 0.4, 0.5, 0.65, 0.9):
        tg, tl = orc.quantile_threshold(g, p), orc.quantile_threshold(l, p)
        # sampling error of an order statistic: sqrt(p(1-p)/n)/density, a few 1e-3 here; fp16 grid 1e-3
        assert abs(tg - np.sqrt(2) * erfinv(p)) < 0.01, (p, tg)
        assert abs(tl + np.log1p(-p)) < 0.015, (p, tl)


def test_threshold_realises_the_level_through_definition_1():
    x = ti.laplace_x(14336, 5)
    for p in (0.25, 0.5, 0.9):
        t = orc.quantile_threshold(x, p)
        kept = orc.sparsify(x, t)[3]
        k = orc.quantile_rank(x.size, p)
        ties = int(np.count_nonzero(np.abs(x.astype(np.float64)) == t))
        assert k <= x.size - kept <= k + ties - 1
