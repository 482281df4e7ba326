"""Pins for the oracle's MLP intermediate h = SiLU(gate) * up (Appendix A.3), which a
kernel fused with the W_down product forms itself.  Its binary32 arithmetic is checked
against the fp64 formula, the binary16 rounding against numpy, and the product against
the composition with Definition 1's oracle.  CPU only."""
import numpy as np
import pytest

import teal_inputs as ti
from oracle import teal_oracle as orc


def silu64(g):
    g = np.asarray(g, np.float64)
    return g / (1.0 + np.exp(-g))


def test_f32_to_f16_rounding_matches_numpy_on_every_boundary():
    # every finite fp16 value, the fp32 neighbours of it, and the fp32 neighbours of the
    # midpoints between consecutive fp16 values (ties and just off ties)
    h = np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16).astype(np.float32)
    mids = (h[:-1].astype(np.float64) + h[1:].astype(np.float64)) / 2
    mids32 = mids.astype(np.float32)            # exact: midpoints have 12 significant bits
    assert np.array_equal(mids32.astype(np.float64), mids)
    cands = [h, np.nextafter(h, np.float32(np.inf)), np.nextafter(h, np.float32(-np.inf)),
             mids32, np.nextafter(mids32, np.float32(np.inf)), np.nextafter(mids32, np.float32(-np.inf)),
             np.array([65504.0, 65519.996, 65520.0, 65535.0, 65536.0, 1e10, np.inf, 2.0 ** -25,
                       np.nextafter(np.float32(2.0 ** -25), np.float32(1)), 2.0 ** -26, 1e-30, 0.0],
                      np.float32)]
    v = np.concatenate(cands)
    v = np.concatenate([v, -v])
    with np.errstate(over="ignore"):
        want = v.astype(np.float16).view(np.uint16)
    got = np.array([orc.f32_to_f16_bits(x) for x in v], np.uint16)
    assert np.array_equal(got, want)
    rng = np.random.Generator(np.random.PCG64(5))
    r = (rng.standard_normal(20000) * np.exp(rng.uniform(-20, 12, 20000))).astype(np.float32)
    with np.errstate(over="ignore"):
        want = r.astype(np.float16).view(np.uint16)
    assert np.array_equal(np.array([orc.f32_to_f16_bits(x) for x in r], np.uint16), want)
    assert orc.f32_to_f16_bits(float("nan")) & 0x7C00 == 0x7C00 and orc.f32_to_f16_bits(float("nan")) & 0x3FF


def test_silu_matches_the_fp64_formula_to_a_few_ulp():
    rng = np.random.Generator(np.random.PCG64(6))
    g = np.concatenate([rng.uniform(-30, 30, 20000), rng.standard_normal(20000),
                        rng.uniform(-90, 90, 2000), np.linspace(-1, 1, 2001)]).astype(np.float32)
    got = np.array([orc.silu_f32(x) for x in g], np.float64)
    want = silu64(g.astype(np.float64))
    # three roundings (exp, reciprocal, product) on top of an exp good to about 1 ulp
    err = np.abs(got - want)
    tol = 4 * np.finfo(np.float32).eps * np.abs(want) + 1e-37
    far = g < -80                     # beyond the clamp: exp(80) stands in, values below 2e-33
    assert np.all(err[~far] <= tol[~far])
    assert np.all(np.abs(got[far]) < 2e-33) and np.all(np.abs(want[far]) < 2e-33)


def test_silu_special_values_and_identities():
    assert orc.silu_f32(0.0) == 0.0
    assert orc.silu_f32(1.0) == pytest.approx(0.7310585786300049, rel=3e-7)
    assert orc.silu_f32(-1.0) == pytest.approx(-0.2689414213699951, rel=3e-7)
    for g in (20.0, 50.0, 100.0, 1e6):
        assert orc.silu_f32(g) == pytest.approx(g, rel=3e-7)      # sigma -> 1
    assert abs(orc.silu_f32(-50.0)) < 1e-19 and orc.silu_f32(-50.0) < 0   # sigma -> 0 from the negative side
    assert np.isnan(orc.silu_f32(float("nan")))
    # sigma(g) + sigma(-g) = 1  =>  SiLU(g) - SiLU(-g) = g
    for g in np.linspace(0.01, 15, 200).astype(np.float32):
        assert orc.silu_f32(float(g)) - orc.silu_f32(float(-g)) == pytest.approx(float(g), rel=1e-6)
    # the minimum of SiLU: about -0.27846 at g = -1.27846
    grid = np.linspace(-2, -0.5, 3001).astype(np.float32)
    vals = np.array([orc.silu_f32(float(x)) for x in grid])
    assert vals.min() == pytest.approx(-0.2784645, abs=2e-6)
    assert grid[vals.argmin()] == pytest.approx(-1.2784645, abs=2e-3)


def test_intermediate_equals_the_rounded_fp64_formula_almost_everywhere():
    rng = np.random.Generator(np.random.PCG64(7))
    m = 50000
    g = (rng.standard_normal(m) * 2.0).astype(np.float32)
    u = rng.standard_normal(m).astype(np.float32)
    h = orc.swiglu_f16(g, u)
    want = (silu64(g) * u.astype(np.float64)).astype(np.float16)
    same = h.view(np.uint16) == want.view(np.uint16)
    assert same.mean() > 0.998          # fp32 and fp64 disagree only within a hair of an fp16 rounding boundary
    # and never by more than one fp16 step
    diff = np.abs(h.view(np.int16).astype(np.int32) - want.view(np.int16).astype(np.int32))
    assert diff[~same].max() == 1
    # element by element it is the scalar definition
    for i in range(0, m, 997):
        s = np.float32(orc.silu_f32(float(g[i])))
        assert h.view(np.uint16)[i] == orc.f32_to_f16_bits(float(s * u[i]))


def test_nan_and_inf_inputs():
    g = np.array([np.nan, 1.0, np.inf, -np.inf, 1.0, 3.0], np.float32)
    u = np.array([1.0, np.nan, 2.0, 2.0, np.inf, 0.0], np.float32)
    h = orc.swiglu_f16(g, u)
    assert np.isnan(h[0]) and np.isnan(h[1])
    assert h[2] == np.inf and h[4] == np.inf and h[5] == 0.0
    assert np.isinf(h[3]) or h[3] == 0      # -inf * sigma: the clamp keeps sigma positive, so -inf
    # NaN is dropped by Definition 1, Inf kept
    _, mask, _, _ = orc.sparsify(h, 0.5)
    assert mask[0] == 0 and mask[1] == 0 and mask[2] == 1 and mask[5] == 0


@pytest.mark.parametrize("n,m", [(24, 300), (40, 1025)])
def test_product_is_the_composition_with_definition_1(n, m):
    rng = np.random.Generator(np.random.PCG64(8 + n))
    g = (rng.standard_normal(m) * 1.5).astype(np.float32)
    u = rng.standard_normal(m).astype(np.float32)
    w = ti.weights_bf16(n, m, 9)
    h = orc.swiglu_f16(g, u)
    W64 = ti.bf16_bits_to_f32(w).astype(np.float64)
    for p in (0.0, 0.5, 0.9):
        t = ti.quantile_threshold(h, p)
        y = orc.sparse_gemv_bf16_swiglu(w, g, u, t)
        assert np.array_equal(y, orc.sparse_gemv_bf16(w, h, t))
        h64 = h.astype(np.float64)
        want = W64 @ np.where(np.abs(h64) > t, h64, 0.0)
        assert np.linalg.norm(y - want) <= 1e-13 * np.linalg.norm(want)


def test_intermediate_of_gaussian_projections_is_peaked_at_zero():
    """Section 4.1 / Figure 2: the MLP intermediate is Laplacian-shaped, more densely
    concentrated around zero than its Gaussian-shaped inputs: excess kurtosis > 0."""
    rng = np.random.Generator(np.random.PCG64(10))
    g = rng.standard_normal(200000).astype(np.float32)
    u = rng.standard_normal(200000).astype(np.float32)
    h = orc.swiglu_f16(g, u).astype(np.float64)
    k = np.mean((h - h.mean()) ** 4) / np.var(h) ** 2
    assert k > 6.0          # a Gaussian has 3, a Laplacian 6
