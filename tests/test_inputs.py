"""Host-side input preparation: format conversion, quantile rule, quantisers, shapes."""
import numpy as np
import pytest
import torch

import teal_inputs as ti


def test_bf16_rounding_matches_torch_round_to_nearest_even():
    rng = np.random.default_rng(0)
    a = np.concatenate([
        (rng.standard_normal(200_000) * 0.02).astype(np.float32),
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40, -1e-40], np.float32),
    ])
    want = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ti.f32_to_bf16_bits(a), want)
    back = ti.bf16_bits_to_f32(want)
    assert np.array_equal(back, torch.from_numpy(a).to(torch.bfloat16).float().numpy())


def test_generators_are_seeded_and_shaped():
    a, b = ti.gaussian_x(4096, 3), ti.gaussian_x(4096, 3)
    assert a.dtype == np.float16 and np.array_equal(a, b)
    assert not np.array_equal(a, ti.gaussian_x(4096, 4))
    g = ti.gaussian_x(200_000, 1).astype(np.float64)
    l = ti.laplace_x(200_000, 2).astype(np.float64)
    assert abs(g.std() - 1.0) < 0.01 and abs(g.mean()) < 0.01
    assert abs(l.std() - np.sqrt(2.0)) < 0.02 and abs(np.mean(np.abs(l)) - 1.0) < 0.01
    w = ti.bf16_bits_to_f32(ti.weights_bf16(256, 512, 9)).astype(np.float64)
    assert w.shape == (256, 512) and abs(w.std() - 0.02) < 2e-4


@pytest.mark.parametrize("p", [0.0, 0.25, 0.4, 0.5, 0.65, 0.8, 0.9, 1.0])
def test_quantile_threshold_is_the_kth_smallest_magnitude(p):
    x = ti.gaussian_x(4096, 77)
    t = ti.quantile_threshold(x, p)
    k = ti.quantile_rank(4096, p)
    mags = np.sort(np.abs(x.astype(np.float64)))
    if k == 0:
        assert t == 0.0
    else:
        assert t == mags[k - 1]
        assert float(np.float16(t)) == t            # no interpolation: an fp16 value


def test_quantile_rank_guards_binary_roundoff():
    assert ti.quantile_rank(4096, 0.4) == 1639
    assert ti.quantile_rank(4096, 0.5) == 2048
    assert ti.quantile_rank(10, 0.3) == 3           # 0.3*10 = 3.0000000000000004 in binary
    assert ti.quantile_rank(11008, 0.65) == 7156


def test_shape_tables():
    assert ti.LAYER_SHAPES["llama2_7b"]["gate"] == (11008, 4096)
    assert ti.LAYER_SHAPES["llama2_7b"]["down"] == (4096, 11008)
    assert ti.LAYER_SHAPES["llama3_8b"]["k"] == (1024, 4096)
    assert ti.LAYER_SHAPES["llama3_8b"]["up"] == (14336, 4096)
    assert ti.LAYER_SHAPES["llama_70b"]["down"] == (8192, 28672)
    total = sum(n * m * 2 for n, m in ti.LAYER_SHAPES["llama2_7b"].values())
    assert total == 404_750_336
    assert ti.x_seed(2, 0, "k") == ti.x_seed(2, 0, "q") == ti.x_seed(2, 0, "v")
    assert ti.x_seed(2, 0, "gate") == ti.x_seed(2, 0, "up") != ti.x_seed(2, 0, "down")


def test_quantisers_value_ranges_and_layout():
    w_bits = ti.weights_bf16(64, 256, 5)
    q, s = ti.quantize_w8(w_bits)
    assert q.dtype == np.int8 and q.shape == (256, 64) and q.min() >= -127
    assert np.abs(q).max(axis=0).min() >= 126        # every channel uses its range
    packed, s4 = ti.quantize_w4(w_bits, 128)
    assert packed.dtype == np.uint8 and packed.shape == (256, 32) and s4.shape == (2, 64)
    lo, hi = packed & 0xF, packed >> 4
    assert not np.any(lo == 8) and not np.any(hi == 8)   # -8 never produced
    t = ti.to_input_channel_major(w_bits)
    assert t.shape == (256, 64) and t[3, 7] == w_bits[7, 3] and t.flags.c_contiguous
