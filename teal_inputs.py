"""Seeded synthetic inputs for the TEAL sparse-GEMV path.

This module serves both the CPU oracle's tests and the HIP path's tests and
benchmark.  It holds input preparation only: random hidden states, random
weights, storage-format conversions, the weight quantisers that produce the
(q, scale) arrays both sides consume, the threshold picked from an empirical
quantile, and the Llama projection shape tables.  None of the method's
arithmetic (thresholding, masking, the matrix-vector product) lives here, and
it imports neither the oracle nor the HIP binding.

Recipe (stands in for real Llama activations and weights, which the paper
samples from C4 / WikiText runs, Section 4.1 and Section 5):
  * hidden states feeding q/k/v and gate/up are Gaussian-shaped, those feeding
    o and down are Laplacian-shaped (Section 4.1, Figure 2) -> N(0,1) or
    Laplace(0,1), rounded to fp16;
  * weights are N(0, 0.02^2) rounded to bf16 (round to nearest even);
  * shapes follow the seven matrices of a Transformer block (Appendix A.3).
"""
from __future__ import annotations

import math

import numpy as np

# ----------------------------------------------------------------------------
# storage formats
# ----------------------------------------------------------------------------


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 array of bfloat16 bit patterns, round to nearest even."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    if np.any((u & 0x7F800000) == 0x7F800000):
        raise ValueError("non-finite value in bf16 conversion input")
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """uint16 bfloat16 bit patterns -> fp32 values (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


# ----------------------------------------------------------------------------
# random hidden states and weights
# ----------------------------------------------------------------------------


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(int(seed)))


def gaussian_x(m: int, seed: int) -> np.ndarray:
    """N(0,1) hidden state of length m as fp16."""
    return _rng(seed).standard_normal(m).astype(np.float16)


def laplace_x(m: int, seed: int) -> np.ndarray:
    """Laplace(0,1) hidden state of length m as fp16."""
    return _rng(seed).laplace(0.0, 1.0, m).astype(np.float16)


def make_x(m: int, seed: int, dist: str) -> np.ndarray:
    if dist == "gaussian":
        return gaussian_x(m, seed)
    if dist == "laplace":
        return laplace_x(m, seed)
    raise ValueError(f"unknown distribution {dist!r}")


def weights_bf16(n: int, m: int, seed: int, std: float = 0.02) -> np.ndarray:
    """Canonical W[n][m] (out x in, row-major) as uint16 bf16 bit patterns."""
    w = _rng(seed).standard_normal((n, m), dtype=np.float32)
    w *= np.float32(std)
    return f32_to_bf16_bits(w)


def to_input_channel_major(w: np.ndarray) -> np.ndarray:
    """Canonical [n][m] -> stored [m][n]: row i holds the weights of input channel i."""
    return np.ascontiguousarray(w.T)


# ----------------------------------------------------------------------------
# threshold from an empirical quantile of |x|
# ----------------------------------------------------------------------------


def quantile_rank(m: int, p: float) -> int:
    """k = ceil(p*m), guarded against binary round-off in p*m."""
    if not 0.0 <= p <= 1.0:
        raise ValueError("sparsity must be in [0, 1]")
    return min(m, int(math.ceil(p * m - 1e-9)))


def quantile_threshold(x_f16: np.ndarray, p: float) -> float:
    """Threshold t with #{|x_i| <= t} >= ceil(p*m): the k-th smallest |x_i|.

    No interpolation, so t is itself an fp16 value (returned as a Python float
    that is exactly representable in fp32).  p == 0 gives t == 0.
    """
    x = np.asarray(x_f16, dtype=np.float16)
    k = quantile_rank(x.size, p)
    if k == 0:
        return 0.0
    a = np.abs(x.astype(np.float32))
    return float(np.partition(a, k - 1)[k - 1])


def mlp_gate_up(m: int, seed: int):
    """The two fp32 vectors from which the input of W_down is formed (Appendix A.3):
    gate = x W_gate^T and up = x W_up^T of a synthetic block, both Gaussian-shaped
    (N(0, 1.5^2) and N(0, 1)); their SiLU-gated product is Laplacian-shaped like the
    real MLP intermediate (Section 4.1, Figure 2).  Returns (gate, up) float32[m]."""
    rng = _rng(seed)
    gate = (rng.standard_normal(m) * 1.5).astype(np.float32)
    up = rng.standard_normal(m).astype(np.float32)
    return gate, up


def norm_inputs(m: int, seed: int):
    """The fp32 hidden state h before the normalisation layer and the layer's weights
    gamma, from which the input of W_q/W_k/W_v (or W_gate/W_up) is formed (Appendix A.3).
    h is Gaussian-shaped, N(0, 2.5^2), with one channel in 512 scaled by 40 (the few
    very large channels of a residual stream, which dominate the sum of squares);
    gamma = 0.5 + 0.1 N(0, 1).  The normalised state comes out Gaussian-shaped with
    unit-order scale, like the inputs of the attention and MLP blocks (Section 4.1,
    Figure 2).  Returns (h, gamma) float32[m]."""
    rng = _rng(seed)
    h = rng.standard_normal(m) * 2.5
    big = rng.random(m) < 1.0 / 512.0
    h = np.where(big, h * 40.0, h).astype(np.float32)
    gamma = (0.5 + 0.1 * rng.standard_normal(m)).astype(np.float32)
    return h, gamma


def make_X(batch: int, m: int, seed: int, dist: str) -> np.ndarray:
    """A small batch of independent hidden states, [batch][m] fp16 (rows drawn
    one after the other from one seeded stream)."""
    rng = _rng(seed)
    if dist == "gaussian":
        X = rng.standard_normal((batch, m))
    elif dist == "laplace":
        X = rng.laplace(0.0, 1.0, (batch, m))
    else:
        raise ValueError(f"unknown distribution {dist!r}")
    return X.astype(np.float16)


def batch_quantile_threshold(X_f16: np.ndarray, p: float) -> float:
    """A threshold for a batch: an fp32 value t such that at least ceil(p*m)
    channels have a batch-averaged magnitude <= t.

    The k-th smallest average magnitude is in general not an fp32 value, so it
    is rounded UP to fp32 (then the k smallest averages are all <= t).  p == 0
    gives t == 0.
    """
    X = np.asarray(X_f16, dtype=np.float16)
    batch, m = X.shape
    k = quantile_rank(m, p)
    if k == 0:
        return 0.0
    mean = np.abs(X.astype(np.float64)).sum(axis=0) / batch
    kth = float(np.partition(mean, k - 1)[k - 1])
    t = np.float32(kth)
    if float(t) < kth:
        t = np.nextafter(t, np.float32(np.inf))
    return float(t)


# ----------------------------------------------------------------------------
# weight quantisers (round to nearest, symmetric); produce what both sides read
# ----------------------------------------------------------------------------


def quantize_w8(w_bits: np.ndarray):
    """8-bit channel-wise round-to-nearest (Section 5.3), symmetric.

    w_bits: canonical [n][m] bf16 bit patterns.
    Returns (q, scale): q int8 [m][n] input-channel-major with values in
    [-127, 127]; scale fp16 [n], one per output channel.
    """
    w = bf16_bits_to_f32(w_bits).astype(np.float64)
    amax = np.abs(w).max(axis=1)
    scale = (amax / 127.0).astype(np.float16)
    scale[scale == 0] = np.float16(1.0)
    q = np.rint(w / scale.astype(np.float64)[:, None])
    q = np.clip(q, -127, 127).astype(np.int8)
    return np.ascontiguousarray(q.T), scale


def quantize_w4(w_bits: np.ndarray, group: int = 128):
    """4-bit symmetric round-to-nearest with one fp16 scale per (group of
    `group` consecutive input channels, output channel).

    Returns (packed, scale): packed uint8 [m][n/2], two signed nibbles per
    byte along the output axis, low nibble = even output channel, values in
    [-7, 7] as two's complement; scale fp16 [m/group][n].
    """
    w = bf16_bits_to_f32(w_bits).astype(np.float64)
    n, m = w.shape
    if m % group or n % 2:
        raise ValueError("m must be a multiple of group and n even")
    g = w.reshape(n, m // group, group)
    amax = np.abs(g).max(axis=2)                       # [n][m/group]
    scale = (amax / 7.0).astype(np.float16)
    scale[scale == 0] = np.float16(1.0)
    q = np.rint(g / scale.astype(np.float64)[:, :, None])
    q = np.clip(q, -7, 7).astype(np.int8).reshape(n, m)
    qt = np.ascontiguousarray(q.T)                     # [m][n]
    nib = (qt & 0x0F).astype(np.uint8)
    packed = (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)
    return np.ascontiguousarray(packed), np.ascontiguousarray(scale.T)


# ----------------------------------------------------------------------------
# projection shape tables (n = output channels, m = input channels)
# ----------------------------------------------------------------------------

PROJ_ORDER = ("q", "k", "v", "o", "gate", "up", "down")
# hidden-state shape by projection role (Section 4.1, Figure 2)
PROJ_DIST = {"q": "gaussian", "k": "gaussian", "v": "gaussian", "o": "laplace",
             "gate": "gaussian", "up": "gaussian", "down": "laplace"}
# projections that read the same hidden state inside a block (Appendix A.3)
PROJ_XGROUP = {"q": 0, "k": 0, "v": 0, "o": 1, "gate": 2, "up": 2, "down": 3}


def _block(d: int, d_kv: int, d_m: int) -> dict:
    return {"q": (d, d), "k": (d_kv, d), "v": (d_kv, d), "o": (d, d),
            "gate": (d_m, d), "up": (d_m, d), "down": (d, d_m)}


LAYER_SHAPES = {
    "llama2_7b": _block(4096, 4096, 11008),
    "llama3_8b": _block(4096, 1024, 14336),
    "llama_70b": _block(8192, 1024, 28672),
}
CONFIG_INDEX = {"single_4096": 1, "llama2_7b": 2, "llama3_8b": 3, "llama_70b": 4}


def weight_seed(config: int, layer: int, proj: str) -> int:
    return 1000 * config + 10 * layer + PROJ_ORDER.index(proj)


def x_seed(config: int, layer: int, proj: str) -> int:
    """Projections sharing a hidden state share a seed (first member's)."""
    first = next(p for p in PROJ_ORDER if PROJ_XGROUP[p] == PROJ_XGROUP[proj])
    return weight_seed(config, layer, first) + 500_000


def layer_inputs(model: str, layer: int = 0):
    """Yield (proj, n, m, w_bits[n][m], x_f16[m]) for one synthetic block."""
    cfg = CONFIG_INDEX[model]
    for proj in PROJ_ORDER:
        n, m = LAYER_SHAPES[model][proj]
        w = weights_bf16(n, m, weight_seed(cfg, layer, proj))
        x = make_x(m, x_seed(cfg, layer, proj), PROJ_DIST[proj])
        yield proj, n, m, w, x
