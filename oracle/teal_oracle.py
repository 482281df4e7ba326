"""Python face of the CPU oracle (oracle/teal_oracle.c).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
cpu_baseline leg may import this; the product path never does, and this
module imports nothing from the GPU package.

It only marshals numpy arrays into the C functions; the arithmetic -- the
sparsification function of Definition 1 (Section 4.2) and the thresholded
matrix-vector product Y = s_t(x) W^T (Sections 3, 4.2, 4.4) in fp64 -- is in
the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "teal_oracle.c")
_LIB = os.path.join(_HERE, "libteal_oracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2 + OpenMP, no tuning flags)."""
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < os.path.getmtime(_SRC))
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.run(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                        "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"], check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(build())
    c = ctypes
    u16p, u8p, i8p = c.POINTER(c.c_uint16), c.POINTER(c.c_uint8), c.POINTER(c.c_int8)
    i32p, f64p = c.POINTER(c.c_int32), c.POINTER(c.c_double)
    lib.oracle_f16_bits_to_f64.restype = c.c_double
    lib.oracle_f16_bits_to_f64.argtypes = [c.c_uint16]
    lib.oracle_bf16_bits_to_f64.restype = c.c_double
    lib.oracle_bf16_bits_to_f64.argtypes = [c.c_uint16]
    lib.oracle_sparsify.restype = c.c_int32
    lib.oracle_sparsify.argtypes = [u16p, c.c_int32, c.c_float, f64p, u8p, i32p]
    lib.oracle_sparse_gemv_bf16.restype = c.c_int32
    lib.oracle_sparse_gemv_bf16.argtypes = [u16p, u16p, c.c_float, f64p,
                                            c.c_int32, c.c_int32, f64p]
    lib.oracle_sparse_gemv_bf16_rows.restype = c.c_int32
    lib.oracle_sparse_gemv_bf16_rows.argtypes = [u16p, u16p, c.c_float, i32p, c.c_int32,
                                                 f64p, c.c_int32, c.c_int32, f64p]
    lib.oracle_sparse_gemv_w8.restype = c.c_int32
    lib.oracle_sparse_gemv_w8.argtypes = [i8p, u16p, u16p, c.c_float, f64p,
                                          c.c_int32, c.c_int32, f64p]
    lib.oracle_sparse_gemv_w4.restype = c.c_int32
    lib.oracle_sparse_gemv_w4.argtypes = [u8p, u16p, c.c_int32, u16p, c.c_float, f64p,
                                          c.c_int32, c.c_int32, f64p]
    lib.oracle_sparsify_batch.restype = c.c_int32
    lib.oracle_sparsify_batch.argtypes = [u16p, c.c_int32, c.c_int32, c.c_float, f64p, u8p, i32p]
    lib.oracle_sparse_gemv_bf16_batch.restype = c.c_int32
    lib.oracle_sparse_gemv_bf16_batch.argtypes = [u16p, u16p, c.c_int32, c.c_float, f64p,
                                                  c.c_int32, c.c_int32, u8p, f64p]
    f32p = c.POINTER(c.c_float)
    lib.oracle_silu_f32.restype = c.c_float
    lib.oracle_silu_f32.argtypes = [c.c_float]
    lib.oracle_f32_to_f16_bits.restype = c.c_uint16
    lib.oracle_f32_to_f16_bits.argtypes = [c.c_float]
    lib.oracle_swiglu_f16.restype = None
    lib.oracle_swiglu_f16.argtypes = [f32p, f32p, c.c_int32, u16p]
    lib.oracle_sum_of_squares.restype = c.c_double
    lib.oracle_sum_of_squares.argtypes = [f32p, c.c_int32]
    lib.oracle_rms_scale.restype = c.c_float
    lib.oracle_rms_scale.argtypes = [f32p, c.c_int32, c.c_float]
    lib.oracle_rmsnorm_f16.restype = None
    lib.oracle_rmsnorm_f16.argtypes = [f32p, f32p, c.c_float, c.c_int32, u16p]
    lib.oracle_sparse_gemv_bf16_rmsnorm.restype = c.c_int32
    lib.oracle_sparse_gemv_bf16_rmsnorm.argtypes = [u16p, f32p, f32p, c.c_float, c.c_float, f64p,
                                                    c.c_int32, c.c_int32, u16p, f64p]
    lib.oracle_sparse_gemv_bf16_swiglu.restype = c.c_int32
    lib.oracle_sparse_gemv_bf16_swiglu.argtypes = [u16p, f32p, f32p, c.c_float, f64p,
                                                   c.c_int32, c.c_int32, u16p, f64p]
    u64p = c.POINTER(c.c_uint64)
    lib.oracle_quantile_rank.restype = c.c_uint64
    lib.oracle_quantile_rank.argtypes = [c.c_uint64, c.c_double]
    lib.oracle_quantile_threshold.restype = c.c_float
    lib.oracle_quantile_threshold.argtypes = [u16p, c.c_uint64, c.c_double, u16p]
    lib.oracle_abs_histogram.restype = None
    lib.oracle_abs_histogram.argtypes = [u16p, c.c_uint64, u64p]
    lib.oracle_num_threads.restype = c.c_int32
    lib.oracle_set_num_threads.argtypes = [c.c_int32]
    _lib = lib
    return lib


def _ptr(a: np.ndarray, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _x_bits(x_f16) -> np.ndarray:
    x = np.ascontiguousarray(x_f16)
    if x.dtype != np.float16 or x.ndim != 1:
        raise TypeError("x must be a 1-D float16 array")
    return x.view(np.uint16)


def _f32(t) -> float:
    tf = float(np.float32(t))
    if tf != float(t):
        raise ValueError("threshold (or eps) must be exactly representable in fp32")
    return tf


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(k: int) -> None:
    _load().oracle_set_num_threads(int(k))


def f16_bits_to_f64(bits: int) -> float:
    return float(_load().oracle_f16_bits_to_f64(int(bits)))


def bf16_bits_to_f64(bits: int) -> float:
    return float(_load().oracle_bf16_bits_to_f64(int(bits)))


def sparsify(x_f16, t):
    """Definition 1. Returns (xs float64[m], mask uint8[m], idx int32[count], count)."""
    xb = _x_bits(x_f16)
    m = xb.size
    xs = np.empty(m, np.float64)
    mask = np.empty(m, np.uint8)
    idx = np.empty(max(m, 1), np.int32)
    count = _load().oracle_sparsify(_ptr(xb, ctypes.c_uint16), m, _f32(t),
                                    _ptr(xs, ctypes.c_double), _ptr(mask, ctypes.c_uint8),
                                    _ptr(idx, ctypes.c_int32))
    return xs, mask, idx[:count].copy(), int(count)


def sparse_gemv_bf16(w_bits, x_f16, t) -> np.ndarray:
    """y float64[n] = s_t(x) W^T for canonical W[n][m] given as bf16 bit patterns."""
    w = np.ascontiguousarray(w_bits)
    if w.dtype != np.uint16 or w.ndim != 2:
        raise TypeError("W must be a 2-D uint16 array of bf16 bit patterns, [n][m]")
    xb = _x_bits(x_f16)
    n, m = w.shape
    if xb.size != m:
        raise ValueError("x length must equal W's input dimension")
    y = np.empty(n, np.float64)
    xs = np.empty(m, np.float64)
    _load().oracle_sparse_gemv_bf16(_ptr(w, ctypes.c_uint16), _ptr(xb, ctypes.c_uint16),
                                    _f32(t), _ptr(y, ctypes.c_double), m, n,
                                    _ptr(xs, ctypes.c_double))
    return y


def sparse_gemv_bf16_rows(w_bits, x_f16, t, rows) -> np.ndarray:
    """Selected output channels of sparse_gemv_bf16, one by one."""
    w = np.ascontiguousarray(w_bits)
    if w.dtype != np.uint16 or w.ndim != 2:
        raise TypeError("W must be a 2-D uint16 array of bf16 bit patterns, [n][m]")
    xb = _x_bits(x_f16)
    n, m = w.shape
    if xb.size != m:
        raise ValueError("x length must equal W's input dimension")
    r = np.ascontiguousarray(rows, dtype=np.int32)
    y = np.empty(r.size, np.float64)
    xs = np.empty(m, np.float64)
    _load().oracle_sparse_gemv_bf16_rows(_ptr(w, ctypes.c_uint16), _ptr(xb, ctypes.c_uint16),
                                         _f32(t), _ptr(r, ctypes.c_int32), r.size,
                                         _ptr(y, ctypes.c_double), m, n,
                                         _ptr(xs, ctypes.c_double))
    return y


def sparse_gemv_w8(q, scale_f16, x_f16, t) -> np.ndarray:
    """q int8 [m][n], scale fp16 [n]; W[j][i] = q[i][j] * scale[j]."""
    q = np.ascontiguousarray(q)
    s = np.ascontiguousarray(scale_f16)
    if q.dtype != np.int8 or q.ndim != 2 or s.dtype != np.float16:
        raise TypeError("q must be int8 [m][n], scale fp16 [n]")
    xb = _x_bits(x_f16)
    m, n = q.shape
    if xb.size != m or s.shape != (n,):
        raise ValueError("shape mismatch")
    y = np.empty(n, np.float64)
    xs = np.empty(m, np.float64)
    _load().oracle_sparse_gemv_w8(_ptr(q, ctypes.c_int8), _ptr(s.view(np.uint16), ctypes.c_uint16),
                                  _ptr(xb, ctypes.c_uint16), _f32(t), _ptr(y, ctypes.c_double),
                                  m, n, _ptr(xs, ctypes.c_double))
    return y


def sparse_gemv_w4(packed, scale_f16, group, x_f16, t) -> np.ndarray:
    """packed uint8 [m][n/2] (low nibble = even j), scale fp16 [m/group][n]."""
    p = np.ascontiguousarray(packed)
    s = np.ascontiguousarray(scale_f16)
    if p.dtype != np.uint8 or p.ndim != 2 or s.dtype != np.float16 or s.ndim != 2:
        raise TypeError("packed must be uint8 [m][n/2], scale fp16 [m/group][n]")
    xb = _x_bits(x_f16)
    m, half = p.shape
    n = 2 * half
    if xb.size != m or m % group or s.shape != (m // group, n):
        raise ValueError("shape mismatch")
    y = np.empty(n, np.float64)
    xs = np.empty(m, np.float64)
    _load().oracle_sparse_gemv_w4(_ptr(p, ctypes.c_uint8), _ptr(s.view(np.uint16), ctypes.c_uint16),
                                  int(group), _ptr(xb, ctypes.c_uint16), _f32(t),
                                  _ptr(y, ctypes.c_double), m, n, _ptr(xs, ctypes.c_double))
    return y


def _X_bits(X_f16) -> np.ndarray:
    X = np.ascontiguousarray(X_f16)
    if X.dtype != np.float16 or X.ndim != 2 or X.shape[0] < 1:
        raise TypeError("X must be a 2-D float16 array, [batch][m]")
    return X.view(np.uint16)


def sparsify_batch(X_f16, t):
    """Section 5.4.4: one mask for the batch from the batch-averaged magnitude.

    Returns (mean_abs float64[m], mask uint8[m], idx int32[count], count)."""
    Xb = _X_bits(X_f16)
    batch, m = Xb.shape
    mean_abs = np.empty(m, np.float64)
    mask = np.empty(m, np.uint8)
    idx = np.empty(max(m, 1), np.int32)
    count = _load().oracle_sparsify_batch(_ptr(Xb, ctypes.c_uint16), batch, m, _f32(t),
                                          _ptr(mean_abs, ctypes.c_double),
                                          _ptr(mask, ctypes.c_uint8), _ptr(idx, ctypes.c_int32))
    return mean_abs, mask, idx[:count].copy(), int(count)


def sparse_gemv_bf16_batch(w_bits, X_f16, t) -> np.ndarray:
    """Y float64[batch][n]: every row of X times W^T over the batch-wide kept channels."""
    w = np.ascontiguousarray(w_bits)
    if w.dtype != np.uint16 or w.ndim != 2:
        raise TypeError("W must be a 2-D uint16 array of bf16 bit patterns, [n][m]")
    Xb = _X_bits(X_f16)
    batch, m = Xb.shape
    n = w.shape[0]
    if w.shape[1] != m:
        raise ValueError("X row length must equal W's input dimension")
    Y = np.empty((batch, n), np.float64)
    mask = np.empty(m, np.uint8)
    xs = np.empty(m, np.float64)
    _load().oracle_sparse_gemv_bf16_batch(_ptr(w, ctypes.c_uint16), _ptr(Xb, ctypes.c_uint16),
                                          batch, _f32(t), _ptr(Y, ctypes.c_double), m, n,
                                          _ptr(mask, ctypes.c_uint8), _ptr(xs, ctypes.c_double))
    return Y


def silu_f32(g: float) -> float:
    """SiLU in the binary32 arithmetic that defines the MLP intermediate."""
    return float(_load().oracle_silu_f32(float(np.float32(g))))


def f32_to_f16_bits(v: float) -> int:
    return int(_load().oracle_f32_to_f16_bits(float(np.float32(v))))


def _f32_vec(a, name) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.float32 or a.ndim != 1:
        raise TypeError(f"{name} must be a 1-D float32 array")
    return a


def swiglu_f16(gate_f32, up_f32) -> np.ndarray:
    """Appendix A.3: h = SiLU(gate) * up, rounded to fp16 (returned as float16[m])."""
    g, u = _f32_vec(gate_f32, "gate"), _f32_vec(up_f32, "up")
    if g.size != u.size:
        raise ValueError("gate and up must have the same length")
    h = np.empty(g.size, np.uint16)
    _load().oracle_swiglu_f16(_ptr(g, ctypes.c_float), _ptr(u, ctypes.c_float), g.size,
                              _ptr(h, ctypes.c_uint16))
    return h.view(np.float16)


def sparse_gemv_bf16_swiglu(w_bits, gate_f32, up_f32, t) -> np.ndarray:
    """y float64[n] = s_t(SiLU(gate) * up) W^T for canonical W[n][m] (the W_down step)."""
    w = np.ascontiguousarray(w_bits)
    if w.dtype != np.uint16 or w.ndim != 2:
        raise TypeError("W must be a 2-D uint16 array of bf16 bit patterns, [n][m]")
    g, u = _f32_vec(gate_f32, "gate"), _f32_vec(up_f32, "up")
    n, m = w.shape
    if g.size != m or u.size != m:
        raise ValueError("gate / up length must equal W's input dimension")
    y = np.empty(n, np.float64)
    h = np.empty(m, np.uint16)
    xs = np.empty(m, np.float64)
    _load().oracle_sparse_gemv_bf16_swiglu(_ptr(w, ctypes.c_uint16), _ptr(g, ctypes.c_float),
                                           _ptr(u, ctypes.c_float), _f32(t),
                                           _ptr(y, ctypes.c_double), m, n,
                                           _ptr(h, ctypes.c_uint16), _ptr(xs, ctypes.c_double))
    return y


def sum_of_squares(h_f32) -> float:
    """The binary64 sum of the squares of h by pairwise summation (see rms_scale)."""
    h = _f32_vec(h_f32, "h")
    return float(_load().oracle_sum_of_squares(_ptr(h, ctypes.c_float), h.size))


def rms_scale(h_f32, eps: float) -> float:
    """r = binary32(1 / sqrt(mean(h^2) + eps)), the sum of squares by pairwise summation
    in binary64 (the normalisation that precedes W_q/W_k/W_v and W_gate/W_up, Appendix A.3)."""
    h = _f32_vec(h_f32, "h")
    if h.size < 1:
        raise ValueError("h must not be empty")
    return float(_load().oracle_rms_scale(_ptr(h, ctypes.c_float), h.size, _f32(eps)))


def rmsnorm_f16(h_f32, gamma_f32, eps: float) -> np.ndarray:
    """x = gamma * h * r rounded to fp16 (returned as float16[m]); r as in rms_scale."""
    h, g = _f32_vec(h_f32, "h"), _f32_vec(gamma_f32, "gamma")
    if h.size != g.size:
        raise ValueError("h and gamma must have the same length")
    x = np.empty(h.size, np.uint16)
    _load().oracle_rmsnorm_f16(_ptr(h, ctypes.c_float), _ptr(g, ctypes.c_float), _f32(eps),
                               h.size, _ptr(x, ctypes.c_uint16))
    return x.view(np.float16)


def sparse_gemv_bf16_rmsnorm(w_bits, h_f32, gamma_f32, eps: float, t) -> np.ndarray:
    """y float64[n] = s_t(rmsnorm(h)) W^T for canonical W[n][m]."""
    w = np.ascontiguousarray(w_bits)
    if w.dtype != np.uint16 or w.ndim != 2:
        raise TypeError("W must be a 2-D uint16 array of bf16 bit patterns, [n][m]")
    h, g = _f32_vec(h_f32, "h"), _f32_vec(gamma_f32, "gamma")
    n, m = w.shape
    if h.size != m or g.size != m:
        raise ValueError("h / gamma length must equal W's input dimension")
    y = np.empty(n, np.float64)
    x = np.empty(m, np.uint16)
    xs = np.empty(m, np.float64)
    _load().oracle_sparse_gemv_bf16_rmsnorm(_ptr(w, ctypes.c_uint16), _ptr(h, ctypes.c_float),
                                            _ptr(g, ctypes.c_float), _f32(eps), _f32(t),
                                            _ptr(y, ctypes.c_double), m, n,
                                            _ptr(x, ctypes.c_uint16), _ptr(xs, ctypes.c_double))
    return y


def quantile_rank(n_valid: int, p: float) -> int:
    return int(_load().oracle_quantile_rank(int(n_valid), float(p)))


def quantile_threshold(x_f16, p: float) -> float:
    """Section 4.2: t_p from a sample, the ceil(p N)-th smallest |x| (NaNs left out)."""
    x = np.ascontiguousarray(x_f16).reshape(-1)
    if x.dtype != np.float16:
        raise TypeError("x must be float16")
    xb = x.view(np.uint16)
    scratch = np.empty(max(xb.size, 1), np.uint16)
    return float(_load().oracle_quantile_threshold(_ptr(xb, ctypes.c_uint16), xb.size, float(p),
                                                   _ptr(scratch, ctypes.c_uint16)))


def abs_histogram(x_f16, hist=None) -> np.ndarray:
    """Counts per fp16 magnitude bit pattern (32768 bins), added into hist if given."""
    x = np.ascontiguousarray(x_f16).reshape(-1)
    if x.dtype != np.float16:
        raise TypeError("x must be float16")
    xb = x.view(np.uint16)
    if hist is None:
        hist = np.zeros(32768, np.uint64)
    _load().oracle_abs_histogram(_ptr(xb, ctypes.c_uint16), xb.size, _ptr(hist, ctypes.c_uint64))
    return hist
