"""ctypes binding of libteal.so: the same names as include/teal.h, argument
marshalling only.  Pointer arguments may be torch tensors (their data_ptr() is
passed; they must be contiguous), plain integer addresses, or None.  `stream`
defaults to torch's current stream on the current device.  Every function
returns the library's status code; check() turns a non-zero one into TealError.
"""
from __future__ import annotations

import ctypes
import os
import threading

TEAL_OK = 0
TEAL_ERR_NULL = 1
TEAL_ERR_SHAPE = 2
TEAL_ERR_ALIGN = 3
TEAL_ERR_THRESHOLD = 4
TEAL_ERR_WORKSPACE = 5
TEAL_ERR_UNSUPPORTED = 6
TEAL_ERR_HIP = 7
TEAL_ERR_STATIC_LIMIT = 8

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libteal.so")
_lib = None

EXPORTS = (
    "teal_status_string", "teal_version", "teal_workspace_bytes", "teal_sparsify",
    "teal_sparse_gemv_bf16", "teal_sparse_gemv_bf16_ex", "teal_sparse_gemv_w8",
    "teal_sparse_gemv_w4", "teal_pack_bf16", "teal_pack_bf16_pitch", "teal_gemv_plan", "teal_sparse_gemv_bf16_multi",
    "teal_abs_histogram", "teal_histogram_thresholds", "teal_workspace_bytes_batch",
    "teal_sparsify_batch", "teal_sparse_gemv_bf16_batch", "teal_sparse_gemv_bf16_batch_ex",
    "teal_sparse_gemv_w8_multi", "teal_sparse_gemv_w4_multi",
    "teal_swiglu_f16", "teal_sparse_gemv_bf16_swiglu", "teal_sparse_gemv_bf16_batch_multi",
    "teal_gemv_plan_multi", "teal_gemv_plan_multi_pitch", "teal_sparse_gemv_bf16_multi_pitch",
    "teal_sparse_gemv_w8_multi_pitch", "teal_sparse_gemv_bf16_rmsnorm_multi_pitch",
    "teal_survivors_offset", "teal_rmsnorm_f16",
    "teal_sparse_gemv_bf16_rmsnorm_multi", "teal_workspace_bytes_stack",
    "teal_sparse_gemv_bf16_stack", "teal_sparse_gemv_w8_stack", "teal_sparse_gemv_w4_stack",
    "teal_stream_read_probe", "teal_sparse_gemv_w8_swiglu", "teal_sparse_gemv_w8_rmsnorm_multi",
    "teal_sparse_gemv_w4_swiglu", "teal_sparse_gemv_w4_rmsnorm_multi",
    "teal_static_scratch_limit", "teal_static_scratch_init", "teal_sparse_gemv_bf16_static",
    "teal_workspace_bytes_mlp", "teal_mlp_down_region_offset", "teal_mlp_status_offset",
    "teal_mlp_plan", "teal_mlp_block_info", "teal_sparse_mlp_bf16", "teal_sparse_mlp_w8",
    "teal_sparse_mlp_w4",
)
TEAL_HIST_BINS = 32768
TEAL_MAX_BATCH = 8


class MlpShape(ctypes.Structure):
    """teal_mlp_shape of include/teal.h."""
    _fields_ = [(name, ctypes.c_int) for name in (
        "gu_lanes_per_row", "gu_tile_cols", "gu_splits", "gu_phase_tiles",
        "down_lanes_per_row", "down_tile_cols", "down_splits", "extra_lds_bytes", "spin_limit",
        "gu_row_pitch", "down_row_pitch")]

    def as_dict(self):
        return {name: getattr(self, name) for name, _ in self._fields_}


class TealError(RuntimeError):
    def __init__(self, status: int):
        self.status = int(status)
        super().__init__(f"libteal status {self.status}: {teal_status_string(self.status)}")


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads the built library; raises if it is not there (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is not built; run `python -m paper_2408_14690_amd.build`")
    lib = ctypes.CDLL(_LIB_PATH)
    c = ctypes
    vp, i, f, sz = c.c_void_p, c.c_int, c.c_float, c.c_size_t
    lib.teal_status_string.restype = c.c_char_p
    lib.teal_status_string.argtypes = [i]
    lib.teal_version.restype = i
    lib.teal_version.argtypes = []
    lib.teal_workspace_bytes.restype = sz
    lib.teal_workspace_bytes.argtypes = [i, i]
    lib.teal_rmsnorm_f16.restype = i
    lib.teal_rmsnorm_f16.argtypes = [vp, vp, f, vp, i, vp]
    lib.teal_sparse_gemv_bf16_rmsnorm_multi.restype = i
    lib.teal_sparse_gemv_bf16_rmsnorm_multi.argtypes = [i, c.POINTER(vp), c.POINTER(f),
                                                        c.POINTER(vp), c.POINTER(i), vp, vp, f, i,
                                                        vp, sz, vp]
    lib.teal_sparse_gemv_bf16_rmsnorm_multi_pitch.restype = i
    lib.teal_sparse_gemv_bf16_rmsnorm_multi_pitch.argtypes = [i, c.POINTER(vp), c.POINTER(i),
                                                              c.POINTER(f), c.POINTER(vp),
                                                              c.POINTER(i), vp, vp, f, i, vp, sz, vp]
    lib.teal_survivors_offset.restype = sz
    lib.teal_survivors_offset.argtypes = []
    lib.teal_sparsify.restype = i
    lib.teal_sparsify.argtypes = [vp, i, f, vp, vp, vp, vp]
    lib.teal_sparse_gemv_bf16.restype = i
    lib.teal_sparse_gemv_bf16.argtypes = [vp, vp, f, vp, i, i, vp, sz, vp]
    lib.teal_static_scratch_limit.restype = sz
    lib.teal_static_scratch_limit.argtypes = []
    lib.teal_static_scratch_init.restype = i
    lib.teal_static_scratch_init.argtypes = []
    lib.teal_sparse_gemv_bf16_static.restype = i
    lib.teal_sparse_gemv_bf16_static.argtypes = [vp, vp, f, vp, i, i, vp]
    lib.teal_sparse_gemv_bf16_ex.restype = i
    lib.teal_sparse_gemv_bf16_ex.argtypes = [vp, vp, f, vp, i, i, vp, sz, vp, i, i, i, i, i]
    lib.teal_sparse_gemv_w8.restype = i
    lib.teal_sparse_gemv_w8.argtypes = [vp, vp, vp, f, vp, i, i, vp, sz, vp]
    lib.teal_sparse_gemv_w4.restype = i
    lib.teal_sparse_gemv_w4.argtypes = [vp, vp, i, vp, f, vp, i, i, vp, sz, vp]
    lib.teal_pack_bf16.restype = i
    lib.teal_pack_bf16.argtypes = [vp, vp, i, i, vp]
    lib.teal_pack_bf16_pitch.restype = i
    lib.teal_pack_bf16_pitch.argtypes = [vp, vp, i, i, i, vp]
    lib.teal_sparse_gemv_bf16_multi.restype = i
    lib.teal_sparse_gemv_bf16_multi.argtypes = [i, c.POINTER(vp), c.POINTER(f), c.POINTER(vp),
                                                c.POINTER(i), vp, i, vp, sz, vp]
    lib.teal_sparse_gemv_bf16_multi_pitch.restype = i
    lib.teal_sparse_gemv_bf16_multi_pitch.argtypes = [i, c.POINTER(vp), c.POINTER(i), c.POINTER(f),
                                                      c.POINTER(vp), c.POINTER(i), vp, i, vp, sz, vp]
    lib.teal_sparse_gemv_w8_multi_pitch.restype = i
    lib.teal_sparse_gemv_w8_multi_pitch.argtypes = [i, c.POINTER(vp), c.POINTER(i), c.POINTER(vp),
                                                    c.POINTER(f), c.POINTER(vp), c.POINTER(i), vp, i,
                                                    vp, sz, vp]
    lib.teal_workspace_bytes_stack.restype = sz
    lib.teal_workspace_bytes_stack.argtypes = [i, c.POINTER(i), c.POINTER(i), c.POINTER(i)]
    lib.teal_sparse_gemv_bf16_stack.restype = i
    lib.teal_sparse_gemv_bf16_stack.argtypes = [i, c.POINTER(i), c.POINTER(vp), c.POINTER(f),
                                                c.POINTER(vp), c.POINTER(i), c.POINTER(vp),
                                                c.POINTER(i), vp, sz, vp]
    lib.teal_sparse_gemv_w8_swiglu.restype = i
    lib.teal_sparse_gemv_w8_swiglu.argtypes = [vp, vp, vp, vp, f, vp, i, i, vp, sz, vp]
    lib.teal_sparse_gemv_w8_rmsnorm_multi.restype = i
    lib.teal_sparse_gemv_w8_rmsnorm_multi.argtypes = [i, c.POINTER(vp), c.POINTER(vp), c.POINTER(f),
                                                      c.POINTER(vp), c.POINTER(i), vp, vp, f, i,
                                                      vp, sz, vp]
    lib.teal_sparse_gemv_w4_swiglu.restype = i
    lib.teal_sparse_gemv_w4_swiglu.argtypes = [vp, vp, i, vp, vp, f, vp, i, i, vp, sz, vp]
    lib.teal_sparse_gemv_w4_rmsnorm_multi.restype = i
    lib.teal_sparse_gemv_w4_rmsnorm_multi.argtypes = [i, c.POINTER(vp), c.POINTER(vp), i,
                                                      c.POINTER(f), c.POINTER(vp), c.POINTER(i),
                                                      vp, vp, f, i, vp, sz, vp]
    lib.teal_stream_read_probe.restype = i
    lib.teal_stream_read_probe.argtypes = [vp, sz, i, c.c_uint32, vp, vp]
    lib.teal_sparse_gemv_w8_stack.restype = i
    lib.teal_sparse_gemv_w8_stack.argtypes = [i, c.POINTER(i), c.POINTER(vp), c.POINTER(vp),
                                              c.POINTER(f), c.POINTER(vp), c.POINTER(i),
                                              c.POINTER(vp), c.POINTER(i), vp, sz, vp]
    lib.teal_sparse_gemv_w4_stack.restype = i
    lib.teal_sparse_gemv_w4_stack.argtypes = [i, c.POINTER(i), c.POINTER(vp), c.POINTER(vp), i,
                                              c.POINTER(f), c.POINTER(vp), c.POINTER(i),
                                              c.POINTER(vp), c.POINTER(i), vp, sz, vp]
    lib.teal_sparse_gemv_w8_multi.restype = i
    lib.teal_sparse_gemv_w8_multi.argtypes = [i, c.POINTER(vp), c.POINTER(vp), c.POINTER(f),
                                              c.POINTER(vp), c.POINTER(i), vp, i, vp, sz, vp]
    lib.teal_sparse_gemv_w4_multi.restype = i
    lib.teal_sparse_gemv_w4_multi.argtypes = [i, c.POINTER(vp), c.POINTER(vp), i, c.POINTER(f),
                                              c.POINTER(vp), c.POINTER(i), vp, i, vp, sz, vp]
    lib.teal_sparse_gemv_bf16_batch_multi.restype = i
    lib.teal_sparse_gemv_bf16_batch_multi.argtypes = [i, c.POINTER(vp), c.POINTER(f), c.POINTER(vp),
                                                      c.POINTER(i), vp, i, i, vp, sz, vp]
    lib.teal_swiglu_f16.restype = i
    lib.teal_swiglu_f16.argtypes = [vp, vp, vp, i, vp]
    lib.teal_sparse_gemv_bf16_swiglu.restype = i
    lib.teal_sparse_gemv_bf16_swiglu.argtypes = [vp, vp, vp, f, vp, i, i, vp, sz, vp]
    lib.teal_abs_histogram.restype = i
    lib.teal_abs_histogram.argtypes = [vp, sz, vp, vp]
    lib.teal_histogram_thresholds.restype = i
    lib.teal_histogram_thresholds.argtypes = [vp, c.POINTER(c.c_double), i, vp, vp]
    lib.teal_workspace_bytes_batch.restype = sz
    lib.teal_workspace_bytes_batch.argtypes = [i, i, i]
    lib.teal_sparsify_batch.restype = i
    lib.teal_sparsify_batch.argtypes = [vp, i, i, f, vp, vp, vp, vp]
    lib.teal_sparse_gemv_bf16_batch.restype = i
    lib.teal_sparse_gemv_bf16_batch.argtypes = [vp, vp, i, f, vp, i, i, vp, sz, vp]
    lib.teal_sparse_gemv_bf16_batch_ex.restype = i
    lib.teal_sparse_gemv_bf16_batch_ex.argtypes = [vp, vp, i, f, vp, i, i, vp, sz, vp, i, i, i]
    shp = c.POINTER(MlpShape)
    lib.teal_workspace_bytes_mlp.restype = sz
    lib.teal_workspace_bytes_mlp.argtypes = [i, i, i]
    lib.teal_mlp_down_region_offset.restype = sz
    lib.teal_mlp_down_region_offset.argtypes = [i, i]
    lib.teal_mlp_status_offset.restype = sz
    lib.teal_mlp_status_offset.argtypes = [i, i, i]
    lib.teal_mlp_plan.restype = i
    lib.teal_mlp_plan.argtypes = [i, i, i, i, shp]
    lib.teal_mlp_block_info.restype = i
    lib.teal_mlp_block_info.argtypes = [i, i, i, i, shp, i, c.POINTER(c.c_int)]
    lib.teal_sparse_mlp_bf16.restype = i
    lib.teal_sparse_mlp_bf16.argtypes = [vp, vp, vp, vp, f, f, f, vp, vp, vp, i, i, i, vp, sz, vp, shp]
    lib.teal_sparse_mlp_w8.restype = i
    lib.teal_sparse_mlp_w8.argtypes = [vp, vp, vp, vp, vp, vp, vp, f, f, f, vp, vp, vp, i, i, i, vp,
                                       sz, vp, shp]
    lib.teal_sparse_mlp_w4.restype = i
    lib.teal_sparse_mlp_w4.argtypes = [vp, vp, vp, vp, vp, vp, i, vp, f, f, f, vp, vp, vp, i, i, i,
                                       vp, sz, vp, shp]
    ip = c.POINTER(c.c_int)
    lib.teal_gemv_plan.restype = i
    lib.teal_gemv_plan.argtypes = [i, i, i, ip, ip, ip, ip, ip]
    lib.teal_gemv_plan_multi.restype = i
    lib.teal_gemv_plan_multi.argtypes = [i, i, ip, i, ip, ip, ip, ip, ip]
    lib.teal_gemv_plan_multi_pitch.restype = i
    lib.teal_gemv_plan_multi_pitch.argtypes = [i, i, ip, ip, i, ip, ip, ip, ip, ip]
    _lib = lib
    return lib


def _ptr(a, need=None, what="argument"):
    """Device address of a tensor (or a raw address).  With `need`, a tensor smaller than
    that many bytes is refused here: the C ABI sees plain pointers and cannot know."""
    if a is None:
        return None
    if isinstance(a, int):
        return a
    if hasattr(a, "data_ptr"):
        if not a.is_contiguous():
            raise ValueError("tensor arguments must be contiguous")
        if need is not None and a.numel() * a.element_size() < int(need):
            raise ValueError(f"{what}: tensor of {a.numel() * a.element_size()} bytes, "
                             f"the call reads or writes {int(need)}")
        return a.data_ptr()
    raise TypeError(f"cannot pass {type(a).__name__} as a device pointer")


def _nbytes(a, given):
    if given is not None:
        return int(given)
    if hasattr(a, "numel"):
        return a.numel() * a.element_size()
    raise TypeError("workspace_bytes is required when workspace is a raw address")


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


_tls = threading.local()      # .recording: the list prepare() fills on THIS host thread


def _call(name, *cargs):
    """Every call that enqueues GPU work goes through here: normally straight into the
    library; while prepare() records on the calling thread, the marshalled arguments are kept
    instead.  Calls from other host threads are not affected by a recording."""
    fn = getattr(load_library(), name)
    recording = getattr(_tls, "recording", None)
    if recording is not None:
        recording.append((fn, cargs))
        return TEAL_OK
    return fn(*cargs)


def prepare(enqueue):
    """Marshals once, calls many times.  `enqueue` is a function that makes one or more
    teal_* calls of this module (device tensors, shapes, thresholds and stream as they will
    be at every later call); nothing reaches the GPU while it runs.  Returns a function
    without arguments that issues exactly those library calls with the arguments as
    marshalled (host arrays are kept alive by it) and returns the first status that is not
    TEAL_OK, else TEAL_OK.  For decode loops that repeat the same calls on the same
    buffers: the per-call cost of building the argument lists is paid once."""
    if getattr(_tls, "recording", None) is not None:
        raise RuntimeError("prepare() does not nest")
    _tls.recording = []
    try:
        enqueue()
        calls = tuple(_tls.recording)
    finally:
        _tls.recording = None
    if len(calls) == 1:
        fn, cargs = calls[0]
        return lambda: fn(*cargs)

    def run():
        for fn, cargs in calls:
            st = fn(*cargs)
            if st != TEAL_OK:
                return st
        return TEAL_OK
    return run


def check(status: int) -> None:
    if status != TEAL_OK:
        raise TealError(status)


def teal_status_string(status: int) -> str:
    return load_library().teal_status_string(int(status)).decode()


def teal_version() -> int:
    return int(load_library().teal_version())


def teal_workspace_bytes(m: int, n: int) -> int:
    return int(load_library().teal_workspace_bytes(int(m), int(n)))


def teal_survivors_offset() -> int:
    return int(load_library().teal_survivors_offset())


def teal_sparsify(x_f16, m, t, mask=None, idx=None, count=None, stream=None) -> int:
    return _call("teal_sparsify", _ptr(x_f16, 2 * m, "x"), int(m), float(t),
                                        _ptr(mask, m, "mask"), _ptr(idx, 4 * m, "idx"),
                                        _ptr(count, 4, "count"), _stream(stream))


def teal_sparse_gemv_bf16(Wt_bf16, x_f16, t, y, m, n, workspace, workspace_bytes=None,
                          stream=None) -> int:
    return _call(
        "teal_sparse_gemv_bf16",
        _ptr(Wt_bf16, 2 * m * n, "Wt"), _ptr(x_f16, 2 * m, "x"), float(t), _ptr(y, 4 * n, "y"),
        int(m), int(n), _ptr(workspace),
        _nbytes(workspace, workspace_bytes), _stream(stream))


def teal_static_scratch_limit() -> int:
    return int(load_library().teal_static_scratch_limit())


def teal_static_scratch_init() -> int:
    return int(load_library().teal_static_scratch_init())


def teal_sparse_gemv_bf16_static(Wt_bf16, x_f16, t, y, m, n, stream=None) -> int:
    return _call(
        "teal_sparse_gemv_bf16_static",
        _ptr(Wt_bf16, 2 * m * n, "Wt"), _ptr(x_f16, 2 * m, "x"), float(t), _ptr(y, 4 * n, "y"),
        int(m), int(n), _stream(stream))


def teal_sparse_gemv_bf16_ex(Wt_bf16, x_f16, t, y, m, n, workspace, workspace_bytes=None,
                             stream=None, lanes_per_row=0, tile_cols=0, splits=0, waves=0,
                             unroll=0) -> int:
    return _call(
        "teal_sparse_gemv_bf16_ex",
        _ptr(Wt_bf16, 2 * m * n, "Wt"), _ptr(x_f16, 2 * m, "x"), float(t), _ptr(y, 4 * n, "y"),
        int(m), int(n), _ptr(workspace),
        _nbytes(workspace, workspace_bytes), _stream(stream), int(lanes_per_row), int(tile_cols),
        int(splits), int(waves), int(unroll))


def teal_sparse_gemv_w8(Wq, scale_f16, x_f16, t, y, m, n, workspace, workspace_bytes=None,
                        stream=None) -> int:
    return _call(
        "teal_sparse_gemv_w8",
        _ptr(Wq, m * n, "Wq"), _ptr(scale_f16, 2 * n, "scale"), _ptr(x_f16, 2 * m, "x"), float(t),
        _ptr(y, 4 * n, "y"), int(m), int(n), _ptr(workspace),
        _nbytes(workspace, workspace_bytes), _stream(stream))


def teal_sparse_gemv_w4(Wq, scale_f16, group, x_f16, t, y, m, n, workspace,
                        workspace_bytes=None, stream=None) -> int:
    return _call(
        "teal_sparse_gemv_w4",
        _ptr(Wq, m * n // 2, "Wq"), _ptr(scale_f16, 2 * n * (m // max(int(group), 1)), "scale"),
        int(group), _ptr(x_f16, 2 * m, "x"), float(t), _ptr(y, 4 * n, "y"), int(m), int(n),
        _ptr(workspace), _nbytes(workspace, workspace_bytes), _stream(stream))


def teal_pack_bf16(W_rowmajor, Wt, m, n, stream=None) -> int:
    return _call("teal_pack_bf16", _ptr(W_rowmajor, 2 * m * n, "W"), _ptr(Wt, 2 * m * n, "Wt"),
                                         int(m), int(n),
                                         _stream(stream))


def teal_pack_bf16_pitch(W_rowmajor, Wt, m, n, row_pitch, stream=None) -> int:
    return _call("teal_pack_bf16_pitch", _ptr(W_rowmajor, 2 * m * n, "W"),
                 _ptr(Wt, 2 * ((m - 1) * max(int(row_pitch), n) + n), "Wt"), int(m), int(n),
                 int(row_pitch), _stream(stream))


def teal_gemv_plan(weight_bits: int, m: int, n: int):
    """Returns (status, dict(lanes_per_row, tile_cols, splits, waves, unroll))."""
    vals = [ctypes.c_int(0) for _ in range(5)]
    st = load_library().teal_gemv_plan(int(weight_bits), int(m), int(n),
                                       *[ctypes.byref(v) for v in vals])
    keys = ("lanes_per_row", "tile_cols", "splits", "waves", "unroll")
    return st, {k: v.value for k, v in zip(keys, vals)}


def teal_gemv_plan_multi(weight_bits: int, m: int, n_list):
    """Returns (status, dict) for a grouped launch of len(n_list) matrices."""
    count = len(n_list)
    N = (ctypes.c_int * max(count, 1))(*[int(n) for n in n_list])
    vals = [ctypes.c_int(0) for _ in range(5)]
    st = load_library().teal_gemv_plan_multi(int(weight_bits), int(m), N, count,
                                             *[ctypes.byref(v) for v in vals])
    keys = ("lanes_per_row", "tile_cols", "splits", "waves", "unroll")
    return st, {k: v.value for k, v in zip(keys, vals)}


def teal_sparse_gemv_bf16_multi(Wt_list, t_list, y_list, n_list, x_f16, m, workspace,
                                workspace_bytes=None, stream=None) -> int:
    """count = len(Wt_list) matrices sharing x; the per-matrix lists become host arrays."""
    count = len(Wt_list)
    if not (len(t_list) == len(y_list) == len(n_list) == count):
        raise ValueError("per-matrix lists must have the same length")
    W = (ctypes.c_void_p * count)(*[_ptr(w, 2 * m * n, "Wt") for w, n in zip(Wt_list, n_list)])
    Y = (ctypes.c_void_p * count)(*[_ptr(y, 4 * n, "y") for y, n in zip(y_list, n_list)])
    Tt = (ctypes.c_float * count)(*[float(t) for t in t_list])
    N = (ctypes.c_int * count)(*[int(n) for n in n_list])
    return _call(
        "teal_sparse_gemv_bf16_multi",
        count, W, Tt, Y, N, _ptr(x_f16, 2 * m, "x"), int(m), _ptr(workspace),
        _nbytes(workspace, workspace_bytes), _stream(stream))


def teal_sparse_gemv_bf16_multi_pitch(Wt_list, pitch_list, t_list, y_list, n_list, x_f16, m, workspace,
                                      workspace_bytes=None, stream=None) -> int:
    """teal_sparse_gemv_bf16_multi on matrices with rows pitch_list[k] elements apart."""
    count = len(Wt_list)
    if not (len(pitch_list) == len(t_list) == len(y_list) == len(n_list) == count):
        raise ValueError("per-matrix lists must have the same length")
    W = (ctypes.c_void_p * count)(*[_ptr(w, 2 * ((m - 1) * max(int(p), n) + n), "Wt")
                                    for w, n, p in zip(Wt_list, n_list, pitch_list)])
    P = (ctypes.c_int * count)(*[int(p) for p in pitch_list])
    Y = (ctypes.c_void_p * count)(*[_ptr(y, 4 * n, "y") for y, n in zip(y_list, n_list)])
    Tt = (ctypes.c_float * count)(*[float(t) for t in t_list])
    N = (ctypes.c_int * count)(*[int(n) for n in n_list])
    return _call(
        "teal_sparse_gemv_bf16_multi_pitch",
        count, W, P, Tt, Y, N, _ptr(x_f16, 2 * m, "x"), int(m), _ptr(workspace),
        _nbytes(workspace, workspace_bytes), _stream(stream))


def teal_sparse_gemv_w8_multi_pitch(Wq_list, pitch_list, scale_list, t_list, y_list, n_list, x_f16, m,
                                    workspace, workspace_bytes=None, stream=None) -> int:
    """teal_sparse_gemv_w8_multi on matrices with rows pitch_list[k] elements (bytes) apart."""
    count = len(Wq_list)
    if not (len(pitch_list) == len(scale_list) == len(t_list) == len(y_list) == len(n_list) == count):
        raise ValueError("per-matrix lists must have the same length")
    W = (ctypes.c_void_p * count)(*[_ptr(w, (m - 1) * max(int(p), n) + n, "Wq")
                                    for w, n, p in zip(Wq_list, n_list, pitch_list)])
    P = (ctypes.c_int * count)(*[int(p) for p in pitch_list])
    S = (ctypes.c_void_p * count)(*[_ptr(sc, 2 * n, "scale") for sc, n in zip(scale_list, n_list)])
    Y = (ctypes.c_void_p * count)(*[_ptr(y, 4 * n, "y") for y, n in zip(y_list, n_list)])
    Tt = (ctypes.c_float * count)(*[float(t) for t in t_list])
    N = (ctypes.c_int * count)(*[int(n) for n in n_list])
    return _call(
        "teal_sparse_gemv_w8_multi_pitch",
        count, W, P, S, Tt, Y, N, _ptr(x_f16, 2 * m, "x"), int(m), _ptr(workspace),
        _nbytes(workspace, workspace_bytes), _stream(stream))


def teal_gemv_plan_multi_pitch(weight_bits: int, m: int, n_list, pitch_list):
    """Returns (status, dict) for a grouped launch on matrices with padded rows."""
    count = len(n_list)
    N = (ctypes.c_int * max(count, 1))(*[int(n) for n in n_list])
    P = (ctypes.c_int * max(count, 1))(*[int(p) for p in pitch_list])
    vals = [ctypes.c_int(0) for _ in range(5)]
    st = load_library().teal_gemv_plan_multi_pitch(int(weight_bits), int(m), N, P, count,
                                                   *[ctypes.byref(v) for v in vals])
    keys = ("lanes_per_row", "tile_cols", "splits", "waves", "unroll")
    return st, {k: v.value for k, v in zip(keys, vals)}


def teal_workspace_bytes_stack(counts, n_list, m_list) -> int:
    """Workspace of a stack call: counts[g] matrices per group, n over all matrices, m per group."""
    C = (ctypes.c_int * len(counts))(*[int(c) for c in counts])
    N = (ctypes.c_int * len(n_list))(*[int(n) for n in n_list])
    M = (ctypes.c_int * len(m_list))(*[int(m) for m in m_list])
    if len(m_list) != len(counts) or sum(int(c) for c in counts) != len(n_list):
        raise ValueError("counts, n and m do not describe the same groups")
    return int(load_library().teal_workspace_bytes_stack(len(counts), C, N, M))


def _stack_arrays(counts, W_list, wbytes, t_list, y_list, n_list, x_list, m_list, scale_list=None,
                  sbytes=None):
    """Host arrays of a stack call; wbytes(m, n) / sbytes(m, n) = bytes the call reads per matrix."""
    groups = len(counts)
    total = sum(int(c) for c in counts)
    if not (len(W_list) == len(t_list) == len(y_list) == len(n_list) == total):
        raise ValueError("per-matrix lists must have one entry per matrix of every group")
    if scale_list is not None and len(scale_list) != total:
        raise ValueError("per-matrix lists must have one entry per matrix of every group")
    if not (len(x_list) == len(m_list) == groups):
        raise ValueError("per-group lists must have one entry per group")
    group_of = [g for g, c in enumerate(counts) for _ in range(int(c))]
    W = (ctypes.c_void_p * total)(*[_ptr(w, wbytes(m_list[g], n), "W")
                                    for w, n, g in zip(W_list, n_list, group_of)])
    S = None
    if scale_list is not None:
        S = (ctypes.c_void_p * total)(*[_ptr(sc, sbytes(m_list[g], n), "scale")
                                        for sc, n, g in zip(scale_list, n_list, group_of)])
    Y = (ctypes.c_void_p * total)(*[_ptr(y, 4 * n, "y") for y, n in zip(y_list, n_list)])
    Tt = (ctypes.c_float * total)(*[float(t) for t in t_list])
    N = (ctypes.c_int * total)(*[int(n) for n in n_list])
    C = (ctypes.c_int * groups)(*[int(c) for c in counts])
    X = (ctypes.c_void_p * groups)(*[_ptr(x, 2 * m, "x") for x, m in zip(x_list, m_list)])
    M = (ctypes.c_int * groups)(*[int(m) for m in m_list])
    return groups, C, W, S, Tt, Y, N, X, M


def teal_sparse_gemv_bf16_stack(counts, Wt_list, t_list, y_list, n_list, x_list, m_list,
                                workspace, workspace_bytes=None, stream=None) -> int:
    """len(counts) independent groups in one launch; matrices listed group after group."""
    groups, C, W, _, Tt, Y, N, X, M = _stack_arrays(counts, Wt_list, lambda m, n: 2 * m * n, t_list,
                                                    y_list, n_list, x_list, m_list)
    return _call(
        "teal_sparse_gemv_bf16_stack",
        groups, C, W, Tt, Y, N, X, M, _ptr(workspace), _nbytes(workspace, workspace_bytes),
        _stream(stream))


def teal_sparse_gemv_w8_stack(counts, Wq_list, scale_list, t_list, y_list, n_list, x_list, m_list,
                              workspace, workspace_bytes=None, stream=None) -> int:
    groups, C, W, S, Tt, Y, N, X, M = _stack_arrays(
        counts, Wq_list, lambda m, n: m * n, t_list, y_list, n_list, x_list, m_list, scale_list,
        lambda m, n: 2 * n)
    return _call(
        "teal_sparse_gemv_w8_stack",
        groups, C, W, S, Tt, Y, N, X, M, _ptr(workspace), _nbytes(workspace, workspace_bytes),
        _stream(stream))


def teal_sparse_gemv_w4_stack(counts, Wq_list, scale_list, group, t_list, y_list, n_list, x_list,
                              m_list, workspace, workspace_bytes=None, stream=None) -> int:
    groups, C, W, S, Tt, Y, N, X, M = _stack_arrays(
        counts, Wq_list, lambda m, n: m * n // 2, t_list, y_list, n_list, x_list, m_list, scale_list,
        lambda m, n: 2 * n * (m // 128))
    return _call(
        "teal_sparse_gemv_w4_stack",
        groups, C, W, S, int(group), Tt, Y, N, X, M, _ptr(workspace),
        _nbytes(workspace, workspace_bytes), _stream(stream))


def teal_stream_read_probe(buf, nbytes, blocks, match, sink, stream=None) -> int:
    """Plain streaming read of nbytes at buf by `blocks` thread blocks (measurement aid)."""
    return _call("teal_stream_read_probe", _ptr(buf, nbytes, "buf"), int(nbytes), int(blocks),
                 int(match) & 0xFFFFFFFF, _ptr(sink, 4 * blocks, "sink"), _stream(stream))


def teal_workspace_bytes_batch(m: int, n: int, batch: int) -> int:
    return int(load_library().teal_workspace_bytes_batch(int(m), int(n), int(batch)))


def teal_sparsify_batch(X_f16, batch, m, t, mask=None, idx=None, count=None, stream=None) -> int:
    return _call("teal_sparsify_batch", _ptr(X_f16, 2 * batch * m, "X"), int(batch), int(m),
                                              float(t), _ptr(mask, m, "mask"),
                                              _ptr(idx, 4 * m, "idx"), _ptr(count, 4, "count"),
                                              _stream(stream))


def teal_sparse_gemv_bf16_batch(Wt_bf16, X_f16, batch, t, Y, m, n, workspace,
                                workspace_bytes=None, stream=None) -> int:
    return _call(
        "teal_sparse_gemv_bf16_batch",
        _ptr(Wt_bf16, 2 * m * n, "Wt"), _ptr(X_f16, 2 * batch * m, "X"), int(batch), float(t),
        _ptr(Y, 4 * batch * n, "Y"), int(m), int(n),
        _ptr(workspace), _nbytes(workspace, workspace_bytes), _stream(stream))


def teal_sparse_gemv_bf16_batch_ex(Wt_bf16, X_f16, batch, t, Y, m, n, workspace,
                                   workspace_bytes=None, stream=None, lanes_per_row=0,
                                   tile_cols=0, splits=0) -> int:
    return _call(
        "teal_sparse_gemv_bf16_batch_ex",
        _ptr(Wt_bf16, 2 * m * n, "Wt"), _ptr(X_f16, 2 * batch * m, "X"), int(batch), float(t),
        _ptr(Y, 4 * batch * n, "Y"), int(m), int(n),
        _ptr(workspace), _nbytes(workspace, workspace_bytes), _stream(stream),
        int(lanes_per_row), int(tile_cols), int(splits))


def teal_sparse_gemv_w8_multi(Wq_list, scale_list, t_list, y_list, n_list, x_f16, m, workspace,
                              workspace_bytes=None, stream=None) -> int:
    """count = len(Wq_list) int8 matrices sharing x; the per-matrix lists become host arrays."""
    count = len(Wq_list)
    if not (len(scale_list) == len(t_list) == len(y_list) == len(n_list) == count):
        raise ValueError("per-matrix lists must have the same length")
    W = (ctypes.c_void_p * count)(*[_ptr(w, m * n, "Wq") for w, n in zip(Wq_list, n_list)])
    S = (ctypes.c_void_p * count)(*[_ptr(sc, 2 * n, "scale") for sc, n in zip(scale_list, n_list)])
    Y = (ctypes.c_void_p * count)(*[_ptr(y, 4 * n, "y") for y, n in zip(y_list, n_list)])
    Tt = (ctypes.c_float * count)(*[float(t) for t in t_list])
    N = (ctypes.c_int * count)(*[int(n) for n in n_list])
    return _call(
        "teal_sparse_gemv_w8_multi",
        count, W, S, Tt, Y, N, _ptr(x_f16, 2 * m, "x"), int(m), _ptr(workspace),
        _nbytes(workspace, workspace_bytes), _stream(stream))


def teal_sparse_gemv_w4_multi(Wq_list, scale_list, group, t_list, y_list, n_list, x_f16, m,
                              workspace, workspace_bytes=None, stream=None) -> int:
    """count = len(Wq_list) int4 matrices sharing x; the per-matrix lists become host arrays."""
    count = len(Wq_list)
    if not (len(scale_list) == len(t_list) == len(y_list) == len(n_list) == count):
        raise ValueError("per-matrix lists must have the same length")
    groups = m // max(int(group), 1)
    W = (ctypes.c_void_p * count)(*[_ptr(w, m * n // 2, "Wq") for w, n in zip(Wq_list, n_list)])
    S = (ctypes.c_void_p * count)(*[_ptr(sc, 2 * n * groups, "scale")
                                    for sc, n in zip(scale_list, n_list)])
    Y = (ctypes.c_void_p * count)(*[_ptr(y, 4 * n, "y") for y, n in zip(y_list, n_list)])
    Tt = (ctypes.c_float * count)(*[float(t) for t in t_list])
    N = (ctypes.c_int * count)(*[int(n) for n in n_list])
    return _call(
        "teal_sparse_gemv_w4_multi",
        count, W, S, int(group), Tt, Y, N, _ptr(x_f16, 2 * m, "x"), int(m), _ptr(workspace),
        _nbytes(workspace, workspace_bytes), _stream(stream))


def teal_sparse_gemv_bf16_batch_multi(Wt_list, t_list, Y_list, n_list, X_f16, batch, m, workspace,
                                      workspace_bytes=None, stream=None) -> int:
    """count = len(Wt_list) matrices sharing the batch X; per-matrix lists become host arrays."""
    count = len(Wt_list)
    if not (len(t_list) == len(Y_list) == len(n_list) == count):
        raise ValueError("per-matrix lists must have the same length")
    W = (ctypes.c_void_p * count)(*[_ptr(w, 2 * m * n, "Wt") for w, n in zip(Wt_list, n_list)])
    Y = (ctypes.c_void_p * count)(*[_ptr(y, 4 * batch * n, "Y") for y, n in zip(Y_list, n_list)])
    Tt = (ctypes.c_float * count)(*[float(t) for t in t_list])
    N = (ctypes.c_int * count)(*[int(n) for n in n_list])
    return _call(
        "teal_sparse_gemv_bf16_batch_multi",
        count, W, Tt, Y, N, _ptr(X_f16, 2 * batch * m, "X"), int(batch), int(m), _ptr(workspace),
        _nbytes(workspace, workspace_bytes), _stream(stream))


def teal_swiglu_f16(gate, up, h_f16, m, stream=None) -> int:
    return _call("teal_swiglu_f16", _ptr(gate, 4 * m, "gate"), _ptr(up, 4 * m, "up"),
                                          _ptr(h_f16, 2 * m, "h"), int(m),
                                          _stream(stream))


def teal_sparse_gemv_bf16_swiglu(Wt_bf16, gate, up, t, y, m, n, workspace, workspace_bytes=None,
                                 stream=None) -> int:
    return _call(
        "teal_sparse_gemv_bf16_swiglu",
        _ptr(Wt_bf16, 2 * m * n, "Wt"), _ptr(gate, 4 * m, "gate"), _ptr(up, 4 * m, "up"), float(t),
        _ptr(y, 4 * n, "y"), int(m), int(n), _ptr(workspace),
        _nbytes(workspace, workspace_bytes), _stream(stream))


def teal_rmsnorm_f16(h, gamma, eps, x_f16, m, stream=None) -> int:
    return _call("teal_rmsnorm_f16", _ptr(h, 4 * m, "h"), _ptr(gamma, 4 * m, "gamma"),
                                           float(eps), _ptr(x_f16, 2 * m, "x"), int(m),
                                           _stream(stream))


def teal_sparse_gemv_bf16_rmsnorm_multi(Wt_list, t_list, y_list, n_list, h, gamma, eps, m,
                                        workspace, workspace_bytes=None, stream=None) -> int:
    """count = len(Wt_list) matrices fed by the normalised h; per-matrix lists become host arrays."""
    count = len(Wt_list)
    if not (len(t_list) == len(y_list) == len(n_list) == count):
        raise ValueError("per-matrix lists must have the same length")
    W = (ctypes.c_void_p * count)(*[_ptr(w, 2 * m * n, "Wt") for w, n in zip(Wt_list, n_list)])
    Y = (ctypes.c_void_p * count)(*[_ptr(y, 4 * n, "y") for y, n in zip(y_list, n_list)])
    Tt = (ctypes.c_float * count)(*[float(t) for t in t_list])
    N = (ctypes.c_int * count)(*[int(n) for n in n_list])
    return _call(
        "teal_sparse_gemv_bf16_rmsnorm_multi",
        count, W, Tt, Y, N, _ptr(h, 4 * m, "h"), _ptr(gamma, 4 * m, "gamma"), float(eps), int(m),
        _ptr(workspace), _nbytes(workspace, workspace_bytes), _stream(stream))


def teal_sparse_gemv_bf16_rmsnorm_multi_pitch(Wt_list, pitch_list, t_list, y_list, n_list, h, gamma,
                                              eps, m, workspace, workspace_bytes=None,
                                              stream=None) -> int:
    """teal_sparse_gemv_bf16_rmsnorm_multi on matrices with rows pitch_list[k] elements apart."""
    count = len(Wt_list)
    if not (len(pitch_list) == len(t_list) == len(y_list) == len(n_list) == count):
        raise ValueError("per-matrix lists must have the same length")
    W = (ctypes.c_void_p * count)(*[_ptr(w, 2 * ((m - 1) * max(int(p), n) + n), "Wt")
                                    for w, n, p in zip(Wt_list, n_list, pitch_list)])
    P = (ctypes.c_int * count)(*[int(p) for p in pitch_list])
    Y = (ctypes.c_void_p * count)(*[_ptr(y, 4 * n, "y") for y, n in zip(y_list, n_list)])
    Tt = (ctypes.c_float * count)(*[float(t) for t in t_list])
    N = (ctypes.c_int * count)(*[int(n) for n in n_list])
    return _call(
        "teal_sparse_gemv_bf16_rmsnorm_multi_pitch",
        count, W, P, Tt, Y, N, _ptr(h, 4 * m, "h"), _ptr(gamma, 4 * m, "gamma"), float(eps), int(m),
        _ptr(workspace), _nbytes(workspace, workspace_bytes), _stream(stream))


def teal_sparse_gemv_w8_swiglu(Wq, scale_f16, gate, up, t, y, m, n, workspace, workspace_bytes=None,
                               stream=None) -> int:
    return _call(
        "teal_sparse_gemv_w8_swiglu",
        _ptr(Wq, m * n, "Wq"), _ptr(scale_f16, 2 * n, "scale"), _ptr(gate, 4 * m, "gate"),
        _ptr(up, 4 * m, "up"), float(t), _ptr(y, 4 * n, "y"), int(m), int(n), _ptr(workspace),
        _nbytes(workspace, workspace_bytes), _stream(stream))


def teal_sparse_gemv_w8_rmsnorm_multi(Wq_list, scale_list, t_list, y_list, n_list, h, gamma, eps, m,
                                      workspace, workspace_bytes=None, stream=None) -> int:
    count = len(Wq_list)
    if not (len(scale_list) == len(t_list) == len(y_list) == len(n_list) == count):
        raise ValueError("per-matrix lists must have the same length")
    W = (ctypes.c_void_p * count)(*[_ptr(w, m * n, "Wq") for w, n in zip(Wq_list, n_list)])
    S = (ctypes.c_void_p * count)(*[_ptr(sc, 2 * n, "scale") for sc, n in zip(scale_list, n_list)])
    Y = (ctypes.c_void_p * count)(*[_ptr(y, 4 * n, "y") for y, n in zip(y_list, n_list)])
    Tt = (ctypes.c_float * count)(*[float(t) for t in t_list])
    N = (ctypes.c_int * count)(*[int(n) for n in n_list])
    return _call(
        "teal_sparse_gemv_w8_rmsnorm_multi",
        count, W, S, Tt, Y, N, _ptr(h, 4 * m, "h"), _ptr(gamma, 4 * m, "gamma"), float(eps), int(m),
        _ptr(workspace), _nbytes(workspace, workspace_bytes), _stream(stream))


def teal_sparse_gemv_w4_swiglu(Wq, scale_f16, group, gate, up, t, y, m, n, workspace,
                               workspace_bytes=None, stream=None) -> int:
    return _call(
        "teal_sparse_gemv_w4_swiglu",
        _ptr(Wq, m * n // 2, "Wq"), _ptr(scale_f16, 2 * n * (m // 128), "scale"), int(group),
        _ptr(gate, 4 * m, "gate"), _ptr(up, 4 * m, "up"), float(t), _ptr(y, 4 * n, "y"), int(m),
        int(n), _ptr(workspace), _nbytes(workspace, workspace_bytes), _stream(stream))


def teal_sparse_gemv_w4_rmsnorm_multi(Wq_list, scale_list, group, t_list, y_list, n_list, h, gamma,
                                      eps, m, workspace, workspace_bytes=None, stream=None) -> int:
    count = len(Wq_list)
    if not (len(scale_list) == len(t_list) == len(y_list) == len(n_list) == count):
        raise ValueError("per-matrix lists must have the same length")
    W = (ctypes.c_void_p * count)(*[_ptr(w, m * n // 2, "Wq") for w, n in zip(Wq_list, n_list)])
    S = (ctypes.c_void_p * count)(*[_ptr(sc, 2 * n * (m // 128), "scale")
                                    for sc, n in zip(scale_list, n_list)])
    Y = (ctypes.c_void_p * count)(*[_ptr(y, 4 * n, "y") for y, n in zip(y_list, n_list)])
    Tt = (ctypes.c_float * count)(*[float(t) for t in t_list])
    N = (ctypes.c_int * count)(*[int(n) for n in n_list])
    return _call(
        "teal_sparse_gemv_w4_rmsnorm_multi",
        count, W, S, int(group), Tt, Y, N, _ptr(h, 4 * m, "h"), _ptr(gamma, 4 * m, "gamma"),
        float(eps), int(m), _ptr(workspace), _nbytes(workspace, workspace_bytes), _stream(stream))


def teal_abs_histogram(x_f16, count, hist, stream=None) -> int:
    return _call("teal_abs_histogram", _ptr(x_f16, 2 * count, "x"), int(count),
                                             _ptr(hist, 8 * TEAL_HIST_BINS, "hist"),
                                             _stream(stream))


def teal_histogram_thresholds(hist, p_list, t, stream=None) -> int:
    """p_list: host levels in [0, 1]; t: device float32 array of the same length."""
    np_ = len(p_list)
    P = (ctypes.c_double * max(np_, 1))(*[float(p) for p in p_list])
    return _call("teal_histogram_thresholds", _ptr(hist, 8 * TEAL_HIST_BINS, "hist"), P, np_,
                                                    _ptr(t, 4 * np_, "t"), _stream(stream))


def teal_workspace_bytes_mlp(m: int, f: int, d: int) -> int:
    return int(load_library().teal_workspace_bytes_mlp(int(m), int(f), int(d)))


def teal_mlp_down_region_offset(m: int, f: int) -> int:
    return int(load_library().teal_mlp_down_region_offset(int(m), int(f)))


def teal_mlp_status_offset(m: int, f: int, d: int) -> int:
    return int(load_library().teal_mlp_status_offset(int(m), int(f), int(d)))


def _mlp_shape(shape):
    """None, an MlpShape, or a dict of its fields (missing fields are zero)."""
    if shape is None or isinstance(shape, MlpShape):
        return shape
    return MlpShape(**{k: int(v) for k, v in dict(shape).items()})


def _mlp_pitches(sh, f, d):
    """Row pitches (elements) a shape gives the matrices: what sizes the weight buffers."""
    pg = sh.gu_row_pitch if sh is not None and sh.gu_row_pitch > f else f
    pd = sh.down_row_pitch if sh is not None and sh.down_row_pitch > d else d
    return int(pg), int(pd)


def teal_mlp_plan(weight_bits: int, m: int, f: int, d: int, gu_row_pitch: int = 0,
                  down_row_pitch: int = 0):
    """Returns (status, MlpShape): the launch shape the library picks for matrices with these
    row pitches (0 = packed rows)."""
    sh = MlpShape()
    sh.gu_row_pitch, sh.down_row_pitch = int(gu_row_pitch), int(down_row_pitch)
    st = load_library().teal_mlp_plan(int(weight_bits), int(m), int(f), int(d), ctypes.byref(sh))
    return st, sh


def teal_mlp_block_info(weight_bits: int, m: int, f: int, d: int, shape, block: int):
    """Returns (status, list of the 8 ints teal.h describes)."""
    sh = _mlp_shape(shape)
    info = (ctypes.c_int * 8)()
    st = load_library().teal_mlp_block_info(int(weight_bits), int(m), int(f), int(d),
                                            ctypes.byref(sh) if sh is not None else None,
                                            int(block), info)
    return st, list(info)


def teal_sparse_mlp_bf16(Wt_gate, Wt_up, Wt_down, x_f16, t_gate, t_up, t_down, gate, up, y, m, f, d,
                         workspace, workspace_bytes=None, stream=None, shape=None) -> int:
    sh = _mlp_shape(shape)
    pg, pd = _mlp_pitches(sh, f, d)
    return _call(
        "teal_sparse_mlp_bf16",
        _ptr(Wt_gate, 2 * ((m - 1) * pg + f), "Wt_gate"), _ptr(Wt_up, 2 * ((m - 1) * pg + f), "Wt_up"),
        _ptr(Wt_down, 2 * ((f - 1) * pd + d), "Wt_down"), _ptr(x_f16, 2 * m, "x"), float(t_gate), float(t_up),
        float(t_down), _ptr(gate, 4 * f, "gate"), _ptr(up, 4 * f, "up"), _ptr(y, 4 * d, "y"),
        int(m), int(f), int(d), _ptr(workspace), _nbytes(workspace, workspace_bytes),
        _stream(stream), ctypes.pointer(sh) if sh is not None else None)


def teal_sparse_mlp_w8(Wq_gate, Wq_up, Wq_down, scale_gate, scale_up, scale_down, x_f16, t_gate,
                       t_up, t_down, gate, up, y, m, f, d, workspace, workspace_bytes=None,
                       stream=None, shape=None) -> int:
    sh = _mlp_shape(shape)
    pg, pd = _mlp_pitches(sh, f, d)
    return _call(
        "teal_sparse_mlp_w8",
        _ptr(Wq_gate, (m - 1) * pg + f, "Wq_gate"), _ptr(Wq_up, (m - 1) * pg + f, "Wq_up"),
        _ptr(Wq_down, (f - 1) * pd + d, "Wq_down"),
        _ptr(scale_gate, 2 * f, "scale_gate"), _ptr(scale_up, 2 * f, "scale_up"),
        _ptr(scale_down, 2 * d, "scale_down"), _ptr(x_f16, 2 * m, "x"), float(t_gate), float(t_up),
        float(t_down), _ptr(gate, 4 * f, "gate"), _ptr(up, 4 * f, "up"), _ptr(y, 4 * d, "y"),
        int(m), int(f), int(d), _ptr(workspace), _nbytes(workspace, workspace_bytes),
        _stream(stream), ctypes.pointer(sh) if sh is not None else None)


def teal_sparse_mlp_w4(Wq_gate, Wq_up, Wq_down, scale_gate, scale_up, scale_down, group, x_f16,
                       t_gate, t_up, t_down, gate, up, y, m, f, d, workspace, workspace_bytes=None,
                       stream=None, shape=None) -> int:
    sh = _mlp_shape(shape)
    g = max(int(group), 1)
    return _call(
        "teal_sparse_mlp_w4",
        _ptr(Wq_gate, m * f // 2, "Wq_gate"), _ptr(Wq_up, m * f // 2, "Wq_up"),
        _ptr(Wq_down, f * d // 2, "Wq_down"), _ptr(scale_gate, 2 * f * (m // g), "scale_gate"),
        _ptr(scale_up, 2 * f * (m // g), "scale_up"), _ptr(scale_down, 2 * d * (f // g), "scale_down"),
        int(group), _ptr(x_f16, 2 * m, "x"), float(t_gate), float(t_up), float(t_down),
        _ptr(gate, 4 * f, "gate"), _ptr(up, 4 * f, "up"), _ptr(y, 4 * d, "y"),
        int(m), int(f), int(d), _ptr(workspace), _nbytes(workspace, workspace_bytes),
        _stream(stream), ctypes.pointer(sh) if sh is not None else None)
