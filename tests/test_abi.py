"""The C-ABI boundary without a GPU: the library loads, exports what
include/teal.h declares, and rejects bad arguments on the host before any GPU
work (so these calls are safe on a machine with no device)."""
import ctypes
import math
import os
import re

import pytest

import paper_2408_14690_amd as T
from paper_2408_14690_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# fake, suitably aligned device addresses: never dereferenced by the checks
W, X, Y, WS, SC = 0x10000, 0x20000, 0x30000, 0x40000, 0x50000
BIG = 1 << 40


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not os.path.exists(T.library_path()):
        from paper_2408_14690_amd import build
        build.build(verbose=False)
    T.load_library()


def _declared_functions():
    """Every function the installed headers declare: teal.h (the method) and teal_probe.h
    (measurement aids, kept apart)."""
    names = set()
    for header in ("teal.h", "teal_probe.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names.update(re.findall(r"\b(teal_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported():
    names = _declared_functions()
    assert set(names) == set(binding.EXPORTS)
    lib = ctypes.CDLL(T.library_path())
    for name in names:
        assert getattr(lib, name) is not None
    # and the Python binding offers the same names
    for name in names:
        assert callable(getattr(T, name))


def test_version_and_status_strings():
    assert T.teal_version() >= 100
    seen = set()
    for code in range(9):
        s = T.teal_status_string(code)
        assert s and s not in seen
        seen.add(s)
    assert T.teal_status_string(0) == "ok"


def test_workspace_bytes():
    assert T.teal_workspace_bytes(0, 8) == 0 and T.teal_workspace_bytes(8, 0) == 0
    # arrival counters (one per 64 output columns of the largest n), the survivor report
    # (64 ints of totals, then 4 matrices x 128 splits of slice counts), 128 fp32 partial rows
    assert T.teal_survivors_offset() == (1 << 24) // 64 * 4
    assert T.teal_workspace_bytes(4096, 4096) == ((1 << 24) // 64 * 4 + (64 + 4 * 128) * 4
                                                   + 128 * 4096 * 4)
    assert T.teal_workspace_bytes(4096, 14336) % 256 == 0
    # very long inputs force more than 128 splits (one block compacts at most 4096 channels)
    assert T.teal_workspace_bytes(1 << 20, 8) >= (1 << 20) // 4096 * 8 * 4
    assert T.teal_workspace_bytes((1 << 24) + 1, 8) == 0


def test_gemv_bf16_argument_errors():
    ok_args = dict(Wt_bf16=W, x_f16=X, t=0.5, y=Y, m=4096, n=4096, workspace=WS,
                   workspace_bytes=BIG, stream=0)

    def call(**kw):
        a = dict(ok_args)
        a.update(kw)
        return T.teal_sparse_gemv_bf16(**a)

    assert call(Wt_bf16=None) == T.TEAL_ERR_NULL
    assert call(x_f16=None) == T.TEAL_ERR_NULL
    assert call(y=None) == T.TEAL_ERR_NULL
    assert call(workspace=None) == T.TEAL_ERR_NULL
    assert call(m=0) == T.TEAL_ERR_SHAPE
    assert call(n=0) == T.TEAL_ERR_SHAPE
    assert call(n=4100) == T.TEAL_ERR_SHAPE           # not a multiple of 8
    assert call(m=(1 << 24) + 1) == T.TEAL_ERR_SHAPE
    assert call(Wt_bf16=W + 8) == T.TEAL_ERR_ALIGN
    assert call(x_f16=X + 1) == T.TEAL_ERR_ALIGN
    assert call(y=Y + 2) == T.TEAL_ERR_ALIGN
    assert call(workspace=WS + 128) == T.TEAL_ERR_ALIGN
    assert call(t=-0.25) == T.TEAL_ERR_THRESHOLD
    assert call(t=math.nan) == T.TEAL_ERR_THRESHOLD
    assert call(t=math.inf) == T.TEAL_ERR_THRESHOLD
    assert call(workspace_bytes=T.teal_workspace_bytes(4096, 4096) - 1) == T.TEAL_ERR_WORKSPACE


def test_gemv_bf16_ex_rejects_unsupported_shapes():
    base = (W, X, 0.5, Y, 4096, 4096, WS, BIG, 0)
    assert T.teal_sparse_gemv_bf16_ex(*base, lanes_per_row=48) == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_sparse_gemv_bf16_ex(*base, splits=129) == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_sparse_gemv_bf16_ex(*base, splits=-1) == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_sparse_gemv_bf16_ex(*base, waves=3) == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_sparse_gemv_bf16_ex(*base, unroll=5) == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_sparse_gemv_bf16_ex(*base, waves=16, unroll=8) == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_sparse_gemv_bf16_ex(*base, tile_cols=12) == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_sparse_gemv_bf16_ex(*base, lanes_per_row=16, tile_cols=136) == T.TEAL_ERR_UNSUPPORTED
    # argument errors win over shape errors
    assert T.teal_sparse_gemv_bf16_ex(None, X, 0.5, Y, 4096, 4096, WS, BIG, 0,
                                      lanes_per_row=48) == T.TEAL_ERR_NULL
    # a caller-chosen tile so narrow that the tiles outnumber the workspace's arrival counters
    wide = (W, X, 0.5, Y, 64, 1 << 22, WS, BIG, 0)
    counters = T.teal_survivors_offset() // 4
    assert (1 << 22) // 8 > counters >= (1 << 22) // 16
    assert T.teal_sparse_gemv_bf16_ex(*wide, lanes_per_row=8, tile_cols=8) == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_sparse_gemv_bf16_batch_ex(W, X, 2, 0.5, Y, 64, 1 << 22, WS, BIG, 0,
                                            lanes_per_row=16, tile_cols=8) == T.TEAL_ERR_UNSUPPORTED


def test_static_scratch_call_argument_errors():
    """The entry point whose scratch is the library's own array: the host checks of
    teal_sparse_gemv_bf16 without those of a workspace, plus its size limit."""
    lim = T.teal_static_scratch_limit()
    assert lim == 65536
    ok = dict(Wt_bf16=W, x_f16=X, t=0.5, y=Y, m=4096, n=4096, stream=0)

    def call(**kw):
        a = dict(ok)
        a.update(kw)
        return T.teal_sparse_gemv_bf16_static(**a)

    assert call(Wt_bf16=None) == T.TEAL_ERR_NULL
    assert call(x_f16=None) == T.TEAL_ERR_NULL
    assert call(y=None) == T.TEAL_ERR_NULL
    assert call(n=4100) == T.TEAL_ERR_SHAPE
    assert call(m=0) == T.TEAL_ERR_SHAPE
    assert call(m=lim + 1) == T.TEAL_ERR_STATIC_LIMIT
    assert call(n=lim + 8) == T.TEAL_ERR_STATIC_LIMIT
    assert call(m=(1 << 24) + 1) == T.TEAL_ERR_SHAPE
    assert call(Wt_bf16=W + 8) == T.TEAL_ERR_ALIGN
    assert call(y=Y + 2) == T.TEAL_ERR_ALIGN
    assert call(t=-1.0) == T.TEAL_ERR_THRESHOLD
    assert call(t=math.inf) == T.TEAL_ERR_THRESHOLD
    assert "static scratch" in T.teal_status_string(T.TEAL_ERR_STATIC_LIMIT)


def test_quantised_argument_errors():
    assert T.teal_sparse_gemv_w8(W, None, X, 0.5, Y, 4096, 4096, WS, BIG, 0) == T.TEAL_ERR_NULL
    assert T.teal_sparse_gemv_w8(W, SC, X, 0.5, Y, 4096, 4104, WS, BIG, 0) == T.TEAL_ERR_SHAPE
    assert T.teal_sparse_gemv_w8(W, SC + 1, X, 0.5, Y, 4096, 4096, WS, BIG, 0) == T.TEAL_ERR_ALIGN
    assert T.teal_sparse_gemv_w8(W, SC, X, -1.0, Y, 4096, 4096, WS, BIG, 0) == T.TEAL_ERR_THRESHOLD
    assert T.teal_sparse_gemv_w4(W, None, 128, X, 0.5, Y, 4096, 4096, WS, BIG, 0) == T.TEAL_ERR_NULL
    assert T.teal_sparse_gemv_w4(W, SC, 128, X, 0.5, Y, 4096, 4112, WS, BIG, 0) == T.TEAL_ERR_SHAPE
    assert T.teal_sparse_gemv_w4(W, SC, 64, X, 0.5, Y, 4096, 4096, WS, BIG, 0) == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_sparse_gemv_w4(W, SC, 128, X, 0.5, Y, 4160, 4096, WS, BIG, 0) == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_sparse_gemv_w4(W, SC + 8, 128, X, 0.5, Y, 4096, 4096, WS, BIG, 0) == T.TEAL_ERR_ALIGN
    assert T.teal_sparse_gemv_w4(W, SC, 128, X, 0.5, Y, 4096, 4096, WS, 16, 0) == T.TEAL_ERR_WORKSPACE


def test_multi_argument_errors():
    ok = dict(Wt_list=[W, W + 0x1000], t_list=[0.5, 0.25], y_list=[Y, Y + 0x1000],
              n_list=[4096, 1024], x_f16=X, m=4096, workspace=WS, workspace_bytes=BIG, stream=0)

    def call(**kw):
        a = dict(ok)
        a.update(kw)
        return T.teal_sparse_gemv_bf16_multi(**a)

    assert call(Wt_list=[W, None]) == T.TEAL_ERR_NULL
    assert call(y_list=[None, Y]) == T.TEAL_ERR_NULL
    assert call(x_f16=None) == T.TEAL_ERR_NULL
    assert call(n_list=[4096, 1020]) == T.TEAL_ERR_SHAPE
    assert call(m=0) == T.TEAL_ERR_SHAPE
    assert call(Wt_list=[W, W + 8]) == T.TEAL_ERR_ALIGN
    assert call(t_list=[0.5, -1.0]) == T.TEAL_ERR_THRESHOLD
    assert call(workspace_bytes=T.teal_workspace_bytes(4096, 5120) - 1) == T.TEAL_ERR_WORKSPACE
    five = dict(Wt_list=[W] * 5, t_list=[0.5] * 5, y_list=[Y] * 5, n_list=[64] * 5)
    assert call(**five) == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_sparse_gemv_bf16_multi([], [], [], [], X, 4096, WS, BIG, 0) == T.TEAL_ERR_UNSUPPORTED


def test_multi_pitch_argument_errors_and_plan():
    """The grouped call on matrices with padded rows: the checks of the packed call plus the
    pitches; the planned shape drops split-K only where the pitches rotate the tiles over the
    address quarters and one 256-byte tile per compute unit exists."""
    ok = dict(Wt_list=[W, W + 0x1000], pitch_list=[4096 + 128, 1024 + 8], t_list=[0.5, 0.25],
              y_list=[Y, Y + 0x1000], n_list=[4096, 1024], x_f16=X, m=4096, workspace=WS,
              workspace_bytes=BIG, stream=0)

    def call(**kw):
        a = dict(ok)
        a.update(kw)
        return T.teal_sparse_gemv_bf16_multi_pitch(**a)

    assert call(Wt_list=[W, None]) == T.TEAL_ERR_NULL
    assert call(n_list=[4096, 1020]) == T.TEAL_ERR_SHAPE
    assert call(pitch_list=[4096 - 8, 1024]) == T.TEAL_ERR_SHAPE        # shorter than the row
    assert call(pitch_list=[4096 + 4, 1024]) == T.TEAL_ERR_SHAPE        # rows not 16-byte aligned
    assert call(Wt_list=[W, W + 8]) == T.TEAL_ERR_ALIGN
    assert call(t_list=[0.5, float("inf")]) == T.TEAL_ERR_THRESHOLD
    assert call(workspace_bytes=T.teal_workspace_bytes(4096, 5120) - 1) == T.TEAL_ERR_WORKSPACE
    q = dict(Wq_list=[W, W + 0x1000], pitch_list=[4096 + 256, 1024], scale_list=[SC, SC],
             t_list=[0.5, 0.25], y_list=[Y, Y + 0x1000], n_list=[4096, 1024], x_f16=X, m=4096,
             workspace=WS, workspace_bytes=BIG, stream=0)
    assert T.teal_sparse_gemv_w8_multi_pitch(**dict(q, pitch_list=[4096 + 8, 1024])) == T.TEAL_ERR_SHAPE
    assert T.teal_sparse_gemv_w8_multi_pitch(**dict(q, scale_list=[SC, None])) == T.TEAL_ERR_NULL
    assert T.teal_sparse_gemv_w8_multi_pitch(**dict(q, workspace_bytes=16)) == T.TEAL_ERR_WORKSPACE

    m, f = 4096, 14336
    packed = T.teal_gemv_plan_multi(16, m, [f, f])
    assert T.teal_gemv_plan_multi_pitch(16, m, [f, f], [f, f]) == packed           # 2 f bytes: a multiple of 1 KiB
    assert T.teal_gemv_plan_multi_pitch(16, m, [f, f], [f + 512, f + 512]) == packed
    assert T.teal_gemv_plan_multi_pitch(16, m, [f, f], [f + 128, f]) == packed     # every matrix must rotate
    st, p = T.teal_gemv_plan_multi_pitch(16, m, [f, f], [f + 128, f + 384])
    assert st == T.TEAL_OK and (p["lanes_per_row"], p["tile_cols"], p["splits"]) == (16, 128, 1)
    st, p = T.teal_gemv_plan_multi_pitch(16, m, [11008, 11008], [11008 + 128] * 2)   # 172 tiles
    assert (p["lanes_per_row"], p["tile_cols"], p["splits"]) == (16, 128, 1)
    st, p = T.teal_gemv_plan_multi_pitch(16, m, [f], [f + 128])                       # one matrix: 128-byte tiles
    assert st == T.TEAL_OK and (p["lanes_per_row"], p["tile_cols"], p["splits"]) == (8, 64, 1)
    # too few tiles (q + k + v of the 8B block: 96 of 128 bytes; one 8192-wide matrix: 128), a slice too long
    assert T.teal_gemv_plan_multi_pitch(16, m, [4096, 1024, 1024], [4096 + 128, 1024 + 128, 1024 + 128]) == \
        T.teal_gemv_plan_multi(16, m, [4096, 1024, 1024])
    assert T.teal_gemv_plan_multi_pitch(16, 8192 + 64, [f, f], [f + 128] * 2) == \
        T.teal_gemv_plan_multi(16, 8192 + 64, [f, f])
    assert T.teal_gemv_plan_multi_pitch(16, 8192, [8192], [8192 + 128]) == T.teal_gemv_plan_multi(16, 8192, [8192])
    # slices of up to 8192 channels: the 70B-sized pair in tiles of 512 bytes; its q + k + v keeps split-K
    st, p = T.teal_gemv_plan_multi_pitch(16, 8192, [28672] * 2, [28672 + 128] * 2)
    assert st == T.TEAL_OK and (p["lanes_per_row"], p["tile_cols"], p["splits"]) == (32, 256, 1)
    qkv = [8192, 1024, 1024]
    assert T.teal_gemv_plan_multi_pitch(16, 8192, qkv, [n + 128 for n in qkv]) == T.teal_gemv_plan_multi(16, 8192, qkv)
    st, p = T.teal_gemv_plan_multi_pitch(8, m, [2 * f, 2 * f], [2 * f + 256] * 2)      # int8: 256 columns per tile
    assert st == T.TEAL_OK and (p["lanes_per_row"], p["tile_cols"], p["splits"]) == (16, 256, 1)
    assert T.teal_gemv_plan_multi_pitch(4, m, [f, f], [f, f])[0] == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_gemv_plan_multi_pitch(16, m, [f, f], [f - 8, f])[0] == T.TEAL_ERR_SHAPE


def test_stack_argument_errors_and_workspace():
    """teal_sparse_gemv_bf16_stack: every check happens on the host before any HIP call; the
    workspace is the sum of the groups' own workspaces."""
    ok = dict(counts=[2, 1], Wt_list=[W, W + 0x1000, W + 0x2000], t_list=[0.5, 0.25, 0.4],
              y_list=[Y, Y + 0x1000, Y + 0x2000], n_list=[4096, 1024, 11008], x_list=[X, X + 0x100],
              m_list=[4096, 2048], workspace=WS, workspace_bytes=BIG, stream=0)

    def call(**kw):
        a = dict(ok)
        a.update(kw)
        return T.teal_sparse_gemv_bf16_stack(**a)

    need = T.teal_workspace_bytes_stack([2, 1], [4096, 1024, 11008], [4096, 2048])
    assert need == T.teal_workspace_bytes(4096, 5120) + T.teal_workspace_bytes(2048, 11008)
    assert call(Wt_list=[W, W, None]) == T.TEAL_ERR_NULL
    assert call(y_list=[Y, None, Y]) == T.TEAL_ERR_NULL
    assert call(x_list=[X, None]) == T.TEAL_ERR_NULL
    assert call(n_list=[4096, 1024, 11004]) == T.TEAL_ERR_SHAPE
    assert call(m_list=[4096, 0]) == T.TEAL_ERR_SHAPE
    assert call(Wt_list=[W, W + 8, W]) == T.TEAL_ERR_ALIGN
    assert call(x_list=[X, X + 1]) == T.TEAL_ERR_ALIGN
    assert call(workspace=WS + 64) == T.TEAL_ERR_ALIGN
    assert call(t_list=[0.5, 0.25, math.nan]) == T.TEAL_ERR_THRESHOLD
    assert call(workspace_bytes=need - 1) == T.TEAL_ERR_WORKSPACE
    assert call(workspace_bytes=T.teal_workspace_bytes(4096, 5120)) == T.TEAL_ERR_WORKSPACE
    five = dict(counts=[5], Wt_list=[W] * 5, t_list=[0.5] * 5, y_list=[Y] * 5, n_list=[64] * 5,
                x_list=[X], m_list=[4096])
    assert call(**five) == T.TEAL_ERR_UNSUPPORTED
    many = dict(counts=[1] * 17, Wt_list=[W] * 17, t_list=[0.5] * 17, y_list=[Y] * 17,
                n_list=[64] * 17, x_list=[X] * 17, m_list=[64] * 17)
    assert call(**many) == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_workspace_bytes_stack([1] * 17, [64] * 17, [64] * 17) == 0
    assert T.teal_workspace_bytes_stack([5], [64] * 5, [64]) == 0
    assert T.teal_workspace_bytes_stack([1], [60], [64]) == 0
    with pytest.raises(ValueError):
        T.teal_sparse_gemv_bf16_stack([2], [W], [0.5], [Y], [64], [X], [64], WS, BIG, 0)


def test_int8_fused_producer_argument_errors():
    G, U, H, GA = 0x70000, 0x80000, 0x90000, 0xA0000
    ok = dict(Wq=W, scale_f16=SC, gate=G, up=U, t=0.5, y=Y, m=4096, n=1024, workspace=WS,
              workspace_bytes=BIG, stream=0)

    def sw(**kw):
        a = dict(ok)
        a.update(kw)
        return T.teal_sparse_gemv_w8_swiglu(**a)

    assert sw(up=None) == T.TEAL_ERR_NULL
    assert sw(scale_f16=None) == T.TEAL_ERR_NULL
    assert sw(n=1032) == T.TEAL_ERR_SHAPE
    assert sw(gate=G + 2) == T.TEAL_ERR_ALIGN
    assert sw(scale_f16=SC + 1) == T.TEAL_ERR_ALIGN
    assert sw(t=-1.0) == T.TEAL_ERR_THRESHOLD
    assert sw(workspace_bytes=64) == T.TEAL_ERR_WORKSPACE
    okn = dict(Wq_list=[W, W + 0x1000], scale_list=[SC, SC + 0x100], t_list=[0.5, 0.25],
               y_list=[Y, Y + 0x1000], n_list=[4096, 1024], h=H, gamma=GA, eps=1e-5, m=4096,
               workspace=WS, workspace_bytes=BIG, stream=0)

    def nm(**kw):
        a = dict(okn)
        a.update(kw)
        return T.teal_sparse_gemv_w8_rmsnorm_multi(**a)

    assert nm(h=None) == T.TEAL_ERR_NULL
    assert nm(scale_list=[SC, None]) == T.TEAL_ERR_NULL
    assert nm(n_list=[4096, 1032]) == T.TEAL_ERR_SHAPE
    assert nm(m=16392) == T.TEAL_ERR_SHAPE
    assert nm(m=4100) == T.TEAL_ERR_SHAPE
    assert nm(h=H + 4) == T.TEAL_ERR_ALIGN
    assert nm(eps=-1.0) == T.TEAL_ERR_THRESHOLD
    assert nm(t_list=[0.5, math.inf]) == T.TEAL_ERR_THRESHOLD
    assert nm(workspace_bytes=64) == T.TEAL_ERR_WORKSPACE
    five = dict(Wq_list=[W] * 5, scale_list=[SC] * 5, t_list=[0.5] * 5, y_list=[Y] * 5, n_list=[64] * 5)
    assert nm(**five) == T.TEAL_ERR_UNSUPPORTED


def test_int4_fused_producer_argument_errors():
    G, U, H, GA = 0x70000, 0x80000, 0x90000, 0xA0000
    ok = dict(Wq=W, scale_f16=SC, group=128, gate=G, up=U, t=0.5, y=Y, m=4096, n=1024, workspace=WS,
              workspace_bytes=BIG, stream=0)

    def sw(**kw):
        a = dict(ok)
        a.update(kw)
        return T.teal_sparse_gemv_w4_swiglu(**a)

    assert sw(up=None) == T.TEAL_ERR_NULL
    assert sw(n=1040) == T.TEAL_ERR_SHAPE
    assert sw(scale_f16=SC + 8) == T.TEAL_ERR_ALIGN
    assert sw(t=math.nan) == T.TEAL_ERR_THRESHOLD
    assert sw(group=32) == T.TEAL_ERR_UNSUPPORTED
    assert sw(m=4160) == T.TEAL_ERR_UNSUPPORTED
    assert sw(workspace_bytes=64) == T.TEAL_ERR_WORKSPACE
    okn = dict(Wq_list=[W, W + 0x1000], scale_list=[SC, SC + 0x100], group=128, t_list=[0.5, 0.25],
               y_list=[Y, Y + 0x1000], n_list=[4096, 1024], h=H, gamma=GA, eps=1e-5, m=4096,
               workspace=WS, workspace_bytes=BIG, stream=0)

    def nm(**kw):
        a = dict(okn)
        a.update(kw)
        return T.teal_sparse_gemv_w4_rmsnorm_multi(**a)

    assert nm(gamma=None) == T.TEAL_ERR_NULL
    assert nm(n_list=[4096, 1040]) == T.TEAL_ERR_SHAPE
    assert nm(m=16512) == T.TEAL_ERR_SHAPE
    assert nm(scale_list=[SC, SC + 8]) == T.TEAL_ERR_ALIGN
    assert nm(eps=math.inf) == T.TEAL_ERR_THRESHOLD
    assert nm(group=64) == T.TEAL_ERR_UNSUPPORTED
    assert nm(m=4104) == T.TEAL_ERR_UNSUPPORTED
    assert nm(workspace_bytes=64) == T.TEAL_ERR_WORKSPACE


def test_stream_read_probe_argument_errors():
    assert T.teal_stream_read_probe(None, 4096, 256, 0, Y, 0) == T.TEAL_ERR_NULL
    assert T.teal_stream_read_probe(W, 4096, 256, 0, None, 0) == T.TEAL_ERR_NULL
    assert T.teal_stream_read_probe(W, 0, 256, 0, Y, 0) == T.TEAL_ERR_SHAPE
    assert T.teal_stream_read_probe(W, 4100, 256, 0, Y, 0) == T.TEAL_ERR_SHAPE
    assert T.teal_stream_read_probe(W, 4096, 0, 0, Y, 0) == T.TEAL_ERR_SHAPE
    assert T.teal_stream_read_probe(W, 4096, 65537, 0, Y, 0) == T.TEAL_ERR_SHAPE
    assert T.teal_stream_read_probe(W + 8, 4096, 256, 0, Y, 0) == T.TEAL_ERR_ALIGN
    assert T.teal_stream_read_probe(W, 4096, 256, 0, Y + 2, 0) == T.TEAL_ERR_ALIGN


def test_quantised_stack_argument_errors():
    ok = dict(counts=[2, 1], Wq_list=[W, W + 0x1000, W + 0x2000], scale_list=[SC, SC + 0x100, SC + 0x200],
              t_list=[0.5, 0.25, 0.4], y_list=[Y, Y + 0x1000, Y + 0x2000], n_list=[4096, 1024, 11008],
              x_list=[X, X + 0x100], m_list=[4096, 2048], workspace=WS, workspace_bytes=BIG, stream=0)

    def w8(**kw):
        a = dict(ok)
        a.update(kw)
        return T.teal_sparse_gemv_w8_stack(**a)

    def w4(**kw):
        a = dict(ok, group=128)
        a.update(kw)
        return T.teal_sparse_gemv_w4_stack(**a)

    for call in (w8, w4):
        assert call(Wq_list=[W, W, None]) == T.TEAL_ERR_NULL
        assert call(scale_list=[SC, None, SC]) == T.TEAL_ERR_NULL
        assert call(x_list=[None, X]) == T.TEAL_ERR_NULL
        assert call(m_list=[4096, 0]) == T.TEAL_ERR_SHAPE
        assert call(Wq_list=[W, W + 8, W]) == T.TEAL_ERR_ALIGN
        assert call(t_list=[0.5, -0.25, 0.4]) == T.TEAL_ERR_THRESHOLD
        assert call(workspace_bytes=4096) == T.TEAL_ERR_WORKSPACE
        assert call(counts=[2, 1] + [1] * 15, Wq_list=[W] * 18, scale_list=[SC] * 18, t_list=[0.5] * 18,
                    y_list=[Y] * 18, n_list=[64] * 18, x_list=[X] * 17, m_list=[128] * 17) \
            == T.TEAL_ERR_UNSUPPORTED
    assert w8(n_list=[4096, 1032, 11008]) == T.TEAL_ERR_SHAPE      # not a multiple of 16
    assert w4(n_list=[4096, 1040, 11008]) == T.TEAL_ERR_SHAPE      # not a multiple of 32
    assert w8(scale_list=[SC, SC + 1, SC]) == T.TEAL_ERR_ALIGN
    assert w4(scale_list=[SC, SC + 8, SC]) == T.TEAL_ERR_ALIGN
    assert w4(group=64) == T.TEAL_ERR_UNSUPPORTED
    assert w4(m_list=[4096, 2112]) == T.TEAL_ERR_UNSUPPORTED       # not a multiple of 128


def test_w8_multi_argument_errors():
    ok = dict(Wq_list=[W, W + 0x1000], scale_list=[SC, SC + 0x100], t_list=[0.5, 0.25],
              y_list=[Y, Y + 0x1000], n_list=[4096, 1024], x_f16=X, m=4096, workspace=WS,
              workspace_bytes=BIG, stream=0)

    def call(**kw):
        a = dict(ok)
        a.update(kw)
        return T.teal_sparse_gemv_w8_multi(**a)

    assert call(Wq_list=[W, None]) == T.TEAL_ERR_NULL
    assert call(scale_list=[SC, None]) == T.TEAL_ERR_NULL
    assert call(y_list=[None, Y]) == T.TEAL_ERR_NULL
    assert call(x_f16=None) == T.TEAL_ERR_NULL
    assert call(n_list=[4096, 1032]) == T.TEAL_ERR_SHAPE          # not a multiple of 16
    assert call(m=0) == T.TEAL_ERR_SHAPE
    assert call(Wq_list=[W, W + 8]) == T.TEAL_ERR_ALIGN
    assert call(scale_list=[SC, SC + 1]) == T.TEAL_ERR_ALIGN
    assert call(t_list=[0.5, math.inf]) == T.TEAL_ERR_THRESHOLD
    assert call(workspace_bytes=T.teal_workspace_bytes(4096, 5120) - 1) == T.TEAL_ERR_WORKSPACE
    five = dict(Wq_list=[W] * 5, scale_list=[SC] * 5, t_list=[0.5] * 5, y_list=[Y] * 5,
                n_list=[64] * 5)
    assert call(**five) == T.TEAL_ERR_UNSUPPORTED


def test_w4_multi_argument_errors():
    ok = dict(Wq_list=[W, W + 0x1000], scale_list=[SC, SC + 0x100], group=128, t_list=[0.5, 0.25],
              y_list=[Y, Y + 0x1000], n_list=[4096, 1024], x_f16=X, m=4096, workspace=WS,
              workspace_bytes=BIG, stream=0)

    def call(**kw):
        a = dict(ok)
        a.update(kw)
        return T.teal_sparse_gemv_w4_multi(**a)

    assert call(Wq_list=[None, W]) == T.TEAL_ERR_NULL
    assert call(scale_list=[SC, None]) == T.TEAL_ERR_NULL
    assert call(n_list=[4096, 1040]) == T.TEAL_ERR_SHAPE          # not a multiple of 32
    assert call(scale_list=[SC, SC + 8]) == T.TEAL_ERR_ALIGN
    assert call(t_list=[-0.5, 0.5]) == T.TEAL_ERR_THRESHOLD
    assert call(group=64) == T.TEAL_ERR_UNSUPPORTED
    assert call(m=4160) == T.TEAL_ERR_UNSUPPORTED
    assert call(workspace_bytes=16) == T.TEAL_ERR_WORKSPACE
    assert T.teal_sparse_gemv_w4_multi([], [], 128, [], [], [], X, 4096, WS, BIG, 0) == T.TEAL_ERR_UNSUPPORTED


def test_swiglu_argument_errors():
    G, U, H = 0x70000, 0x80000, 0x90000
    assert T.teal_swiglu_f16(None, U, H, 16, stream=0) == T.TEAL_ERR_NULL
    assert T.teal_swiglu_f16(G, None, H, 16, stream=0) == T.TEAL_ERR_NULL
    assert T.teal_swiglu_f16(G, U, None, 16, stream=0) == T.TEAL_ERR_NULL
    assert T.teal_swiglu_f16(G, U, H, -1, stream=0) == T.TEAL_ERR_SHAPE
    assert T.teal_swiglu_f16(G + 2, U, H, 16, stream=0) == T.TEAL_ERR_ALIGN
    assert T.teal_swiglu_f16(G, U, H + 1, 16, stream=0) == T.TEAL_ERR_ALIGN
    assert T.teal_swiglu_f16(None, None, None, 0, stream=0) == T.TEAL_OK
    ok = dict(Wt_bf16=W, gate=G, up=U, t=0.5, y=Y, m=14336, n=4096, workspace=WS,
              workspace_bytes=BIG, stream=0)

    def call(**kw):
        a = dict(ok)
        a.update(kw)
        return T.teal_sparse_gemv_bf16_swiglu(**a)

    assert call(gate=None) == T.TEAL_ERR_NULL
    assert call(up=None) == T.TEAL_ERR_NULL
    assert call(Wt_bf16=None) == T.TEAL_ERR_NULL
    assert call(n=4100) == T.TEAL_ERR_SHAPE
    assert call(gate=G + 2) == T.TEAL_ERR_ALIGN
    assert call(up=U + 1) == T.TEAL_ERR_ALIGN
    assert call(t=-1.0) == T.TEAL_ERR_THRESHOLD
    assert call(workspace_bytes=16) == T.TEAL_ERR_WORKSPACE


def test_plan_is_reported():
    st, plan = T.teal_gemv_plan(16, 4096, 14336)
    assert st == T.TEAL_OK
    assert plan["tile_cols"] % 64 == 0 and plan["tile_cols"] <= 8 * plan["lanes_per_row"]
    assert 1 <= plan["splits"] <= 16 and plan["waves"] in (4, 8, 16)
    assert T.teal_gemv_plan(12, 4096, 4096)[0] == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_gemv_plan(16, 0, 4096)[0] == T.TEAL_ERR_SHAPE
    # grouped launches: one matrix is the single plan; several fill the chip once
    assert T.teal_gemv_plan_multi(16, 4096, [14336]) == T.teal_gemv_plan(16, 4096, 14336)
    for bits, ns in ((16, [4096, 4096, 4096]), (16, [4096, 1024, 1024]), (8, [14336, 14336]),
                     (4, [4096, 1024, 1024])):
        st, pl = T.teal_gemv_plan_multi(bits, 4096, ns)
        assert st == T.TEAL_OK
        tiles = sum(-(-n // pl["tile_cols"]) for n in ns)
        assert 128 <= tiles * pl["splits"] <= 256
        assert pl["tile_cols"] <= pl["lanes_per_row"] * {16: 8, 8: 16, 4: 32}[bits]
    # inputs too long for 16 splits: as many as the 4096-channel slices need, and no
    # more partial rows than the workspace holds
    for m in (70000, 1 << 20):
        st, pl = T.teal_gemv_plan_multi(16, m, [4096, 4096])
        assert st == T.TEAL_OK and pl["splits"] >= -(-m // 4096)
        assert (pl["splits"] * 8192 * 4 + (1 << 24) // 64 * 4) <= T.teal_workspace_bytes(m, 8192)
    assert T.teal_gemv_plan_multi(16, 4096, [])[0] == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_gemv_plan_multi(16, 4096, [64] * 5)[0] == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_gemv_plan_multi(12, 4096, [64, 64])[0] == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_gemv_plan_multi(16, 4096, [64, 0])[0] == T.TEAL_ERR_SHAPE


# (lanes per row, tile columns, splits, thread blocks) the launch rule gives for the
# projections of the benchmark configurations: the shapes the measured figures belong to.
PLANNED_GRIDS = {
    ("llama2_7b", 16): {"q": (16, 128, 8, 256), "gate": (64, 384, 8, 232), "down": (16, 128, 8, 256),
                        "q+k+v": (32, 256, 5, 240), "gate+up": (64, 448, 5, 250)},
    ("llama3_8b", 16): {"q": (16, 128, 8, 256), "k": (16, 128, 16, 128), "gate": (64, 448, 8, 256),
                        "down": (16, 128, 8, 256), "q+k+v": (16, 128, 5, 240), "gate+up": (64, 448, 4, 256)},
    ("llama_70b", 16): {"q": (32, 256, 8, 256), "k": (16, 128, 16, 128), "gate": (64, 512, 4, 224),
                        "down": (32, 256, 8, 256), "q+k+v": (16, 128, 3, 240), "gate+up": (64, 448, 2, 256)},
    ("llama3_8b", 8): {"q": (8, 128, 8, 256), "gate": (32, 512, 8, 224), "down": (8, 128, 8, 256),
                       "q+k+v": (8, 128, 5, 240), "gate+up": (64, 896, 8, 256)},
    ("llama3_8b", 4): {"q": (16, 512, 16, 128), "gate": (16, 512, 8, 224), "down": (16, 512, 16, 128),
                       "q+k+v": (16, 512, 16, 192), "gate+up": (32, 1024, 8, 224)},
}


@pytest.mark.parametrize("model,bits", sorted(PLANNED_GRIDS))
def test_planned_grids_of_the_benchmark_configurations(model, bits):
    """The launch rule is a set of constants from sweeps on one chip (256 compute units): about
    one block of 8 wavefronts per unit, at most 16 splits, tiles on 128-byte boundaries.  This
    pins what it yields for the benchmark's shapes, so a change of the rule shows up here."""
    import teal_inputs as ti
    shapes = ti.LAYER_SHAPES[model]
    for name, want in PLANNED_GRIDS[(model, bits)].items():
        members = name.split("+")
        ns = [shapes[p][0] for p in members]
        m = shapes[members[0]][1]
        if len(ns) == 1:
            st, p = T.teal_gemv_plan(bits, m, ns[0])
        else:
            st, p = T.teal_gemv_plan_multi(bits, m, ns)
        assert st == T.TEAL_OK
        blocks = sum(-(-n // p["tile_cols"]) for n in ns) * p["splits"]
        assert (p["lanes_per_row"], p["tile_cols"], p["splits"], blocks) == want, (name, p, blocks)
        assert p["waves"] == 8 and p["unroll"] == 4
        assert blocks <= 256 and p["tile_cols"] * bits % (8 * 128) == 0   # fills the chip once; 128-byte edges


def test_sparsify_and_pack_argument_errors():
    assert T.teal_sparsify(None, 16, 0.5, Y, None, None, stream=0) == T.TEAL_ERR_NULL
    assert T.teal_sparsify(X, -1, 0.5, Y, None, None, stream=0) == T.TEAL_ERR_SHAPE
    assert T.teal_sparsify(X + 1, 16, 0.5, Y, None, None, stream=0) == T.TEAL_ERR_ALIGN
    assert T.teal_sparsify(X, 16, 0.5, None, Y + 2, None, stream=0) == T.TEAL_ERR_ALIGN
    assert T.teal_sparsify(X, 16, -0.5, Y, None, None, stream=0) == T.TEAL_ERR_THRESHOLD
    # nothing requested: accepted, nothing launched
    assert T.teal_sparsify(X, 16, 0.5, None, None, None, stream=0) == T.TEAL_OK
    assert T.teal_pack_bf16(None, Y, 8, 8, stream=0) == T.TEAL_ERR_NULL
    assert T.teal_pack_bf16(X, None, 8, 8, stream=0) == T.TEAL_ERR_NULL
    assert T.teal_pack_bf16(X, Y, 0, 8, stream=0) == T.TEAL_ERR_SHAPE
    assert T.teal_pack_bf16(X + 1, Y, 8, 8, stream=0) == T.TEAL_ERR_ALIGN


def test_calibration_argument_errors():
    H = 0x60000
    assert T.teal_abs_histogram(None, 16, H, stream=0) == T.TEAL_ERR_NULL
    assert T.teal_abs_histogram(X, 16, None, stream=0) == T.TEAL_ERR_NULL
    assert T.teal_abs_histogram(X + 1, 16, H, stream=0) == T.TEAL_ERR_ALIGN
    assert T.teal_abs_histogram(X, 16, H + 4, stream=0) == T.TEAL_ERR_ALIGN
    assert T.teal_abs_histogram(X, (1 << 38) + 1, H, stream=0) == T.TEAL_ERR_SHAPE
    assert T.teal_abs_histogram(None, 0, H, stream=0) == T.TEAL_OK        # empty batch: nothing to do
    assert T.teal_histogram_thresholds(None, [0.5], Y, stream=0) == T.TEAL_ERR_NULL
    assert T.teal_histogram_thresholds(H, [0.5], None, stream=0) == T.TEAL_ERR_NULL
    assert T.teal_histogram_thresholds(H, [], Y, stream=0) == T.TEAL_ERR_SHAPE
    assert T.teal_histogram_thresholds(H, [0.5] * 17, Y, stream=0) == T.TEAL_ERR_SHAPE
    assert T.teal_histogram_thresholds(H, [1.5], Y, stream=0) == T.TEAL_ERR_THRESHOLD
    assert T.teal_histogram_thresholds(H, [float("nan")], Y, stream=0) == T.TEAL_ERR_THRESHOLD
    assert T.teal_histogram_thresholds(H + 4, [0.5], Y, stream=0) == T.TEAL_ERR_ALIGN


def test_batch_argument_errors():
    ok = dict(Wt_bf16=W, X_f16=X, batch=4, t=0.5, Y=Y, m=4096, n=4096, workspace=WS,
              workspace_bytes=BIG, stream=0)

    def call(**kw):
        a = dict(ok)
        a.update(kw)
        return T.teal_sparse_gemv_bf16_batch(**a)

    assert call(Wt_bf16=None) == T.TEAL_ERR_NULL
    assert call(X_f16=None) == T.TEAL_ERR_NULL
    assert call(Y=None) == T.TEAL_ERR_NULL
    assert call(workspace=None) == T.TEAL_ERR_NULL
    assert call(batch=0) == T.TEAL_ERR_SHAPE
    assert call(batch=T.TEAL_MAX_BATCH + 1) == T.TEAL_ERR_SHAPE
    assert call(n=4100) == T.TEAL_ERR_SHAPE
    assert call(m=0) == T.TEAL_ERR_SHAPE
    assert call(Wt_bf16=W + 8) == T.TEAL_ERR_ALIGN
    assert call(X_f16=X + 1) == T.TEAL_ERR_ALIGN
    assert call(t=-1.0) == T.TEAL_ERR_THRESHOLD
    assert call(t=math.nan) == T.TEAL_ERR_THRESHOLD
    need = T.teal_workspace_bytes_batch(4096, 4096, 4)
    assert need % 256 == 0 and need >= (1 << 24) // 64 * 4 + 16 * 4 * 4096 * 4
    assert call(workspace_bytes=need - 1) == T.TEAL_ERR_WORKSPACE
    assert T.teal_workspace_bytes_batch(4096, 4096, 0) == 0
    assert T.teal_workspace_bytes_batch(4096, 4096, 9) == 0
    # long inputs: a block compacts at most 2048 channels of a batch, so more partial rows
    assert T.teal_workspace_bytes_batch(1 << 16, 8, 2) >= (1 << 16) // 2048 * 2 * 8 * 4
    base = (W, X, 8, 0.5, Y, 4096, 4096, WS, BIG, 0)
    assert T.teal_sparse_gemv_bf16_batch_ex(*base, lanes_per_row=64) == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_sparse_gemv_bf16_batch_ex(*base, lanes_per_row=8) == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_sparse_gemv_bf16_batch_ex(*base, splits=1) == T.TEAL_ERR_UNSUPPORTED   # slice of 4096
    assert T.teal_sparse_gemv_bf16_batch_ex(*base, splits=64) == T.TEAL_ERR_UNSUPPORTED  # partial rows
    assert T.teal_sparse_gemv_bf16_batch_ex(*base, tile_cols=12) == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_sparsify_batch(None, 2, 16, 0.5, Y, None, None, stream=0) == T.TEAL_ERR_NULL
    assert T.teal_sparsify_batch(X, 0, 16, 0.5, Y, None, None, stream=0) == T.TEAL_ERR_SHAPE
    assert T.teal_sparsify_batch(X, 9, 16, 0.5, Y, None, None, stream=0) == T.TEAL_ERR_SHAPE
    assert T.teal_sparsify_batch(X, 2, -1, 0.5, Y, None, None, stream=0) == T.TEAL_ERR_SHAPE
    assert T.teal_sparsify_batch(X + 1, 2, 16, 0.5, Y, None, None, stream=0) == T.TEAL_ERR_ALIGN
    assert T.teal_sparsify_batch(X, 2, 16, -0.5, Y, None, None, stream=0) == T.TEAL_ERR_THRESHOLD
    assert T.teal_sparsify_batch(X, 2, 16, 0.5, None, None, None, stream=0) == T.TEAL_OK


def test_batch_multi_argument_errors():
    ok = dict(Wt_list=[W, W + 0x1000], t_list=[0.5, 0.25], Y_list=[Y, Y + 0x1000],
              n_list=[4096, 1024], X_f16=X, batch=4, m=4096, workspace=WS, workspace_bytes=BIG,
              stream=0)

    def call(**kw):
        a = dict(ok)
        a.update(kw)
        return T.teal_sparse_gemv_bf16_batch_multi(**a)

    assert call(Wt_list=[W, None]) == T.TEAL_ERR_NULL
    assert call(X_f16=None) == T.TEAL_ERR_NULL
    assert call(batch=0) == T.TEAL_ERR_SHAPE
    assert call(batch=9) == T.TEAL_ERR_SHAPE
    assert call(n_list=[4096, 1020]) == T.TEAL_ERR_SHAPE
    assert call(Wt_list=[W, W + 8]) == T.TEAL_ERR_ALIGN
    assert call(t_list=[0.5, -1.0]) == T.TEAL_ERR_THRESHOLD
    assert call(workspace_bytes=T.teal_workspace_bytes_batch(4096, 5120, 4) - 1) == T.TEAL_ERR_WORKSPACE
    five = dict(Wt_list=[W] * 5, t_list=[0.5] * 5, Y_list=[Y] * 5, n_list=[64] * 5)
    assert call(**five) == T.TEAL_ERR_UNSUPPORTED


def test_check_raises_with_message():
    with pytest.raises(T.TealError) as e:
        T.check(T.TEAL_ERR_WORKSPACE)
    assert "workspace" in str(e.value) and e.value.status == T.TEAL_ERR_WORKSPACE
    T.check(T.TEAL_OK)


def test_binding_refuses_tensors_smaller_than_the_call_touches():
    """The C ABI sees plain pointers; the binding knows a tensor's size and refuses a
    buffer the kernels would run past (CPU tensors stand in: the check is on sizes)."""
    torch = pytest.importorskip("torch")
    m = 256
    ws = torch.zeros(T.teal_workspace_bytes(m, 128), dtype=torch.uint8)
    x = torch.zeros(m, dtype=torch.int16)
    wt = torch.zeros(m * 64, dtype=torch.int16)
    y = torch.zeros(64)
    with pytest.raises(ValueError, match="Wt"):
        T.teal_sparse_gemv_bf16(wt, x, 0.5, torch.zeros(128), m, 128, ws, stream=0)
    with pytest.raises(ValueError, match="y:"):
        T.teal_sparse_gemv_bf16(wt, x, 0.5, torch.zeros(32), m, 64, ws, stream=0)
    with pytest.raises(ValueError, match="x:"):
        T.teal_sparse_gemv_bf16(wt, x[:100].clone(), 0.5, y, m, 64, ws, stream=0)
    # grouped calls: every per-matrix list must be in the same order
    q = [torch.zeros(m * n // 2, dtype=torch.uint8) for n in (64, 32)]
    sc = [torch.zeros(m // 128 * n, dtype=torch.int16) for n in (64, 32)]
    ys = [torch.zeros(n) for n in (32, 64)]
    with pytest.raises(ValueError, match="Wq"):
        T.teal_sparse_gemv_w4_multi(q, sc, 128, [0.1, 0.1], ys, [32, 64], x, m, ws, stream=0)
    with pytest.raises(ValueError, match="Y:"):
        T.teal_sparse_gemv_bf16_batch(wt, torch.zeros(2 * m, dtype=torch.int16), 2, 0.5,
                                      torch.zeros(64), m, 64, ws, stream=0)
    with pytest.raises(ValueError, match="gate"):
        T.teal_sparse_gemv_bf16_swiglu(wt, torch.zeros(m - 1), torch.zeros(m), 0.5, y, m, 64, ws,
                                       stream=0)


def test_rmsnorm_argument_errors():
    H, G = 1 << 20, 2 << 20                       # fake 16-byte aligned device addresses
    assert T.teal_rmsnorm_f16(None, G, 1e-5, X, 4096, stream=0) == T.TEAL_ERR_NULL
    assert T.teal_rmsnorm_f16(H, G, 1e-5, X, 0, stream=0) == T.TEAL_ERR_SHAPE
    assert T.teal_rmsnorm_f16(H, G, 1e-5, X, 4100, stream=0) == T.TEAL_ERR_SHAPE        # m % 8
    assert T.teal_rmsnorm_f16(H, G, 1e-5, X, 16392, stream=0) == T.TEAL_ERR_SHAPE       # > 16384
    assert T.teal_rmsnorm_f16(H + 4, G, 1e-5, X, 4096, stream=0) == T.TEAL_ERR_ALIGN
    assert T.teal_rmsnorm_f16(H, G, -1.0, X, 4096, stream=0) == T.TEAL_ERR_THRESHOLD
    assert T.teal_rmsnorm_f16(H, G, float("nan"), X, 4096, stream=0) == T.TEAL_ERR_THRESHOLD

    def call(count=2, t=(0.5, 0.5), n=(4096, 1024), h=H, gamma=G, eps=1e-5, m=4096, ws=WS,
             ws_bytes=BIG, w=None, y=None):
        w = [W] * count if w is None else w
        y = [Y] * count if y is None else y
        return T.teal_sparse_gemv_bf16_rmsnorm_multi(w, list(t), y, list(n), h, gamma, eps, m, ws,
                                                     ws_bytes, stream=0)

    assert call(h=None) == T.TEAL_ERR_NULL
    assert call(gamma=None) == T.TEAL_ERR_NULL
    assert call(w=[W, None]) == T.TEAL_ERR_NULL
    assert call(m=4100) == T.TEAL_ERR_SHAPE
    assert call(m=32768) == T.TEAL_ERR_SHAPE
    assert call(n=(4096, 1020)) == T.TEAL_ERR_SHAPE
    assert call(h=H + 8) == T.TEAL_ERR_ALIGN
    assert call(t=(0.5, -1.0)) == T.TEAL_ERR_THRESHOLD
    assert call(eps=float("inf")) == T.TEAL_ERR_THRESHOLD
    assert call(ws_bytes=64) == T.TEAL_ERR_WORKSPACE
    assert call(count=5, t=(0.5,) * 5, n=(64,) * 5) == T.TEAL_ERR_UNSUPPORTED


def test_rmsnorm_multi_pitch_argument_errors():
    H, G = 0x60000, 0x70000
    ok = dict(Wt_list=[W, W + 0x1000], pitch_list=[4096 + 128, 1024 + 128], t_list=[0.5, 0.25],
              y_list=[Y, Y + 0x1000], n_list=[4096, 1024], h=H, gamma=G, eps=1e-5, m=4096,
              workspace=WS, workspace_bytes=BIG, stream=0)

    def call(**kw):
        a = dict(ok)
        a.update(kw)
        return T.teal_sparse_gemv_bf16_rmsnorm_multi_pitch(**a)

    assert call(h=None) == T.TEAL_ERR_NULL
    assert call(Wt_list=[None, W]) == T.TEAL_ERR_NULL
    assert call(pitch_list=[4096 - 8, 1024]) == T.TEAL_ERR_SHAPE
    assert call(pitch_list=[4096 + 4, 1024]) == T.TEAL_ERR_SHAPE
    assert call(m=4100) == T.TEAL_ERR_SHAPE
    assert call(h=H + 4) == T.TEAL_ERR_ALIGN
    assert call(eps=-1.0) == T.TEAL_ERR_THRESHOLD
    assert call(workspace_bytes=64) == T.TEAL_ERR_WORKSPACE


def test_plans_of_random_shapes_are_always_launchable():
    """Host logic: for any accepted shape the chosen launch shape satisfies what the kernels
    and the workspace assume (tile width a multiple of the vector width and within the lanes,
    slices within the LDS list, partial rows within the workspace)."""
    import numpy as np
    rng = np.random.Generator(np.random.PCG64(2024))
    epl = {16: 8, 8: 16, 4: 32}
    for _ in range(3000):
        bits = int(rng.choice([16, 8, 4]))
        m = int(np.exp(rng.uniform(0, np.log(1 << 21))))
        count = int(rng.integers(1, 5))
        ns = [max(epl[bits], int(np.exp(rng.uniform(np.log(8), np.log(1 << 17)))) // epl[bits] * epl[bits])
              for _ in range(count)]
        if bits == 4:
            m = max(128, m // 128 * 128)
        st, pl = T.teal_gemv_plan_multi(bits, m, ns)
        assert st == T.TEAL_OK, (bits, m, ns)
        assert pl["lanes_per_row"] in (8, 16, 32, 64) and pl["waves"] == 8 and pl["unroll"] == 4
        assert pl["tile_cols"] % epl[bits] == 0 and 0 < pl["tile_cols"] <= pl["lanes_per_row"] * epl[bits]
        ks = -(-m // pl["splits"])
        mult = 128 if bits == 4 else 64
        ks = -(-ks // mult) * mult
        assert ks <= 4096 or pl["splits"] == -(-m // 4096), (bits, m, ns, pl)
        splits = -(-m // min(ks, 4096))
        need = (1 << 24) // 64 * 4 + splits * sum(ns) * 4
        assert need <= T.teal_workspace_bytes(m, sum(ns)), (bits, m, ns, pl)
        if count == 1:
            assert T.teal_gemv_plan(bits, m, ns[0]) == (st, pl)


def test_header_is_plain_c_and_links_against_the_library(tmp_path):
    """include/teal.h compiles as C99 with warnings as errors, and a C program that takes the
    address of every declared function links against the built library (no C++ names, no
    torch types in the signatures)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    names = _declared_functions()
    src = tmp_path / "use_teal.c"
    body = "\n".join(f"    p[{i}] = (void (*)(void))&{n};" for i, n in enumerate(names))
    src.write_text('#include "teal.h"\n#include "teal_probe.h"\n#include <stdio.h>\nint main(void)\n{\n'
                   f"    void (*p[{len(names)}])(void);\n{body}\n"
                   f"    printf(\"%d %s\\n\", teal_version(), teal_status_string(TEAL_OK));\n"
                   f"    return p[0] == 0;\n}}\n")
    exe = tmp_path / "use_teal"
    libdir = os.path.dirname(T.library_path())
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror",
                    "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe),
                    "-L", libdir, "-l:libteal.so", f"-Wl,-rpath,{libdir}"], check=True)
    res = subprocess.run([str(exe)], capture_output=True, text=True, check=True)
    assert res.stdout.split()[0] == str(T.teal_version())


def test_prepared_calls_marshal_once():
    """prepare() records the marshalled arguments of the calls a function makes (nothing is
    enqueued meanwhile) and returns a function that re-issues them; shown here on calls that
    the host checks reject, so no GPU is touched."""
    made = []

    def two_calls():
        made.append(T.teal_sparse_gemv_bf16(W, X, 0.5, Y, 4096, 4096, WS, 16, stream=0))
        made.append(T.teal_sparse_gemv_bf16(W, X, -1.0, Y, 4096, 4096, WS, BIG, stream=0))

    run = T.prepare(two_calls)
    assert made == [T.TEAL_OK, T.TEAL_OK]                 # recorded, not executed
    assert run() == T.TEAL_ERR_WORKSPACE                  # the first failing status
    assert run() == T.TEAL_ERR_WORKSPACE
    one = T.prepare(lambda: T.teal_sparse_gemv_bf16_multi([W, W], [0.5, float("nan")], [Y, Y],
                                                          [64, 64], X, 4096, WS, BIG, stream=0))
    assert one() == T.TEAL_ERR_THRESHOLD
    with pytest.raises(RuntimeError):
        T.prepare(lambda: T.prepare(lambda: None))
    # and the module is back to calling straight through
    assert T.teal_sparse_gemv_bf16(W, X, -1.0, Y, 4096, 4096, WS, BIG, stream=0) == T.TEAL_ERR_THRESHOLD


def test_a_recording_does_not_swallow_other_threads_calls():
    """While one host thread records with prepare(), a call made by another thread goes
    straight to the library (and here comes back with the host check's status)."""
    import threading
    entered, release, seen = threading.Event(), threading.Event(), []

    def slow_enqueue():
        T.teal_sparse_gemv_bf16(W, X, -1.0, Y, 4096, 4096, WS, BIG, stream=0)
        entered.set()
        release.wait(10)

    def other():
        entered.wait(10)
        seen.append(T.teal_sparse_gemv_bf16(W, X, -1.0, Y, 4096, 4096, WS, BIG, stream=0))
        release.set()

    th = threading.Thread(target=other)
    th.start()
    run = T.prepare(slow_enqueue)
    th.join()
    assert seen == [T.TEAL_ERR_THRESHOLD]                 # executed, not recorded
    assert run() == T.TEAL_ERR_THRESHOLD                  # only the recording thread's call
