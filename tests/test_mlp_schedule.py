"""The block schedule of the one-launch MLP (Appendix A.3) without a GPU: the library
describes every thread block of a launch through teal_mlp_block_info (the same integer
arithmetic the kernel runs), and a small model of a GPU's block dispatcher -- blocks start in
index order as slots free up, running blocks finish in any order, a block of W_down cannot
finish before the gate / up tiles it waits for -- checks that the work is covered exactly
once, that every wait is for exactly the tiles that hold the waiting block's inputs, and that
no order of completion and no number of slots can leave a block waiting for ever."""
import os
import random

import pytest

import paper_2408_14690_amd as T

GATE, UP, DOWN = 0, 1, 2


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not os.path.exists(T.library_path()):
        from paper_2408_14690_amd import build
        build.build(verbose=False)
    T.load_library()


def blocks_of(bits, m, f, d, shape):
    st, info = T.teal_mlp_block_info(bits, m, f, d, shape, -1)
    assert st == T.TEAL_OK
    out = []
    for b in range(info[0]):
        st, i = T.teal_mlp_block_info(bits, m, f, d, shape, b)
        assert st == T.TEAL_OK and i[0] == info[0]
        out.append(dict(kind=i[1], tile=i[2], split=i[3], lo=i[4], hi=i[5], a=i[6], b=i[7]))
    return out


def shape_of(bits, m, f, d, **over):
    st, sh = T.teal_mlp_plan(bits, m, f, d)
    assert st == T.TEAL_OK
    for k, v in over.items():
        setattr(sh, k, v)
    return sh


def simulate(blocks, slots, rng, order=None):
    """In-order dispatch into `slots` slots; running blocks complete in random order, a
    consumer only once its slice's counter has reached the value it waits for.  Returns the
    completion order, or None if a state is reached in which nothing can complete."""
    order = list(range(len(blocks))) if order is None else order
    splits_gu = 1 + max(b["split"] for b in blocks if b["kind"] != DOWN)
    arrived, ready = {}, {}
    running, nxt, done = [], 0, []
    while len(done) < len(blocks):
        while nxt < len(order) and len(running) < slots:
            running.append(order[nxt])
            nxt += 1
        can = [i for i in running
               if blocks[i]["kind"] != DOWN or ready.get(blocks[i]["a"], 0) == blocks[i]["b"]]
        if not can:
            return None
        i = rng.choice(can)
        running.remove(i)
        done.append(i)
        blk = blocks[i]
        if blk["kind"] != DOWN:
            key = (blk["kind"], blk["tile"])
            arrived[key] = arrived.get(key, 0) + 1
            if arrived[key] == splits_gu:                 # the block that combines the K-slices
                for s in range(blk["a"], blk["b"] + 1):
                    ready[s] = ready.get(s, 0) + 1
    return done


SHAPES = [
    (16, 4096, 14336, 4096, {}),
    (16, 4096, 14336, 4096, dict(gu_phase_tiles=4)),
    (16, 4096, 14336, 4096, dict(gu_lanes_per_row=16, gu_tile_cols=128, gu_splits=2, gu_phase_tiles=14,
                                 down_lanes_per_row=32, down_tile_cols=256, down_splits=16)),
    (16, 4096, 11008, 4096, dict(gu_phase_tiles=3)),
    (16, 8192, 28672, 8192, dict(gu_phase_tiles=8)),
    (16, 520, 1224, 264, dict(gu_lanes_per_row=16, gu_tile_cols=120, gu_splits=3, gu_phase_tiles=2,
                              down_lanes_per_row=16, down_tile_cols=72, down_splits=5)),
    (8, 4096, 14336, 4096, dict(gu_phase_tiles=2)),
    (4, 4096, 14336, 4096, dict(gu_phase_tiles=5)),
]


@pytest.mark.parametrize("bits,m,f,d,over", SHAPES)
def test_every_tile_and_slice_is_covered_exactly_once(bits, m, f, d, over):
    sh = shape_of(bits, m, f, d, **over)
    blocks = blocks_of(bits, m, f, d, sh)
    gu = [b for b in blocks if b["kind"] != DOWN]
    dn = [b for b in blocks if b["kind"] == DOWN]
    # producers first, then consumers
    first_down = min(i for i, b in enumerate(blocks) if b["kind"] == DOWN)
    assert all(b["kind"] != DOWN for b in blocks[:first_down])
    assert all(b["kind"] == DOWN for b in blocks[first_down:])
    # each (matrix, tile, K-slice) once; the tiles of a matrix cover [0, f) without overlap
    seen = {(b["kind"], b["tile"], b["split"]) for b in gu}
    assert len(seen) == len(gu)
    for kind in (GATE, UP):
        tiles = sorted({(b["tile"], b["lo"], b["hi"]) for b in gu if b["kind"] == kind})
        assert tiles[0][1] == 0 and tiles[-1][2] == f
        assert all(a[2] == b[1] for a, b in zip(tiles, tiles[1:]))
        splits = {b["split"] for b in gu if b["kind"] == kind}
        assert splits == set(range(len(splits)))
        assert len([b for b in gu if b["kind"] == kind]) == len(tiles) * len(splits)
    # W_down: each (tile, K-slice) once; the slices cover [0, f) without overlap
    assert len({(b["tile"], b["split"]) for b in dn}) == len(dn)
    slices = sorted({(b["split"], b["lo"], b["hi"]) for b in dn})
    assert slices[0][1] == 0 and slices[-1][2] == f
    assert all(a[2] == b[1] for a, b in zip(slices, slices[1:]))
    # a slice waits for exactly the gate and up tiles that hold one of its channels, and
    # exactly those tiles tell it
    for s, k0, k1 in slices:
        for kind in (GATE, UP):
            overlapping = {b["tile"] for b in gu if b["kind"] == kind and b["lo"] < k1 and b["hi"] > k0}
            telling = {b["tile"] for b in gu if b["kind"] == kind and b["a"] <= s <= b["b"]}
            assert overlapping == telling
        expected = {b["b"] for b in dn if b["split"] == s}
        assert expected == {2 * len(overlapping)}


@pytest.mark.parametrize("bits,m,f,d,over", SHAPES)
def test_phases_finish_the_first_columns_first(bits, m, f, d, over):
    sh = shape_of(bits, m, f, d, **over)
    blocks = blocks_of(bits, m, f, d, sh)
    gu = [b for b in blocks if b["kind"] != DOWN]
    tiles = 1 + max(b["tile"] for b in gu)
    per = sh.gu_phase_tiles or tiles
    phase = [b["tile"] // per for b in gu]
    assert phase == sorted(phase)                      # a phase's blocks are contiguous, in order
    # inside a phase gate and up alternate, so both halves of a column range finish together
    for p in set(phase):
        kinds = [b["kind"] for b, q in zip(gu, phase) if q == p]
        assert kinds[0::2] == [GATE] * (len(kinds) // 2) and kinds[1::2] == [UP] * (len(kinds) // 2)
    # blocks of W_down come in the order of the columns they read
    dn = [b for b in blocks if b["kind"] == DOWN]
    assert [b["lo"] for b in dn] == sorted(b["lo"] for b in dn)


@pytest.mark.parametrize("bits,m,f,d,over", SHAPES[:6])
@pytest.mark.parametrize("slots", [1, 2, 7, 256, 768, 100000])
def test_no_wait_lasts_for_ever_whatever_finishes_first(bits, m, f, d, over, slots):
    sh = shape_of(bits, m, f, d, **over)
    blocks = blocks_of(bits, m, f, d, sh)
    for seed in range(3):
        done = simulate(blocks, slots, random.Random(1000 * slots + seed))
        assert done is not None and sorted(done) == list(range(len(blocks)))


def test_the_model_sees_a_schedule_that_can_wait_for_ever():
    """The same model with the consumers placed BEFORE their producers and fewer slots than
    consumers: nothing can complete.  (The mistake is planted in the model's dispatch order,
    on the CPU; the kernel's order is the one checked above.)"""
    sh = shape_of(16, 4096, 14336, 4096, gu_lanes_per_row=64, gu_tile_cols=448, gu_splits=4)
    blocks = blocks_of(16, 4096, 14336, 4096, sh)
    n_down = sum(b["kind"] == DOWN for b in blocks)
    wrong = sorted(range(len(blocks)), key=lambda i: blocks[i]["kind"] != DOWN)
    assert simulate(blocks, n_down // 2, random.Random(1), order=wrong) is None
    assert simulate(blocks, len(blocks), random.Random(1), order=wrong) is not None


def test_plan_and_argument_errors():
    W, X, Y, WS = 0x10000, 0x20000, 0x30000, 0x40000
    BIG = 1 << 40
    m, f, d = 4096, 14336, 4096
    st, sh = T.teal_mlp_plan(16, m, f, d)
    assert st == T.TEAL_OK
    # the library's choice: W_down as its own call; gate / up without split-K in tiles of 256
    # bytes of a row where that gives about one block per compute unit (224 here), else the
    # shape of the grouped gate + up call (the 70B-sized layer; int8, where 256 bytes are 256
    # columns and the blocks would be too few)
    st2, dn = T.teal_gemv_plan(16, f, d)
    assert st2 == T.TEAL_OK
    assert (sh.gu_lanes_per_row, sh.gu_tile_cols, sh.gu_splits) == (16, 128, 1)
    assert (sh.down_lanes_per_row, sh.down_tile_cols, sh.down_splits) == (dn["lanes_per_row"], dn["tile_cols"], dn["splits"])
    for bits, (mm, ff, dd) in ((16, (8192, 28672, 8192)), (8, (m, f, d)), (4, (m, f, d))):
        st, big = T.teal_mlp_plan(bits, mm, ff, dd)
        st2, gu = T.teal_gemv_plan_multi(bits, mm, [ff, ff])
        assert st == st2 == T.TEAL_OK
        assert (big.gu_lanes_per_row, big.gu_tile_cols, big.gu_splits) == (gu["lanes_per_row"], gu["tile_cols"], gu["splits"])
    assert T.teal_mlp_plan(5, m, f, d)[0] == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_mlp_plan(16, m, f + 4, d)[0] == T.TEAL_ERR_SHAPE
    need = T.teal_workspace_bytes_mlp(m, f, d)
    control = 128 * (1 + 4096)          # status word + one counter line per W_down block
    assert need == T.teal_workspace_bytes(m, 2 * f) + T.teal_workspace_bytes(f, d) + control
    assert T.teal_mlp_down_region_offset(m, f) == T.teal_workspace_bytes(m, 2 * f)
    assert T.teal_mlp_status_offset(m, f, d) == need - control
    assert T.teal_workspace_bytes_mlp(m, 0, d) == 0

    ok = dict(Wt_gate=W, Wt_up=W, Wt_down=W, x_f16=X, t_gate=0.5, t_up=0.5, t_down=0.1, gate=Y,
              up=Y + 0x100000, y=Y + 0x200000, m=m, f=f, d=d, workspace=WS, workspace_bytes=BIG,
              stream=0)

    def call(**kw):
        a = dict(ok)
        a.update(kw)
        return T.teal_sparse_mlp_bf16(**a)

    assert call(Wt_up=None) == T.TEAL_ERR_NULL
    assert call(gate=None) == T.TEAL_ERR_NULL
    assert call(workspace=None) == T.TEAL_ERR_NULL
    assert call(f=f + 4) == T.TEAL_ERR_SHAPE
    assert call(d=0) == T.TEAL_ERR_SHAPE
    assert call(Wt_down=W + 8) == T.TEAL_ERR_ALIGN
    assert call(up=Y + 2) == T.TEAL_ERR_ALIGN
    assert call(t_down=-1.0) == T.TEAL_ERR_THRESHOLD
    assert call(t_up=float("nan")) == T.TEAL_ERR_THRESHOLD
    assert call(workspace_bytes=need - 1) == T.TEAL_ERR_WORKSPACE
    bad = T.MlpShape(**sh.as_dict())
    bad.gu_lanes_per_row = 48
    assert call(shape=bad) == T.TEAL_ERR_UNSUPPORTED
    bad = T.MlpShape(**sh.as_dict())
    bad.down_splits = 224                                   # more blocks than readiness counters
    bad.down_tile_cols = 128
    assert call(shape=bad) == T.TEAL_ERR_UNSUPPORTED
    bad = T.MlpShape(**sh.as_dict())
    bad.extra_lds_bytes = 1 << 20
    assert call(shape=bad) == T.TEAL_ERR_UNSUPPORTED
    # row pitches: 0 (packed rows) is the library's choice; else at least the row and rows 16-byte aligned
    assert (sh.gu_row_pitch, sh.down_row_pitch) == (0, 0)
    for field, value in (("gu_row_pitch", f - 8), ("gu_row_pitch", f + 4), ("gu_row_pitch", -8),
                         ("down_row_pitch", d - 8), ("down_row_pitch", d + 12)):
        bad = T.MlpShape(**sh.as_dict())
        setattr(bad, field, value)
        assert call(shape=bad) == T.TEAL_ERR_UNSUPPORTED
        assert T.teal_mlp_block_info(16, m, f, d, bad, 0)[0] == T.TEAL_ERR_UNSUPPORTED
    # the plan follows the layout the caller names: narrow tiles without split-K on rotating rows
    st, p70 = T.teal_mlp_plan(16, 8192, 28672, 8192, gu_row_pitch=28672 + 128, down_row_pitch=8192 + 128)
    assert st == T.TEAL_OK and (p70.gu_lanes_per_row, p70.gu_tile_cols, p70.gu_splits) == (32, 256, 1)
    assert (p70.gu_row_pitch, p70.down_row_pitch) == (28672 + 128, 8192 + 128)
    st, p8 = T.teal_mlp_plan(8, m, f, d, gu_row_pitch=f + 256)
    assert st == T.TEAL_OK and (p8.gu_lanes_per_row, p8.gu_tile_cols, p8.gu_splits) == (8, 128, 1)
    st, pb = T.teal_mlp_plan(16, m, f, d, gu_row_pitch=f + 128)
    assert (pb.gu_lanes_per_row, pb.gu_tile_cols, pb.gu_splits) == (16, 128, 1)
    st, pc = T.teal_mlp_plan(16, 8192, 28672, 8192, gu_row_pitch=28672 + 512)      # not rotating
    st0, p0 = T.teal_mlp_plan(16, 8192, 28672, 8192)
    assert (pc.gu_lanes_per_row, pc.gu_tile_cols, pc.gu_splits) == (p0.gu_lanes_per_row, p0.gu_tile_cols, p0.gu_splits)
    # bf16 tiles of 128 bytes (8 lanes) have no instance in this kernel: the packed choice stays
    st, pn = T.teal_mlp_plan(16, m, 8192, d, gu_row_pitch=8192 + 128)
    st0, pn0 = T.teal_mlp_plan(16, m, 8192, d)
    assert (pn.gu_lanes_per_row, pn.gu_tile_cols, pn.gu_splits) == (pn0.gu_lanes_per_row, pn0.gu_tile_cols, pn0.gu_splits)
    assert T.teal_mlp_plan(16, m, f, d, gu_row_pitch=f - 8)[0] == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_mlp_plan(4, m, f, d, gu_row_pitch=f + 128)[0] == T.TEAL_ERR_UNSUPPORTED
    good = T.MlpShape(**sh.as_dict())
    good.gu_row_pitch, good.down_row_pitch = f + 128, d + 128
    assert T.teal_mlp_block_info(16, m, f, d, good, -1)[1][0] == T.teal_mlp_block_info(16, m, f, d, sh, -1)[1][0]
    assert T.teal_pack_bf16_pitch(W, X, 64, 64, 63, stream=0) == T.TEAL_ERR_SHAPE
    assert T.teal_pack_bf16_pitch(None, X, 64, 64, 64, stream=0) == T.TEAL_ERR_NULL
    assert T.teal_pack_bf16_pitch(W, X + 1, 64, 64, 72, stream=0) == T.TEAL_ERR_ALIGN
    # quantised: scales required, int4 group size
    q = dict(Wq_gate=W, Wq_up=W, Wq_down=W, scale_gate=X, scale_up=X, scale_down=X, x_f16=X,
             t_gate=0.5, t_up=0.5, t_down=0.1, gate=Y, up=Y + 0x100000, y=Y + 0x200000, m=m, f=f,
             d=d, workspace=WS, workspace_bytes=BIG, stream=0)
    assert T.teal_sparse_mlp_w8(**dict(q, scale_up=None)) == T.TEAL_ERR_NULL
    assert T.teal_sparse_mlp_w8(**dict(q, d=4104)) == T.TEAL_ERR_SHAPE
    assert T.teal_sparse_mlp_w4(group=64, **q) == T.TEAL_ERR_UNSUPPORTED
    assert T.teal_sparse_mlp_w4(group=128, **dict(q, scale_down=X + 2)) == T.TEAL_ERR_ALIGN
    st, s4 = T.teal_mlp_plan(4, m, f, d)
    assert st == T.TEAL_OK
    s4.gu_row_pitch = f + 128                               # int4 rows are always packed
    assert T.teal_sparse_mlp_w4(group=128, shape=s4, **q) == T.TEAL_ERR_UNSUPPORTED
    st, s8 = T.teal_mlp_plan(8, m, f, d)
    s8.down_row_pitch = d + 8                               # int8 rows: a multiple of 16
    assert T.teal_sparse_mlp_w8(shape=s8, **q) == T.TEAL_ERR_UNSUPPORTED


def test_every_plan_for_padded_rows_is_a_shape_the_launch_accepts():
    """teal_mlp_plan told the row pitches never names a shape teal_mlp_block_info (which
    validates like the launch) refuses, whatever the sizes."""
    for bits in (16, 8):
        pad = 256 * 8 // bits
        for m in (512, 2048, 4096, 5120, 8192, 16384):
            for f in (1024, 3584, 5504, 8192, 14336, 28672, 57344):
                for d in (512, 4096, 8192):
                    for extra in (pad, 2 * pad, 5 * pad):
                        st, sh = T.teal_mlp_plan(bits, m, f, d, f + extra, d + pad)
                        assert st == T.TEAL_OK, (bits, m, f, d, extra)
                        assert (sh.gu_row_pitch, sh.down_row_pitch) == (f + extra, d + pad)
                        if sh.gu_splits == 1:
                            assert m <= 8192
                        st, _ = T.teal_mlp_block_info(bits, m, f, d, sh, 0)
                        assert st == T.TEAL_OK, (bits, m, f, d, extra, sh.as_dict())
