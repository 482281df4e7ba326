"""Host-side logic of bench.py that needs no GPU: the algorithmic-byte formula the roofline
figures rest on, the argument contract, and the grouping of a block's projections."""
import json
import subprocess
import sys
import os

import pytest

import bench
import teal_inputs as ti

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_algorithmic_bytes_formula():
    """Bytes the method must move for one call: the surviving rows, x, y and the scales
    (n*b bytes per surviving channel: 2, 1, 0.5 for bf16, int8, int4)."""
    m, n, nnz = 4096, 14336, 2048
    assert bench.algorithmic_bytes("bf16", nnz, m, n) == nnz * n * 2 + 2 * m + 4 * n
    assert bench.algorithmic_bytes("w8", nnz, m, n) == nnz * n + 2 * m + 4 * n + 2 * n
    assert bench.algorithmic_bytes("w4", nnz, m, n) == nnz * n // 2 + 2 * m + 4 * n + 2 * n * (m // 128)
    # a batch re-reads nothing: the rows once, x and y per batch row
    assert bench.algorithmic_bytes("bf16", nnz, m, n, 4) == nnz * n * 2 + 4 * (2 * m + 4 * n)
    # the sizes quoted for the 4096 x 14336-class projections: 117.4 MB dense, 58.7 MB at 50 %
    assert round(bench.algorithmic_bytes("bf16", m, m, n) / 1e6, 1) == 117.5
    assert round(bench.algorithmic_bytes("bf16", nnz, m, n) / 1e6, 1) == 58.8
    # at the 8 TB/s peak: 14.7 us dense, 7.3 us at 50 %
    assert round(bench.algorithmic_bytes("bf16", m, m, n) / bench.HBM_PEAK_GBS / 1e3, 1) == 14.7
    assert round(bench.algorithmic_bytes("bf16", nnz, m, n) / bench.HBM_PEAK_GBS / 1e3, 1) == 7.3


def test_block_shapes_and_input_groups():
    """The seven matrices of a block (Appendix A.3) and which of them read the same state."""
    for model, (d, dkv, dm) in {"llama2_7b": (4096, 4096, 11008), "llama3_8b": (4096, 1024, 14336),
                                "llama_70b": (8192, 1024, 28672)}.items():
        s = ti.LAYER_SHAPES[model]
        assert [s[p] for p in ti.PROJ_ORDER] == [(d, d), (dkv, d), (dkv, d), (d, d), (dm, d), (dm, d), (d, dm)]
    groups = {}
    for p in ti.PROJ_ORDER:
        groups.setdefault(ti.PROJ_XGROUP[p], []).append(p)
    assert list(groups.values()) == [["q", "k", "v"], ["o"], ["gate", "up"], ["down"]]
    # projections that share a state share its seed; the others do not
    assert ti.x_seed(2, 0, "q") == ti.x_seed(2, 0, "k") == ti.x_seed(2, 0, "v")
    assert ti.x_seed(2, 0, "gate") == ti.x_seed(2, 0, "up")
    assert len({ti.x_seed(2, 0, p) for p in ("q", "o", "gate", "down")}) == 4


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_measured_traffic_table_is_close_to_the_algorithmic_bytes():
    """The HBM bytes per launch copied from the rocprofv3 summaries stay within 3 % of the
    algorithmic bytes of the same launches (they include the partial rows and x per tile)."""
    # no GPU: the 50 % bytes of the Llama-2-7B block recomputed from its shapes
    shapes = ti.LAYER_SHAPES["llama2_7b"]
    per_proj = sum(bench.algorithmic_bytes("bf16", m // 2, m, n) for n, m in shapes.values())
    grouped = per_proj - 2 * 4096 * 3          # x read once for q+k+v and once for gate+up
    t = bench.MEASURED_TRAFFIC_BYTES
    assert abs(t[("llama2_7b", "bf16", 0.5, 1, True)] * 4 / grouped - 1) < 0.03
    assert abs(t[("llama2_7b", "bf16", 0.5, 1, False)] * 7 / per_proj - 1) < 0.03
    assert abs(t[("llama2_7b", "bf16", 0.5, 1, "stack")] / grouped - 1) < 0.03
