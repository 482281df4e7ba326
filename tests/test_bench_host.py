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


def test_measured_traffic_comes_from_a_profile_summary_of_the_same_kernels(tmp_path):
    """roofline.traffic is read from a rocprofv3 counter summary under profiles/, and only from
    one taken for the same workload, format, sparsity, launch mode AND library version: a
    summary of older kernels gives no figure, with the reason."""
    import bench_lib
    (tmp_path / "a.txt").write_text(
        "header\n"
        "TRAFFIC workload=llama_70b format=bf16 sparsity=0.5 layers=80 launches=grouped "
        "library_version=400 fetch_bytes_per_launch=1000 write_bytes_per_launch=24\n"
        "TRAFFIC workload=llama3_8b format=bf16 sparsity=0.5 layers=1 launches=grouped "
        "library_version=399 fetch_bytes_per_launch=5 write_bytes_per_launch=5\n")
    got, src = bench_lib.measured_traffic("llama_70b", "bf16", 0.5, 80, "grouped", 400, str(tmp_path))
    assert got == 1024.0 and src.endswith("a.txt")
    got, why = bench_lib.measured_traffic("llama3_8b", "bf16", 0.5, 1, "grouped", 400, str(tmp_path))
    assert got is None and "399" in why
    got, why = bench_lib.measured_traffic("llama2_7b", "w8", 0.5, 1, "stack", 400, str(tmp_path))
    assert got is None and "no rocprofv3" in why


def test_committed_traffic_summaries_are_close_to_the_algorithmic_bytes():
    """Every TRAFFIC line committed under profiles/ stays within 3 % of the algorithmic bytes
    it states beside the counters (partial rows re-read, x read once per tile)."""
    import glob
    lines = [l for f in glob.glob(os.path.join(ROOT, "profiles", "*.txt")) for l in open(f)
             if l.startswith("TRAFFIC ")]
    for l in lines:
        kv = dict(t.split("=", 1) for t in l.split()[1:] if "=" in t)
        total = float(kv["fetch_bytes_per_launch"]) + float(kv["write_bytes_per_launch"])
        assert abs(total / float(kv["algorithmic_bytes_per_launch"]) - 1) < 0.03, l


def test_headline_defaults_name_the_largest_single_gpu_configuration():
    assert bench.DEFAULT_LAYERS["llama_70b"] == 80
    src = open(os.path.join(ROOT, "bench.py")).read()
    assert 'default="llama_70b"' in src
    # 80 blocks of the 70B-shaped layer: 137 GB of bf16 weights
    per_block = sum(2 * n * m for n, m in ti.LAYER_SHAPES["llama_70b"].values())
    assert round(80 * per_block / 1e9) == 137
