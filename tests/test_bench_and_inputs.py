"""Host-only checks of the benchmark's argument handling and of the workload table."""
import os
import subprocess
import sys

import numpy as np

import rar_inputs as ri

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_bytes_match_the_schedule():
    """Per rank: reads M + L*2M/G + M/G, writes M/G + L*M/G + M (Section 4.1 phases, Section 4.3 sizes)."""
    sys.path.insert(0, ROOT)
    import bench
    for name, want in (("c1", 3407872), ("c2", 16777216), ("c3", 159383552), ("c4", 738197504)):
        w = ri.WORKLOADS[name]
        assert bench.algorithmic_bytes(w.P, w.G, w.N, w.bytes_per_rank) == want
        L, M = w.N.bit_length() - 1, w.bytes_per_rank
        reads = M + L * 2 * M // w.G + M // w.G
        writes = M // w.G + L * M // w.G + M
        assert w.P * (reads + writes) == want


def test_moved_bytes_are_what_the_fused_kernel_touches():
    """Per rank: reads M (reduce-scatter) + L*M/G (one peer partial per step), writes L*M/G (its own
    partial for every step but the last) + M (all-gather): never more than the schedule's count."""
    sys.path.insert(0, ROOT)
    import bench
    for name, want in (("c1", 2621440), ("c2", 12582912), ("c3", 117440512), ("c4", 536870912)):
        w = ri.WORKLOADS[name]
        assert bench.moved_bytes(w.P, w.G, w.N, w.bytes_per_rank) == want
        assert want < bench.algorithmic_bytes(w.P, w.G, w.N, w.bytes_per_rank)


def test_workload_table():
    shapes = {"c1": (8, 4, 128 << 10), "c2": (16, 4, 256 << 10), "c3": (32, 4, 1 << 20), "c4": (64, 4, 2 << 20)}
    for name, (P, G, nbytes) in shapes.items():
        w = ri.WORKLOADS[name]
        assert (w.P, w.G, w.bytes_per_rank, w.dtype) == (P, G, nbytes, "bf16")
        assert w.N & (w.N - 1) == 0
    x = ri.make_inputs(ri.WORKLOADS["c1"])
    assert x.shape == (8, 65536) and x.dtype == np.uint16
    assert np.array_equal(x, ri.make_inputs(ri.WORKLOADS["c1"]))          # seeded: the same bits every time
    ints = ri.bf16_bits_to_f32(ri.make_inputs(ri.WORKLOADS["c1_int"]))
    assert np.array_equal(ints, np.round(ints)) and np.abs(ints).max() <= 8
    c2 = ri.bf16_bits_to_f32(ri.make_inputs(ri.WORKLOADS["c2"]))
    outliers = np.abs(c2) == 20.0
    assert 0.0003 < outliers.mean() < 0.003                                 # 0.1 % outliers at +-20
    f = ri.make_inputs(ri.sweep_workload(8, 4, 8 << 10, "f32"))
    assert f.shape == (8, 2048) and f.dtype == np.float32
