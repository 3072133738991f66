"""The useful-MAC and byte counts the benchmark reports, pinned without a GPU."""
import numpy as np
import pytest

import oracle
from paper_2209_03704_amd import metrics
from paper_2209_03704_amd import workloads as wl


def count_segregated_macs(N, n):
    """Count, by walking the quad sweep of Section 3.3, the taps of every stored output."""
    M = 2 * N - n
    total = 0
    for i in range((M + 1) // 2):
        for j in range((M + 1) // 2):
            for r in (0, 1):
                for s in (0, 1):
                    if 2 * i + r < M and 2 * j + s < M:
                        total += len(range(r, n, 2)) * len(range(s, n, 2))
    return total


@pytest.mark.parametrize("N,n", [(4, 3), (5, 4), (6, 5), (3, 1), (3, 2), (9, 7), (8, 5), (16, 4)])
def test_useful_macs_matches_a_walk_of_the_quad_sweep(N, n):
    layer = wl.Layer("t", 3, 5, 7, N, n, "f32", "normal")
    assert metrics.useful_macs(layer) == count_segregated_macs(N, n) * 3 * 5 * 7


def test_even_kernels_need_exactly_a_quarter_as_table4_reports():
    # Table 4, DCGAN layer 2 is 536,870,912 -> 134,217,728: the ratio 4 of an even kernel.
    for N, n in [(16, 4), (8, 2), (12, 6)]:
        layer = wl.Layer("t", 2, 3, 4, N, n, "f32", "normal")
        assert 4 * metrics.useful_macs(layer) == metrics.conventional_macs(layer)
        assert metrics.conventional_macs(layer) == oracle.conventional_ops(3, 4, N, n)[0] * 2


def test_benchmark_layer_counts():
    want = {
        "cfg1_tiny_1ch": (8_464, 33_489, 19_016),
        "cfg2_1ch_bandwidth": (415_507_456, 1_661_377_600, 332_929_380),
        "cfg3_gan_n4": (52_613_349_376, 210_453_397_504, 178_257_920),
        "cfg4_deep_n5": (26_306_674_688, 101_502_156_800, 85_065_728),
        "cfg5_late_bf16": (37_060_870_144, 147_456_000_000, 323_698_688),
    }
    for layer in wl.LAYERS:
        u, c, b = want[layer.name]
        assert metrics.useful_macs(layer) == u
        assert metrics.conventional_macs(layer) == c
        assert metrics.algorithmic_bytes(layer) == b


def test_workloads_are_seeded_and_bf16_is_rounded_once():
    layer = wl.Layer("t", 2, 3, 4, 6, 3, "bf16", "relu_normal")
    x1, w1 = wl.make_tensors(layer, 7)
    x2, w2 = wl.make_tensors(layer, 7)
    assert x1.dtype == w1.dtype and str(x1.dtype) == "torch.bfloat16"
    assert (x1 == x2).all() and (w1 == w2).all()
    assert (x1 >= 0).all()
    x64 = wl.to_f64(x1)
    assert x64.dtype == np.float64
    assert np.array_equal(x64.astype(np.float32).astype(np.float64), x64)


def test_bench_reads_traffic_from_the_committed_counter_summary():
    """bench.py's roofline.traffic comes from profiles/hbm_traffic_pmc.txt, not from constants in
    the script: the four benchmark layers with a counter measurement are found there, and each
    figure lies between the layer's algorithmic bytes and ten times that."""
    import bench
    from paper_2209_03704_amd import metrics, workloads as wl
    traffic = bench.measured_traffic()
    for name in ("cfg2_1ch_bandwidth", "cfg3_gan_n4", "cfg4_deep_n5", "cfg5_late_bf16"):
        alg = metrics.algorithmic_bytes(wl.layer_by_name(name))
        assert alg <= traffic[name] <= 10 * alg, name


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)
