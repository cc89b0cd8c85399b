"""CPU checks of the measurement side: the byte model behind every GB/s figure and the benchmark's refusals.

The byte model is pinned to the survey's per-configuration figures (every needed input element read once, every
output written once, 4 bytes each); the benchmark must refuse more than one GPU and must not fall back to the CPU.
"""
import os
import subprocess
import sys

import pytest

from paper_1610_03618_amd import roofline as rl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_transform_bytes_of_config_2():
    # 128 x 96 x 55 x 55 floats: 148.68 MB each side
    assert rl.transform_bytes(128, 96, 55, 55) == 2 * 148_684_800


def test_pool_bytes_of_config_4_first_tensor():
    # 64 x 64 x 224 x 224 in (822.08 MB), 64 x 64 x 112 x 112 out (205.52 MB)
    assert rl.pool_bytes(64, 64, 224, 224, 2, 2, 2, 2) == 822_083_584 + 205_520_896


def test_pool_bytes_count_only_the_rows_and_columns_some_window_covers():
    # 3x3 / stride 2 on 56 x 56: Ho = 27, the windows cover rows and columns 0..54 only
    assert rl.pooled_extent(56, 3, 2, 0) == 27
    assert rl.pool_bytes(1, 1, 56, 56, 3, 3, 2, 2) == 4 * (55 * 55 + 27 * 27)
    # with padding 1 the last window reaches row 55: the whole plane is needed
    assert rl.pooled_extent(56, 3, 2, 1) == 28
    assert rl.pool_bytes(1, 1, 56, 56, 3, 3, 2, 2, 1, 1) == 4 * (56 * 56 + 28 * 28)


def test_softmax_bytes_of_config_5():
    # 4096 x 21841 floats: 357.84 MB each way
    assert rl.softmax_bytes(4096, 21841) == 2 * 357_842_944


def test_backward_bytes():
    # average: gradient in, gradient out; maximum: the forward input as well
    assert rl.pool_backward_bytes(64, 64, 224, 224, 2, 2, 2, 2, needs_input=False) == 822_083_584 + 205_520_896
    assert rl.pool_backward_bytes(64, 64, 224, 224, 2, 2, 2, 2) == 2 * 822_083_584 + 205_520_896
    assert rl.softmax_backward_bytes(4096, 21841) == 3 * 357_842_944


def test_peak_is_the_published_hbm_figure():
    assert rl.PEAK_HBM_GBPS == 8000.0


def run_bench(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          cwd=ROOT, timeout=300)


def test_bench_refuses_more_than_one_gpu():
    r = run_bench("--gpus", "2")
    assert r.returncode == 2
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""


def test_bench_has_no_cpu_fallback():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    r = run_bench("--steps", "1", "--warmup", "0")
    assert r.returncode == 2
    assert "no CPU fallback" in r.stderr
    assert r.stdout.strip() == ""
