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


# ---- HBM traffic tables under profiles/ -------------------------------------------------------------------

def _traffic_tables():
    import glob
    return sorted(glob.glob(os.path.join(ROOT, "profiles", "hbm_traffic_*.json")))


def test_traffic_tables_are_consistent_with_their_counters():
    """Every `traffic` figure that bench.py may print equals FETCH_SIZE / factor + WRITE_SIZE / factor (KiB -> bytes)
    of the same table, and the factors are the calibration copy's counters over its known size."""
    import json
    tables = _traffic_tables()
    assert tables, "profiles/ holds no counter summary"
    for path in tables:
        t = json.load(open(path))
        cal = t["calibration"]
        assert abs(cal["fetch_kib"] / cal["copy_kib_each_way"] - cal["fetch_factor"]) < 1e-5
        assert abs(cal["write_kib"] / cal["copy_kib_each_way"] - cal["write_factor"]) < 1e-5
        assert t["ops"], path
        for name, op in t["ops"].items():
            want = (op["fetch_kib"] / cal["fetch_factor"] + op["write_kib"] / cal["write_factor"]) * 1024
            assert abs(op["traffic"] - want) <= 1e-3 * want, (path, name)
            assert abs(op["traffic"] - (op["read_bytes"] + op["write_bytes"])) <= 2, (path, name)
            assert abs(op["traffic_over_algorithmic"] - op["traffic"] / op["alg_bytes"]) < 1e-3, (path, name)


def test_headline_traffic_table_matches_the_markdown_summary_and_the_byte_model():
    import json
    t = json.load(open(os.path.join(ROOT, "profiles", "hbm_traffic_largest_configs.json")))
    assert set(t["ops"]) == {"transform_nchw_to_chwn", "transform_chwn_to_nchw", "pool_max_nchw", "pool_max_chwn",
                             "pool_avg_nchw", "pool_avg_chwn", "softmax"}
    assert t["ops"]["transform_nchw_to_chwn"]["alg_bytes"] == rl.transform_bytes(128, 96, 55, 55)
    assert t["ops"]["pool_max_chwn"]["alg_bytes"] == rl.pool_bytes(64, 64, 224, 224, 2, 2, 2, 2)
    assert t["ops"]["softmax"]["alg_bytes"] == rl.softmax_bytes(4096, 21841)
    md = open(os.path.join(ROOT, "profiles", "bench_largest_configs_hbm_traffic.md")).read()
    rows = {}
    for line in md.splitlines():
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) == 9 and cells[0] in t["ops"]:
            rows[cells[0]] = cells
    assert set(rows) == set(t["ops"])
    for name, cells in rows.items():
        op = t["ops"][name]
        assert abs(float(cells[2]) - op["fetch_kib"]) < 0.06 and abs(float(cells[3]) - op["write_kib"]) < 0.06
        assert abs(float(cells[6]) - op["traffic"] / 1e6) < 0.006
        assert abs(float(cells[8]) - op["traffic_over_algorithmic"]) < 1e-4
    assert t["sources_digest"] in md


def test_traffic_is_only_reported_for_the_sources_it_was_measured_on(tmp_path):
    import json
    from paper_1610_03618_amd import counters
    path = os.path.join(ROOT, "profiles", "hbm_traffic_largest_configs.json")
    t = json.load(open(path))
    assert counters.load_for(path, t["sources_digest"])["ops"] == t["ops"]
    assert counters.load_for(path, "0" * 16) is None
    assert counters.load_for(str(tmp_path / "missing.json"), t["sources_digest"]) is None
    assert len(counters.sources_digest()) == 16
