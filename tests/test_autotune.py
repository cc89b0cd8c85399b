"""Pooling auto-tuner: the hill-climbing rule of Section V.A on synthetic cost
curves (CPU), and the real search on a small layer (GPU)."""
import numpy as np
import pytest

from paper_1610_03618_amd import autotune


def test_hill_climb_follows_the_papers_rule():
    # start at 2, keep growing while faster, stop at the first step that is not
    cost = {1: 10.0, 2: 8.0, 3: 7.0, 4: 7.5}
    best, seen = autotune.hill_climb(cost.__getitem__, 1, 4)
    assert best == 3 and set(seen) == {1, 2, 3, 4}
    cost = {1: 10.0, 2: 11.0, 3: 1.0, 4: 0.5}            # worse at 2: stop there, never look further
    best, seen = autotune.hill_climb(cost.__getitem__, 1, 4)
    assert best == 1 and set(seen) == {1, 2}
    cost = {1: 10.0, 2: 9.0, 3: 8.0, 4: 7.0}             # improves all the way: capped by hi
    best, seen = autotune.hill_climb(cost.__getitem__, 1, 4)
    assert best == 4 and set(seen) == {1, 2, 3, 4}
    best, seen = autotune.hill_climb({1: 3.0, 2: 2.0}.__getitem__, 1, 2)
    assert best == 2
    calls = []
    autotune.hill_climb(lambda f: calls.append(f) or 1.0, 1, 4)      # equal time is not an improvement
    assert calls == [1, 2]


@pytest.mark.gpu
@pytest.mark.parametrize("layout", [0, 1])
def test_tune_pool_returns_a_valid_tuning_that_changes_no_result(layout):
    import torch

    import oracle
    import paper_1610_03618_amd as cm
    N, C, H, W, k, s = 16, 8, 27, 27, 3, 2
    best, hist = autotune.tune_pool(N, C, H, W, layout, cm.POOL_MAX, k, s, iters=4)
    assert len(hist) >= 4 and all(h["ms"] > 0 for h in hist)
    assert set(best) <= {"rows_per_lane", "cols_per_lane", "workgroups_per_cu", "nchw_kernel", "slab_lanes"}
    x = np.random.default_rng(4).standard_normal((N, C, H, W), dtype=np.float32)
    src = x if layout == 0 else oracle.transform(x, N, C, H, W, 0, 1)
    want = oracle.pool(src, N, C, H, W, layout, 0, k, k, s, s)
    got = cm.pool(torch.from_numpy(src).cuda(), N, C, H, W, layout, cm.POOL_MAX, k, k, s, s, tuning=best)
    np.testing.assert_array_equal(got.cpu().numpy(), want)


def test_tuning_table_round_trip(tmp_path):
    """The shape -> tuning table the tool writes can be read back and looked up by shape."""
    import json
    from paper_1610_03618_amd import autotune
    written = {
        "PL5 ...": dict(shape=dict(N=128, C=96, H=55, W=55, k=3, s=2, p=0, layout=1, mode=0),
                        tuning=dict(rows_per_lane=3, cols_per_lane=1, workgroups_per_cu=3), gbps=5190.0),
        "PL1 ...": dict(shape=dict(N=128, C=16, H=28, W=28, k=2, s=2, p=0, layout=0, mode=0),
                        tuning=dict(nchw_kernel=2, slab_lanes=1024, workgroups_per_cu=6), gbps=622.0),
    }
    path = tmp_path / "table.json"
    path.write_text(json.dumps(written))
    table = autotune.load_table(str(path))
    assert autotune.lookup(table, 128, 96, 55, 55, 3, 2, 0, 1, 0) == dict(rows_per_lane=3, cols_per_lane=1,
                                                                            workgroups_per_cu=3)
    assert autotune.lookup(table, 128, 16, 28, 28, 2, 2, 0, 0, 0)["slab_lanes"] == 1024
    assert autotune.lookup(table, 64, 16, 28, 28, 2, 2, 0, 0, 0) is None
