"""The five benchmark configurations at full size, HIP path against the oracle,
every element, in the launch configuration the benchmark times (default
dispatch, torch's current stream)."""
import numpy as np
import pytest
import torch

import oracle
import paper_1610_03618_amd as cm
from paper_1610_03618_amd import workloads as wl

pytestmark = pytest.mark.gpu

NCHW, CHWN, MAX, AVG = cm.NCHW, cm.CHWN, cm.POOL_MAX, cm.POOL_AVG


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def same_bits(a, b):
    return a.shape == b.shape and np.array_equal(a.view(np.uint32), b.view(np.uint32))


def softmax_ok(got, want):
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    tol = np.maximum(2e-6 * np.abs(want.astype(np.float64)), 1e-7)
    return bool(np.all(err <= tol)), float((err / tol).max())


def run_transform_round_trip(x, t):
    want = oracle.transform(x, t.N, t.C, t.H, t.W, NCHW, CHWN)
    d_x = dev(x)
    d_c = cm.transform(d_x, t.N, t.C, t.H, t.W, NCHW, CHWN)
    assert same_bits(host(d_c), want)
    d_back = cm.transform(d_c, t.N, t.C, t.H, t.W, CHWN, NCHW)
    assert same_bits(host(d_back), x)
    return want


def run_pool_both_layouts(x, xc, t, spec):
    k, s, p = spec.k, spec.s, spec.p
    for layout, src in ((NCHW, x), (CHWN, xc)):
        want = oracle.pool(src, t.N, t.C, t.H, t.W, layout, spec.mode, k, k, s, s, p, p)
        got = host(cm.pool(dev(src), t.N, t.C, t.H, t.W, layout, spec.mode, k, k, s, s, p, p))
        if spec.mode == MAX:
            assert same_bits(got, want), (t.name, layout)       # inputs are >= +0 or canonical
        else:
            # inputs are non-negative: 1e-6 relative to the result itself
            err = np.abs(got.astype(np.float64) - want.astype(np.float64))
            assert np.all(err <= 1e-6 * np.abs(want.astype(np.float64))), (t.name, layout, float(err.max()))
    return want


def test_config1_maxpool_both_layouts():
    cfg = wl.config(1)
    t = cfg.transforms[0]
    x = wl.make_tensor(t, wl.rng_for(1))
    xc = run_transform_round_trip(x, t)
    spec = cfg.pools[0]
    run_pool_both_layouts(x, xc, t, spec)
    # "also emitted and checked in CHWN": pooling the CHWN copy equals the CHWN copy of the NCHW result
    Ho, Wo = oracle.pool_out_dims(t.H, t.W, 3, 3, 2, 2, 0, 0)
    assert (Ho, Wo) == (15, 15)
    p_n = cm.pool(dev(x), t.N, t.C, t.H, t.W, NCHW, MAX, 3, 3, 2, 2)
    p_c = cm.pool(dev(xc), t.N, t.C, t.H, t.W, CHWN, MAX, 3, 3, 2, 2)
    assert same_bits(host(cm.transform(p_n, t.N, t.C, Ho, Wo, NCHW, CHWN)), host(p_c))


def test_config2_transform_round_trip_and_softmax():
    cfg = wl.config(2)
    rng = wl.rng_for(2)
    t = cfg.transforms[0]
    x = wl.make_tensor(t, rng)
    run_transform_round_trip(x, t)
    z = wl.make_logits(cfg.softmaxes[0], rng)
    ok, worst = softmax_ok(host(cm.softmax(dev(z))), oracle.softmax(z))
    assert ok, worst


@pytest.mark.parametrize("which", [0, 1, 2])
def test_config3_alexnet_pooling_stack(which):
    cfg = wl.config(3)
    spec = cfg.pools[which]
    t = spec.tensor
    x = wl.make_tensor(t, wl.rng_for(3, which))
    xc = run_transform_round_trip(x, t)
    pooled = run_pool_both_layouts(x, xc, t, spec)
    # transforms on the pooled tensor's shape as well (CHWN result -> NCHW result)
    Ho, Wo = oracle.pool_out_dims(t.H, t.W, spec.k, spec.k, spec.s, spec.s, 0, 0)
    d_pc = dev(pooled)                                          # `pooled` is the CHWN-layout oracle result
    back = cm.transform(d_pc, t.N, t.C, Ho, Wo, CHWN, NCHW)
    assert same_bits(host(back), oracle.transform(pooled, t.N, t.C, Ho, Wo, CHWN, NCHW))


@pytest.mark.parametrize("which", [0, 1, 2, 3, 4])
def test_config4_vgg_pooling(which):
    cfg = wl.config(4)
    specs = [p for p in cfg.pools if p.tensor.name == f"x{which + 1}"]
    t = specs[0].tensor
    x = wl.make_tensor(t, wl.rng_for(4, which))
    xc = oracle.transform(x, t.N, t.C, t.H, t.W, NCHW, CHWN)
    for spec in specs:
        run_pool_both_layouts(x, xc, t, spec)


def test_config5_large_softmax_and_transform():
    cfg = wl.config(5)
    s = cfg.softmaxes[0]
    z = wl.make_logits(s, wl.rng_for(5, 0))
    assert float(z.max()) >= 50.0
    want = oracle.softmax(z)
    got = host(cm.softmax(dev(z)))
    ok, worst = softmax_ok(got, want)
    assert ok, worst
    sums = got.astype(np.float64).sum(axis=1)
    assert np.all(np.abs(sums - 1.0) <= 1e-5)
    # the largest probability sits on a column that holds the row's maximum logit
    assert np.all(z[np.arange(s.N), got.argmax(axis=1)] == z.max(axis=1))
    t = cfg.transforms[0]
    x = wl.make_tensor(t, wl.rng_for(5, 1))
    run_transform_round_trip(x, t)
