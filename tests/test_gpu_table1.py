"""Every pooling and classifier layer of Table 1 at its full size, both layouts,
HIP path against the oracle (the second workload next to the five benchmark
configurations; extents follow the floor rule, so PL3 / PL4 / PL9 give 11 / 5 /
12 outputs per side)."""
import numpy as np
import pytest
import torch

import oracle
import paper_1610_03618_amd as cm
from paper_1610_03618_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("row", wl.TABLE1_POOLS, ids=[r[0] for r in wl.TABLE1_POOLS])
def test_table1_pooling_layer_full_size(row):
    name, N, hw, k, C, s = row
    rng = np.random.default_rng(sum(map(ord, name)))
    x = wl.relu_normal(rng, (N, C, hw, hw))
    xc = oracle.transform(x, N, C, hw, hw, 0, 1)
    Ho, Wo = oracle.pool_out_dims(hw, hw, k, k, s, s, 0, 0)
    for layout, src in ((cm.NCHW, x), (cm.CHWN, xc)):
        d = torch.from_numpy(src).cuda()
        want = oracle.pool(src, N, C, hw, hw, layout, 0, k, k, s, s)
        got = cm.pool(d, N, C, hw, hw, layout, cm.POOL_MAX, k, k, s, s).cpu().numpy()
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), (name, layout)
        want = oracle.pool(src, N, C, hw, hw, layout, 1, k, k, s, s).astype(np.float64)
        got = cm.pool(d, N, C, hw, hw, layout, cm.POOL_AVG, k, k, s, s).cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got - want) <= 1e-6 * np.abs(want)), (name, layout)
    # and the transform on the pooled shape, both ways
    p = oracle.pool(x, N, C, hw, hw, 0, 0, k, k, s, s)
    pc = cm.transform(torch.from_numpy(p).cuda(), N, C, Ho, Wo, cm.NCHW, cm.CHWN)
    assert np.array_equal(pc.cpu().numpy().view(np.uint32), oracle.transform(p, N, C, Ho, Wo, 0, 1).view(np.uint32))
    back = cm.transform(pc, N, C, Ho, Wo, cm.CHWN, cm.NCHW)
    assert np.array_equal(back.cpu().numpy().view(np.uint32), p.view(np.uint32))


@pytest.mark.parametrize("row", wl.TABLE1_CLASSIFIERS, ids=[r[0] for r in wl.TABLE1_CLASSIFIERS])
def test_table1_classifier_full_size(row):
    name, n, c = row
    rng = np.random.default_rng(n * 7 + c)
    z = wl.plant_outliers(wl.normal_logits(rng, n, c, 3.0), rng) if c > 10 else wl.normal_logits(rng, n, c, 3.0)
    want = oracle.softmax(z).astype(np.float64)
    got = cm.softmax(torch.from_numpy(z).cuda()).cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - want) <= np.maximum(2e-6 * want, 1e-7)), name
    assert np.all(np.abs(got.sum(axis=1) - 1.0) <= 1e-6)


@pytest.mark.parametrize("shape", wl.SOFTMAX_SWEEP, ids=[f"{n}x{c}" for n, c in wl.SOFTMAX_SWEEP])
def test_softmax_sweep_batch_by_categories(shape):
    """The batch x categories range of Fig. 13 (10 to 10000 categories)."""
    n, c = shape
    rng = np.random.default_rng(n * 13 + c)
    z = wl.normal_logits(rng, n, c, 3.0)
    want = oracle.softmax(z).astype(np.float64)
    got = cm.softmax(torch.from_numpy(z).cuda()).cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - want) <= np.maximum(2e-6 * want, 1e-7)), shape
    assert np.all(np.abs(got.sum(axis=1) - 1.0) <= 1e-5)
    rows = np.arange(n)
    assert np.array_equal(got[rows, z.argmax(axis=1)], got.max(axis=1))   # the largest logit keeps the largest probability
