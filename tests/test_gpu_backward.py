"""Backward passes of pooling and softmax on the GPU against the oracle.

Tolerances: a pooling gradient is a sum of at most ceil(k/s)^2 fp32 terms (fp64 in the
oracle): |error| <= 1e-6 * (sum of |terms|), the bound the forward average uses; where a
single window contributes (2x2 / stride 2) the maximum's gradient is bit-exact.  The
softmax gradient carries the error of an fp32 dot product over the row:
|error| <= 2e-6 * |p| * (|dp| + sum_k |dp_k p_k|)."""
import numpy as np
import pytest
import torch

import oracle
import paper_1610_03618_amd as cm
from paper_1610_03618_amd import workloads as wl

pytestmark = pytest.mark.gpu

CASES = [  # N, C, H, W, k, s, p
    (16, 8, 32, 32, 3, 2, 0), (8, 4, 55, 55, 3, 2, 0), (8, 3, 27, 27, 3, 2, 0), (16, 6, 28, 28, 2, 2, 0),
    (8, 5, 14, 14, 2, 2, 0), (8, 3, 13, 13, 3, 1, 1), (8, 2, 17, 19, 3, 2, 1), (6, 3, 15, 15, 3, 2, 0),
    (4, 3, 30, 24, 2, 2, 0), (8, 2, 9, 9, 5, 3, 2), (3, 2, 7, 5, 2, 1, 0), (4, 2, 20, 20, 9, 4, 3),
    (4, 2, 12, 12, 4, 4, 0), (8, 2, 11, 11, 2, 3, 0),
    # planes larger than the LDS budget: strips of input rows (cells and single elements), with and without padding
    (4, 3, 150, 150, 3, 2, 0), (4, 2, 224, 224, 3, 2, 1), (4, 2, 300, 40, 5, 3, 2), (4, 2, 111, 113, 3, 2, 0),
    (4, 1, 130, 130, 2, 2, 0), (8, 2, 97, 200, 3, 1, 1),
    # batches that are multiples of 32: the CHWN patch kernel (ragged patches, one-cell images, several chunks)
    (32, 3, 27, 27, 3, 2, 0), (64, 2, 55, 55, 3, 2, 0), (32, 2, 13, 13, 3, 2, 0), (32, 1, 5, 5, 3, 2, 0),
    (32, 2, 64, 70, 3, 2, 0), (96, 1, 3, 3, 3, 2, 0), (32, 1, 9, 40, 3, 2, 0),
    # thousands of small planes: several planes per workgroup in NCHW, several rows per wavefront
    (64, 128, 13, 13, 3, 2, 0), (128, 96, 7, 7, 3, 2, 0), (64, 96, 8, 6, 3, 2, 0),
]


def check_pool_backward(x, dy, N, C, H, W, k, s, p, mode, what):
    Ho, Wo = oracle.pool_out_dims(H, W, k, k, s, s, p, p)
    xc = oracle.transform(x, N, C, H, W, 0, 1)
    dyc = oracle.transform(dy, N, C, Ho, Wo, 0, 1)
    for layout, hx, hdy in ((cm.NCHW, x, dy), (cm.CHWN, xc, dyc)):
        want = oracle.pool_backward(hx, hdy, N, C, H, W, layout, mode, k, k, s, s, p, p).astype(np.float64)
        bound = 1e-6 * oracle.pool_backward(hx, np.abs(hdy), N, C, H, W, layout, mode, k, k, s, s, p, p) + 1e-30
        src = torch.from_numpy(hx).cuda() if mode == cm.POOL_MAX else None
        got = cm.pool_backward(src, torch.from_numpy(hdy).cuda(), N, C, H, W, layout, mode, k, k, s, s, p, p)
        got = got.cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got - want) <= bound), (what, layout, float(np.abs(got - want).max()))
        if mode == cm.POOL_MAX and k <= s:            # disjoint windows: one term, no rounding at all
            assert np.array_equal(got, want), (what, layout)


@pytest.mark.parametrize("mode", [cm.POOL_MAX, cm.POOL_AVG], ids=["max", "avg"])
@pytest.mark.parametrize("case", CASES, ids=["-".join(map(str, c)) for c in CASES])
def test_pool_backward_matches_oracle(case, mode):
    N, C, H, W, k, s, p = case
    rng = np.random.default_rng(sum(case) + mode)
    x = wl.relu_normal(rng, (N, C, H, W))                 # the zeros of a ReLU layer give plenty of ties
    Ho, Wo = oracle.pool_out_dims(H, W, k, k, s, s, p, p)
    dy = rng.standard_normal((N, C, Ho, Wo), dtype=np.float32)
    check_pool_backward(x, dy, N, C, H, W, k, s, p, mode, case)


def test_pool_backward_generic_paths_for_odd_batches_and_misaligned_views():
    N, C, H, W, k, s = 6, 3, 12, 12, 3, 2                  # N % 4 != 0: CHWN takes the generic kernel
    rng = np.random.default_rng(8)
    x = wl.relu_normal(rng, (N, C, H, W))
    dy = rng.standard_normal((N, C, 5, 5), dtype=np.float32)
    check_pool_backward(x, dy, N, C, H, W, k, s, 0, cm.POOL_MAX, "odd batch")
    # misaligned NCHW 2x2 / stride 2
    N, C, H, W = 4, 2, 8, 8
    x = wl.relu_normal(rng, (N, C, H, W))
    dy = rng.standard_normal((N, C, 4, 4), dtype=np.float32)
    n = x.size
    xb = torch.zeros(n + 4, device="cuda")
    xb[1:1 + n] = torch.from_numpy(x).cuda().reshape(-1)
    out = torch.full((n + 4,), -9.0, device="cuda")
    st = cm.cnnmem_pool_backward(xb[1:], torch.from_numpy(dy).cuda(), out[1:], N, C, H, W, cm.NCHW, cm.POOL_MAX,
                                 2, 2, 2, 2, 0, 0)
    assert st == 0
    got = out.cpu().numpy()
    want = oracle.pool_backward(x, dy, N, C, H, W, 0, 0, 2, 2, 2, 2).ravel()
    assert np.array_equal(got[1:1 + n], want) and got[0] == -9.0 and np.all(got[1 + n:] == -9.0)


def test_config4_and_config3_pool_backward_reduced_batch():
    rng = np.random.default_rng(44)
    for (N, C, H, W, k, s) in [(8, 64, 224, 224, 2, 2), (16, 96, 55, 55, 3, 2)]:
        x = wl.relu_normal(rng, (N, C, H, W))
        Ho, Wo = oracle.pool_out_dims(H, W, k, k, s, s, 0, 0)
        dy = rng.standard_normal((N, C, Ho, Wo), dtype=np.float32)
        for mode in (cm.POOL_MAX, cm.POOL_AVG):
            check_pool_backward(x, dy, N, C, H, W, k, s, 0, mode, (N, C, H, W, mode))


S_SHAPES = [(7, 1), (5, 7), (33, 10), (40, 100), (128, 1000), (64, 1001), (9, 4096), (6, 21841), (3, 70001), (300, 257)]


@pytest.mark.parametrize("shape", S_SHAPES, ids=[f"{n}x{c}" for n, c in S_SHAPES])
def test_softmax_backward_matches_oracle(shape):
    n, c = shape
    rng = np.random.default_rng(n * 17 + c)
    p = oracle.softmax(wl.normal_logits(rng, n, c, 3.0))
    dp = rng.standard_normal((n, c), dtype=np.float32)
    want = oracle.softmax_backward(p, dp).astype(np.float64)
    got = cm.softmax_backward(torch.from_numpy(p).cuda(), torch.from_numpy(dp).cuda()).cpu().numpy().astype(np.float64)
    pd = p.astype(np.float64)
    bound = 2e-6 * pd * (np.abs(dp) + np.abs(dp * pd).sum(axis=1, keepdims=True)) + 1e-30
    assert np.all(np.abs(got - want) <= bound), float(np.abs(got - want).max())


def test_softmax_backward_misaligned_mixed_phase_and_in_place():
    n, c = 19, 777
    rng = np.random.default_rng(2)
    p = oracle.softmax(wl.normal_logits(rng, n, c, 3.0))
    dp = rng.standard_normal((n, c), dtype=np.float32)
    want = oracle.softmax_backward(p, dp).astype(np.float64)
    pd = p.astype(np.float64)
    bound = 2e-6 * pd * (np.abs(dp) + np.abs(dp * pd).sum(axis=1, keepdims=True)) + 1e-30
    for a, b, z in [(1, 1, 1), (0, 1, 2), (3, 3, 0), (4, 4, 4)]:
        pb = torch.zeros(n * c + 8, device="cuda")
        db = torch.zeros(n * c + 8, device="cuda")
        zb = torch.zeros(n * c + 8, device="cuda")
        pb[a:a + n * c] = torch.from_numpy(p).cuda().reshape(-1)
        db[b:b + n * c] = torch.from_numpy(dp).cuda().reshape(-1)
        assert cm.cnnmem_softmax_backward(pb[a:], db[b:], zb[z:], n, c) == 0
        got = zb.cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got[z:z + n * c].reshape(n, c) - want) <= bound), (a, b, z)
        assert not got[:z].any() and not got[z + n * c:].any()
    d = torch.from_numpy(dp).cuda()
    assert cm.cnnmem_softmax_backward(torch.from_numpy(p).cuda(), d, d, n, c) == 0        # in place over dprobs
    assert np.all(np.abs(d.cpu().numpy().astype(np.float64) - want) <= bound)


def test_config5_softmax_backward_full_size():
    s = wl.config(5).softmaxes[0]
    z = wl.make_logits(s, wl.rng_for(5, 0))
    p = oracle.softmax(z)
    dp = np.random.default_rng(55).standard_normal(p.shape, dtype=np.float32)
    want = oracle.softmax_backward(p, dp).astype(np.float64)
    got = cm.softmax_backward(torch.from_numpy(p).cuda(), torch.from_numpy(dp).cuda()).cpu().numpy().astype(np.float64)
    pd = p.astype(np.float64)
    bound = 2e-6 * pd * (np.abs(dp) + np.abs(dp * pd).sum(axis=1, keepdims=True)) + 1e-30
    assert np.all(np.abs(got - want) <= bound)
