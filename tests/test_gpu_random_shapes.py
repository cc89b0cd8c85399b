"""GPU parity on seeded random shapes: every entry point against the oracle on shapes nobody picked by hand.

The hand-written cases in the other files aim at known kernel boundaries; these walk the space between them
(batches that are and are not multiples of 4 / 8 / 32, odd and even planes, windows up to 5, strides up to 3,
padding up to half the window, planes below and above one LDS slab).  Same bars as everywhere else: transforms and
the maximum bit-exact, averages 1e-6 of the mean tap magnitude, softmax max(2e-6 |ref|, 1e-7); 16-bit results within
one unit in the last place of the storage format.
"""
import itertools

import numpy as np
import pytest
import torch

import oracle
import paper_1610_03618_amd as cm
from paper_1610_03618_amd import workloads as wl

pytestmark = pytest.mark.gpu

SEEDS = list(range(12))


def bits32(a):
    return np.ascontiguousarray(a).view(np.uint32)


def draw_tensor(rng, big):
    """A 4-D shape with at most ~1.5M (big: ~6M) elements; batch and plane extents of every parity."""
    N = int(rng.choice([1, 2, 3, 4, 5, 8, 12, 16, 20, 32, 33, 64, 96, 128]))
    H = int(rng.integers(1, 70 if not big else 160))
    W = int(rng.integers(1, 70 if not big else 160))
    budget = (6_000_000 if big else 1_500_000) // (N * H * W) + 1
    C = int(rng.integers(1, min(budget, 40) + 1))
    return N, C, H, W


def draw_window(rng, H, W):
    for _ in range(100):
        k = int(rng.integers(1, 6))
        s = int(rng.integers(1, 4))
        p = int(rng.integers(0, k // 2 + 1))
        if H + 2 * p >= k and W + 2 * p >= k:
            return k, s, p
    return 1, 1, 0


@pytest.mark.parametrize("seed", SEEDS)
def test_transform_and_named_orders(seed):
    rng = np.random.default_rng(1000 + seed)
    for _ in range(4):
        N, C, H, W = draw_tensor(rng, big=False)
        x = rng.integers(0, 1 << 32, size=(N, C, H, W), dtype=np.uint64).astype(np.uint32).view(np.float32)
        d = torch.from_numpy(x).cuda()
        got = cm.transform(d, N, C, H, W, cm.NCHW, cm.CHWN)
        want = oracle.transform(x, N, C, H, W, 0, 1)
        assert np.array_equal(bits32(got.cpu().numpy()), bits32(want)), (N, C, H, W)
        back = cm.transform(got, N, C, H, W, cm.CHWN, cm.NCHW)
        assert np.array_equal(bits32(back.cpu().numpy()), bits32(x)), (N, C, H, W)
        order = "".join(rng.permutation(list("NCHW")))
        got = cm.relayout(d, N, C, H, W, "NCHW", order)
        want = oracle.relayout(x, N, C, H, W, "NCHW", order)
        assert np.array_equal(bits32(got.cpu().numpy()).ravel(), bits32(want).ravel()), (N, C, H, W, order)
        back = cm.relayout(got, N, C, H, W, order, "NCHW")
        assert np.array_equal(bits32(back.cpu().numpy()).ravel(), bits32(x).ravel()), (N, C, H, W, order)


@pytest.mark.parametrize("seed", SEEDS)
def test_pool_forward_and_backward(seed):
    rng = np.random.default_rng(2000 + seed)
    for trial in range(4):
        N, C, H, W = draw_tensor(rng, big=(trial == 0))
        k, s, p = draw_window(rng, H, W)
        what = (N, C, H, W, k, s, p)
        Ho, Wo = oracle.pool_out_dims(H, W, k, k, s, s, p, p)
        x = wl.relu_normal(rng, (N, C, H, W)) + np.float32(0.0)
        dy = rng.standard_normal((N, C, Ho, Wo), dtype=np.float32)
        xc = oracle.transform(x, N, C, H, W, 0, 1)
        dyc = oracle.transform(dy, N, C, Ho, Wo, 0, 1)
        tol = 1e-6 * oracle.pool(np.abs(x), N, C, H, W, 0, 1, k, k, s, s, p, p).astype(np.float64)
        tolc = oracle.transform(tol.astype(np.float32), N, C, Ho, Wo, 0, 1).astype(np.float64) * (1 + 1e-6)
        for layout, hx, hdy, t in ((cm.NCHW, x, dy, tol), (cm.CHWN, xc, dyc, tolc)):
            dx = torch.from_numpy(hx).cuda()
            want = oracle.pool(hx, N, C, H, W, layout, 0, k, k, s, s, p, p)
            got = cm.pool(dx, N, C, H, W, layout, cm.POOL_MAX, k, k, s, s, p, p).cpu().numpy()
            assert np.array_equal(bits32(got + np.float32(0.0)), bits32(want + np.float32(0.0))), (what, layout, "max")
            want = oracle.pool(hx, N, C, H, W, layout, 1, k, k, s, s, p, p)
            got = cm.pool(dx, N, C, H, W, layout, cm.POOL_AVG, k, k, s, s, p, p).cpu().numpy()
            err = np.abs(got.astype(np.float64) - want.astype(np.float64))
            assert np.all(err <= t + 1e-45), (what, layout, "avg", float(err.max()))
            for mode in (cm.POOL_MAX, cm.POOL_AVG):
                want = oracle.pool_backward(hx, hdy, N, C, H, W, layout, mode, k, k, s, s, p, p).astype(np.float64)
                bound = 1e-6 * oracle.pool_backward(hx, np.abs(hdy), N, C, H, W, layout, mode, k, k, s, s, p, p) + 1e-30
                got = cm.pool_backward(dx if mode == cm.POOL_MAX else None, torch.from_numpy(hdy).cuda(),
                                       N, C, H, W, layout, mode, k, k, s, s, p, p).cpu().numpy().astype(np.float64)
                assert np.all(np.abs(got - want) <= bound), (what, layout, mode, float(np.abs(got - want).max()))


@pytest.mark.parametrize("seed", SEEDS[:8])
def test_pool_rectangular_windows(seed):
    """Windows up to 7 x 7 with different extents, strides and padding per axis (the run-time-window kernels: several
    output rows per lane, window rows dealt over lanes, clipped loops), fp32 and fp16, forward and backward."""
    rng = np.random.default_rng(5000 + seed)
    for trial in range(3):
        N, C, H, W = draw_tensor(rng, big=False)
        for _ in range(100):
            kh, kw = int(rng.integers(1, 8)), int(rng.integers(1, 8))
            sh, sw = int(rng.integers(1, 5)), int(rng.integers(1, 5))
            ph, pw = int(rng.integers(0, kh // 2 + 1)), int(rng.integers(0, kw // 2 + 1))
            if H + 2 * ph >= kh and W + 2 * pw >= kw and (kh, kw) != (sh, sw):
                break
        else:
            kh = kw = sh = sw = 1
            ph = pw = 0
        what = (N, C, H, W, kh, kw, sh, sw, ph, pw)
        Ho, Wo = oracle.pool_out_dims(H, W, kh, kw, sh, sw, ph, pw)
        x = wl.relu_normal(rng, (N, C, H, W)) + np.float32(0.25)
        dy = rng.standard_normal((N, C, Ho, Wo), dtype=np.float32)
        xc = oracle.transform(x, N, C, H, W, 0, 1)
        dyc = oracle.transform(dy, N, C, Ho, Wo, 0, 1)
        tol = 1e-6 * oracle.pool(np.abs(x), N, C, H, W, 0, 1, kh, kw, sh, sw, ph, pw).astype(np.float64)
        tolc = oracle.transform(tol.astype(np.float32), N, C, Ho, Wo, 0, 1).astype(np.float64) * (1 + 1e-6)
        xh = torch.from_numpy(x).cuda().half()
        xhb = xh.view(torch.int16).cpu().numpy().view(np.uint16)
        xhc = cm.transform(xh, N, C, H, W, cm.NCHW, cm.CHWN)
        xhcb = oracle.transform16(xhb, N, C, H, W, 0, 1)
        for layout, hx, hdy, t, d16, b16 in ((cm.NCHW, x, dy, tol, xh, xhb), (cm.CHWN, xc, dyc, tolc, xhc, xhcb)):
            dx = torch.from_numpy(hx).cuda()
            want = oracle.pool(hx, N, C, H, W, layout, 0, kh, kw, sh, sw, ph, pw)
            got = cm.pool(dx, N, C, H, W, layout, cm.POOL_MAX, kh, kw, sh, sw, ph, pw).cpu().numpy()
            assert np.array_equal(bits32(got), bits32(want)), (what, layout, "max")
            want = oracle.pool(hx, N, C, H, W, layout, 1, kh, kw, sh, sw, ph, pw)
            got = cm.pool(dx, N, C, H, W, layout, cm.POOL_AVG, kh, kw, sh, sw, ph, pw).cpu().numpy()
            err = np.abs(got.astype(np.float64) - want.astype(np.float64))
            assert np.all(err <= t + 1e-45), (what, layout, "avg", float(err.max()))
            want = oracle.pool16(b16, N, C, H, W, layout, 0, kh, kw, sh, sw, ph, pw, cm.F16)
            out = cm.pool(d16, N, C, H, W, layout, cm.POOL_MAX, kh, kw, sh, sw, ph, pw)
            assert np.array_equal(out.view(torch.int16).cpu().numpy().view(np.uint16), want), (what, layout, "max16")
            want = oracle.pool16(b16, N, C, H, W, layout, 1, kh, kw, sh, sw, ph, pw, cm.F16)
            out = cm.pool(d16, N, C, H, W, layout, cm.POOL_AVG, kh, kw, sh, sw, ph, pw)
            dist = ulp16(out.view(torch.int16).cpu().numpy().view(np.uint16), want)
            assert dist.max() <= 1, (what, layout, "avg16", int(dist.max()))
            for mode in (cm.POOL_MAX, cm.POOL_AVG):
                want = oracle.pool_backward(hx, hdy, N, C, H, W, layout, mode, kh, kw, sh, sw, ph, pw).astype(np.float64)
                bound = 1e-6 * oracle.pool_backward(hx, np.abs(hdy), N, C, H, W, layout, mode, kh, kw, sh, sw, ph, pw) + 1e-30
                got = cm.pool_backward(dx if mode == cm.POOL_MAX else None, torch.from_numpy(hdy).cuda(),
                                       N, C, H, W, layout, mode, kh, kw, sh, sw, ph, pw).cpu().numpy().astype(np.float64)
                assert np.all(np.abs(got - want) <= bound), (what, layout, mode, float(np.abs(got - want).max()))


@pytest.mark.parametrize("seed", SEEDS)
def test_softmax_forward_and_backward(seed):
    rng = np.random.default_rng(3000 + seed)
    for _ in range(4):
        classes = int(rng.choice([1, 2, 3, 7, 10, 33, 100, 159, 160, 257, 1000, 1001, 4097, 21841, 70001]))
        rows = int(rng.integers(1, max(2, min(600, 1_500_000 // classes))))
        z = (3.0 * rng.standard_normal((rows, classes))).astype(np.float32)
        want = oracle.softmax(z)
        got = cm.softmax(torch.from_numpy(z).cuda()).cpu().numpy()
        err = np.abs(got.astype(np.float64) - want.astype(np.float64))
        assert np.all(err <= np.maximum(2e-6 * np.abs(want.astype(np.float64)), 1e-7)), (rows, classes, float(err.max()))
        dp = rng.standard_normal((rows, classes), dtype=np.float32)
        wantb = oracle.softmax_backward(want, dp).astype(np.float64)
        gotb = cm.softmax_backward(torch.from_numpy(want).cuda(), torch.from_numpy(dp).cuda()).cpu().numpy()
        p64, dp64 = want.astype(np.float64), dp.astype(np.float64)
        bound = 2e-6 * p64 * (np.abs(dp64) + np.sum(np.abs(dp64 * p64), axis=1, keepdims=True)) + 1e-30
        assert np.all(np.abs(gotb.astype(np.float64) - wantb) <= bound), (rows, classes)


def ulp16(a, b):
    def key(u):
        u = u.astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7fff), u & 0x7fff)
    return np.abs(key(a) - key(b))


@pytest.mark.parametrize("seed", SEEDS[:8])
@pytest.mark.parametrize("dtype", [cm.F16, cm.BF16], ids=["f16", "bf16"])
def test_16bit_storage(seed, dtype):
    rng = np.random.default_rng(4000 + seed + 100 * dtype)
    tdt = torch.float16 if dtype == cm.F16 else torch.bfloat16
    for _ in range(3):
        N, C, H, W = draw_tensor(rng, big=False)
        k, s, p = draw_window(rng, H, W)
        what = (N, C, H, W, k, s, p)
        xf = wl.relu_normal(rng, (N, C, H, W)) + np.float32(0.25)
        xd = torch.from_numpy(xf).cuda().to(tdt)
        xb = xd.view(torch.int16).cpu().numpy().view(np.uint16)
        got = cm.transform(xd, N, C, H, W, cm.NCHW, cm.CHWN)
        xcb = oracle.transform16(xb, N, C, H, W, 0, 1)
        assert np.array_equal(got.view(torch.int16).cpu().numpy().view(np.uint16), xcb), what
        for layout, hb, d in ((cm.NCHW, xb, xd), (cm.CHWN, xcb, got)):
            want = oracle.pool16(hb, N, C, H, W, layout, 0, k, k, s, s, p, p, dtype)
            out = cm.pool(d, N, C, H, W, layout, cm.POOL_MAX, k, k, s, s, p, p)
            assert np.array_equal(out.view(torch.int16).cpu().numpy().view(np.uint16), want), (what, layout, "max")
            want = oracle.pool16(hb, N, C, H, W, layout, 1, k, k, s, s, p, p, dtype)
            out = cm.pool(d, N, C, H, W, layout, cm.POOL_AVG, k, k, s, s, p, p)
            dist = ulp16(out.view(torch.int16).cpu().numpy().view(np.uint16), want)
            assert dist.max() <= 1, (what, layout, "avg", int(dist.max()))
        classes = int(rng.choice([1, 5, 10, 100, 255, 256, 1000, 4099, 21841]))
        rows = int(rng.integers(1, max(2, min(300, 600_000 // classes))))
        zd = torch.from_numpy((3.0 * rng.standard_normal((rows, classes))).astype(np.float32)).cuda().to(tdt)
        zb = zd.view(torch.int16).cpu().numpy().view(np.uint16)
        want = oracle.softmax16(zb, dtype)
        out = cm.softmax(zd)
        dist = ulp16(out.view(torch.int16).cpu().numpy().view(np.uint16), want)
        assert dist.max() <= 1, (rows, classes, int(dist.max()))
