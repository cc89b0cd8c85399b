"""Tensors with more than 2^31 elements (64-bit offsets inside the kernels).
Inputs are generated on the device; outputs are checked on sampled elements
that the oracle computes one by one (index arithmetic, small windows, rows)."""
import numpy as np
import pytest
import torch

import oracle
import paper_1610_03618_amd as cm

pytestmark = pytest.mark.gpu
NCHW, CHWN, MAX, AVG = cm.NCHW, cm.CHWN, cm.POOL_MAX, cm.POOL_AVG


def _free_gib():
    free, _ = torch.cuda.mem_get_info()
    return free / 2**30


def test_transform_beyond_2g_elements_sampled():
    if _free_gib() < 24:
        pytest.skip("needs ~20 GiB of free device memory")
    N, C, H, W = 128, 1000, 100, 170                        # 2 176 000 000 elements, 8.7 GB
    total = N * C * H * W
    assert total > 2**31
    # word i holds i mod 2^31 as an int32 bit pattern, moved as fp32
    src = (torch.arange(total, dtype=torch.int64, device="cuda") & 0x7FFFFFFF).to(torch.int32).view(torch.float32)
    dst = torch.empty(total, dtype=torch.float32, device="cuda")
    assert cm.cnnmem_transform(src, dst, N, C, H, W, NCHW, CHWN) == 0
    rng = np.random.default_rng(7)
    pts = np.stack([rng.integers(0, d, size=4000) for d in (N, C, H, W)], axis=1)
    pts[:8] = [[0, 0, 0, 0], [N - 1, C - 1, H - 1, W - 1], [N - 1, 0, 0, 0], [0, C - 1, H - 1, W - 1],
               [127, 999, 99, 168], [64, 500, 50, 85], [1, 999, 99, 169], [126, 0, 0, 1]]
    si = torch.tensor([oracle.index(NCHW, N, C, H, W, *map(int, p)) for p in pts], device="cuda")
    di = torch.tensor([oracle.index(CHWN, N, C, H, W, *map(int, p)) for p in pts], device="cuda")
    assert int(di.max()) > 2**31
    got = dst.view(torch.int32)[di].cpu().numpy()
    want = (si & 0x7FFFFFFF).to(torch.int32).cpu().numpy()
    np.testing.assert_array_equal(got, want)
    # and back: the round trip is the identity on a strided sample of words
    back = torch.empty(total, dtype=torch.float32, device="cuda")
    assert cm.cnnmem_transform(dst, back, N, C, H, W, CHWN, NCHW) == 0
    probe = torch.arange(0, total, 1000003, device="cuda")
    assert torch.equal(back.view(torch.int32)[probe], src.view(torch.int32)[probe])
    assert torch.equal(back.view(torch.int32)[-4096:], src.view(torch.int32)[-4096:])


@pytest.mark.parametrize("layout", [NCHW, CHWN])
def test_pool_beyond_2g_elements_sampled(layout):
    if _free_gib() < 16:
        pytest.skip("needs ~12 GiB of free device memory")
    N, C, H, W = 64, 64, 736, 736                           # 2 218 786 816 elements
    k, s = (2, 2) if layout == NCHW else (3, 2)
    assert N * C * H * W > 2**31
    g = torch.Generator(device="cuda").manual_seed(11)
    x = torch.empty(N * C * H * W, dtype=torch.float32, device="cuda")
    x.uniform_(0.0, 1.0, generator=g)
    Ho, Wo = oracle.pool_out_dims(H, W, k, k, s, s, 0, 0)
    rng = np.random.default_rng(8)
    pts = np.stack([rng.integers(0, d, size=600) for d in (N, C, Ho, Wo)], axis=1)
    pts[:4] = [[0, 0, 0, 0], [N - 1, C - 1, Ho - 1, Wo - 1], [N - 1, C - 1, 0, Wo - 1], [0, C - 1, Ho - 1, 0]]
    for mode in (MAX, AVG):
        out = torch.empty(N * C * Ho * Wo, dtype=torch.float32, device="cuda")
        assert cm.cnnmem_pool(x, out, N, C, H, W, layout, mode, k, k, s, s, 0, 0) == 0
        # gather each sampled window and its output, then let the oracle pool the k x k patch
        idx = np.array([[oracle.index(layout, N, C, H, W, int(n), int(c), int(i) * s + y, int(j) * s + xx)
                         for y in range(k) for xx in range(k)] for (n, c, i, j) in pts], dtype=np.int64)
        oidx = np.array([oracle.index(layout, N, C, Ho, Wo, *map(int, p)) for p in pts], dtype=np.int64)
        patches = x[torch.from_numpy(idx).cuda()].cpu().numpy().reshape(-1, 1, k, k)    # (samples, 1, k, k)
        got = out[torch.from_numpy(oidx).cuda()].cpu().numpy()
        want = oracle.pool(np.ascontiguousarray(patches), patches.shape[0], 1, k, k, NCHW, mode, k, k, s, s).ravel()
        if mode == MAX:
            np.testing.assert_array_equal(got, want)
        else:
            assert np.all(np.abs(got.astype(np.float64) - want) <= 1e-6 * np.abs(want))
        del out


def test_softmax_beyond_2g_elements_sampled_rows():
    if _free_gib() < 22:
        pytest.skip("needs ~18 GiB of free device memory")
    N, classes = 70001, 32771                               # 2 294 002 771 elements, odd row length
    assert N * classes > 2**31
    g = torch.Generator(device="cuda").manual_seed(12)
    z = torch.empty((N, classes), dtype=torch.float32, device="cuda")
    z.normal_(0.0, 3.0, generator=g)
    z[N - 1, 17] = 50.0
    p = torch.empty_like(z)
    assert cm.cnnmem_softmax(z, p, N, classes) == 0
    rows = [0, 1, 7, 65535, 65536, 65537, N // 2, N - 2, N - 1]
    want = oracle.softmax(np.ascontiguousarray(z[rows].cpu().numpy())).astype(np.float64)
    got = p[rows].cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - want) <= np.maximum(2e-6 * want, 1e-7))
    sums = p.sum(dim=1, dtype=torch.float64)
    assert float((sums - 1.0).abs().max()) <= 1e-5


def _letter_index(layout: str, ext: dict, coord: dict) -> int:
    """Linear index of a coordinate in a spelled layout (slowest axis first): plain positional arithmetic."""
    idx = 0
    for letter in layout:
        idx = idx * ext[letter] + coord[letter]
    return idx


@pytest.mark.parametrize("dst_layout", ["NHWC", "HWCN", "CNHW"])
def test_relayout_beyond_2g_elements_sampled(dst_layout):
    """Strided tile kernel (NHWC, HWCN) and row-move kernel (CNHW, several launches) with 64-bit offsets."""
    if _free_gib() < 24:
        pytest.skip("needs ~20 GiB of free device memory")
    N, C, H, W = 96, 340, 257, 257                           # 2 155 839 360 elements
    total = N * C * H * W
    assert total > 2**31
    src = (torch.arange(total, dtype=torch.int64, device="cuda") & 0x7FFFFFFF).to(torch.int32).view(torch.float32)
    dst = torch.zeros(total, dtype=torch.float32, device="cuda")
    st = cm.cnnmem_relayout(src, dst, N, C, H, W, "NCHW", dst_layout)
    assert st == 0
    ext = dict(N=N, C=C, H=H, W=W)
    rng = np.random.default_rng(9)
    pts = np.stack([rng.integers(0, d, size=4000) for d in (N, C, H, W)], axis=1)
    pts[:4] = [[0, 0, 0, 0], [N - 1, C - 1, H - 1, W - 1], [N - 1, 0, H - 1, 0], [0, C - 1, 0, W - 1]]
    si = np.array([_letter_index("NCHW", ext, dict(zip("NCHW", map(int, p)))) for p in pts], dtype=np.int64)
    di = np.array([_letter_index(dst_layout, ext, dict(zip("NCHW", map(int, p)))) for p in pts], dtype=np.int64)
    assert di.max() > 2**31
    got = dst.view(torch.int32)[torch.from_numpy(di).cuda()].cpu().numpy()
    np.testing.assert_array_equal(got, (si & 0x7FFFFFFF).astype(np.int32))
    back = torch.empty(total, dtype=torch.float32, device="cuda")
    assert cm.cnnmem_relayout(dst, back, N, C, H, W, dst_layout, "NCHW") == 0
    probe = torch.arange(0, total, 1000003, device="cuda")
    assert torch.equal(back.view(torch.int32)[probe], src.view(torch.int32)[probe])
    assert torch.equal(back.view(torch.int32)[-4096:], src.view(torch.int32)[-4096:])


def test_transform16_beyond_2g_elements_sampled():
    if _free_gib() < 14:
        pytest.skip("needs ~10 GiB of free device memory")
    N, C, H, W = 128, 1000, 100, 170                        # 2 176 000 000 16-bit words
    total = N * C * H * W
    src = (torch.arange(total, dtype=torch.int64, device="cuda") % 65521).to(torch.int16)
    dst = torch.empty(total, dtype=torch.int16, device="cuda")
    st = cm.library().cnnmem_transform_dtype(src.data_ptr(), dst.data_ptr(), N, C, H, W, NCHW, CHWN, cm.F16,
                                             torch.cuda.current_stream().cuda_stream or None)
    assert st == 0
    rng = np.random.default_rng(10)
    pts = np.stack([rng.integers(0, d, size=4000) for d in (N, C, H, W)], axis=1)
    pts[:4] = [[0, 0, 0, 0], [N - 1, C - 1, H - 1, W - 1], [N - 1, 0, 0, 0], [0, C - 1, H - 1, W - 1]]
    si = np.array([oracle.index(NCHW, N, C, H, W, *map(int, p)) for p in pts], dtype=np.int64)
    di = torch.tensor([oracle.index(CHWN, N, C, H, W, *map(int, p)) for p in pts], device="cuda")
    assert int(di.max()) > 2**31
    got = dst[di].cpu().numpy().astype(np.int64) & 0xFFFF
    np.testing.assert_array_equal(got, si % 65521)


@pytest.mark.parametrize("layout,k", [(NCHW, 2), (CHWN, 2), (NCHW, 3), (CHWN, 3)])
def test_pool_backward_beyond_2g_elements_sampled(layout, k):
    """Every backward kernel family (row pairs, cells, LDS slab, LDS patches) with 64-bit offsets: sampled input
    gradients against the oracle run on the small region that holds every window touching the sample."""
    if _free_gib() < 26:
        pytest.skip("needs ~22 GiB of free device memory")
    N, C, H, W, s = 64, 64, 736, 736, 2                     # 2 218 786 816 input elements
    assert N * C * H * W > 2**31
    Ho, Wo = oracle.pool_out_dims(H, W, k, k, s, s, 0, 0)
    g = torch.Generator(device="cuda").manual_seed(21 + k)
    x = torch.empty(N * C * H * W, dtype=torch.float32, device="cuda")
    x.uniform_(0.0, 1.0, generator=g)
    x.mul_(8).floor_().div_(8)                               # few distinct values: plenty of tied windows
    dy = torch.empty(N * C * Ho * Wo, dtype=torch.float32, device="cuda")
    dy.normal_(generator=g)
    rng = np.random.default_rng(9 + k)
    pts = np.stack([rng.integers(0, d, size=300) for d in (N, C, H, W)], axis=1)
    pts[:4] = [[0, 0, 0, 0], [N - 1, C - 1, H - 1, W - 1], [N - 1, C - 1, 0, W - 1], [0, C - 1, H - 1, 0]]
    for mode in (MAX, AVG):
        dx = torch.full((N * C * H * W,), 7.0, dtype=torch.float32, device="cuda")
        assert cm.cnnmem_pool_backward(x if mode == MAX else None, dy, dx, N, C, H, W, layout, mode,
                                       k, k, s, s, 0, 0) == 0
        for (n, c, h, w) in pts:
            n, c, h, w = int(n), int(c), int(h), int(w)
            # windows (along each axis) that contain the sample, clipped to the output
            i_lo, i_hi = max(0, -(-(h - k + 1) // s)), min(Ho - 1, h // s)
            j_lo, j_hi = max(0, -(-(w - k + 1) // s)), min(Wo - 1, w // s)
            got = float(dx[oracle.index(layout, N, C, H, W, n, c, h, w)])
            if i_lo > i_hi or j_lo > j_hi:                   # last row / column that no window covers
                assert got == 0.0
                continue
            r0, q0 = i_lo * s, j_lo * s
            R, Q = (i_hi - i_lo) * s + k, (j_hi - j_lo) * s + k
            idx = np.array([oracle.index(layout, N, C, H, W, n, c, r0 + a, q0 + b) for a in range(R) for b in range(Q)],
                           dtype=np.int64)
            gidx = np.array([oracle.index(layout, N, C, Ho, Wo, n, c, i, j)
                             for i in range(i_lo, i_hi + 1) for j in range(j_lo, j_hi + 1)], dtype=np.int64)
            region = x[torch.from_numpy(idx).cuda()].cpu().numpy().reshape(1, 1, R, Q)
            grads = dy[torch.from_numpy(gidx).cuda()].cpu().numpy().reshape(1, 1, i_hi - i_lo + 1, j_hi - j_lo + 1)
            want = oracle.pool_backward(region, grads, 1, 1, R, Q, NCHW, mode, k, k, s, s, 0, 0)[0, 0, h - r0, w - q0]
            bound = 1e-6 * float(np.abs(grads).sum()) + 1e-30
            assert abs(got - float(want)) <= bound, (layout, k, mode, n, c, h, w, got, float(want))
        del dx
