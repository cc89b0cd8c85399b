"""General storage-order changes on the GPU against the oracle, word for word
(Section I: 24 orders; Section IV.A: CHWN / HWCN; NHWC)."""
import itertools

import numpy as np
import pytest
import torch

import oracle
import paper_1610_03618_amd as cm
from paper_1610_03618_amd import workloads as wl

pytestmark = pytest.mark.gpu

PERMS = list(itertools.permutations(range(4)))
LAYOUTS = ["".join(p) for p in itertools.permutations("NCHW")]


def bits(a):
    return np.ascontiguousarray(a).view(np.uint32)


def random_words(rng, shape):
    return rng.integers(0, 2**32, size=shape, dtype=np.uint32).view(np.float32)    # every bit pattern, NaNs too


# extents chosen to hit every kernel: all multiples of 4 (128-bit both sides), odd fastest extents (dword on
# one side or both), several tiles with ragged edges, extents of 1 (merged away), short and long fastest axes
SHAPES = [(8, 16, 20, 24), (5, 12, 70, 36), (3, 7, 9, 130), (2, 3, 129, 67), (4, 68, 5, 72), (1, 96, 7, 7),
          (4, 1, 33, 5), (6, 4, 1, 260), (2, 300, 2, 4), (1, 1, 1, 9), (1, 1, 1, 1), (3, 3, 3, 3)]


@pytest.mark.parametrize("dims", SHAPES, ids=["x".join(map(str, s)) for s in SHAPES])
def test_every_permutation_matches_oracle(dims):
    rng = np.random.default_rng(sum(dims))
    x = random_words(rng, dims)
    d = torch.from_numpy(x).cuda()
    for perm in PERMS:
        want = oracle.permute(x, dims, perm)
        got = cm.permute(d, dims, perm).cpu().numpy()
        assert got.shape == want.shape
        assert np.array_equal(bits(got), bits(want)), (dims, perm)


def test_every_pair_of_spelled_layouts():
    N, C, H, W = 6, 20, 9, 12
    rng = np.random.default_rng(24)
    canon = random_words(rng, (N, C, H, W))
    for src in LAYOUTS:
        x = oracle.relayout(canon, N, C, H, W, "NCHW", src)
        d = torch.from_numpy(x).cuda()
        for dst in LAYOUTS:
            want = oracle.relayout(x, N, C, H, W, src, dst)
            got = cm.relayout(d, N, C, H, W, src, dst).cpu().numpy()
            assert np.array_equal(bits(got), bits(want)), (src, dst)


def test_relayout_agrees_with_the_two_layout_transform():
    N, C, H, W = 32, 24, 13, 13
    x = wl.uniform_pm1(np.random.default_rng(5), (N, C, H, W))
    d = torch.from_numpy(x).cuda()
    a = cm.relayout(d, N, C, H, W, "NCHW", "CHWN")
    b = cm.transform(d, N, C, H, W, cm.NCHW, cm.CHWN)
    assert torch.equal(a.view(torch.int32), b.view(torch.int32))
    back = cm.relayout(a, N, C, H, W, "CHWN", "NCHW")
    assert torch.equal(back.view(torch.int32), d.view(torch.int32))


@pytest.mark.parametrize("src_off,dst_off", [(1, 0), (0, 1), (3, 2), (4, 4)])
def test_misaligned_buffers_take_the_dword_paths(src_off, dst_off):
    dims = (3, 8, 36, 20)
    n = int(np.prod(dims))
    rng = np.random.default_rng(src_off * 10 + dst_off)
    x = random_words(rng, dims)
    sbuf = torch.zeros(n + 8, dtype=torch.float32, device="cuda")
    sbuf[src_off:src_off + n] = torch.from_numpy(x).cuda().reshape(-1)
    for perm in [(0, 2, 3, 1), (3, 2, 1, 0), (1, 0, 2, 3), (0, 3, 1, 2), (2, 0, 1, 3)]:
        dbuf = torch.full((n + 8,), -1.0, dtype=torch.float32, device="cuda")
        st = cm.cnnmem_permute(sbuf[src_off:], dbuf[dst_off:], dims, perm)
        assert st == 0
        got = dbuf.cpu().numpy()
        want = oracle.permute(x, dims, perm).ravel()
        assert np.array_equal(bits(got[dst_off:dst_off + n]), bits(want)), perm
        assert np.all(got[:dst_off] == -1.0) and np.all(got[dst_off + n:] == -1.0)      # nothing written outside


FULL = [("NCHW", "NHWC"), ("NHWC", "NCHW"), ("CHWN", "HWCN"), ("HWCN", "CHWN"), ("NCHW", "HWCN"), ("NHWC", "CHWN"),
        ("NCHW", "CNHW"), ("NCHW", "NCWH")]


@pytest.mark.parametrize("src,dst", FULL, ids=[f"{a}-{b}" for a, b in FULL])
def test_config2_tensor_full_size(src, dst):
    t = wl.config(2).transforms[0]                       # 128 x 96 x 55 x 55: odd image extents
    canon = wl.make_tensor(t, wl.rng_for(2))
    x = oracle.relayout(canon, t.N, t.C, t.H, t.W, "NCHW", src)
    want = oracle.relayout(x, t.N, t.C, t.H, t.W, src, dst)
    got = cm.relayout(torch.from_numpy(x).cuda(), t.N, t.C, t.H, t.W, src, dst).cpu().numpy()
    assert np.array_equal(bits(got), bits(want))


@pytest.mark.parametrize("src,dst", [("NCHW", "NHWC"), ("NHWC", "NCHW"), ("NCHW", "HWCN")])
def test_vgg_tensor_full_size(src, dst):
    N, C, H, W = 64, 64, 112, 112                        # extents all multiples of 4: 128-bit both sides
    canon = wl.relu_normal(np.random.default_rng(112), (N, C, H, W))
    x = oracle.relayout(canon, N, C, H, W, "NCHW", src)
    want = oracle.relayout(x, N, C, H, W, src, dst)
    got = cm.relayout(torch.from_numpy(x).cuda(), N, C, H, W, src, dst).cpu().numpy()
    assert np.array_equal(bits(got), bits(want))


def test_first_layer_rgb_tensor():
    N, C, H, W = 32, 3, 224, 224                         # three feature maps: a very short fastest axis in NHWC
    canon = wl.uniform_pm1(np.random.default_rng(3), (N, C, H, W))
    for src, dst in [("NCHW", "NHWC"), ("NHWC", "NCHW"), ("NHWC", "CHWN")]:
        x = oracle.relayout(canon, N, C, H, W, "NCHW", src)
        want = oracle.relayout(x, N, C, H, W, src, dst)
        got = cm.relayout(torch.from_numpy(x).cuda(), N, C, H, W, src, dst).cpu().numpy()
        assert np.array_equal(bits(got), bits(want)), (src, dst)


@pytest.mark.parametrize("T", [2, 3, 4, 5, 6, 7, 8])
def test_thin_axes_both_directions(T):
    """Two to eight feature maps: the thin-plane kernels, several blocks with a ragged last one."""
    for (N, H, W) in [(2, 37, 61), (1, 50, 50), (3, 1, 1025), (2, 1, 3)]:
        rng = np.random.default_rng(T * 100 + H)
        canon = random_words(rng, (N, T, H, W))
        d = torch.from_numpy(canon).cuda()
        nhwc = cm.relayout(d, N, T, H, W, "NCHW", "NHWC")
        assert np.array_equal(bits(nhwc.cpu().numpy()), bits(oracle.relayout(canon, N, T, H, W, "NCHW", "NHWC")))
        back = cm.relayout(nhwc, N, T, H, W, "NHWC", "NCHW")
        assert np.array_equal(bits(back.cpu().numpy()), bits(canon))
        # thin batch: T images, N-fastest layouts
        chwn = cm.relayout(d, N, T, H, W, "NCHW", "CHWN")
        assert np.array_equal(bits(chwn.cpu().numpy()), bits(oracle.relayout(canon, N, T, H, W, "NCHW", "CHWN")))
        x2 = random_words(rng, (T, 5, H, W))
        d2 = torch.from_numpy(x2).cuda()
        got = cm.relayout(d2, T, 5, H, W, "NCHW", "CHWN")
        assert np.array_equal(bits(got.cpu().numpy()), bits(oracle.relayout(x2, T, 5, H, W, "NCHW", "CHWN")))
        got = cm.relayout(got, T, 5, H, W, "CHWN", "NCHW")
        assert np.array_equal(bits(got.cpu().numpy()), bits(x2))
