"""Pins of the oracle's general storage-order changes (Section I: a 4-D tensor
can be stored in 24 orders; Section IV.A: CHWN / HWCN; NHWC in the comparison
libraries).  Nothing here goes through the oracle's own index formulae: the
expected values are hand-worked, come from numpy's transpose, or are structural
properties (inverse, composition, agreement of the two independent routines)."""
import itertools

import numpy as np
import pytest

import oracle

PERMS = list(itertools.permutations(range(4)))
LAYOUTS = ["".join(p) for p in itertools.permutations("NCHW")]


def bits(a):
    return np.ascontiguousarray(a).view(np.uint32)


def test_permute_hand_worked():
    # dims (2,1,2,2), values = source linear index; perm (3,0,1,2): the fastest axis becomes the slowest
    x = np.arange(8, dtype=np.float32).reshape(2, 1, 2, 2)
    got = oracle.permute(x, (2, 1, 2, 2), (3, 0, 1, 2))
    # destination [w][a][b][h]: element (w,a,0,h) = x[a,0,h,w] = 4a + 2h + w
    want = np.array([0, 2, 4, 6, 1, 3, 5, 7], dtype=np.float32).reshape(2, 2, 1, 2)
    assert got.shape == (2, 2, 1, 2)
    assert np.array_equal(got, want)


def test_relayout_hand_worked_nchw_to_nhwc():
    # N=1, C=2, H=1, W=3: NCHW [c][w] = [[0,1,2],[3,4,5]] -> NHWC [w][c] = [[0,3],[1,4],[2,5]]
    x = np.arange(6, dtype=np.float32)
    got = oracle.relayout(x, 1, 2, 1, 3, "NCHW", "NHWC").ravel()
    assert got.tolist() == [0, 3, 1, 4, 2, 5]
    back = oracle.relayout(got, 1, 2, 1, 3, "NHWC", "NCHW").ravel()
    assert back.tolist() == [0, 1, 2, 3, 4, 5]


@pytest.mark.parametrize("perm", PERMS)
def test_permute_is_numpy_transpose(perm):
    rng = np.random.default_rng(7)
    dims = (3, 5, 4, 7)
    x = rng.integers(0, 2**32, size=dims, dtype=np.uint32).view(np.float32)   # all bit patterns, NaNs included
    got = oracle.permute(x, dims, perm)
    assert np.array_equal(bits(got), bits(x.transpose(perm)))


@pytest.mark.parametrize("perm", PERMS)
def test_permute_inverse_restores(perm):
    rng = np.random.default_rng(8)
    dims = (2, 6, 3, 5)
    x = rng.standard_normal(dims, dtype=np.float32)
    y = oracle.permute(x, dims, perm)
    inv = [perm.index(a) for a in range(4)]
    assert np.array_equal(bits(oracle.permute(y, y.shape, inv)), bits(x))


def test_permute_composition():
    rng = np.random.default_rng(9)
    dims = (4, 3, 5, 2)
    x = rng.standard_normal(dims, dtype=np.float32)
    p, q = (2, 0, 3, 1), (1, 3, 0, 2)
    two_steps = oracle.permute(oracle.permute(x, dims, p), tuple(dims[a] for a in p), q)
    one_step = oracle.permute(x, dims, tuple(p[a] for a in q))
    assert np.array_equal(bits(two_steps), bits(one_step))


@pytest.mark.parametrize("src", LAYOUTS)
def test_relayout_against_numpy_for_every_pair(src):
    N, C, H, W = 3, 4, 2, 5
    ext = dict(N=N, C=C, H=H, W=W)
    rng = np.random.default_rng(10)
    canon = rng.integers(0, 2**32, size=(N, C, H, W), dtype=np.uint32).view(np.float32)
    x = np.ascontiguousarray(canon.transpose(["NCHW".index(l) for l in src]))
    assert x.shape == tuple(ext[l] for l in src)
    for dst in LAYOUTS:
        got = oracle.relayout(x, N, C, H, W, src, dst)
        want = canon.transpose(["NCHW".index(l) for l in dst])
        assert got.shape == want.shape
        assert np.array_equal(bits(got), bits(want)), (src, dst)


def test_relayout_and_permute_agree_and_extend_the_two_layout_transform():
    N, C, H, W = 4, 3, 5, 6
    rng = np.random.default_rng(11)
    x = rng.standard_normal((N, C, H, W), dtype=np.float32)
    # CHWN is source axes (1, 2, 3, 0) of NCHW
    a = oracle.relayout(x, N, C, H, W, "NCHW", "CHWN")
    b = oracle.permute(x, (N, C, H, W), (1, 2, 3, 0))
    c = oracle.transform(x, N, C, H, W, oracle.NCHW, oracle.CHWN)
    assert np.array_equal(bits(a), bits(b)) and np.array_equal(bits(a), bits(c))
    # HWCN keeps N fastest like CHWN (Section IV.A): both are [M][N] matrices with the rows reordered
    hwcn = oracle.relayout(x, N, C, H, W, "NCHW", "HWCN")
    assert np.array_equal(bits(hwcn), bits(a.transpose(1, 2, 0, 3)))


def test_index_tagged_words_land_where_the_layout_says():
    N, C, H, W = 2, 3, 4, 5
    x = np.arange(N * C * H * W, dtype=np.uint32).view(np.float32).reshape(N, C, H, W)
    y = bits(oracle.relayout(x, N, C, H, W, "NCHW", "WHCN"))       # [w][h][c][n]
    for (n, c, h, w) in [(0, 0, 0, 0), (1, 2, 3, 4), (1, 0, 2, 3), (0, 2, 1, 4)]:
        assert y[w, h, c, n] == ((n * C + c) * H + h) * W + w


def test_rejects_bad_arguments():
    x = np.zeros(16, dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.permute(x, (2, 2, 2, 2), (0, 1, 1, 3))
    with pytest.raises(ValueError):
        oracle.relayout(x, 2, 2, 2, 2, "NCHW", "NCHH")
    with pytest.raises(ValueError):
        oracle.relayout(x, 2, 2, 2, 2, "NCH", "NCHW")
