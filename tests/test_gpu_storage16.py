"""The hot path on 16-bit storage (fp16, bf16) against the oracle.

Bars: transforms and max-pooling bit for bit; average pooling and softmax are
computed in fp32 and rounded once to 16 bits, the oracle computes in fp64 and
rounds once, so a result may differ by one unit in the last place of the storage
format where the exact value lies within fp32 rounding of a tie (rare: the tests
also require at least 99.9 % / 99 % of the outputs to be identical)."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_1610_03618_amd as cm
from paper_1610_03618_amd import workloads as wl

pytestmark = pytest.mark.gpu

TORCH = {cm.F16: torch.float16, cm.BF16: torch.bfloat16}
IDS = {cm.F16: "fp16", cm.BF16: "bf16"}
DTYPES = [cm.F16, cm.BF16]


def to16(x32: np.ndarray, dtype):
    """float32 array -> (uint16 bit patterns for the oracle, torch tensor on the GPU)."""
    t = torch.from_numpy(np.ascontiguousarray(x32)).to(TORCH[dtype])
    return t.view(torch.int16).numpy().view(np.uint16), t.cuda()


def bits_of(t: torch.Tensor) -> np.ndarray:
    return t.cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def ulp_distance(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    def key(u):
        u = u.astype(np.int32)
        return np.where(u < 0x8000, u, 0x8000 - u)
    return np.abs(key(a) - key(b))


def check_rounded(got: np.ndarray, want: np.ndarray, min_equal: float, what):
    d = ulp_distance(got, want)
    assert d.max() <= 1, (what, int(d.max()))
    assert (d == 0).mean() >= min_equal, (what, float((d == 0).mean()))


# ---- transform -------------------------------------------------------------------

T_SHAPES = [(16, 64, 32, 32), (6, 7, 9, 10), (3, 5, 7, 11), (128, 3, 9, 10), (2, 96, 13, 13), (130, 2, 33, 4),
            (1, 8, 8, 8), (64, 1, 1, 1), (8, 1, 1, 7), (34, 4, 5, 6), (256, 16, 6, 6),
            # 2..8 images: thin-plane kernels (several blocks, ragged and odd ends, blocks of fewer than 8 columns)
            (2, 3, 37, 61), (3, 5, 21, 33), (4, 16, 28, 28), (5, 1, 1, 2049), (6, 2, 50, 50), (7, 3, 19, 23),
            (8, 8, 32, 32), (8, 1, 1, 9), (4, 1, 1, 8), (2, 1, 1, 4), (3, 1, 1, 4099), (1, 3, 17, 19),
            (100, 4, 16, 16), (96, 8, 8, 8)]


@pytest.mark.parametrize("shape", T_SHAPES, ids=["x".join(map(str, s)) for s in T_SHAPES])
def test_transform16_matches_oracle(shape):
    N, C, H, W = shape
    rng = np.random.default_rng(sum(shape))
    x = rng.integers(0, 65536, size=shape).astype(np.uint16)            # every bit pattern
    d = torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16)
    want = oracle.transform16(x, N, C, H, W, oracle.NCHW, oracle.CHWN)
    got = cm.transform(d, N, C, H, W, cm.NCHW, cm.CHWN)
    assert np.array_equal(bits_of(got), want)
    back = cm.transform(got, N, C, H, W, cm.CHWN, cm.NCHW)
    assert np.array_equal(bits_of(back), x)
    same = cm.transform(d, N, C, H, W, cm.NCHW, cm.NCHW)
    assert np.array_equal(bits_of(same), x)


@pytest.mark.parametrize("odd", [False, True], ids=["even", "odd"])
@pytest.mark.parametrize("tile", list(range(17)))
def test_transform16_every_tile_shape(tile, odd):
    # 150 x 924: even extents, ragged in every tile shape; 151 x 1001: odd extents (shifted accesses / word tiles)
    N, C, H, W = (151, 7, 11, 13) if odd else (150, 6, 11, 14)
    rng = np.random.default_rng(tile)
    x = rng.integers(0, 65536, size=(N, C, H, W)).astype(np.uint16)
    d = torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
    os.environ["CNNMEM_TRANSFORM16_TILE"] = str(tile)
    try:
        got = cm.transform(d, N, C, H, W, cm.NCHW, cm.CHWN)
        back = cm.transform(got, N, C, H, W, cm.CHWN, cm.NCHW)
    finally:
        del os.environ["CNNMEM_TRANSFORM16_TILE"]
    assert np.array_equal(bits_of(got), oracle.transform16(x, N, C, H, W, 0, 1))
    assert np.array_equal(bits_of(back), x)


def test_transform16_misaligned_views():
    N, C, H, W = 12, 6, 5, 8
    n = N * C * H * W
    rng = np.random.default_rng(5)
    x = rng.integers(0, 65536, size=(N, C, H, W)).astype(np.uint16)
    for so, do in [(1, 0), (0, 1), (2, 2), (3, 5)]:
        sbuf = torch.zeros(n + 8, dtype=torch.float16, device="cuda")
        sbuf[so:so + n] = torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16).reshape(-1)
        dbuf = torch.zeros(n + 8, dtype=torch.float16, device="cuda")
        st = cm.cnnmem_transform_dtype(sbuf[so:], dbuf[do:], N, C, H, W, cm.NCHW, cm.CHWN, cm.F16)
        assert st == 0
        got = bits_of(dbuf)
        assert np.array_equal(got[do:do + n], oracle.transform16(x, N, C, H, W, 0, 1).ravel()), (so, do)
        assert not got[:do].any() and not got[do + n:].any()


# ---- pooling ---------------------------------------------------------------------

P_CASES = [  # N, C, H, W, k, s, p
    (16, 8, 32, 32, 3, 2, 0), (8, 4, 55, 55, 3, 2, 0), (8, 3, 27, 27, 3, 2, 0), (16, 6, 28, 28, 2, 2, 0),
    (8, 5, 14, 14, 2, 2, 0), (8, 3, 13, 13, 3, 1, 1), (8, 2, 17, 19, 3, 2, 1), (6, 3, 15, 15, 3, 2, 0),
    (8, 2, 64, 64, 2, 2, 0), (4, 3, 30, 24, 2, 2, 0), (8, 2, 9, 9, 5, 3, 2), (24, 2, 150, 150, 3, 2, 0),
    (8, 1, 224, 224, 2, 2, 0), (3, 2, 7, 5, 2, 1, 0), (4, 2, 224, 224, 3, 2, 1), (4, 2, 300, 40, 5, 3, 2),
    (8, 2, 129, 131, 3, 2, 0), (16, 3, 7, 7, 7, 7, 0), (8, 2, 20, 21, 4, 3, 1), (24, 2, 33, 35, 5, 3, 2),
]


@pytest.mark.parametrize("dtype", DTYPES, ids=[IDS[d] for d in DTYPES])
@pytest.mark.parametrize("case", P_CASES, ids=["-".join(map(str, c)) for c in P_CASES])
def test_pool16_matches_oracle(case, dtype):
    N, C, H, W, k, s, p = case
    rng = np.random.default_rng(sum(case))
    xb, xd = to16(wl.relu_normal(rng, (N, C, H, W)) + np.float32(0.25), dtype)
    xcb = oracle.transform16(xb, N, C, H, W, 0, 1)
    xcd = cm.transform(xd, N, C, H, W, cm.NCHW, cm.CHWN)
    for layout, hb, dev in ((cm.NCHW, xb, xd), (cm.CHWN, xcb, xcd)):
        want = oracle.pool16(hb, N, C, H, W, layout, 0, k, k, s, s, p, p, dtype)
        got = cm.pool(dev, N, C, H, W, layout, cm.POOL_MAX, k, k, s, s, p, p)
        assert np.array_equal(bits_of(got), want), (case, layout, "max")
        want = oracle.pool16(hb, N, C, H, W, layout, 1, k, k, s, s, p, p, dtype)
        got = cm.pool(dev, N, C, H, W, layout, cm.POOL_AVG, k, k, s, s, p, p)
        check_rounded(bits_of(got), want, 0.999, (case, layout, "avg"))


@pytest.mark.parametrize("dtype", DTYPES, ids=[IDS[d] for d in DTYPES])
def test_pool16_max_orders_every_finite_pattern(dtype):
    """Subnormals, the largest finite values and infinities: the maximum of random bit patterns
    (NaNs and the negative zero excluded) is the oracle's, bit for bit, in every kernel."""
    rng = np.random.default_rng(1616)
    N, C, H, W = 8, 6, 24, 24
    bits = rng.integers(0, 65536, size=(N, C, H, W)).astype(np.uint16)
    exp_mask, frac_mask = (0x7c00, 0x03ff) if dtype == cm.F16 else (0x7f80, 0x007f)
    nan = ((bits & exp_mask) == exp_mask) & ((bits & frac_mask) != 0)
    bits[nan | (bits == 0x8000)] = 0x0001                              # the smallest subnormal instead
    xd = torch.from_numpy(bits.view(np.int16)).cuda().view(TORCH[dtype])
    xcb = oracle.transform16(bits, N, C, H, W, 0, 1)
    xcd = cm.transform(xd, N, C, H, W, cm.NCHW, cm.CHWN)
    for (k, s) in [(2, 2), (3, 2), (3, 1), (5, 3), (4, 2), (24, 24)]:      # the last three: run-time-window kernels
        for layout, hb, dev in ((cm.NCHW, bits, xd), (cm.CHWN, xcb, xcd)):
            want = oracle.pool16(hb, N, C, H, W, layout, 0, k, k, s, s, 0, 0, dtype)
            got = cm.pool(dev, N, C, H, W, layout, cm.POOL_MAX, k, k, s, s)
            assert np.array_equal(bits_of(got), want), (k, s, layout)


@pytest.mark.parametrize("dtype", DTYPES, ids=[IDS[d] for d in DTYPES])
def test_pool16_average_of_infinities_and_exact_ties(dtype):
    """The average divides by a reciprocal with one residual step and a fix-up: windows that hold an infinity give
    that infinity, and window sums that are exact multiples of the area (averages exactly representable, many of
    them on rounding ties of the storage format) come out bit-exact."""
    rng = np.random.default_rng(77)
    N, C, H, W = 8, 4, 21, 23
    small = rng.integers(0, 64, size=(N, C, H, W)).astype(np.float32) / np.float32(8.0)    # multiples of 1/8
    xb, _ = to16(small, dtype)
    inf16 = np.uint16(0x7c00 if dtype == cm.F16 else 0x7f80)
    xb = xb.copy()
    xb[0, 0, 3, 4] = inf16
    xb[1, 2, 10, 11] = inf16 | np.uint16(0x8000)
    xd = torch.from_numpy(xb.view(np.int16)).cuda().view(TORCH[dtype])
    xcb = oracle.transform16(xb, N, C, H, W, 0, 1)
    xcd = torch.from_numpy(xcb.view(np.int16)).cuda().view(TORCH[dtype])
    for (kh, kw, s, p) in [(3, 3, 2, 0), (3, 3, 1, 1), (5, 3, 2, 1), (2, 2, 2, 0), (21, 23, 21, 0)]:
        for layout, hb, dev in ((cm.NCHW, xb, xd), (cm.CHWN, xcb, xcd)):
            want = oracle.pool16(hb, N, C, H, W, layout, 1, kh, kw, s, s, p, p, dtype)
            got = bits_of(cm.pool(dev, N, C, H, W, layout, cm.POOL_AVG, kh, kw, s, s, p, p))
            assert np.array_equal(got, want), (kh, kw, s, p, layout, int((got != want).sum()))


@pytest.mark.parametrize("rows", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("dtype", DTYPES, ids=[IDS[d] for d in DTYPES])
def test_pool16_nchw_slab_rows_per_lane(rows, dtype, monkeypatch):
    """The LDS kernel's 2 x OY output blocks: padding clamps, odd Wo (unaligned pairs), ragged row blocks, strips."""
    monkeypatch.setenv("CNNMEM_SLAB16_ROWS", str(rows))
    for case in [(3, 5, 13, 17, 3, 1, 1), (2, 3, 57, 57, 3, 1, 0), (1, 2, 150, 131, 3, 1, 1), (3, 5, 13, 17, 3, 2, 1),
                 (2, 3, 57, 57, 3, 2, 0), (1, 2, 260, 131, 3, 2, 1), (2, 2, 9, 300, 3, 1, 1), (2, 2, 300, 9, 3, 2, 1)]:
        N, C, H, W, k, s, p = case
        rng = np.random.default_rng(sum(case) + rows)
        xb, xd = to16(wl.relu_normal(rng, (N, C, H, W)) + np.float32(0.25), dtype)
        want = oracle.pool16(xb, N, C, H, W, cm.NCHW, 0, k, k, s, s, p, p, dtype)
        got = cm.pool(xd, N, C, H, W, cm.NCHW, cm.POOL_MAX, k, k, s, s, p, p)
        assert np.array_equal(bits_of(got), want), (case, "max")
        want = oracle.pool16(xb, N, C, H, W, cm.NCHW, 1, k, k, s, s, p, p, dtype)
        got = cm.pool(xd, N, C, H, W, cm.NCHW, cm.POOL_AVG, k, k, s, s, p, p)
        check_rounded(bits_of(got), want, 0.999, (case, "avg"))


@pytest.mark.parametrize("rows", [1, 2, 3])
@pytest.mark.parametrize("dtype", DTYPES, ids=[IDS[d] for d in DTYPES])
def test_pool16_chwn_any_window_rows_per_lane(rows, dtype, monkeypatch):
    """The run-time-window CHWN kernel with 1..3 output rows per lane: ragged row blocks, padding, rectangular
    windows, a window as large as the image."""
    monkeypatch.setenv("CNNMEM_CHWN16_ANY_ROWS", str(rows))
    for case in [(8, 3, 17, 19, 5, 5, 3, 3, 2, 2), (16, 2, 20, 21, 5, 5, 2, 2, 2, 2), (8, 2, 11, 13, 5, 5, 1, 1, 2, 2),
                 (8, 3, 16, 16, 4, 4, 2, 2, 1, 1), (8, 2, 7, 7, 7, 7, 7, 7, 0, 0), (8, 2, 9, 30, 5, 3, 1, 2, 2, 1),
                 (8, 2, 30, 9, 3, 5, 2, 1, 1, 2), (24, 1, 10, 10, 4, 4, 3, 3, 2, 2)]:
        N, C, H, W, kh, kw, sh, sw, ph, pw = case
        rng = np.random.default_rng(sum(case) + rows)
        xb, _ = to16(wl.relu_normal(rng, (N, C, H, W)) + np.float32(0.25), dtype)
        xcb = oracle.transform16(xb, N, C, H, W, 0, 1)
        xcd = torch.from_numpy(xcb.view(np.int16)).cuda().view(TORCH[dtype])
        want = oracle.pool16(xcb, N, C, H, W, cm.CHWN, 0, kh, kw, sh, sw, ph, pw, dtype)
        got = cm.pool(xcd, N, C, H, W, cm.CHWN, cm.POOL_MAX, kh, kw, sh, sw, ph, pw)
        assert np.array_equal(bits_of(got), want), (case, "max")
        want = oracle.pool16(xcb, N, C, H, W, cm.CHWN, 1, kh, kw, sh, sw, ph, pw, dtype)
        got = cm.pool(xcd, N, C, H, W, cm.CHWN, cm.POOL_AVG, kh, kw, sh, sw, ph, pw)
        check_rounded(bits_of(got), want, 0.999, (case, "avg"))


@pytest.mark.parametrize("split", [0, 4, 8])
@pytest.mark.parametrize("dtype", DTYPES, ids=[IDS[d] for d in DTYPES])
def test_pool16_chwn_window_rows_dealt_over_lanes(split, dtype, monkeypatch):
    """Few outputs, tall windows: the rows of a window dealt over 4 or 8 lanes, partial results combined in LDS."""
    if split:
        monkeypatch.setenv("CNNMEM_CHWN_SPLIT", str(split))
    monkeypatch.setenv("CNNMEM_CHWN16_ANY_ROWS", "1")
    for case in [(128, 20, 7, 7, 7, 7, 7, 7, 0, 0), (8, 3, 14, 14, 14, 14, 14, 14, 0, 0), (8, 5, 9, 11, 5, 5, 3, 3, 2, 2),
                 (24, 2, 8, 8, 8, 8, 1, 1, 4, 4), (8, 3, 13, 6, 6, 4, 2, 1, 3, 2), (40, 7, 10, 10, 4, 4, 2, 2, 1, 1)]:
        N, C, H, W, kh, kw, sh, sw, ph, pw = case
        rng = np.random.default_rng(sum(case) + split)
        xb, _ = to16(wl.relu_normal(rng, (N, C, H, W)) + np.float32(0.25), dtype)
        xcb = oracle.transform16(xb, N, C, H, W, 0, 1)
        xcd = torch.from_numpy(xcb.view(np.int16)).cuda().view(TORCH[dtype])
        want = oracle.pool16(xcb, N, C, H, W, cm.CHWN, 0, kh, kw, sh, sw, ph, pw, dtype)
        got = cm.pool(xcd, N, C, H, W, cm.CHWN, cm.POOL_MAX, kh, kw, sh, sw, ph, pw)
        assert np.array_equal(bits_of(got), want), (case, "max")
        want = oracle.pool16(xcb, N, C, H, W, cm.CHWN, 1, kh, kw, sh, sw, ph, pw, dtype)
        got = cm.pool(xcd, N, C, H, W, cm.CHWN, cm.POOL_AVG, kh, kw, sh, sw, ph, pw)
        check_rounded(bits_of(got), want, 0.999, (case, "avg"))


def test_pool16_misaligned_views_take_the_generic_kernel():
    N, C, H, W, k, s = 8, 3, 12, 12, 3, 2
    rng = np.random.default_rng(77)
    xb, xd = to16(wl.relu_normal(rng, (N, C, H, W)), cm.F16)
    n = xb.size
    buf = torch.zeros(n + 8, dtype=torch.float16, device="cuda")
    buf[1:1 + n] = xd.reshape(-1)
    Ho, Wo = oracle.pool_out_dims(H, W, k, k, s, s, 0, 0)
    out = torch.zeros(N * C * Ho * Wo + 8, dtype=torch.float16, device="cuda")
    for layout in (cm.NCHW, cm.CHWN):
        hb = xb if layout == cm.NCHW else oracle.transform16(xb, N, C, H, W, 0, 1)
        buf[1:1 + n] = torch.from_numpy(hb.view(np.int16)).cuda().view(torch.float16).reshape(-1)
        st = cm.cnnmem_pool_dtype(buf[1:], out[3:], N, C, H, W, layout, cm.POOL_MAX, k, k, s, s, 0, 0, cm.F16)
        assert st == 0
        want = oracle.pool16(hb, N, C, H, W, layout, 0, k, k, s, s, 0, 0, oracle.F16).ravel()
        assert np.array_equal(bits_of(out)[3:3 + want.size], want), layout


# ---- softmax ---------------------------------------------------------------------

S_SHAPES = [(7, 1), (5, 10), (33, 31), (33, 32), (40, 100), (128, 1000), (64, 1001), (9, 4096), (6, 21841),
            (3, 70001), (300, 257), (17, 8200),
            # 32768 < categories <= 65536: the long-row kernel that keeps only 16-bit words in registers
            (5, 50257), (3, 65536), (4, 40000), (2, 33001), (3, 65535)]


@pytest.mark.parametrize("dtype", DTYPES, ids=[IDS[d] for d in DTYPES])
@pytest.mark.parametrize("shape", S_SHAPES, ids=[f"{n}x{c}" for n, c in S_SHAPES])
def test_softmax16_matches_oracle(shape, dtype):
    n, c = shape
    rng = np.random.default_rng(n * 31 + c)
    z = wl.normal_logits(rng, n, c, 3.0)
    if c > 10:
        z = wl.plant_outliers(z, rng)
    zb, zd = to16(z, dtype)
    want = oracle.softmax16(zb, dtype)
    got = bits_of(cm.softmax(zd))
    check_rounded(got, want, 0.99, shape)


@pytest.mark.parametrize("dtype", DTYPES, ids=[IDS[d] for d in DTYPES])
def test_softmax16_misaligned_and_mixed_phase(dtype):
    n, c = 19, 777
    rng = np.random.default_rng(4)
    zb, zd = to16(wl.normal_logits(rng, n, c, 3.0), dtype)
    want = oracle.softmax16(zb, dtype)
    for so, do in [(1, 1), (0, 1), (3, 0), (8, 8), (4, 12)]:
        src = torch.zeros(n * c + 16, dtype=TORCH[dtype], device="cuda")
        dst = torch.zeros(n * c + 16, dtype=TORCH[dtype], device="cuda")
        src[so:so + n * c] = zd.reshape(-1)
        st = cm.cnnmem_softmax_dtype(src[so:], dst[do:], n, c, dtype)
        assert st == 0
        got = bits_of(dst)
        check_rounded(got[do:do + n * c].reshape(n, c), want, 0.99, (so, do))
        assert not got[:do].any() and not got[do + n * c:].any()


def test_softmax16_in_place():
    n, c = 50, 3000
    zb, zd = to16(wl.normal_logits(np.random.default_rng(6), n, c, 2.0), cm.BF16)
    want = oracle.softmax16(zb, oracle.BF16)
    st = cm.cnnmem_softmax_dtype(zd, zd, n, c, cm.BF16)
    assert st == 0
    check_rounded(bits_of(zd), want, 0.99, "in place")


# ---- the benchmark configurations' largest tensors, 16-bit --------------------------

@pytest.mark.parametrize("dtype", DTYPES, ids=[IDS[d] for d in DTYPES])
def test_config2_transform16_full_size(dtype):
    t = wl.config(2).transforms[0]
    xb, xd = to16(wl.make_tensor(t, wl.rng_for(2)), dtype)
    got = cm.transform(xd, t.N, t.C, t.H, t.W, cm.NCHW, cm.CHWN)
    assert np.array_equal(bits_of(got), oracle.transform16(xb, t.N, t.C, t.H, t.W, 0, 1))
    back = cm.transform(got, t.N, t.C, t.H, t.W, cm.CHWN, cm.NCHW)
    assert np.array_equal(bits_of(back), xb)


@pytest.mark.parametrize("dtype", DTYPES, ids=[IDS[d] for d in DTYPES])
def test_config4_pool16_second_tensor_full_size(dtype):
    p = wl.config(4).pools[2].tensor                     # 64 x 128 x 112 x 112
    xb, xd = to16(wl.make_tensor(p, wl.rng_for(4, 1)), dtype)
    xcb = oracle.transform16(xb, p.N, p.C, p.H, p.W, 0, 1)
    xcd = cm.transform(xd, p.N, p.C, p.H, p.W, cm.NCHW, cm.CHWN)
    for layout, hb, dev in ((cm.NCHW, xb, xd), (cm.CHWN, xcb, xcd)):
        want = oracle.pool16(hb, p.N, p.C, p.H, p.W, layout, 0, 2, 2, 2, 2, 0, 0, dtype)
        assert np.array_equal(bits_of(cm.pool(dev, p.N, p.C, p.H, p.W, layout, cm.POOL_MAX, 2, 2, 2, 2)), want)
        want = oracle.pool16(hb, p.N, p.C, p.H, p.W, layout, 1, 2, 2, 2, 2, 0, 0, dtype)
        check_rounded(bits_of(cm.pool(dev, p.N, p.C, p.H, p.W, layout, cm.POOL_AVG, 2, 2, 2, 2)), want, 0.999, layout)


@pytest.mark.parametrize("dtype", DTYPES, ids=[IDS[d] for d in DTYPES])
def test_config3_pool16_first_tensor_full_size(dtype):
    p = wl.config(3).pools[0].tensor                     # 128 x 96 x 55 x 55, 3x3 / stride 2
    xb, xd = to16(wl.make_tensor(p, wl.rng_for(3, 0)), dtype)
    xcb = oracle.transform16(xb, p.N, p.C, p.H, p.W, 0, 1)
    xcd = cm.transform(xd, p.N, p.C, p.H, p.W, cm.NCHW, cm.CHWN)
    for layout, hb, dev in ((cm.NCHW, xb, xd), (cm.CHWN, xcb, xcd)):
        want = oracle.pool16(hb, p.N, p.C, p.H, p.W, layout, 0, 3, 3, 2, 2, 0, 0, dtype)
        assert np.array_equal(bits_of(cm.pool(dev, p.N, p.C, p.H, p.W, layout, cm.POOL_MAX, 3, 3, 2, 2)), want)


@pytest.mark.parametrize("dtype", DTYPES, ids=[IDS[d] for d in DTYPES])
def test_config5_softmax16_full_size(dtype):
    s = wl.config(5).softmaxes[0]
    zb, zd = to16(wl.make_logits(s, wl.rng_for(5, 0)), dtype)
    want = oracle.softmax16(zb, dtype)
    check_rounded(bits_of(cm.softmax(zd)), want, 0.99, "config 5")


# ---- any storage order, 16-bit words ------------------------------------------------

import itertools

P16_SHAPES = [(8, 16, 20, 24), (5, 12, 70, 36), (3, 7, 9, 130), (2, 3, 129, 67), (4, 68, 6, 72), (1, 96, 7, 7),
              (4, 1, 33, 5), (6, 4, 1, 260), (2, 300, 2, 4), (1, 1, 1, 9), (3, 3, 3, 3), (2, 130, 34, 18)]


@pytest.mark.parametrize("dims", P16_SHAPES, ids=["x".join(map(str, s)) for s in P16_SHAPES])
def test_permute16_every_permutation_matches_oracle(dims):
    rng = np.random.default_rng(sum(dims) + 16)
    x = rng.integers(0, 65536, size=dims).astype(np.uint16)
    d = torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
    for perm in itertools.permutations(range(4)):
        want = oracle.permute16(x, dims, perm)
        got = cm.permute(d, dims, perm)
        assert tuple(got.shape) == want.shape
        assert np.array_equal(bits_of(got), want), (dims, perm)


@pytest.mark.parametrize("T", [2, 3, 4, 5, 6, 7, 8])
def test_relayout16_thin_axes_both_directions(T):
    """Two to eight feature maps in 16-bit storage: the thin-plane kernels inside a batch of planes."""
    for (N, H, W) in [(2, 37, 61), (1, 50, 50), (3, 1, 2049), (2, 1, 5)]:
        rng = np.random.default_rng(T * 100 + H)
        x = rng.integers(0, 65536, size=(N, T, H, W)).astype(np.uint16)
        d = torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16)
        nhwc = cm.relayout(d, N, T, H, W, "NCHW", "NHWC")
        want = oracle.permute16(x, (N, T, H, W), (0, 2, 3, 1))
        assert np.array_equal(bits_of(nhwc).reshape(-1), want.reshape(-1)), (T, N, H, W)
        back = cm.relayout(nhwc, N, T, H, W, "NHWC", "NCHW")
        assert np.array_equal(bits_of(back).reshape(-1), x.reshape(-1)), (T, N, H, W)


def test_relayout16_named_orders_full_size_and_misaligned():
    t = wl.config(2).transforms[0]                       # 128 x 96 x 55 x 55: odd image extents
    N, C, H, W = t.N, t.C, t.H, t.W
    canon = np.random.default_rng(2).integers(0, 65536, size=(N, C, H, W)).astype(np.uint16)
    d = torch.from_numpy(canon.view(np.int16)).cuda().view(torch.float16)
    for dst, perm in [("NHWC", (0, 2, 3, 1)), ("HWCN", (2, 3, 1, 0)), ("CNHW", (1, 0, 2, 3))]:
        want = oracle.permute16(canon, (N, C, H, W), perm)
        got = cm.relayout(d, N, C, H, W, "NCHW", dst)
        assert np.array_equal(bits_of(got), want), dst
        back = cm.relayout(got, N, C, H, W, dst, "NCHW")
        assert np.array_equal(bits_of(back), canon), dst
    # buffers that are only 2-byte aligned take the word-by-word kernels
    dims, n = (3, 8, 36, 20), 3 * 8 * 36 * 20
    x = np.random.default_rng(3).integers(0, 65536, size=dims).astype(np.uint16)
    for so, do in [(1, 0), (0, 1), (3, 3)]:
        sbuf = torch.zeros(n + 8, dtype=torch.float16, device="cuda")
        sbuf[so:so + n] = torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16).reshape(-1)
        for perm in [(0, 2, 3, 1), (3, 2, 1, 0), (1, 0, 2, 3), (2, 0, 1, 3)]:
            dbuf = torch.zeros(n + 8, dtype=torch.float16, device="cuda")
            assert cm.cnnmem_permute_dtype(sbuf[so:], dbuf[do:], dims, perm, cm.F16) == 0
            got = bits_of(dbuf)
            assert np.array_equal(got[do:do + n], oracle.permute16(x, dims, perm).ravel()), (so, do, perm)
            assert not got[:do].any() and not got[do + n:].any()
