"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element
by element, on seeded inputs.

Bars: transforms and max-pool bit-exact; avg-pool 1e-6 relative (to the mean
magnitude of the taps, which equals the result for the non-negative inputs of
the benchmark configurations); softmax |gpu - ref| <= max(2e-6 |ref|, 1e-7).
"""
import numpy as np
import pytest
import torch

import oracle
import paper_1610_03618_amd as cm
from paper_1610_03618_amd import workloads as wl

pytestmark = pytest.mark.gpu

NCHW, CHWN, MAX, AVG = cm.NCHW, cm.CHWN, cm.POOL_MAX, cm.POOL_AVG


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t: torch.Tensor) -> np.ndarray:
    torch.cuda.synchronize()
    return t.cpu().numpy()


def same_bits(a: np.ndarray, b: np.ndarray) -> bool:
    return a.shape == b.shape and np.array_equal(a.view(np.uint32), b.view(np.uint32))


def test_extension_is_loaded_and_device_is_gfx950():
    assert cm.library() is not None
    assert torch.cuda.is_available()
    name = torch.cuda.get_device_properties(0).gcnArchName
    assert "gfx950" in name, name


# ------------------------------------------------------------------ transform

TRANSFORM_SHAPES = [
    (1, 1, 1, 1), (2, 2, 1, 2), (4, 1, 1, 4), (16, 3, 8, 8), (128, 3, 7, 12), (64, 5, 13, 12),
    (32, 6, 10, 10), (8, 16, 9, 4), (256, 2, 17, 4), (100, 4, 5, 9), (132, 3, 11, 4),   # vector paths, ragged tiles
    (5, 7, 3, 3), (3, 2, 55, 55), (127, 1, 9, 7), (16, 3, 5, 5), (66, 1, 1, 129),       # scalar path
    (20, 8, 6, 2), (12, 4, 4, 4),
    (256, 4, 17, 16), (260, 8, 12, 12), (512, 4, 24, 24),                               # 256 images and more: XCD-ordered tiles
    (1, 3, 17, 19), (1, 64, 8, 8),                                                      # one image: a copy
    (2, 3, 37, 61), (3, 5, 21, 33), (4, 16, 28, 28), (5, 1, 1, 1025), (6, 2, 50, 50),   # 2..8 images: thin-plane kernels,
    (7, 3, 19, 23), (8, 8, 32, 32), (8, 1, 1, 3), (4, 1, 1, 1), (2, 1, 1, 2),           # several blocks, ragged ends
    (100, 4, 16, 16), (96, 8, 8, 8), (72, 64, 4, 4),                                     # 65..127 images: 128-wide tiles
]


@pytest.mark.parametrize("shape", TRANSFORM_SHAPES)
def test_transform_matches_oracle_bit_for_bit(shape):
    N, C, H, W = shape
    rng = np.random.default_rng(hash(shape) % (1 << 32))
    bits = rng.integers(0, 1 << 32, size=N * C * H * W, dtype=np.uint64).astype(np.uint32)
    bits[: min(4, bits.size)] = [0x7FC00001, 0xFFC12345, 0x80000000, 0x7F800000][: min(4, bits.size)]
    x = bits.view(np.float32).reshape(N, C, H, W)
    want = oracle.transform(x, N, C, H, W, NCHW, CHWN)
    got = cm.transform(dev(x), N, C, H, W, NCHW, CHWN)
    assert same_bits(host(got), want)
    back = cm.transform(got, N, C, H, W, CHWN, NCHW)
    assert same_bits(host(back), x)
    assert same_bits(host(back), oracle.transform(want, N, C, H, W, CHWN, NCHW))
    same = cm.transform(dev(x), N, C, H, W, NCHW, NCHW)
    assert same_bits(host(same), x)


@pytest.mark.parametrize("tile", list(range(15)))
def test_transform_every_tile_shape(tile, monkeypatch):
    monkeypatch.setenv("CNNMEM_TRANSFORM_TILE", str(tile))
    for (N, C, H, W) in [(128, 3, 9, 12), (20, 5, 7, 4), (260, 1, 33, 4)]:
        x = np.arange(N * C * H * W, dtype=np.uint32).view(np.float32).reshape(N, C, H, W)
        want = oracle.transform(x, N, C, H, W, NCHW, CHWN)
        got = cm.transform(dev(x), N, C, H, W, NCHW, CHWN)
        assert same_bits(host(got), want)
        assert same_bits(host(cm.transform(got, N, C, H, W, CHWN, NCHW)), x)


def test_transform_misaligned_views_take_the_scalar_path():
    N, C, H, W = 64, 4, 6, 4
    n = N * C * H * W
    x = np.arange(n, dtype=np.uint32).view(np.float32)
    buf_in = torch.zeros(n + 8, dtype=torch.float32, device="cuda")
    buf_out = torch.full((n + 8,), -7.0, dtype=torch.float32, device="cuda")
    for off_in, off_out in [(1, 0), (0, 3), (2, 2)]:
        buf_in[off_in:off_in + n] = dev(x)
        buf_out.fill_(-7.0)
        st = cm.cnnmem_transform(buf_in.data_ptr() + 4 * off_in, buf_out.data_ptr() + 4 * off_out,
                                 N, C, H, W, NCHW, CHWN)
        assert st == 0
        out = host(buf_out)
        assert same_bits(out[off_out:off_out + n].reshape(C, H, W, N),
                         oracle.transform(x.reshape(N, C, H, W), N, C, H, W, NCHW, CHWN))
        assert np.all(out[:off_out] == -7.0) and np.all(out[off_out + n:] == -7.0)   # nothing outside


# ------------------------------------------------------------------ pooling

def avg_tolerance(x_nchw, N, C, H, W, geom):
    """1e-6 times the mean magnitude of each window's taps (NCHW order)."""
    kh, kw, sh, sw, ph, pw = geom
    return 1e-6 * oracle.pool(np.abs(x_nchw), N, C, H, W, NCHW, AVG, kh, kw, sh, sw, ph, pw).astype(np.float64)


def check_pool(x, N, C, H, W, geom, modes=(MAX, AVG), layouts=(NCHW, CHWN), tuning=None):
    kh, kw, sh, sw, ph, pw = geom
    Ho, Wo = oracle.pool_out_dims(H, W, kh, kw, sh, sw, ph, pw)
    x = x + np.float32(0.0)                       # -0 -> +0: the sign of a zero maximum is unspecified
    xc = oracle.transform(x, N, C, H, W, NCHW, CHWN)
    tol_n = avg_tolerance(x, N, C, H, W, geom) if AVG in modes else None
    for layout in layouts:
        src = x if layout == NCHW else xc
        d_src = dev(src)
        for mode in modes:
            want = oracle.pool(src, N, C, H, W, layout, mode, kh, kw, sh, sw, ph, pw)
            got = host(cm.pool(d_src, N, C, H, W, layout, mode, kh, kw, sh, sw, ph, pw, tuning=tuning))
            assert got.shape == want.shape
            if mode == MAX:
                assert same_bits(got + np.float32(0.0), want + np.float32(0.0)), (layout, geom)
            else:
                tol = tol_n if layout == NCHW else oracle.transform(
                    tol_n.astype(np.float32), N, C, Ho, Wo, NCHW, CHWN).astype(np.float64) * (1 + 1e-6)
                err = np.abs(got.astype(np.float64) - want.astype(np.float64))
                assert np.all(err <= tol + 1e-45), (layout, geom, float(err.max()))


POOL_CASES = [
    # (N, C, H, W), (kh, kw, sh, sw, ph, pw)
    ((16, 64, 32, 32), (3, 3, 2, 2, 0, 0)),      # config 1 (also run at full size below)
    ((4, 3, 13, 13), (3, 3, 2, 2, 0, 0)),
    ((8, 5, 27, 27), (3, 3, 2, 2, 0, 0)),
    ((12, 2, 55, 55), (3, 3, 2, 2, 0, 0)),
    ((4, 2, 110, 110), (3, 3, 2, 2, 0, 0)),      # plane larger than one LDS slab: row strips with halo
    ((4, 3, 24, 24), (3, 3, 2, 2, 0, 0)),
    ((8, 3, 28, 28), (2, 2, 2, 2, 0, 0)),        # W % 8 != 0
    ((4, 3, 224, 224), (2, 2, 2, 2, 0, 0)),
    ((4, 2, 14, 14), (2, 2, 2, 2, 0, 0)),        # W % 4 != 0: slab path
    ((4, 3, 15, 15), (2, 2, 2, 2, 0, 0)),        # odd H and W, last row/col unused
    ((5, 3, 9, 11), (3, 3, 2, 2, 0, 0)),         # N % 4 != 0: generic CHWN path
    ((4, 3, 9, 11), (3, 3, 2, 2, 1, 1)),         # padded
    ((8, 2, 12, 10), (2, 2, 2, 2, 1, 1)),
    ((4, 2, 17, 19), (3, 3, 1, 1, 1, 1)),
    ((4, 2, 17, 19), (3, 2, 2, 1, 1, 0)),        # rectangular window and stride
    ((4, 2, 20, 9), (5, 3, 3, 2, 2, 1)),
    ((4, 2, 7, 7), (7, 7, 1, 1, 0, 0)),          # window = image
    ((4, 2, 6, 6), (1, 1, 1, 1, 0, 0)),          # identity
    ((4, 2, 9, 9), (2, 2, 3, 3, 0, 0)),          # stride > window
    ((4, 1, 1, 12), (1, 4, 1, 2, 0, 0)),         # Fig. 8 geometry
    ((1, 1, 2, 2), (2, 2, 2, 2, 0, 0)),
    ((4, 2, 150, 70), (3, 3, 2, 2, 1, 1)),       # padded + strips
    ((64, 2, 8, 8), (2, 2, 2, 2, 0, 0)),
    ((128, 1, 6, 5), (3, 3, 2, 2, 0, 0)),
]


@pytest.mark.parametrize("shape,geom", POOL_CASES)
def test_pool_matches_oracle(shape, geom):
    N, C, H, W = shape
    rng = np.random.default_rng(abs(hash((shape, geom))) % (1 << 32))
    x = rng.standard_normal(shape, dtype=np.float32)
    check_pool(x, N, C, H, W, geom)


@pytest.mark.parametrize("rows", [1, 2, 3])
def test_pool_chwn_any_window_rows_per_lane(rows, monkeypatch):
    """The run-time-window CHWN kernel with 1..3 output rows per lane: ragged row blocks, padding, rectangular
    windows, windows as large as the image."""
    monkeypatch.setenv("CNNMEM_CHWN_ANY_ROWS", str(rows))
    rng = np.random.default_rng(60 + rows)
    for shape, geom in [((8, 3, 17, 19), (5, 5, 3, 3, 2, 2)), ((4, 2, 20, 21), (5, 5, 2, 2, 2, 2)),
                        ((8, 2, 11, 13), (5, 5, 1, 1, 2, 2)), ((4, 3, 16, 16), (4, 4, 2, 2, 1, 1)),
                        ((8, 2, 7, 7), (7, 7, 7, 7, 0, 0)), ((4, 2, 9, 30), (5, 3, 1, 2, 2, 1)),
                        ((4, 2, 30, 9), (3, 5, 2, 1, 1, 2)), ((12, 1, 10, 10), (4, 4, 3, 3, 2, 2))]:
        x = rng.standard_normal(shape, dtype=np.float32)
        check_pool(x, *shape, geom, layouts=(CHWN,))


@pytest.mark.parametrize("split", [0, 4, 8])
def test_pool_chwn_window_rows_dealt_over_lanes(split, monkeypatch):
    """Few outputs, tall windows: the rows of a window are dealt over 4 or 8 lanes and the partial results meet in
    LDS.  Global pooling, padded windows shorter than the number of parts, a ragged last workgroup."""
    if split:
        monkeypatch.setenv("CNNMEM_CHWN_SPLIT", str(split))
    monkeypatch.setenv("CNNMEM_CHWN_ANY_ROWS", "1")
    rng = np.random.default_rng(70 + split)
    for shape, geom in [((128, 20, 7, 7), (7, 7, 7, 7, 0, 0)), ((8, 3, 14, 14), (14, 14, 14, 14, 0, 0)),
                        ((4, 5, 9, 11), (5, 5, 3, 3, 2, 2)), ((12, 2, 8, 8), (8, 8, 1, 1, 4, 4)),
                        ((4, 3, 13, 6), (6, 4, 2, 1, 3, 2)), ((36, 7, 10, 10), (4, 4, 2, 2, 1, 1))]:
        x = rng.standard_normal(shape, dtype=np.float32)
        check_pool(x, *shape, geom)                 # NCHW too: its LDS kernel shares such outputs among eight lanes


@pytest.mark.parametrize("oy", [1, 2, 3, 4])
@pytest.mark.parametrize("ox", [1, 2])
def test_pool_chwn_every_working_set_shape(oy, ox):
    rng = np.random.default_rng(10 * oy + ox)
    for shape, geom in [((8, 3, 27, 27), (3, 3, 2, 2, 0, 0)), ((8, 3, 13, 15), (3, 3, 2, 2, 1, 1)),
                        ((8, 3, 14, 30), (2, 2, 2, 2, 0, 0)), ((4, 2, 12, 11), (3, 3, 1, 1, 1, 1)),
                        ((16, 2, 9, 7), (2, 2, 2, 2, 1, 1)), ((8, 2, 17, 16), (5, 5, 3, 3, 2, 2)),
                        ((4, 3, 12, 14), (4, 6, 2, 1, 1, 3))]:    # the last two: the run-time-window kernel
        x = rng.standard_normal(shape, dtype=np.float32)
        check_pool(x, *shape, geom, layouts=(CHWN,), tuning=dict(rows_per_lane=oy, cols_per_lane=ox))


@pytest.mark.parametrize("tuning", [dict(nchw_kernel=2), dict(nchw_kernel=2, slab_lanes=256),
                                    dict(nchw_kernel=2, slab_lanes=1024), dict(workgroups_per_cu=6),
                                    dict(workgroups_per_cu=2), dict(workgroups_per_cu=-1)])
def test_pool_nchw_every_kernel_choice(tuning):
    rng = np.random.default_rng(9)
    for shape, geom in [((4, 5, 32, 48), (2, 2, 2, 2, 0, 0)), ((4, 3, 27, 27), (3, 3, 2, 2, 0, 0)),
                        ((2, 2, 110, 110), (3, 3, 2, 2, 0, 0))]:
        x = rng.standard_normal(shape, dtype=np.float32)
        check_pool(x, *shape, geom, layouts=(NCHW,), tuning=tuning)
    x = rng.standard_normal((8, 4, 16, 16), dtype=np.float32)
    check_pool(x, 8, 4, 16, 16, (2, 2, 2, 2, 0, 0), layouts=(CHWN,), tuning=tuning)


@pytest.mark.parametrize("rows", [0, 1, 2, 3, 4])
def test_pool_nchw_slab_rows_per_lane(rows, monkeypatch):
    """The LDS kernel's several-outputs-per-lane variants (padding clamps, ragged row blocks, strips with halo)."""
    monkeypatch.setenv("CNNMEM_SLAB_ROWS", str(rows))
    rng = np.random.default_rng(40 + rows)
    for shape, geom in [((3, 5, 13, 17), (3, 3, 1, 1, 1, 1)), ((2, 3, 57, 57), (3, 3, 1, 1, 0, 0)),
                        ((1, 2, 130, 131), (3, 3, 1, 1, 1, 1)), ((3, 5, 13, 17), (3, 3, 2, 2, 1, 1)),
                        ((2, 3, 57, 57), (3, 3, 2, 2, 0, 0)), ((1, 2, 230, 131), (3, 3, 2, 2, 1, 1)),
                        ((2, 2, 9, 300), (3, 3, 1, 1, 1, 0)), ((2, 2, 300, 9), (3, 3, 2, 2, 0, 1))]:
        x = rng.standard_normal(shape, dtype=np.float32)
        check_pool(x, *shape, geom, layouts=(NCHW,))


def test_pool_misaligned_views():
    N, C, H, W = 8, 3, 9, 9
    geom = (3, 3, 2, 2, 0, 0)
    x = np.random.default_rng(10).standard_normal((N, C, H, W), dtype=np.float32)
    Ho, Wo = oracle.pool_out_dims(H, W, 3, 3, 2, 2, 0, 0)
    n_in, n_out = x.size, N * C * Ho * Wo
    for layout in (NCHW, CHWN):
        src = x if layout == NCHW else oracle.transform(x, N, C, H, W, NCHW, CHWN)
        want = oracle.pool(src, N, C, H, W, layout, MAX, *geom)
        for off_in, off_out in [(1, 0), (0, 1), (3, 2)]:
            buf_in = torch.zeros(n_in + 8, dtype=torch.float32, device="cuda")
            buf_out = torch.full((n_out + 8,), -7.0, dtype=torch.float32, device="cuda")
            buf_in[off_in:off_in + n_in] = dev(src.ravel())
            st = cm.cnnmem_pool(buf_in.data_ptr() + 4 * off_in, buf_out.data_ptr() + 4 * off_out,
                                N, C, H, W, layout, MAX, *geom)
            assert st == 0
            out = host(buf_out)
            assert same_bits(out[off_out:off_out + n_out], want.ravel())
            assert np.all(out[:off_out] == -7.0) and np.all(out[off_out + n_out:] == -7.0)


@pytest.mark.parametrize("row", wl.TABLE1_POOLS, ids=[r[0] for r in wl.TABLE1_POOLS])
def test_pool_table1_shapes_reduced_batch(row):
    name, N, hw, k, C, s = row
    N, C = 8, min(C, 8)                           # Table 1 plane sizes and windows, fewer planes
    x = wl.relu_normal(np.random.default_rng(len(name) + hw), (N, C, hw, hw))
    check_pool(x, N, C, hw, hw, (k, k, s, s, 0, 0))


# ------------------------------------------------------------------ softmax

def check_softmax(z: np.ndarray, in_place=False):
    want = oracle.softmax(z)
    d = dev(z)
    got = host(cm.softmax(d, out=d if in_place else None))
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    tol = np.maximum(2e-6 * np.abs(want.astype(np.float64)), 1e-7)
    assert np.all(err <= tol), float((err / tol).max())
    sums = got.astype(np.float64).sum(axis=1)
    assert np.all(np.abs(sums - 1.0) <= 1e-5)
    assert np.all(got >= 0) and np.all(got <= 1)
    return got


SOFTMAX_SHAPES = [(1, 1), (3, 2), (9, 5), (300, 7), (4, 8), (5, 9), (3, 11), (128, 10), (5, 63), (9, 64), (7, 65), (128, 1000), (7, 1001), (33, 1023),
                  (6, 2049), (10, 4097), (5, 8191), (3, 10000), (5, 21841), (3, 32768), (2, 49153),
                  (2, 65530), (2, 70001), (1, 140000)]


@pytest.mark.parametrize("shape", SOFTMAX_SHAPES)
def test_softmax_matches_oracle(shape):
    n, c = shape
    rng = np.random.default_rng(n * 100003 + c)
    z = wl.normal_logits(rng, n, c, 3.0)
    z[0, rng.integers(0, c)] += 50.0
    check_softmax(z)
    check_softmax(z, in_place=True)


@pytest.mark.parametrize("tpr", [64, 128, 256, 512, 1024])
def test_softmax_every_lane_group_width(tpr, monkeypatch):
    monkeypatch.setenv("CNNMEM_SOFTMAX_TPR", str(tpr))
    rng = np.random.default_rng(tpr)
    for n, c in [(9, 257), (5, 1000), (3, 4099)]:
        check_softmax(wl.normal_logits(rng, n, c, 2.0))


def test_softmax_planted_outliers_ties_and_large_shift():
    rng = np.random.default_rng(77)
    z = wl.plant_outliers(wl.normal_logits(rng, 64, 1531, 3.0), rng)
    z[3, :] = 0.25                                   # constant row -> exactly uniform
    z[5, 7] = 100.0                                  # exp(100) overflows fp32 without the max shift
    z[6, :] += 1000.0
    got = check_softmax(z)
    assert np.all(np.isfinite(got))
    np.testing.assert_allclose(got[3], 1.0 / 1531, rtol=2e-6)
    assert got[5, 7] == 1.0


def test_softmax_misaligned_and_mixed_phase_views():
    n, c = 6, 1003
    z = wl.normal_logits(np.random.default_rng(5), n, c, 2.0)
    want = oracle.softmax(z)
    for off_in, off_out in [(1, 1), (2, 2), (3, 3), (0, 1), (2, 0)]:
        buf_in = torch.zeros(n * c + 8, dtype=torch.float32, device="cuda")
        buf_out = torch.full((n * c + 8,), -7.0, dtype=torch.float32, device="cuda")
        buf_in[off_in:off_in + n * c] = dev(z.ravel())
        st = cm.cnnmem_softmax(buf_in.data_ptr() + 4 * off_in, buf_out.data_ptr() + 4 * off_out, n, c)
        assert st == 0
        out = host(buf_out)
        got = out[off_out:off_out + n * c].reshape(n, c)
        err = np.abs(got.astype(np.float64) - want.astype(np.float64))
        assert np.all(err <= np.maximum(2e-6 * np.abs(want.astype(np.float64)), 1e-7))
        assert np.all(out[:off_out] == -7.0) and np.all(out[off_out + n * c:] == -7.0)


@pytest.mark.parametrize("row", wl.TABLE1_CLASSIFIERS, ids=[r[0] for r in wl.TABLE1_CLASSIFIERS])
def test_softmax_table1_classifiers(row):
    _, n, c = row
    check_softmax(wl.normal_logits(np.random.default_rng(n + c), n, c, 2.0))


def test_non_default_stream():
    s = torch.cuda.Stream()
    z = wl.normal_logits(np.random.default_rng(1), 32, 777, 2.0)
    d = dev(z)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        out = cm.softmax(d)
    s.synchronize()
    want = oracle.softmax(z)
    err = np.abs(out.cpu().numpy().astype(np.float64) - want)
    assert np.all(err <= np.maximum(2e-6 * np.abs(want), 1e-7))


@pytest.mark.parametrize("shape", [(1000, 4), (777, 5), (300, 10), (129, 31), (64, 63), (50, 100), (33, 159), (17, 160),
                                   (9, 257), (5, 512), (3, 70001), (2, 131073), (1, 262147)],
                         ids=lambda s: f"{s[0]}x{s[1]}")
def test_softmax_short_and_very_long_rows(shape):
    """Sub-wavefront row groups (4 .. 32 lanes per row) and the two-sweep kernel for rows beyond the register budget."""
    n, c = shape
    rng = np.random.default_rng(n + c)
    z = wl.normal_logits(rng, n, c, 3.0)
    if c > 10:
        z = wl.plant_outliers(z, rng)
    want = oracle.softmax(z).astype(np.float64)
    got = cm.softmax(torch.from_numpy(z).cuda()).cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - want) <= np.maximum(2e-6 * want, 1e-7)), shape
    # a view one float into a buffer: rows start at every dword phase
    buf = torch.zeros(n * c + 4, device="cuda")
    buf[1:1 + n * c] = torch.from_numpy(z).cuda().reshape(-1)
    out = torch.zeros(n * c + 4, device="cuda")
    assert cm.cnnmem_softmax(buf[1:], out[3:], n, c) == 0
    got = out.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got[3:3 + n * c].reshape(n, c) - want) <= np.maximum(2e-6 * want, 1e-7)), shape
    assert not got[:3].any() and not got[3 + n * c:].any()
