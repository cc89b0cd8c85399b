"""Pins for the CPU oracle: values the paper fixes, hand-worked cases, closed
forms, invariants, brute force on tiny inputs and library routines.  None of
these goes through the oracle's own formulae."""
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from oracle import CHWN, NCHW, POOL_AVG, POOL_MAX

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


# ---------------------------------------------------------------- transform

def test_transform_hand_worked_2x2x1x2():
    # N=2, C=2, H=1, W=2; value = NCHW linear index.  In CHWN the element
    # (c, h, w, n) sits at ((c*1+h)*2+w)*2+n, so reading CHWN in order gives
    # n-pairs of each (c, w): [0,4, 1,5, 2,6, 3,7].
    src = np.arange(8, dtype=np.float32)
    out = oracle.transform(src, 2, 2, 1, 2, NCHW, CHWN)
    assert out.ravel().tolist() == [0, 4, 1, 5, 2, 6, 3, 7]
    back = oracle.transform(out, 2, 2, 1, 2, CHWN, NCHW)
    assert back.ravel().tolist() == list(range(8))


def test_transform_hand_worked_3x1x2x1():
    # N=3, C=1, H=2, W=1: NCHW [n][h] = [[0,1],[2,3],[4,5]] -> CHWN [h][n].
    src = np.arange(6, dtype=np.float32)
    out = oracle.transform(src, 3, 1, 2, 1, NCHW, CHWN)
    assert out.ravel().tolist() == [0, 2, 4, 1, 3, 5]


@pytest.mark.parametrize("shape", [(2, 3, 4, 5), (7, 1, 1, 9), (1, 5, 3, 2), (16, 3, 5, 7), (5, 4, 1, 1)])
def test_transform_matches_library_permute(shape):
    N, C, H, W = shape
    rng = np.random.default_rng(1)
    x = rng.standard_normal(shape, dtype=np.float32)
    chwn = oracle.transform(x, N, C, H, W, NCHW, CHWN)
    assert chwn.shape == (C, H, W, N)
    np.testing.assert_array_equal(chwn, np.ascontiguousarray(x.transpose(1, 2, 3, 0)))
    nchw = oracle.transform(chwn, N, C, H, W, CHWN, NCHW)
    np.testing.assert_array_equal(nchw, x)


def test_transform_is_2d_transpose_of_flattened_chw():
    # Section IV.C: NCHW == [N][C*H*W], CHWN == [C*H*W][N].
    N, C, H, W = 6, 3, 4, 5
    x = np.arange(N * C * H * W, dtype=np.float32).reshape(N, C * H * W)
    out = oracle.transform(x.reshape(N, C, H, W), N, C, H, W, NCHW, CHWN)
    np.testing.assert_array_equal(out.reshape(C * H * W, N), x.T)


def test_transform_round_trip_preserves_every_bit_pattern():
    N, C, H, W = 5, 3, 4, 7
    rng = np.random.default_rng(2)
    bits = rng.integers(0, 2**32, size=N * C * H * W, dtype=np.uint64).astype(np.uint32)
    bits[:4] = [0x7FC00001, 0xFFC12345, 0x80000000, 0x7F800000]  # NaN payloads, -0, inf
    x = bits.view(np.float32).reshape(N, C, H, W)
    y = oracle.transform(x, N, C, H, W, NCHW, CHWN)
    z = oracle.transform(y, N, C, H, W, CHWN, NCHW)
    assert z.view(np.uint32).tobytes() == x.view(np.uint32).tobytes()
    assert sorted(y.view(np.uint32).ravel().tolist()) == sorted(bits.tolist())


def test_transform_index_tagged():
    # Each word holds its own source index; the destination index decodes to
    # the same (n, c, h, w).
    N, C, H, W = 3, 2, 3, 4
    tags = np.arange(N * C * H * W, dtype=np.uint32).view(np.float32)
    out = oracle.transform(tags, N, C, H, W, NCHW, CHWN).view(np.uint32).ravel()
    for d, s in enumerate(out.tolist()):
        n, rem = d % N, d // N
        w, rem = rem % W, rem // W
        h, c = rem % H, rem // H
        assert s == ((n * C + c) * H + h) * W + w


def test_transform_special_cases():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((1, 4, 3, 5), dtype=np.float32)         # N=1: identity copy
    np.testing.assert_array_equal(oracle.transform(x, 1, 4, 3, 5, NCHW, CHWN).ravel(), x.ravel())
    m = rng.standard_normal((7, 1, 1, 9), dtype=np.float32)         # C=H=1: matrix transpose
    np.testing.assert_array_equal(oracle.transform(m, 7, 1, 1, 9, NCHW, CHWN).reshape(9, 7),
                                  m.reshape(7, 9).T)
    same = oracle.transform(x, 1, 4, 3, 5, NCHW, NCHW)               # same layout: copy
    np.testing.assert_array_equal(same, x)


def test_transform_rejects_bad_arguments():
    x = np.zeros(4, dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.transform(x, 2, 2, 1, 1, NCHW, 7)


# ---------------------------------------------------------------- pooling

def test_pool_fig8_worked_example():
    (L, k, s, outputs, loads), = [[int(v) for v in r] for r in _rows("fig8_overlapped_pooling.txt")]
    assert oracle.pool_out_dims(1, L, 1, k, 1, s, 0, 0) == (1, outputs)
    assert oracle.naive_pool_loads_1d(L, k, s) == loads
    # the same signal actually pooled: 12 inputs 0..11, window 4, stride 2
    x = np.arange(L, dtype=np.float32).reshape(1, 1, 1, L)
    mx = oracle.pool(x, 1, 1, 1, L, NCHW, POOL_MAX, 1, k, 1, s)
    av = oracle.pool(x, 1, 1, 1, L, NCHW, POOL_AVG, 1, k, 1, s)
    assert mx.ravel().tolist() == [3, 5, 7, 9, 11]
    assert av.ravel().tolist() == [1.5, 3.5, 5.5, 7.5, 9.5]


def test_pool_extent_floor_rule():
    assert oracle.pool_out_dims(32, 32, 3, 3, 2, 2, 0, 0) == (15, 15)     # config 1: 32 -> 15
    for name, N, hw, k, C, s, expect in _rows("table1_pooling_shapes.txt"):
        assert oracle.pool_out_dims(int(hw), int(hw), int(k), int(k), int(s), int(s), 0, 0) == \
            (int(expect), int(expect)), name
    assert oracle.pool_out_dims(224, 112, 2, 2, 2, 2, 0, 0) == (112, 56)
    assert oracle.pool_out_dims(5, 5, 3, 3, 2, 2, 1, 1) == (3, 3)


def test_pool_hand_worked_ramp_4x4():
    x = np.arange(16, dtype=np.float32).reshape(1, 1, 4, 4)
    assert oracle.pool(x, 1, 1, 4, 4, NCHW, POOL_MAX, 2, 2, 2, 2).ravel().tolist() == [5, 7, 13, 15]
    assert oracle.pool(x, 1, 1, 4, 4, NCHW, POOL_AVG, 2, 2, 2, 2).ravel().tolist() == \
        [2.5, 4.5, 10.5, 12.5]
    # 3x3 stride 2 on 4x4: floor((4-3)/2)+1 = 1 output over rows/cols 0..2
    assert oracle.pool(x, 1, 1, 4, 4, NCHW, POOL_MAX, 3, 3, 2, 2).ravel().tolist() == [10]
    assert oracle.pool(x, 1, 1, 4, 4, NCHW, POOL_AVG, 3, 3, 2, 2).ravel().tolist() == [5.0]
    # rectangular window 1x2 / stride (1,2): distinguishes kh from kw and sh from sw
    got = oracle.pool(x, 1, 1, 4, 4, NCHW, POOL_MAX, 1, 2, 1, 2).reshape(4, 2)
    assert got.tolist() == [[1, 3], [5, 7], [9, 11], [13, 15]]
    got = oracle.pool(x, 1, 1, 4, 4, NCHW, POOL_MAX, 2, 1, 2, 1).reshape(2, 4)
    assert got.tolist() == [[4, 5, 6, 7], [12, 13, 14, 15]]


def test_pool_brute_force_2x2_inputs():
    a, b, c, d = 3.0, -1.0, 0.5, 2.0
    x = np.array([a, b, c, d], dtype=np.float32).reshape(1, 1, 2, 2)
    assert oracle.pool(x, 1, 1, 2, 2, NCHW, POOL_MAX, 2, 2, 2, 2).ravel().tolist() == [3.0]
    assert oracle.pool(x, 1, 1, 2, 2, NCHW, POOL_AVG, 2, 2, 2, 2).ravel().tolist() == [1.125]
    ident = oracle.pool(x, 1, 1, 2, 2, NCHW, POOL_MAX, 1, 1, 1, 1)
    np.testing.assert_array_equal(ident, x)
    ident = oracle.pool(x, 1, 1, 2, 2, NCHW, POOL_AVG, 1, 1, 1, 1)
    np.testing.assert_array_equal(ident, x)
    # 2x2 window, stride 1, pad 1 -> 3x3 outputs, enumerated by hand.
    # Taps outside the image are skipped by max and count as 0 in the average
    # (divisor stays 4).
    mx = oracle.pool(x, 1, 1, 2, 2, NCHW, POOL_MAX, 2, 2, 1, 1, 1, 1).reshape(3, 3)
    assert mx.tolist() == [[a, a, b], [a, a, d], [c, d, d]]
    av = oracle.pool(x, 1, 1, 2, 2, NCHW, POOL_AVG, 2, 2, 1, 1, 1, 1).reshape(3, 3)
    expect = [[a / 4, (a + b) / 4, b / 4],
              [(a + c) / 4, (a + b + c + d) / 4, (b + d) / 4],
              [c / 4, (c + d) / 4, d / 4]]
    assert av.tolist() == expect


def _brute_pool(x, mode, kh, kw, sh, sw, ph, pw):
    """Independent pure-Python pooling over an (N, C, H, W) array, exact rational-free fp64."""
    N, C, H, W = x.shape
    Ho = (H + 2 * ph - kh) // sh + 1
    Wo = (W + 2 * pw - kw) // sw + 1
    out = np.empty((N, C, Ho, Wo), dtype=np.float32)
    for n in range(N):
        for c in range(C):
            for i in range(Ho):
                for j in range(Wo):
                    taps = [float(x[n, c, r, q])
                            for r in range(i * sh - ph, i * sh - ph + kh) if 0 <= r < H
                            for q in range(j * sw - pw, j * sw - pw + kw) if 0 <= q < W]
                    out[n, c, i, j] = max(taps) if mode == POOL_MAX else \
                        np.float32(math.fsum(taps) / (kh * kw))
    return out


@pytest.mark.parametrize("geom", [(3, 3, 2, 2, 0, 0), (2, 2, 2, 2, 0, 0), (3, 2, 1, 2, 1, 0),
                                  (4, 4, 2, 2, 2, 1), (2, 3, 3, 1, 0, 1), (5, 5, 3, 3, 2, 2)])
@pytest.mark.parametrize("layout", [NCHW, CHWN])
def test_pool_matches_brute_force_small(geom, layout):
    kh, kw, sh, sw, ph, pw = geom
    N, C, H, W = 3, 2, 9, 8
    rng = np.random.default_rng(11)
    x = rng.standard_normal((N, C, H, W), dtype=np.float32)
    src = x if layout == NCHW else np.ascontiguousarray(x.transpose(1, 2, 3, 0))
    for mode in (POOL_MAX, POOL_AVG):
        got = oracle.pool(src, N, C, H, W, layout, mode, kh, kw, sh, sw, ph, pw)
        want = _brute_pool(x, mode, kh, kw, sh, sw, ph, pw)
        if layout == CHWN:
            want = np.ascontiguousarray(want.transpose(1, 2, 3, 0))
        if mode == POOL_MAX:
            np.testing.assert_array_equal(got, want)
        else:
            np.testing.assert_allclose(got, want, rtol=0, atol=1e-7)


@pytest.mark.parametrize("geom", [(3, 3, 2, 2, 0, 0), (2, 2, 2, 2, 0, 0), (3, 3, 2, 2, 1, 1),
                                  (3, 2, 2, 1, 1, 0), (5, 3, 1, 2, 2, 1)])
def test_pool_matches_library_routine_fp64(geom):
    kh, kw, sh, sw, ph, pw = geom
    N, C, H, W = 4, 5, 17, 13
    rng = np.random.default_rng(12)
    x = rng.standard_normal((N, C, H, W), dtype=np.float32)
    t = torch.from_numpy(x).double()
    want_max = F.max_pool2d(t, (kh, kw), (sh, sw), (ph, pw)).float().numpy()
    want_avg = F.avg_pool2d(t, (kh, kw), (sh, sw), (ph, pw), ceil_mode=False,
                            count_include_pad=True).float().numpy()
    np.testing.assert_array_equal(
        oracle.pool(x, N, C, H, W, NCHW, POOL_MAX, kh, kw, sh, sw, ph, pw), want_max)
    np.testing.assert_allclose(
        oracle.pool(x, N, C, H, W, NCHW, POOL_AVG, kh, kw, sh, sw, ph, pw), want_avg,
        rtol=0, atol=1e-7)


def test_pool_invariants():
    N, C, H, W = 4, 3, 11, 10
    rng = np.random.default_rng(13)
    # small integers: 2x+1 and sums are exact in fp32
    x = rng.integers(-50, 50, size=(N, C, H, W)).astype(np.float32)
    p = oracle.pool(x, N, C, H, W, NCHW, POOL_MAX, 3, 3, 2, 2)
    q = oracle.pool(2 * x + 1, N, C, H, W, NCHW, POOL_MAX, 3, 3, 2, 2)
    np.testing.assert_array_equal(q, 2 * p + 1)                     # commutes with monotone map
    assert set(np.unique(p)).issubset(set(np.unique(x)))             # outputs are inputs
    a = oracle.pool(x, N, C, H, W, NCHW, POOL_AVG, 3, 3, 2, 2)
    assert np.all(a <= p) and np.all(a >= -50)                        # mean <= max
    const = np.full((N, C, H, W), 0.3, dtype=np.float32)
    np.testing.assert_array_equal(
        oracle.pool(const, N, C, H, W, NCHW, POOL_AVG, 3, 3, 2, 2), np.float32(0.3))
    np.testing.assert_array_equal(oracle.pool(x, N, C, H, W, NCHW, POOL_MAX, 1, 1, 1, 1), x)
    # layouts commute: pooling the CHWN copy equals the CHWN copy of the pooled tensor
    xc = oracle.transform(x, N, C, H, W, NCHW, CHWN)
    for mode in (POOL_MAX, POOL_AVG):
        pn = oracle.pool(x, N, C, H, W, NCHW, mode, 3, 3, 2, 2)
        pc = oracle.pool(xc, N, C, H, W, CHWN, mode, 3, 3, 2, 2)
        Ho, Wo = oracle.pool_out_dims(H, W, 3, 3, 2, 2, 0, 0)
        np.testing.assert_array_equal(pc, oracle.transform(pn, N, C, Ho, Wo, NCHW, CHWN))


def test_pool_rejects_bad_arguments():
    x = np.zeros(16, dtype=np.float32)
    for bad in [dict(kh=5), dict(sh=0), dict(ph=2), dict(mode=3), dict(layout=2), dict(ph=-1)]:
        args = dict(N=1, C=1, H=4, W=4, layout=NCHW, mode=POOL_MAX, kh=2, kw=2, sh=2, sw=2, ph=0, pw=0)
        args.update(bad)
        with pytest.raises(ValueError):
            oracle.pool(x, **args)


# ---------------------------------------------------------------- softmax

def test_softmax_hand_worked_rows():
    z = np.array([[0.0, 0.0]], dtype=np.float32)
    assert oracle.softmax(z).tolist() == [[0.5, 0.5]]
    z = np.array([[0.0, math.log(3.0)]], dtype=np.float32)
    np.testing.assert_allclose(oracle.softmax(z), [[0.25, 0.75]], rtol=1e-7)
    z = np.full((1, 4), 1.7, dtype=np.float32)
    assert oracle.softmax(z).tolist() == [[0.25] * 4]
    z = np.array([[50.0, 0.0, 0.0]], dtype=np.float32)
    out = oracle.softmax(z)[0]
    assert out[0] == np.float32(1.0)
    np.testing.assert_allclose(out[1:], math.exp(-50.0), rtol=1e-6)   # 1.9287e-22
    assert oracle.softmax(np.array([[3.25]], dtype=np.float32)).tolist() == [[1.0]]  # one class


def test_softmax_two_classes_is_logistic():
    rng = np.random.default_rng(21)
    z = (4 * rng.standard_normal((64, 2))).astype(np.float32)
    out = oracle.softmax(z)
    for (a, b), (pa, pb) in zip(z.astype(np.float64), out):
        assert abs(pa - 1.0 / (1.0 + math.exp(-(a - b)))) <= 1e-7
        assert abs(pb - 1.0 / (1.0 + math.exp(-(b - a)))) <= 1e-7


def test_softmax_brute_force_high_precision():
    rng = np.random.default_rng(22)
    z = (3 * rng.standard_normal((5, 37))).astype(np.float32)
    out = oracle.softmax(z)
    for row, got in zip(z, out):
        m = max(float(v) for v in row)
        e = [math.exp(float(v) - m) for v in row]
        s = math.fsum(e)
        want = np.array([v / s for v in e], dtype=np.float32)
        np.testing.assert_array_equal(got, want)       # double result rounded once to fp32


def test_softmax_invariants():
    rng = np.random.default_rng(23)
    z = (3 * rng.standard_normal((16, 1000))).astype(np.float32)
    out = oracle.softmax(z)
    assert np.all(out >= 0) and np.all(out <= 1)
    assert np.all(np.abs(out.astype(np.float64).sum(axis=1) - 1.0) <= 1e-6)   # rows sum to 1
    np.testing.assert_array_equal(out.argmax(axis=1), z.argmax(axis=1))       # argmax kept
    order = np.argsort(z[0], kind="stable")
    assert np.all(np.diff(out[0][order]) >= 0)                                # monotone in logit
    # shift by a power of two keeps these inputs exactly representable
    zq = np.round(z * 64) / 64
    for k in (8.0, 64.0):
        shifted = oracle.softmax((zq + np.float32(k)).astype(np.float32))
        np.testing.assert_array_equal(shifted, oracle.softmax(zq.astype(np.float32)))


def test_softmax_needs_max_subtraction():
    # exp(100) overflows fp32 and exp(800) overflows fp64: only a shifted
    # evaluation gives finite probabilities.
    z = np.array([[100.0, 99.0, 0.0], [800.0, 800.0, -800.0]], dtype=np.float32)
    out = oracle.softmax(z)
    assert np.all(np.isfinite(out))
    np.testing.assert_allclose(out[0, :2], [1 / (1 + math.exp(-1.0)), 1 / (1 + math.exp(1.0))], rtol=1e-7)
    assert out[1].tolist() == [0.5, 0.5, 0.0]


def test_softmax_matches_library_routine_fp64():
    rng = np.random.default_rng(24)
    for n, c in [(3, 1), (4, 10), (7, 1000), (2, 21841)]:
        z = (3 * rng.standard_normal((n, c))).astype(np.float32)
        z[0, rng.integers(0, c)] = 50.0
        want = torch.softmax(torch.from_numpy(z).double(), dim=1).float().numpy()
        got = oracle.softmax(z)
        np.testing.assert_allclose(got, want, rtol=1e-7, atol=1e-12)
        assert abs(float(got.astype(np.float64).sum(axis=1)[0]) - 1.0) <= 1e-5


def test_softmax_ties_at_planted_maximum():
    z = np.zeros((1, 9), dtype=np.float32)
    z[0, [1, 4, 7]] = 50.0
    out = oracle.softmax(z)[0]
    np.testing.assert_allclose(out[[1, 4, 7]], 1 / 3, rtol=1e-7)
    assert np.all(out[[0, 2, 3, 5, 6, 8]] < 1e-21)


def test_oracle_reports_threads():
    assert oracle.threads() >= 1


def test_index_matches_numpy_strides():
    N, C, H, W = 3, 4, 5, 6
    a = np.arange(N * C * H * W).reshape(N, C, H, W)            # NCHW order: value = linear index
    b = np.ascontiguousarray(a.transpose(1, 2, 3, 0))           # CHWN copy
    for (n, c, h, w) in [(0, 0, 0, 0), (2, 3, 4, 5), (1, 2, 3, 4), (2, 0, 4, 1)]:
        assert oracle.index(NCHW, N, C, H, W, n, c, h, w) == a[n, c, h, w]
        assert b.ravel()[oracle.index(CHWN, N, C, H, W, n, c, h, w)] == a[n, c, h, w]
    big = oracle.index(CHWN, 128, 1000, 100, 170, 127, 999, 99, 169)
    assert big == 128 * 1000 * 100 * 170 - 1 and big > 2**31
