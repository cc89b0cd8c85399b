"""Pins of the oracle's 16-bit storage variants (fp16 = IEEE binary16, bf16 = upper
half of binary32).  The conversions are pinned exhaustively against numpy's /
torch's own conversions; the layer functions are pinned against library routines
run in float64 on the widened inputs, and against the defining property of a
correctly rounded result (no neighbouring 16-bit value is closer to the exact one)."""
import numpy as np
import pytest
import torch

import oracle

F16, BF16 = oracle.F16, oracle.BF16
ALL = np.arange(65536, dtype=np.uint32).astype(np.uint16)


def widen(bits, dtype):
    """Library widening of uint16 patterns to float64 (numpy for fp16, bit shift for bf16)."""
    bits = np.asarray(bits, dtype=np.uint16)
    if dtype == F16:
        return bits.view(np.float16).astype(np.float64)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def from_f32(x, dtype):
    """Library narrowing of float32 values (numpy for fp16, torch for bf16)."""
    x = np.asarray(x, dtype=np.float32)
    if dtype == F16:
        return x.astype(np.float16).view(np.uint16)
    return torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


@pytest.mark.parametrize("dtype", [F16, BF16])
def test_widening_is_exhaustively_the_library_value(dtype):
    want = widen(ALL, dtype)
    got = np.array([oracle.widen16(int(b), dtype) for b in ALL])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


@pytest.mark.parametrize("dtype", [F16, BF16])
def test_narrowing_inverts_widening_for_every_pattern(dtype):
    vals = widen(ALL, dtype)
    for b, v in zip(ALL, vals):
        if np.isnan(v):
            continue
        assert oracle.narrow16(float(v), dtype) == int(b)


@pytest.mark.parametrize("dtype", [F16, BF16])
def test_narrowing_rounds_midpoints_to_even_and_matches_library(dtype):
    # midpoints between consecutive positive finite values are exact in float32 for both formats
    last_finite = 0x7bff if dtype == F16 else 0x7f7f
    lo = np.arange(0, last_finite, dtype=np.uint32).astype(np.uint16)
    a, b = widen(lo, dtype), widen(lo + 1, dtype)
    mid = (a + b) / 2
    f32 = mid.astype(np.float32)
    exact = f32.astype(np.float64) == mid
    lib = from_f32(f32, dtype)
    for k in range(0, lo.size, 7):
        got = oracle.narrow16(float(mid[k]), dtype)
        assert got in (int(lo[k]), int(lo[k]) + 1)
        assert got % 2 == 0                                  # the even neighbour
        if exact[k]:
            assert got == int(lib[k])
        # just off the midpoint the nearer neighbour wins
        assert oracle.narrow16(float(np.nextafter(mid[k], np.inf)), dtype) == int(lo[k]) + 1
        assert oracle.narrow16(float(np.nextafter(mid[k], -np.inf)), dtype) == int(lo[k])


@pytest.mark.parametrize("dtype", [F16, BF16])
def test_narrowing_matches_library_on_random_float32(dtype):
    rng = np.random.default_rng(16)
    x = np.concatenate([rng.standard_normal(4000) * s for s in (1e-8, 1e-5, 1e-3, 1.0, 50.0, 3e4, 1e6)]).astype(np.float32)
    lib = from_f32(x, dtype)
    got = np.array([oracle.narrow16(float(v), dtype) for v in x], dtype=np.uint16)
    assert np.array_equal(got, lib)


def test_fp16_narrowing_from_double_matches_numpy_single_rounding():
    rng = np.random.default_rng(17)
    x = np.concatenate([rng.standard_normal(3000) * s for s in (1e-8, 6e-8, 1e-5, 1.0, 1000.0, 7e4)])
    lib = x.astype(np.float16).view(np.uint16)               # numpy rounds double -> half in one step
    got = np.array([oracle.narrow16(float(v), F16) for v in x], dtype=np.uint16)
    assert np.array_equal(got, lib)


def test_special_values():
    assert oracle.narrow16(65504.0, F16) == 0x7bff and oracle.narrow16(65519.999, F16) == 0x7bff
    assert oracle.narrow16(65520.0, F16) == 0x7c00          # tie between max and 2^16 goes to the even one: infinity
    assert oracle.narrow16(float("inf"), F16) == 0x7c00 and oracle.narrow16(float("-inf"), BF16) == 0xff80
    assert oracle.narrow16(0.0, F16) == 0 and oracle.narrow16(-0.0, BF16) == 0x8000
    assert oracle.narrow16(2.0 ** -24, F16) == 1 and oracle.narrow16(2.0 ** -25, F16) == 0   # tie to even (zero)
    assert oracle.narrow16(2.0 ** -25 * 1.0001, F16) == 1
    assert oracle.narrow16(1.0, BF16) == 0x3f80 and oracle.narrow16(1.0 + 2.0 ** -8, BF16) == 0x3f80
    assert oracle.narrow16(1.0 + 3 * 2.0 ** -8, BF16) == 0x3f82
    assert np.isnan(oracle.widen16(oracle.narrow16(float("nan"), F16), F16))


def nearest_ok(out_bits, exact, dtype):
    """Every output is a 16-bit value with no closer neighbour to the exact result."""
    out_bits = out_bits.astype(np.int64)
    v = widen(out_bits.astype(np.uint16), dtype)
    err = np.abs(v - exact)
    mag = out_bits & 0x7fff
    up = widen(np.where(mag < 0x7fff, out_bits + 1, out_bits).astype(np.uint16), dtype)
    dn_bits = np.where(mag > 0, out_bits - 1, out_bits ^ 0x8000)      # below +0 comes -0 (same value)
    dn = widen(dn_bits.astype(np.uint16), dtype)
    with np.errstate(invalid="ignore"):
        ok_up = ~np.isfinite(up) | (err <= np.abs(up - exact))
        ok_dn = ~np.isfinite(dn) | (err <= np.abs(dn - exact))
    return bool(np.all(ok_up & ok_dn))


def make16(rng, shape, dtype, relu=True, scale=1.0):
    x = rng.standard_normal(shape).astype(np.float32) * np.float32(scale)
    if relu:
        x = np.maximum(x, 0)
    return from_f32(x, dtype).reshape(shape)


def test_transform16_is_numpy_transpose():
    rng = np.random.default_rng(18)
    N, C, H, W = 3, 4, 5, 6
    x = rng.integers(0, 65536, size=(N, C, H, W)).astype(np.uint16)
    y = oracle.transform16(x, N, C, H, W, oracle.NCHW, oracle.CHWN)
    assert np.array_equal(y, x.transpose(1, 2, 3, 0))
    assert np.array_equal(oracle.transform16(y, N, C, H, W, oracle.CHWN, oracle.NCHW), x)


@pytest.mark.parametrize("dtype", [F16, BF16])
@pytest.mark.parametrize("k,s,p", [(2, 2, 0), (3, 2, 0), (3, 1, 1), (3, 2, 1)])
def test_pool16_against_float64_library_pooling(dtype, k, s, p):
    rng = np.random.default_rng(19 + k + s)
    N, C, H, W = 2, 3, 11, 13
    x = make16(rng, (N, C, H, W), dtype, relu=False, scale=3.0)
    xd = torch.from_numpy(widen(x, dtype))
    got_max = oracle.pool16(x, N, C, H, W, oracle.NCHW, oracle.POOL_MAX, k, k, s, s, p, p, dtype)
    want_max = torch.nn.functional.max_pool2d(xd, k, s, p).numpy()
    assert np.array_equal(widen(got_max, dtype), want_max)              # the maximum is one of the inputs, exactly
    got_avg = oracle.pool16(x, N, C, H, W, oracle.NCHW, oracle.POOL_AVG, k, k, s, s, p, p, dtype)
    exact = torch.nn.functional.avg_pool2d(xd, k, s, p, count_include_pad=True).numpy()
    assert nearest_ok(got_avg, exact, dtype)
    if dtype == F16:
        assert np.array_equal(got_avg, exact.astype(np.float16).view(np.uint16))
    # CHWN gives the same numbers in the other order
    xc = oracle.transform16(x, N, C, H, W, oracle.NCHW, oracle.CHWN)
    got_c = oracle.pool16(xc, N, C, H, W, oracle.CHWN, oracle.POOL_AVG, k, k, s, s, p, p, dtype)
    Ho, Wo = oracle.pool_out_dims(H, W, k, k, s, s, p, p)
    assert np.array_equal(oracle.transform16(got_c, N, C, Ho, Wo, oracle.CHWN, oracle.NCHW), got_avg)


def test_pool16_hand_worked():
    # 1x1x2x2, window 2: fp16 values 1, 2, 3, 4.5 -> max 4.5, mean 2.625 (exact in fp16)
    x = np.array([1.0, 2.0, 3.0, 4.5], dtype=np.float16).view(np.uint16).reshape(1, 1, 2, 2)
    assert oracle.pool16(x, 1, 1, 2, 2, 0, 0, 2, 2, 2, 2, dtype=F16).view(np.float16).item() == 4.5
    assert oracle.pool16(x, 1, 1, 2, 2, 0, 1, 2, 2, 2, 2, dtype=F16).view(np.float16).item() == 2.625
    # bf16 keeps 8 significant bits: mean of 1, 1, 1, 1.0078125 = 1.001953125 -> rounds to 1.0
    b = from_f32(np.array([1.0, 1.0, 1.0, 1.0078125], dtype=np.float32), BF16).reshape(1, 1, 2, 2)
    assert oracle.pool16(b, 1, 1, 2, 2, 0, 1, 2, 2, 2, 2, dtype=BF16).item() == 0x3f80
    # mean of 1, 1.0078125 x3 = 1.005859375: nearer to 1.0078125 (0x3f81) than to 1.0
    b = from_f32(np.array([1.0, 1.0078125, 1.0078125, 1.0078125], dtype=np.float32), BF16).reshape(1, 1, 2, 2)
    assert oracle.pool16(b, 1, 1, 2, 2, 0, 1, 2, 2, 2, 2, dtype=BF16).item() == 0x3f81


@pytest.mark.parametrize("dtype", [F16, BF16])
def test_softmax16_is_the_correctly_rounded_float64_softmax(dtype):
    rng = np.random.default_rng(23)
    z = make16(rng, (17, 301), dtype, relu=False, scale=3.0)
    z[0, 5] = from_f32(np.array([40.0], dtype=np.float32), dtype)[0]    # an outlier row
    got = oracle.softmax16(z, dtype)
    exact = torch.softmax(torch.from_numpy(widen(z, dtype)), dim=1).numpy()
    assert nearest_ok(got, exact, dtype)
    if dtype == F16:
        assert np.array_equal(got, exact.astype(np.float16).view(np.uint16))
    assert np.all(np.abs(widen(got, dtype).sum(axis=1) - 1.0) < (3e-3 if dtype == F16 else 2e-2))


@pytest.mark.parametrize("dtype", [F16, BF16])
def test_softmax16_hand_rows(dtype):
    one, half, quarter = (oracle.narrow16(v, dtype) for v in (1.0, 0.5, 0.25))
    z = np.array([[0, 0]], dtype=np.uint16)
    assert oracle.softmax16(z, dtype).tolist() == [[half, half]]
    z = from_f32(np.array([[3.0, 3.0, 3.0, 3.0]], dtype=np.float32), dtype).reshape(1, 4)
    assert oracle.softmax16(z, dtype).tolist() == [[quarter] * 4]
    z = from_f32(np.array([[7.0]], dtype=np.float32), dtype).reshape(1, 1)
    assert oracle.softmax16(z, dtype).tolist() == [[one]]
    z = from_f32(np.array([[60.0, 0.0]], dtype=np.float32), dtype).reshape(1, 2)   # e^-60 underflows both formats' ... fp16 only
    out = oracle.softmax16(z, dtype)
    assert out[0, 0] == one
    assert out[0, 1] == (0 if dtype == F16 else oracle.narrow16(np.exp(-60.0) / (1 + np.exp(-60.0)), dtype))


def test_permute16_is_numpy_transpose_for_every_permutation():
    import itertools
    rng = np.random.default_rng(29)
    dims = (3, 4, 5, 6)
    x = rng.integers(0, 65536, size=dims).astype(np.uint16)
    for perm in itertools.permutations(range(4)):
        got = oracle.permute16(x, dims, perm)
        assert np.array_equal(got, x.transpose(perm)), perm
    # hand-worked: 1x2x1x3 [c][w] = [[0,1,2],[3,4,5]] with the last two real axes swapped -> [[0,3],[1,4],[2,5]]
    y = oracle.permute16(np.arange(6, dtype=np.uint16).reshape(1, 2, 1, 3), (1, 2, 1, 3), (0, 2, 3, 1))
    assert y.ravel().tolist() == [0, 3, 1, 4, 2, 5]
