"""Pins of the oracle's backward passes: hand-worked cases, conservation laws, finite
differences of the (already pinned) forward oracle, and torch's autograd in float64."""
import numpy as np
import pytest
import torch

import oracle


def test_max_pool_backward_hand_worked_with_ties():
    # 1x1x2x4, window 2x2 / stride 2: windows [[1, 5], [5, 0]] and [[2, 2], [2, 2]]
    x = np.array([[1, 5, 2, 2], [5, 0, 2, 2]], dtype=np.float32).reshape(1, 1, 2, 4)
    dy = np.array([10.0, 7.0], dtype=np.float32).reshape(1, 1, 1, 2)
    dx = oracle.pool_backward(x, dy, 1, 1, 2, 4, 0, 0, 2, 2, 2, 2)
    # first maximum in scan order: (0,1) for the left window, (0,2) for the right one
    assert dx.reshape(2, 4).tolist() == [[0, 10, 7, 0], [0, 0, 0, 0]]


def test_avg_pool_backward_hand_worked_overlap():
    # 1-D flavour: 1x1x1x5, window 1x3 / stride 2 -> outputs cover columns 0-2 and 2-4
    dy = np.array([3.0, 6.0], dtype=np.float32).reshape(1, 1, 1, 2)
    dx = oracle.pool_backward(None, dy, 1, 1, 1, 5, 0, 1, 1, 3, 1, 2)
    assert np.allclose(dx.ravel(), [1, 1, 3, 2, 2])


@pytest.mark.parametrize("k,s,p", [(2, 2, 0), (3, 2, 0), (3, 1, 1), (3, 2, 1), (5, 3, 2)])
@pytest.mark.parametrize("mode", [0, 1])
def test_pool_backward_is_torch_autograd(k, s, p, mode):
    rng = np.random.default_rng(k * 10 + s + mode)
    N, C, H, W = 2, 3, 11, 13
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    x[0, 0, :4, :4] = 1.5                                          # a block of ties
    xt = torch.from_numpy(x).double().requires_grad_(True)
    if mode == 0:
        y = torch.nn.functional.max_pool2d(xt, k, s, p)
    else:
        y = torch.nn.functional.avg_pool2d(xt, k, s, p, count_include_pad=True)
    dy = rng.standard_normal(tuple(y.shape)).astype(np.float32)
    y.backward(torch.from_numpy(dy).double())
    want = xt.grad.numpy()
    got = oracle.pool_backward(x, dy, N, C, H, W, oracle.NCHW, mode, k, k, s, s, p, p)
    assert np.allclose(got, want, rtol=1e-6, atol=1e-6)
    # CHWN gives the same numbers in the other order
    xc = oracle.transform(x, N, C, H, W, 0, 1)
    Ho, Wo = y.shape[2], y.shape[3]
    dyc = oracle.transform(dy, N, C, Ho, Wo, 0, 1)
    gotc = oracle.pool_backward(xc, dyc, N, C, H, W, oracle.CHWN, mode, k, k, s, s, p, p)
    assert np.array_equal(oracle.transform(gotc, N, C, H, W, 1, 0), got)


def test_pool_backward_conserves_the_gradient_without_padding():
    rng = np.random.default_rng(3)
    N, C, H, W = 2, 2, 9, 9
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    dy = rng.standard_normal((N, C, 4, 4)).astype(np.float32)
    for mode in (0, 1):
        dx = oracle.pool_backward(x, dy, N, C, H, W, 0, mode, 3, 3, 2, 2)
        assert np.allclose(dx.sum(axis=(2, 3), dtype=np.float64), dy.sum(axis=(2, 3), dtype=np.float64), atol=1e-5)


def test_avg_pool_backward_is_the_adjoint_of_the_forward():
    # <pool(x), dy> == <x, pool_backward(dy)> for the linear (average) case
    rng = np.random.default_rng(4)
    N, C, H, W = 2, 3, 10, 12
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    y = oracle.pool(x, N, C, H, W, 0, 1, 3, 3, 2, 2, 1, 1)
    dy = rng.standard_normal(y.shape).astype(np.float32)
    dx = oracle.pool_backward(None, dy, N, C, H, W, 0, 1, 3, 3, 2, 2, 1, 1)
    assert abs(np.vdot(y.astype(np.float64), dy) - np.vdot(x.astype(np.float64), dx)) < 1e-4


def test_softmax_backward_hand_worked():
    p = np.array([[0.5, 0.5]], dtype=np.float32)
    dp = np.array([[1.0, 0.0]], dtype=np.float32)
    # dot = 0.5 -> dz = [0.5 * 0.5, 0.5 * -0.5]
    assert oracle.softmax_backward(p, dp).tolist() == [[0.25, -0.25]]
    # a gradient that is constant along the row changes nothing (rows of p sum to one)
    p = oracle.softmax(np.array([[1.0, 2.0, 3.0, -1.0]], dtype=np.float32))
    assert np.allclose(oracle.softmax_backward(p, np.full_like(p, 3.0)), 0, atol=1e-6)


def test_softmax_backward_is_torch_autograd_and_finite_differences():
    rng = np.random.default_rng(5)
    z = (rng.standard_normal((7, 33)) * 2).astype(np.float32)
    dp = rng.standard_normal((7, 33)).astype(np.float32)
    zt = torch.from_numpy(z).double().requires_grad_(True)
    pt = torch.softmax(zt, dim=1)
    pt.backward(torch.from_numpy(dp).double())
    p = pt.detach().numpy().astype(np.float32)
    got = oracle.softmax_backward(p, dp)
    assert np.allclose(got, zt.grad.numpy(), rtol=1e-5, atol=1e-7)
    # finite difference of the forward oracle along one coordinate
    eps = 1e-3
    zp, zm = z.copy(), z.copy()
    zp[2, 5] += eps
    zm[2, 5] -= eps
    fd = ((oracle.softmax(zp).astype(np.float64) - oracle.softmax(zm)) * dp).sum() / (2 * eps)
    assert abs(fd - got[2, 5]) < 2e-3 * max(1.0, abs(got[2, 5]))
    assert np.all(np.abs(got.sum(axis=1)) < 1e-5)                 # gradients of a row sum to zero
