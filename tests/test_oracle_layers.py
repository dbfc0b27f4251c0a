"""Pins for the oracle's layer primitives (CPU only).

Each primitive is checked against something that is not the oracle itself: pure-Python brute force on
tiny shapes, torch's CPU fp64 library routines, algebraic identities (adjointness of forward / weight
gradient / data gradient; depthwise-separable == rank-structured full convolution; BatchNorm moments),
and hand-computed numbers.
"""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import block as ob

RNG = np.random.default_rng(12345)


def brute_conv3x3(a, W, s):
    N, Ci, H, Wd = a.shape
    Co = W.shape[0]
    Ho, Wo = (H - 1) // s + 1, (Wd - 1) // s + 1
    z = np.zeros((N, Co, Ho, Wo))
    for n, o, i, j, c, ky, kx in itertools.product(range(N), range(Co), range(Ho), range(Wo), range(Ci), range(3), range(3)):
        y, x = s * i + ky - 1, s * j + kx - 1
        if 0 <= y < H and 0 <= x < Wd:
            z[n, o, i, j] += W[o, c, ky, kx] * a[n, c, y, x]
    return z


@pytest.mark.parametrize("s", [1, 2])
@pytest.mark.parametrize("shape", [(2, 3, 5, 4), (1, 2, 6, 7), (2, 1, 1, 1), (1, 2, 2, 3)])
def test_conv3x3_fwd_brute_force(shape, s):
    a = RNG.standard_normal(shape)
    W = RNG.standard_normal((3, shape[1], 3, 3))
    np.testing.assert_allclose(ob.conv3x3_fwd(a, W, s), brute_conv3x3(a, W, s), rtol=0, atol=1e-13)


@pytest.mark.parametrize("s", [1, 2])
def test_dw_and_1x1_brute_force(s):
    a = RNG.standard_normal((2, 3, 5, 6))
    D = RNG.standard_normal((3, 1, 3, 3))
    # depthwise == full conv whose weight is zero off the channel diagonal
    Wfull = np.zeros((3, 3, 3, 3))
    for c in range(3):
        Wfull[c, c] = D[c, 0]
    np.testing.assert_allclose(ob.dw3x3_fwd(a, D, s), brute_conv3x3(a, Wfull, s), atol=1e-13)
    P = RNG.standard_normal((4, 3))
    z = ob.conv1x1_fwd(a, P, s)
    ref = np.einsum("oc,nchw->nohw", P, a[:, :, ::s, ::s])
    np.testing.assert_allclose(z, ref, atol=1e-13)


@pytest.mark.parametrize("s", [1, 2])
@pytest.mark.parametrize("hw", [(8, 8), (7, 9), (2, 2), (1, 3)])
def test_forward_matches_torch_library(hw, s):
    a = RNG.standard_normal((3, 4) + hw)
    W = RNG.standard_normal((5, 4, 3, 3))
    D = RNG.standard_normal((4, 1, 3, 3))
    P = RNG.standard_normal((6, 4))
    ta = torch.from_numpy(a)
    np.testing.assert_allclose(ob.conv3x3_fwd(a, W, s), F.conv2d(ta, torch.from_numpy(W), stride=s, padding=1).numpy(), atol=1e-12)
    np.testing.assert_allclose(ob.dw3x3_fwd(a, D, s), F.conv2d(ta, torch.from_numpy(D), stride=s, padding=1, groups=4).numpy(), atol=1e-12)
    np.testing.assert_allclose(ob.conv1x1_fwd(a, P, s), F.conv2d(ta, torch.from_numpy(P[:, :, None, None]), stride=s).numpy(), atol=1e-12)


def test_identity_kernels_reproduce_input():
    a = RNG.standard_normal((2, 3, 6, 5))
    D = np.zeros((3, 1, 3, 3))
    D[:, 0, 1, 1] = 1.0
    np.testing.assert_array_equal(ob.dw3x3_fwd(a, D, 1), a)
    np.testing.assert_array_equal(ob.conv1x1_fwd(a, np.eye(3), 1), a)
    W = np.zeros((3, 3, 3, 3))
    for c in range(3):
        W[c, c, 1, 1] = 1.0
    np.testing.assert_array_equal(ob.conv3x3_fwd(a, W, 1), a)
    # a one-pixel shift kernel: tap (ky=1,kx=0) reads the left neighbour, zero at the left border
    D2 = np.zeros((3, 1, 3, 3))
    D2[:, 0, 1, 0] = 1.0
    sh = ob.dw3x3_fwd(a, D2, 1)
    np.testing.assert_array_equal(sh[..., 1:], a[..., :-1])
    np.testing.assert_array_equal(sh[..., 0], 0 * a[..., 0])
    # stride 2 with the centre tap picks the even pixels
    np.testing.assert_array_equal(ob.dw3x3_fwd(a, D, 2), a[:, :, ::2, ::2])


@pytest.mark.parametrize("s", [1, 2])
def test_depthwise_separable_equals_rank_structured_full_conv(s):
    """pw(dw(a)) == conv3x3(a; W) with W[o,c,ky,kx] = P[o,c] * D[c,ky,kx]  (two independent code paths)."""
    a = RNG.standard_normal((2, 5, 7, 6))
    D = RNG.standard_normal((5, 1, 3, 3))
    P = RNG.standard_normal((4, 5))
    W = P[:, :, None, None] * D[None, :, 0]
    ds = ob.conv1x1_fwd(ob.dw3x3_fwd(a, D, s), P, 1)
    np.testing.assert_allclose(ds, ob.conv3x3_fwd(a, W, s), atol=1e-12)


@pytest.mark.parametrize("s", [1, 2])
@pytest.mark.parametrize("hw", [(6, 5), (7, 8), (2, 2)])
def test_backward_primitives_are_adjoints_of_forward(hw, s):
    """<dz, fwd(a, W)> is bilinear: it equals <wgrad(dz,a), W> and <dgrad(dz,W), a>."""
    a = RNG.standard_normal((2, 3) + hw)
    W = RNG.standard_normal((4, 3, 3, 3))
    z = ob.conv3x3_fwd(a, W, s)
    dz = RNG.standard_normal(z.shape)
    ref = np.sum(dz * z)
    assert np.isclose(np.sum(ob.conv3x3_wgrad(dz, a, s) * W), ref, rtol=1e-12)
    assert np.isclose(np.sum(ob.conv3x3_dgrad(dz, W, hw, s) * a), ref, rtol=1e-12)
    D = RNG.standard_normal((3, 1, 3, 3))
    u = ob.dw3x3_fwd(a, D, s)
    du = RNG.standard_normal(u.shape)
    ref = np.sum(du * u)
    assert np.isclose(np.sum(ob.dw3x3_wgrad(du, a, s) * D), ref, rtol=1e-12)
    assert np.isclose(np.sum(ob.dw3x3_dgrad(du, D, hw, s) * a), ref, rtol=1e-12)
    P = RNG.standard_normal((5, 3))
    z1 = ob.conv1x1_fwd(a, P, s)
    dz1 = RNG.standard_normal(z1.shape)
    ref = np.sum(dz1 * z1)
    assert np.isclose(np.sum(ob.conv1x1_wgrad(dz1, a, s) * P), ref, rtol=1e-12)
    assert np.isclose(np.sum(ob.conv1x1_dgrad(dz1, P, hw, s) * a), ref, rtol=1e-12)


@pytest.mark.parametrize("s", [1, 2])
def test_backward_primitives_match_torch_autograd(s):
    a = torch.from_numpy(RNG.standard_normal((2, 3, 7, 6))).requires_grad_()
    W = torch.from_numpy(RNG.standard_normal((4, 3, 3, 3))).requires_grad_()
    D = torch.from_numpy(RNG.standard_normal((3, 1, 3, 3))).requires_grad_()
    z = F.conv2d(a, W, stride=s, padding=1)
    dz = torch.from_numpy(RNG.standard_normal(tuple(z.shape)))
    ga, gW = torch.autograd.grad(z, (a, W), dz)
    np.testing.assert_allclose(ob.conv3x3_wgrad(dz.numpy(), a.detach().numpy(), s), gW.numpy(), atol=1e-12)
    np.testing.assert_allclose(ob.conv3x3_dgrad(dz.numpy(), W.detach().numpy(), (7, 6), s), ga.numpy(), atol=1e-12)
    u = F.conv2d(a, D, stride=s, padding=1, groups=3)
    du = torch.from_numpy(RNG.standard_normal(tuple(u.shape)))
    ga, gD = torch.autograd.grad(u, (a, D), du)
    np.testing.assert_allclose(ob.dw3x3_wgrad(du.numpy(), a.detach().numpy(), s), gD.numpy(), atol=1e-12)
    np.testing.assert_allclose(ob.dw3x3_dgrad(du.numpy(), D.detach().numpy(), (7, 6), s), ga.numpy(), atol=1e-12)


def test_bn_moments_and_special_cases():
    z = 3.0 + 2.0 * RNG.standard_normal((4, 3, 5, 5))
    z[:, 1] = 7.25                                   # a constant channel
    gamma = np.array([1.5, 0.7, -0.4])
    beta = np.array([0.1, -0.2, 0.3])
    eps = 1e-5
    xhat, b, mean, rstd = ob.bn_fwd(z, gamma, beta, eps)
    var = z.var(axis=(0, 2, 3))                      # numpy's default is the biased variance
    np.testing.assert_allclose(mean, z.mean(axis=(0, 2, 3)), rtol=1e-13)
    np.testing.assert_allclose(rstd, 1 / np.sqrt(var + eps), rtol=1e-12)
    np.testing.assert_allclose(xhat.mean(axis=(0, 2, 3)), 0, atol=1e-13)
    np.testing.assert_allclose(xhat.var(axis=(0, 2, 3)), var / (var + eps), rtol=1e-10, atol=1e-13)
    np.testing.assert_array_equal(xhat[:, 1], 0 * xhat[:, 1])
    np.testing.assert_allclose(b, gamma[None, :, None, None] * xhat + beta[None, :, None, None], atol=1e-14)
    tb = F.batch_norm(torch.from_numpy(z), None, None, torch.from_numpy(gamma), torch.from_numpy(beta), True, 0.1, eps)
    np.testing.assert_allclose(b, tb.numpy(), atol=1e-11)


def test_bn_hand_example():
    # one channel, values 1,2,3,4: mean 2.5, biased variance 1.25
    z = np.array([1.0, 2.0, 3.0, 4.0]).reshape(2, 1, 1, 2)
    xhat, b, mean, rstd = ob.bn_fwd(z, np.array([2.0]), np.array([1.0]), 0.0)
    assert mean[0] == 2.5 and np.isclose(rstd[0], 1 / np.sqrt(1.25))
    np.testing.assert_allclose(xhat.ravel(), np.array([-1.5, -0.5, 0.5, 1.5]) / np.sqrt(1.25), rtol=1e-14)
    np.testing.assert_allclose(b.ravel(), 2 * xhat.ravel() + 1, rtol=1e-14)


def test_bn_backward_projections_and_torch():
    z = RNG.standard_normal((3, 4, 5, 2)) + 1.0
    gamma = RNG.uniform(0.5, 1.5, 4)
    beta = RNG.standard_normal(4)
    g = RNG.standard_normal(z.shape)
    xhat, b, mean, rstd = ob.bn_fwd(z, gamma, beta, 1e-5)
    dz, dgamma, dbeta = ob.bn_bwd(g, xhat, gamma, rstd)
    # dz is orthogonal to the constant in every channel, and to xhat up to the eps term:
    # sum dz*xhat = gamma*rstd*dgamma*(1 - sum(xhat^2)/m) = gamma*rstd*dgamma*eps*rstd^2
    np.testing.assert_allclose(dz.sum(axis=(0, 2, 3)), 0, atol=1e-12)
    np.testing.assert_allclose((dz * xhat).sum(axis=(0, 2, 3)), gamma * rstd ** 3 * dgamma * 1e-5, rtol=1e-8, atol=1e-13)
    np.testing.assert_allclose(dbeta, g.sum(axis=(0, 2, 3)), rtol=1e-13)
    np.testing.assert_allclose(dgamma, (g * xhat).sum(axis=(0, 2, 3)), rtol=1e-13)
    tz = torch.from_numpy(z).requires_grad_()
    tg = torch.from_numpy(gamma).requires_grad_()
    tbt = torch.from_numpy(beta).requires_grad_()
    out = F.batch_norm(tz, None, None, tg, tbt, True, 0.1, 1e-5)
    gz, gg, gb = torch.autograd.grad(out, (tz, tg, tbt), torch.from_numpy(g))
    np.testing.assert_allclose(dz, gz.numpy(), atol=1e-11)
    np.testing.assert_allclose(dgamma, gg.numpy(), atol=1e-11)
    np.testing.assert_allclose(dbeta, gb.numpy(), atol=1e-11)


def test_maxpool_first_max_tie_break_and_torch():
    y = np.zeros((1, 1, 2, 4))
    y[0, 0] = [[1.0, 1.0, 0.0, 5.0],
               [1.0, 0.5, 5.0, 5.0]]
    p, arg = ob.maxpool2x2_fwd(y)
    np.testing.assert_array_equal(p[0, 0], [[1.0, 5.0]])
    np.testing.assert_array_equal(arg[0, 0], [[0, 1]])       # first maximum in row-major window order
    dy = ob.maxpool2x2_bwd(np.array([[[[10.0, 20.0]]]]), arg, (2, 4))
    np.testing.assert_array_equal(dy[0, 0], [[10.0, 0, 0, 20.0], [0, 0, 0, 0]])
    # odd sizes: last row / column dropped
    y = RNG.standard_normal((2, 3, 5, 7))
    p, arg = ob.maxpool2x2_fwd(y)
    tp = F.max_pool2d(torch.from_numpy(y), 2)
    np.testing.assert_array_equal(p, tp.numpy())
    ty = torch.from_numpy(y).requires_grad_()
    dp = RNG.standard_normal(p.shape)
    (gy,) = torch.autograd.grad(F.max_pool2d(ty, 2), ty, torch.from_numpy(dp))
    np.testing.assert_array_equal(ob.maxpool2x2_bwd(dp, arg, (5, 7)), gy.numpy())


def test_loss_hand_example():
    """Eq. 3 on a 2-image batch of 2-element feature maps, worked by hand in tests/golden."""
    import json
    import os
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "loss_hand_example.json")))
    p = np.array(g["student"]).reshape(2, 1, 2, 1)
    t = np.array(g["teacher"]).reshape(2, 1, 2, 1)
    np.testing.assert_array_equal(((p - t) ** 2).sum(axis=(1, 2, 3)), g["per_image_squared_norm"])
    assert ob.local_loss(p, t, 1) == (g["eq3_sum_over_batch_size"], 2)
    assert ob.local_loss(p, t, 0) == (g["mean_over_elements"], 4)
