"""Pins for the CPU oracle's primitives (BN, ReLU, conv) against things other
than the oracle itself: definitions written out by brute force, closed-form
invariants, adjoint identities, textbook special cases and float64 library
routines.  A dropped term, wrong sign/index or transposed operand in
oracle/dnb_oracle.c fails at least one of these."""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F


def rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------ conv

def brute_conv(x, w):
    """Definition written out on an explicitly zero-padded copy (cross-correlation)."""
    n, ci, H, W = x.shape
    co, _, ks, _ = w.shape
    pad = (ks - 1) // 2
    xp = np.zeros((n, ci, H + 2 * pad, W + 2 * pad))
    xp[:, :, pad:pad + H, pad:pad + W] = x
    out = np.zeros((n, co, H, W))
    for b, o, y, xx in itertools.product(range(n), range(co), range(H), range(W)):
        s = 0.0
        for c, i, j in itertools.product(range(ci), range(ks), range(ks)):
            s += w[o, c, i, j] * xp[b, c, y + i, xx + j]
        out[b, o, y, xx] = s
    return out


@pytest.mark.parametrize("ks,shape", [(1, (2, 3, 4, 5)), (3, (2, 3, 4, 5)), (3, (1, 2, 1, 1)), (3, (1, 1, 2, 3))])
def test_conv_forward_bruteforce(oracle, ks, shape):
    r = rng(10)
    x = r.standard_normal(shape)
    w = r.standard_normal((4, shape[1], ks, ks))
    np.testing.assert_allclose(oracle.conv_forward(x, w), brute_conv(x, w), rtol=0, atol=1e-13)


@pytest.mark.parametrize("ks", [1, 3])
def test_conv_matches_library_float64(oracle, ks):
    r = rng(11)
    x = r.standard_normal((3, 5, 7, 6))
    w = r.standard_normal((4, 5, ks, ks))
    g = r.standard_normal((3, 4, 7, 6))
    xt = torch.tensor(x, requires_grad=True)
    wt = torch.tensor(w, requires_grad=True)
    out = F.conv2d(xt, wt, padding=(ks - 1) // 2)
    out.backward(torch.tensor(g))
    np.testing.assert_allclose(oracle.conv_forward(x, w), out.detach().numpy(), atol=1e-12)
    np.testing.assert_allclose(oracle.conv_dgrad(g, w), xt.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(oracle.conv_wgrad(x, g, ks), wt.grad.numpy(), atol=1e-11)


def test_conv_center_tap_equals_1x1(oracle):
    r = rng(12)
    x = r.standard_normal((2, 4, 5, 5))
    w1 = r.standard_normal((3, 4, 1, 1))
    w3 = np.zeros((3, 4, 3, 3))
    w3[:, :, 1, 1] = w1[:, :, 0, 0]
    np.testing.assert_array_equal(oracle.conv_forward(x, w3), oracle.conv_forward(x, w1))


def test_conv_single_tap_is_a_shift(oracle):
    """A 3x3 kernel with only tap (i,j) set copies the input shifted by (i-1,j-1):
    pins the correlation (not convolution) orientation and the padding."""
    x = rng(13).standard_normal((1, 1, 4, 5))
    for i, j in itertools.product(range(3), range(3)):
        w = np.zeros((1, 1, 3, 3))
        w[0, 0, i, j] = 1.0
        out = oracle.conv_forward(x, w)[0, 0]
        exp = np.zeros((4, 5))
        for y, xx in itertools.product(range(4), range(5)):
            yy, xs = y + i - 1, xx + j - 1
            if 0 <= yy < 4 and 0 <= xs < 5:
                exp[y, xx] = x[0, 0, yy, xs]
        np.testing.assert_array_equal(out, exp)


@pytest.mark.parametrize("ks", [1, 3])
def test_conv_adjoint_identities(oracle, ks):
    """<conv(a,W), g> = <a, dgrad(g,W)> = <W, wgrad(a,g)>."""
    r = rng(14)
    a = r.standard_normal((2, 6, 5, 4))
    w = r.standard_normal((3, 6, ks, ks))
    g = r.standard_normal((2, 3, 5, 4))
    lhs = np.sum(oracle.conv_forward(a, w) * g)
    assert abs(lhs - np.sum(a * oracle.conv_dgrad(g, w))) < 1e-10 * max(1.0, abs(lhs))
    assert abs(lhs - np.sum(w * oracle.conv_wgrad(a, g, ks))) < 1e-10 * max(1.0, abs(lhs))


def test_conv_1x1_is_a_matmul(oracle):
    r = rng(15)
    x = r.standard_normal((2, 5, 3, 3))
    w = r.standard_normal((4, 5, 1, 1))
    exp = np.einsum("oc,nchw->nohw", w[:, :, 0, 0], x)
    np.testing.assert_allclose(oracle.conv_forward(x, w), exp, atol=1e-13)


# ------------------------------------------------------------------- BN

def test_bn_forward_invariants(oracle):
    """Pre-affine normalised values: mean 0, biased variance v/(v+eps)."""
    r = rng(20)
    u = r.standard_normal((4, 6, 5, 3)) * r.uniform(0.1, 5, (1, 6, 1, 1)) + r.uniform(-3, 3, (1, 6, 1, 1))
    eps = 1e-5
    xhat, mean, var = oracle.bn_forward(u, np.ones(6), np.zeros(6), eps)
    np.testing.assert_allclose(mean, u.mean(axis=(0, 2, 3)), atol=1e-13)
    np.testing.assert_allclose(var, u.var(axis=(0, 2, 3)), rtol=1e-12)  # numpy var is biased
    assert np.max(np.abs(xhat.mean(axis=(0, 2, 3)))) < 1e-12
    np.testing.assert_allclose(xhat.var(axis=(0, 2, 3)), var / (var + eps), rtol=1e-11)


def test_bn_forward_affine_and_library(oracle):
    r = rng(21)
    u = r.standard_normal((3, 4, 2, 5)) * 2 + 1
    g, b = r.standard_normal(4), r.standard_normal(4)
    z, mean, var = oracle.bn_forward(u, g, b, 1e-5)
    xhat, _, _ = oracle.bn_forward(u, np.ones(4), np.zeros(4), 1e-5)
    np.testing.assert_allclose(z, g[None, :, None, None] * xhat + b[None, :, None, None], atol=1e-13)
    zt = F.batch_norm(torch.tensor(u), None, None, torch.tensor(g), torch.tensor(b), True, 0.0, 1e-5)
    np.testing.assert_allclose(z, zt.numpy(), atol=1e-12)


def test_bn_eps_is_inside_the_square_root(oracle):
    """With a constant channel (variance 0) the output is beta and stays finite;
    with variance v the scale is exactly 1/sqrt(v+eps)."""
    u = np.full((2, 1, 2, 2), 3.0)
    z, mean, var = oracle.bn_forward(u, [2.0], [0.5], 1e-5)
    np.testing.assert_array_equal(z, np.full_like(u, 0.5))
    u = np.array([1.0, -1.0]).reshape(2, 1, 1, 1)  # mean 0, biased var 1
    z, mean, var = oracle.bn_forward(u, [1.0], [0.0], 0.21)
    np.testing.assert_allclose(z.ravel(), np.array([1.0, -1.0]) / np.sqrt(1.21), rtol=1e-15)


def test_bn_backward_invariants_and_library(oracle):
    """Closed-form properties of the BN gradient: per channel sum(du)=0 and
    sum(du*xhat) = gamma*istd*dgamma*eps/(var+eps) (zero as eps -> 0); and equality
    with float64 autograd of the library routine."""
    r = rng(22)
    u = r.standard_normal((3, 5, 4, 4)) * 1.7 - 0.4
    g, b = r.standard_normal(5), r.standard_normal(5)
    dz = r.standard_normal(u.shape)
    eps = 1e-5
    _, mean, var = oracle.bn_forward(u, g, b, eps)
    xhat, _, _ = oracle.bn_forward(u, np.ones(5), np.zeros(5), eps)
    du, dg, db = oracle.bn_backward(u, dz, g, mean, var, eps)
    assert np.max(np.abs(du.sum(axis=(0, 2, 3)))) < 1e-12
    # sum(du*xhat) = gamma*istd*dgamma*(1 - sum(xhat^2)/P) = gamma*istd*dgamma*eps/(var+eps)
    closed = g / np.sqrt(var + eps) * dg * eps / (var + eps)
    np.testing.assert_allclose((du * xhat).sum(axis=(0, 2, 3)), closed, atol=1e-12)
    np.testing.assert_allclose(db, dz.sum(axis=(0, 2, 3)), atol=1e-12)
    np.testing.assert_allclose(dg, (dz * xhat).sum(axis=(0, 2, 3)), atol=1e-12)
    ut = torch.tensor(u, requires_grad=True)
    gt = torch.tensor(g, requires_grad=True)
    bt = torch.tensor(b, requires_grad=True)
    F.batch_norm(ut, None, None, gt, bt, True, 0.0, eps).backward(torch.tensor(dz))
    np.testing.assert_allclose(du, ut.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dg, gt.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(db, bt.grad.numpy(), atol=1e-12)


def test_bn_backward_finite_difference(oracle):
    r = rng(23)
    u = r.standard_normal((2, 2, 3, 2))
    g, b = r.standard_normal(2) + 1.5, r.standard_normal(2)
    t = r.standard_normal(u.shape)
    eps = 1e-3

    def loss(uu):
        return float(np.sum(oracle.bn_forward(uu, g, b, eps)[0] * t))

    _, mean, var = oracle.bn_forward(u, g, b, eps)
    du, _, _ = oracle.bn_backward(u, t, g, mean, var, eps)
    h = 1e-6
    for idx in itertools.product(*[range(s) for s in u.shape]):
        up, um = u.copy(), u.copy()
        up[idx] += h
        um[idx] -= h
        fd = (loss(up) - loss(um)) / (2 * h)
        assert abs(fd - du[idx]) < 1e-7 * max(1.0, abs(fd))


# ----------------------------------------------------------------- ReLU

def test_relu_and_its_derivative_at_zero(oracle):
    z = np.array([-2.0, -0.0, 0.0, 1e-300, 3.0])
    a = oracle.relu(z)
    np.testing.assert_array_equal(a, np.array([0.0, 0.0, 0.0, 1e-300, 3.0]))
    np.testing.assert_array_equal(oracle.relu_backward(a, np.ones(5)), np.array([0.0, 0.0, 0.0, 1.0, 1.0]))
