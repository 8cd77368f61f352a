"""Pins for the oracle of the non-convolutional layers (Section 4.1's layer list): closed
forms, special cases that reduce to other routines, finite differences, brute force."""
import itertools
import math

import numpy as np
import pytest

import oracle
from oracle import netlayers as on

RNG = np.random.default_rng(20171202)


def numeric_grad(f, x, h=1e-6):
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        xp, xm = x.copy(), x.copy()
        xp[i] += h
        xm[i] -= h
        g[i] = (f(xp) - f(xm)) / (2 * h)
    return g


# ---- normalisation -------------------------------------------------------------------------
def test_norm_window_of_one_is_a_pointwise_closed_form():
    x = RNG.normal(size=(2, 3, 2, 2))
    y = on.norm_fwd(x, size=1, kappa=2.0, alpha=0.5, beta=0.75)
    assert np.allclose(y, x * (2.0 + 0.5 * x * x) ** -0.75, rtol=1e-14)


def test_norm_window_covering_all_channels_uses_the_whole_pixel_energy():
    x = RNG.normal(size=(2, 3, 2, 2))
    y = on.norm_fwd(x, size=7, kappa=1.0, alpha=0.1, beta=0.5)
    energy = (x ** 2).sum(axis=1, keepdims=True)
    assert np.allclose(y, x / np.sqrt(1.0 + 0.1 * energy), rtol=1e-14)


def test_norm_windows_are_centred_and_clipped():
    x = np.zeros((1, 6, 1, 1))
    x[0, :, 0, 0] = [1, 2, 3, 4, 5, 6]
    s = on.norm_scale(x, size=3, kappa=0.0, alpha=1.0)[0, :, 0, 0]
    assert s.tolist() == [1 + 4, 1 + 4 + 9, 4 + 9 + 16, 9 + 16 + 25, 16 + 25 + 36, 25 + 36]


def test_norm_backward_is_the_gradient():
    x = RNG.normal(size=(2, 6, 2, 2))
    dy = RNG.normal(size=x.shape)
    kw = dict(size=5, kappa=1.5, alpha=0.3, beta=0.75)
    g = numeric_grad(lambda v: float(np.sum(on.norm_fwd(v, **kw) * dy)), x)
    assert np.allclose(on.norm_bwd(x, dy, **kw), g, rtol=1e-6, atol=1e-8)


# ---- pooling -------------------------------------------------------------------------------
def test_pool_known_values_and_extent():
    x = np.arange(16.0).reshape(1, 1, 4, 4)
    assert on.pool_fwd(x, 2, 2)[0, 0].tolist() == [[5, 7], [13, 15]]
    assert on.pool_fwd(np.zeros((1, 1, 28, 28)), 2, 2).shape == (1, 1, 14, 14)   # the paper's 28 -> 14
    assert on.pool_fwd(np.zeros((1, 1, 10, 10)), 2, 2).shape == (1, 1, 5, 5)
    assert on.pool_fwd(np.zeros((1, 1, 7, 7)), 3, 2).shape == (1, 1, 3, 3)


def test_pool_brute_force_and_gradient_routing():
    x = RNG.normal(size=(2, 3, 7, 6))
    y = on.pool_fwd(x, 3, 2)
    dy = RNG.normal(size=y.shape)
    dx = on.pool_bwd(x, dy, 3, 2)
    want = np.zeros_like(x)
    for n, c, p, q in itertools.product(range(2), range(3), range(y.shape[2]), range(y.shape[3])):
        best, arg = -math.inf, None
        for i, j in itertools.product(range(3), range(3)):
            v = x[n, c, 2 * p + i, 2 * q + j]
            if v > best:
                best, arg = v, (2 * p + i, 2 * q + j)
        assert y[n, c, p, q] == best
        want[n, c, arg[0], arg[1]] += dy[n, c, p, q]
    assert np.array_equal(dx, want)
    assert math.isclose(dx.sum(), dy.sum(), rel_tol=1e-12)      # every window passes its gradient to one input


def test_pool_ties_go_to_the_first_maximum():
    x = np.ones((1, 1, 2, 2))
    assert on.pool_bwd(x, np.full((1, 1, 1, 1), 3.0), 2, 2)[0, 0].tolist() == [[3.0, 0.0], [0.0, 0.0]]


# ---- fully connected -----------------------------------------------------------------------
def test_fc_is_a_convolution_with_filters_as_large_as_the_input():
    x = RNG.normal(size=(3, 4, 5, 5))
    W = RNG.normal(size=(7, 4 * 5 * 5))
    sh = oracle.Shape(3, 4, 5, 5, 7, 5, 5, 1, 1, 0, 0, 0, 7)
    y_conv = oracle.conv_fwd(sh, x, W.reshape(7, 4, 5, 5))[:, :, 0, 0]
    assert np.allclose(on.fc_fwd(x, W, np.zeros(7)), y_conv, rtol=1e-12)
    dy = RNG.normal(size=(3, 7))
    dx, dW, db = on.fc_bwd(x, W, dy)
    assert np.allclose(dx, oracle.conv_bwd_data(sh, dy.reshape(3, 7, 1, 1), W.reshape(7, 4, 5, 5)), rtol=1e-12)
    assert np.allclose(dW.reshape(7, 4, 5, 5), oracle.conv_bwd_weight(sh, x, dy.reshape(3, 7, 1, 1)), rtol=1e-12)
    assert np.allclose(db, dy.sum(axis=0))


def test_fc_brute_force_with_bias():
    x = RNG.normal(size=(2, 6))
    W = RNG.normal(size=(3, 6))
    b = RNG.normal(size=3)
    y = on.fc_fwd(x, W, b)
    for n, o in itertools.product(range(2), range(3)):
        assert math.isclose(y[n, o], sum(x[n, i] * W[o, i] for i in range(6)) + b[o], rel_tol=1e-12, abs_tol=1e-14)


# ---- softmax loss --------------------------------------------------------------------------
def test_softmax_loss_closed_forms():
    z = np.zeros((4, 10))
    assert math.isclose(on.softmax_loss_fwd(z, [0, 3, 9, 5]), math.log(10), rel_tol=1e-15)   # ten CIFAR classes
    z = np.array([[math.log(1), math.log(2), math.log(5)]])
    assert math.isclose(on.softmax_loss_fwd(z, [2]), -math.log(5 / 8), rel_tol=1e-14)
    assert np.allclose(on.softmax(z), [[1 / 8, 2 / 8, 5 / 8]], rtol=1e-14)
    # invariance under a shift of the logits, also a huge one
    assert math.isclose(on.softmax_loss_fwd(z + 1e4, [2]), -math.log(5 / 8), rel_tol=1e-10)


def test_softmax_loss_backward_is_the_gradient_and_sums_to_zero():
    z = RNG.normal(size=(5, 10))
    labels = [1, 0, 9, 3, 3]
    g = numeric_grad(lambda v: on.softmax_loss_fwd(v, labels), z)
    dz = on.softmax_loss_bwd(z, labels)
    assert np.allclose(dz, g, rtol=1e-6, atol=1e-9)
    assert np.allclose(dz.sum(axis=1), 0.0, atol=1e-15)


def test_sgd_step():
    assert on.sgd_update(np.array([1.0, 2.0]), np.array([10.0, -10.0]), 0.1).tolist() == [0.0, 3.0]
