"""The network's other layers on the GPU (normalisation, pooling, fully connected, softmax
loss, SGD step; Section 4.1) against the fp64 oracle, element by element, at small ragged
sizes and at the sizes the paper's largest network has."""
import numpy as np
import pytest

import paper_1712_02546_amd as cs
from helpers import rel_err
from oracle import netlayers as on

pytestmark = pytest.mark.gpu

TOL = 1e-4        # fp32 against fp64, metric of helpers.rel_err


def dev(a, dtype=None):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is None:
        t = t.float()
    return t.to("cuda:0")


def empty(shape):
    import torch
    return torch.empty(shape, dtype=torch.float32, device="cuda:0")


def host(t):
    import torch
    torch.cuda.synchronize()
    return t.double().cpu().numpy()


def f32(a):
    return np.asarray(a, dtype=np.float32).astype(np.float64)


@pytest.mark.parametrize("N,C,H,W,size,kappa,alpha,beta", [
    (3, 7, 5, 4, 5, 1.0, 1e-4, 0.75),
    (2, 33, 3, 3, 3, 2.0, 0.3, 0.5),
    (5, 4, 6, 5, 9, 1.0, 0.05, 0.75),       # window wider than the channel count
    (2, 5, 2, 2, 1, 1.5, 0.2, 1.0),         # window of one channel
    (4, 6, 4, 6, 9, 1.0, 0.05, 0.75),       # four pixels per thread, window wider than the channel count
    (16, 500, 28, 28, 5, 1.0, 1e-4, 0.75),  # after C1 of the largest network (batch reduced)
])
def test_normalisation(N, C, H, W, size, kappa, alpha, beta):
    rng = np.random.default_rng(N * 1000 + C)
    x = f32(rng.normal(size=(N, C, H, W)) * 3.0)
    dy = f32(rng.normal(size=x.shape))
    xd, dyd = dev(x), dev(dy)
    y, scale, dx = empty(x.shape), empty(x.shape), empty(x.shape)
    cs.net_norm_fwd(xd, y, scale, N, C, H * W, size, kappa, alpha, beta)
    cs.net_norm_bwd(xd, y, scale, dyd, dx, N, C, H * W, size, kappa, alpha, beta)
    assert rel_err(host(y), on.norm_fwd(x, size, kappa, alpha, beta)) <= TOL
    assert rel_err(host(scale), on.norm_scale(x, size, kappa, alpha)) <= TOL
    assert rel_err(host(dx), on.norm_bwd(x, dy, size, kappa, alpha, beta)) <= TOL


@pytest.mark.parametrize("N,C,H,W,win,stride", [
    (2, 3, 4, 4, 2, 2), (3, 5, 7, 6, 3, 2), (2, 2, 9, 9, 2, 3), (1, 4, 5, 5, 5, 1), (2, 3, 8, 7, 3, 1),
    (16, 500, 28, 28, 2, 2), (16, 1500, 10, 10, 2, 2),   # the two pooling layers of the largest network
])
def test_max_pooling(N, C, H, W, win, stride):
    rng = np.random.default_rng(H * 100 + W)
    # few distinct values, so that ties inside a window are common
    x = f32(rng.integers(-3, 4, size=(N, C, H, W)).astype(np.float64) / 2)
    P, Q = on.pool_out(H, win, stride), on.pool_out(W, win, stride)
    dy = f32(rng.normal(size=(N, C, P, Q)))
    xd, dyd = dev(x), dev(dy)
    y, dx = empty((N, C, P, Q)), empty(x.shape)
    cs.net_pool_fwd(xd, y, N * C, H, W, win, stride)
    cs.net_pool_bwd(xd, dyd, dx, N * C, H, W, win, stride)
    assert np.array_equal(host(y), on.pool_fwd(x, win, stride))          # selection: exact
    assert rel_err(host(dx), on.pool_bwd(x, dy, win, stride)) <= 1e-6    # sums of at most a few terms


@pytest.mark.parametrize("N,I,O", [(3, 10, 4), (5, 1000, 10), (2, 257, 9), (7, 300, 17), (128, 37500, 10)])
def test_fully_connected(N, I, O):
    rng = np.random.default_rng(I)
    x = f32(rng.normal(size=(N, I)))
    W = f32(rng.normal(size=(O, I)) * 0.05)
    b = f32(rng.normal(size=O))
    dy = f32(rng.normal(size=(N, O)))
    xd, Wd, bd, dyd = dev(x), dev(W), dev(b), dev(dy)
    y, dx, dW, db = empty((N, O)), empty((N, I)), empty((O, I)), empty((O,))
    cs.net_fc_fwd(xd, Wd, bd, y, N, I, O)
    cs.net_fc_bwd(xd, Wd, dyd, dx, dW, db, N, I, O)
    rdx, rdW, rdb = on.fc_bwd(x, W, dy)
    assert rel_err(host(y), on.fc_fwd(x, W, b)) <= TOL
    assert rel_err(host(dx), rdx) <= TOL
    assert rel_err(host(dW), rdW) <= TOL
    assert rel_err(host(db), rdb) <= TOL


@pytest.mark.parametrize("N,O", [(1, 2), (5, 10), (128, 10), (1000, 10), (300, 37)])
def test_softmax_loss(N, O):
    import torch
    rng = np.random.default_rng(N + O)
    z = f32(rng.normal(size=(N, O)) * 4.0)
    labels = rng.integers(0, O, size=N).astype(np.int32)
    zd, ld = dev(z), dev(labels, dtype="int")
    loss, dz = empty((1,)), empty((N, O))
    cs.net_softmax_loss_fwd(zd, ld, loss, N, O)
    cs.net_softmax_loss_bwd(zd, ld, dz, N, O)
    want = on.softmax_loss_fwd(z, labels)
    assert abs(float(host(loss)[0]) - want) <= 1e-5 * max(1.0, abs(want))
    assert rel_err(host(dz), on.softmax_loss_bwd(z, labels)) <= TOL
    # a second run gives the same bits (fixed summation order)
    loss2 = empty((1,))
    cs.net_softmax_loss_fwd(zd, ld, loss2, N, O)
    assert torch.equal(loss, loss2)


def test_sgd_update():
    rng = np.random.default_rng(9)
    w = f32(rng.normal(size=100003))
    dw = f32(rng.normal(size=100003))
    wd, dwd = dev(w), dev(dw)
    cs.net_sgd_update(wd, dwd, 0.01, w.size)
    assert rel_err(host(wd), on.sgd_update(w, dw, np.float32(0.01).astype(np.float64))) <= 1e-6
