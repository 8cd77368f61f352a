"""Pins for the CPU oracle: what mathematics fixes about a convolution layer's three passes.

The paper (arXiv 1712.02546) prints no value of a convolution, so nothing here
is a paper-printed number; every check is a closed form, an invariant, a special
case that reduces to a library routine, or brute force on a tiny input.  Each is
chosen so that a plausible slip in the oracle (dropped term, wrong sign or
index, transposed operand, off-by-one in padding or stride) fails at least one.
"""
import itertools

import numpy as np
import pytest

import oracle
from oracle import Shape

RNG = np.random.default_rng(171202546)

SMALL_SHAPES = [
    Shape(N=2, C=3, H=7, W=6, K=4, R=3, S=2, sh=1, sw=1, ph=0, pw=0),
    Shape(N=2, C=3, H=7, W=6, K=4, R=3, S=2, sh=2, sw=1, ph=1, pw=2),
    Shape(N=1, C=2, H=9, W=8, K=3, R=3, S=3, sh=3, sw=2, ph=2, pw=0),
    Shape(N=3, C=1, H=5, W=5, K=2, R=5, S=5, sh=1, sw=1, ph=2, pw=2),
    Shape(N=2, C=2, H=11, W=10, K=5, R=4, S=3, sh=4, sw=3, ph=1, pw=1, k0=1, k1=4),
]


def rand(*shape):
    return RNG.standard_normal(shape)


def tensors(sh):
    sh = sh.resolved()
    P, Q = oracle.out_hw(sh)
    return rand(sh.N, sh.C, sh.H, sh.W), rand(sh.K, sh.C, sh.R, sh.S), rand(sh.N, sh.K, P, Q)


def loss(sh, x, w, dy):
    return float(np.sum(oracle.conv_fwd(sh, x, w) * dy))


# ---------------------------------------------------------------- output extent
@pytest.mark.parametrize("H,R,s,p,P", [(32, 5, 1, 0, 28), (14, 5, 1, 0, 10), (224, 11, 4, 2, 55),
                                       (27, 5, 1, 2, 27), (34, 5, 4, 0, 8), (5, 5, 1, 0, 1)])
def test_output_extent_floor_formula(H, R, s, p, P):
    sh = Shape(N=1, C=1, H=H, W=H, K=1, R=R, S=R, sh=s, sw=s, ph=p, pw=p)
    assert oracle.out_hw(sh) == (P, P)


def test_rejects_bad_shapes():
    with pytest.raises(ValueError):
        oracle.out_hw(Shape(N=1, C=1, H=3, W=3, K=1, R=5, S=5))
    with pytest.raises(ValueError):
        oracle.out_hw(Shape(N=1, C=1, H=8, W=8, K=4, R=3, S=3, k0=3, k1=2))
    with pytest.raises(ValueError):
        oracle.out_hw(Shape(N=1, C=1, H=8, W=8, K=4, R=3, S=3, k0=0, k1=5))


# ------------------------------------------------- brute-force finite differences
@pytest.mark.parametrize("sh", SMALL_SHAPES[:3] + SMALL_SHAPES[4:])
def test_gradients_equal_exact_finite_differences(sh):
    """<conv(x,w),dy> is linear in x and in w separately, so a central difference
    with any step is the exact derivative (up to fp64 rounding)."""
    x, w, dy = tensors(sh)
    dx = oracle.conv_bwd_data(sh, dy, w)
    dw = oracle.conv_bwd_weight(sh, x, dy)
    h = 0.5
    for i in range(x.size):
        e = np.zeros(x.size)
        e[i] = h
        e = e.reshape(x.shape)
        fd = (loss(sh, x + e, w, dy) - loss(sh, x - e, w, dy)) / (2 * h)
        assert abs(fd - dx.flat[i]) <= 1e-10 * (1 + abs(fd)), (i, fd, dx.flat[i])
    for i in range(w.size):
        e = np.zeros(w.size)
        e[i] = h
        e = e.reshape(w.shape)
        fd = (loss(sh, x, w + e, dy) - loss(sh, x, w - e, dy)) / (2 * h)
        assert abs(fd - dw.flat[i]) <= 1e-10 * (1 + abs(fd)), (i, fd, dw.flat[i])


# ------------------------------------------------------------ adjoint identities
STRIDE_PAD = [(1, 0), (1, 2), (2, 1), (3, 2), (4, 2)]


@pytest.mark.parametrize("stride,pad", STRIDE_PAD)
def test_adjoint_identities(stride, pad):
    sh = Shape(N=3, C=4, H=13, W=12, K=6, R=5, S=4, sh=stride, sw=stride, ph=pad, pw=pad, k0=1, k1=5)
    x, w, dy = tensors(sh)
    a = loss(sh, x, w, dy)
    b = float(np.sum(x * oracle.conv_bwd_data(sh, dy, w)))
    c = float(np.sum(w * oracle.conv_bwd_weight(sh, x, dy)))
    assert abs(a - b) <= 1e-11 * abs(a)
    assert abs(a - c) <= 1e-11 * abs(a)


# -------------------------------------------------------------- slice identities
@pytest.mark.parametrize("cuts", [(0, 7), (0, 3, 7), (0, 1, 2, 7), (0, 0, 7)])
def test_kernel_slices_concatenate_to_full_layer(cuts):
    """Same inputs, disjoint kernel blocks, results concatenated by the master
    (Section 4.1.2): y and dw blocks are the full result's blocks bit for bit,
    dx partial sums add up to the full dx."""
    base = dict(N=2, C=3, H=9, W=8, K=7, R=3, S=3, sh=2, sw=1, ph=1, pw=1)
    full = Shape(**base)
    x, w, dy = tensors(full)
    y_full = oracle.conv_fwd(full, x, w)
    dw_full = oracle.conv_bwd_weight(full, x, dy)
    dx_full = oracle.conv_bwd_data(full, dy, w)
    y_cat = np.zeros_like(y_full)
    dw_cat = np.zeros_like(dw_full)
    dx_sum = np.zeros_like(dx_full)
    for k0, k1 in zip(cuts[:-1], cuts[1:]):
        sl = Shape(**base, k0=k0, k1=k1)
        y = oracle.conv_fwd(sl, x, w)
        dw = oracle.conv_bwd_weight(sl, x, dy)
        assert not y[:, :k0].any() and not y[:, k1:].any()
        assert not dw[:k0].any() and not dw[k1:].any()
        y_cat += y
        dw_cat += dw
        dx_sum += oracle.conv_bwd_data(sl, dy, w)
    assert np.array_equal(y_cat, y_full)
    assert np.array_equal(dw_cat, dw_full)
    assert np.allclose(dx_sum, dx_full, rtol=0, atol=1e-12 * np.abs(dx_full).max())


def test_empty_slice_is_all_zero():
    sh = Shape(N=1, C=2, H=6, W=6, K=3, R=3, S=3, k0=2, k1=2)
    x, w, dy = tensors(sh)
    assert not oracle.conv_fwd(sh, x, w).any()
    assert not oracle.conv_bwd_data(sh, dy, w).any()
    assert not oracle.conv_bwd_weight(sh, x, dy).any()


def test_packed_device_view_equals_slice_of_full_layer():
    """A device that holds only its own kernels and maps (Algorithm 2) computes
    the same numbers as the slice call on full-layer tensors."""
    full = Shape(N=2, C=3, H=8, W=8, K=6, R=3, S=3, k0=2, k1=5)
    x, w, dy = tensors(full)
    packed = Shape(N=2, C=3, H=8, W=8, K=3, R=3, S=3)
    assert np.array_equal(oracle.conv_fwd(full, x, w)[:, 2:5], oracle.conv_fwd(packed, x, w[2:5]))
    assert np.array_equal(oracle.conv_bwd_weight(full, x, dy)[2:5],
                          oracle.conv_bwd_weight(packed, x, dy[:, 2:5]))
    assert np.array_equal(oracle.conv_bwd_data(full, dy, w),
                          oracle.conv_bwd_data(packed, dy[:, 2:5], w[2:5]))


# ------------------------------------------- special cases with a textbook answer
def test_1x1_filter_is_a_per_pixel_matrix_product():
    sh = Shape(N=2, C=5, H=4, W=3, K=6, R=1, S=1)
    x, w, dy = tensors(sh)
    W2 = w.reshape(6, 5)
    y = np.einsum("kc,nchw->nkhw", W2, x)
    assert np.allclose(oracle.conv_fwd(sh, x, w), y, rtol=1e-13, atol=1e-13)
    dx = np.einsum("kc,nkhw->nchw", W2, dy)
    assert np.allclose(oracle.conv_bwd_data(sh, dy, w), dx, rtol=1e-13, atol=1e-13)
    dw = np.einsum("nkhw,nchw->kc", dy, x).reshape(6, 5, 1, 1)
    assert np.allclose(oracle.conv_bwd_weight(sh, x, dy), dw, rtol=1e-13, atol=1e-13)


def test_full_size_filter_is_a_fully_connected_layer():
    sh = Shape(N=3, C=2, H=4, W=5, K=3, R=4, S=5)
    x, w, dy = tensors(sh)
    assert oracle.out_hw(sh) == (1, 1)
    y = x.reshape(3, -1) @ w.reshape(3, -1).T
    assert np.allclose(oracle.conv_fwd(sh, x, w).reshape(3, 3), y, rtol=1e-13, atol=1e-13)
    dx = dy.reshape(3, 3) @ w.reshape(3, -1)
    assert np.allclose(oracle.conv_bwd_data(sh, dy, w).reshape(3, -1), dx, rtol=1e-13, atol=1e-13)
    dw = dy.reshape(3, 3).T @ x.reshape(3, -1)
    assert np.allclose(oracle.conv_bwd_weight(sh, x, dy).reshape(3, -1), dw, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("r0,s0,pad", [(0, 0, 0), (2, 1, 0), (1, 3, 2), (4, 0, 1)])
def test_one_hot_filter_shifts_the_input(r0, s0, pad):
    """w[k,c,r0,s0] = delta(k,c): cross-correlation picks x at offset (r0-pad, s0-pad);
    a flipped (true convolution) kernel would pick the mirrored offset."""
    C, H, W, R, S = 3, 8, 9, 5, 4
    sh = Shape(N=2, C=C, H=H, W=W, K=C, R=R, S=S, ph=pad, pw=pad)
    P, Q = oracle.out_hw(sh)
    x = rand(2, C, H, W)
    w = np.zeros((C, C, R, S))
    for c in range(C):
        w[c, c, r0, s0] = 1.0
    xp = np.zeros((2, C, H + 2 * pad, W + 2 * pad))
    xp[:, :, pad:pad + H, pad:pad + W] = x
    expect = xp[:, :, r0:r0 + P, s0:s0 + Q]
    assert np.array_equal(oracle.conv_fwd(sh, x, w), expect)


@pytest.mark.parametrize("stride,pad", STRIDE_PAD)
def test_all_ones_counts_in_range_taps(stride, pad):
    C, H, W, R, S = 3, 11, 9, 5, 3
    sh = Shape(N=1, C=C, H=H, W=W, K=2, R=R, S=S, sh=stride, sw=stride, ph=pad, pw=pad)
    P, Q = oracle.out_hw(sh)
    y = oracle.conv_fwd(sh, np.ones((1, C, H, W)), np.ones((2, C, R, S)))
    rows = [sum(0 <= p * stride - pad + r < H for r in range(R)) for p in range(P)]
    cols = [sum(0 <= q * stride - pad + s < W for s in range(S)) for q in range(Q)]
    expect = C * np.outer(rows, cols)
    assert np.array_equal(y[0, 0], expect) and np.array_equal(y[0, 1], expect)
    # all-ones upstream gradient: dx counts the windows that cover each pixel
    dx = oracle.conv_bwd_data(sh, np.ones((1, 2, P, Q)), np.ones((2, C, R, S)))
    cover_r = [sum(1 for p in range(P) for r in range(R) if p * stride - pad + r == h) for h in range(H)]
    cover_c = [sum(1 for q in range(Q) for s in range(S) if q * stride - pad + s == v) for v in range(W)]
    assert np.array_equal(dx[0, 0], 2 * np.outer(cover_r, cover_c))


def test_rows_no_window_reaches_get_zero_gradient():
    sh = Shape(N=1, C=1, H=34, W=34, K=2, R=5, S=5, sh=4, sw=4)
    assert oracle.out_hw(sh) == (8, 8)
    x, w, dy = tensors(sh)
    dx = oracle.conv_bwd_data(sh, dy, w)
    assert not dx[:, :, 33, :].any() and not dx[:, :, :, 33].any()
    assert dx[:, :, 32, :33].all()
    x2 = x.copy()
    x2[:, :, 33, :] += 7.0
    assert np.array_equal(oracle.conv_fwd(sh, x, w), oracle.conv_fwd(sh, x2, w))


# --------------------------------------------------- hand-written tiny brute force
def test_tiny_case_against_python_loops():
    sh = Shape(N=2, C=2, H=5, W=4, K=3, R=2, S=3, sh=2, sw=1, ph=1, pw=1, k0=1, k1=3)
    x, w, dy = tensors(sh)
    P, Q = oracle.out_hw(sh)
    y = np.zeros((2, 3, P, Q))
    dx = np.zeros_like(x)
    dw = np.zeros_like(w)
    for n, k, p, q, c, r, s in itertools.product(range(2), range(1, 3), range(P), range(Q),
                                                 range(2), range(2), range(3)):
        h, v = 2 * p - 1 + r, q - 1 + s
        if 0 <= h < 5 and 0 <= v < 4:
            y[n, k, p, q] += x[n, c, h, v] * w[k, c, r, s]
            dx[n, c, h, v] += dy[n, k, p, q] * w[k, c, r, s]
            dw[k, c, r, s] += dy[n, k, p, q] * x[n, c, h, v]
    assert np.allclose(oracle.conv_fwd(sh, x, w), y, rtol=1e-13, atol=1e-14)
    assert np.allclose(oracle.conv_bwd_data(sh, dy, w), dx, rtol=1e-13, atol=1e-14)
    assert np.allclose(oracle.conv_bwd_weight(sh, x, dy), dw, rtol=1e-13, atol=1e-14)


# ------------------------------------------------ independent library cross-check
@pytest.mark.parametrize("sh", SMALL_SHAPES + [
    Shape(N=2, C=3, H=32, W=32, K=16, R=5, S=5),                       # tiny CIFAR-shaped layer
    Shape(N=1, C=3, H=35, W=35, K=4, R=11, S=11, sh=4, sw=4, ph=2, pw=2),  # 11x11 stride 4 pad 2
])
def test_against_library_cross_correlation_and_autograd(sh):
    torch = pytest.importorskip("torch")
    sh = sh.resolved()
    x, w, dy = tensors(sh)
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    wt = torch.tensor(w[sh.k0:sh.k1], dtype=torch.float64, requires_grad=True)
    yt = torch.nn.functional.conv2d(xt, wt, stride=(sh.sh, sh.sw), padding=(sh.ph, sh.pw))
    (yt * torch.tensor(dy[:, sh.k0:sh.k1])).sum().backward()
    y = oracle.conv_fwd(sh, x, w)
    assert np.allclose(y[:, sh.k0:sh.k1], yt.detach().numpy(), rtol=1e-12, atol=1e-12)
    assert np.allclose(oracle.conv_bwd_data(sh, dy, w), xt.grad.numpy(), rtol=1e-12, atol=1e-12)
    dw = oracle.conv_bwd_weight(sh, x, dy)
    assert np.allclose(dw[sh.k0:sh.k1], wt.grad.numpy(), rtol=1e-12, atol=1e-12)


# ------------------------------------------------------------------- linearity
def test_forward_is_linear_and_shift_equivariant():
    sh = Shape(N=1, C=2, H=12, W=12, K=3, R=3, S=3, sh=2, sw=2)
    x1, w, _ = tensors(sh)
    x2 = rand(*x1.shape)
    lhs = oracle.conv_fwd(sh, 2.0 * x1 - 3.0 * x2, w)
    rhs = 2.0 * oracle.conv_fwd(sh, x1, w) - 3.0 * oracle.conv_fwd(sh, x2, w)
    assert np.allclose(lhs, rhs, rtol=1e-12, atol=1e-12)
    xs = np.zeros_like(x1)
    xs[:, :, 2:, :] = x1[:, :, :-2, :]          # shift down by one stride
    y, ys = oracle.conv_fwd(sh, x1, w), oracle.conv_fwd(sh, xs, w)
    assert np.array_equal(ys[:, :, 1:, :], y[:, :, :-1, :])


# ------------------------------------------------------------ sampled versions
@pytest.mark.parametrize("sh", SMALL_SHAPES)
def test_single_element_versions_match_full_loops(sh):
    """The *_at functions are written differently (bwd_data searches for covering
    windows instead of scattering), so agreement checks both."""
    x, w, dy = tensors(sh)
    y = oracle.conv_fwd(sh, x, w)
    dx = oracle.conv_bwd_data(sh, dy, w)
    dw = oracle.conv_bwd_weight(sh, x, dy)
    assert np.array_equal(oracle.conv_fwd_at(sh, x, w, np.arange(y.size)), y.ravel())
    assert np.allclose(oracle.conv_bwd_data_at(sh, dy, w, np.arange(dx.size)), dx.ravel(),
                       rtol=1e-13, atol=1e-13)
    assert np.array_equal(oracle.conv_bwd_weight_at(sh, x, dy, np.arange(dw.size)), dw.ravel())
    with pytest.raises(ValueError):
        oracle.conv_fwd_at(sh, x, w, [y.size])


def test_float32_inputs_are_widened_exactly():
    sh = Shape(N=1, C=2, H=6, W=6, K=2, R=3, S=3)
    x, w, _ = tensors(sh)
    x32, w32 = x.astype(np.float32), w.astype(np.float32)
    assert np.array_equal(oracle.conv_fwd(sh, x32, w32),
                          oracle.conv_fwd(sh, x32.astype(np.float64), w32.astype(np.float64)))
