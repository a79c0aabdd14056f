"""Pins for the fp64 oracle: each function is checked against something other than itself - pure-Python
brute force on tiny inputs, library routines on the special cases that reduce to them, closed forms,
finite differences and algebraic identities.  No GPU needed."""
import itertools
import math

import numpy as np
import pytest
import scipy.signal
import scipy.special
import torch

import oracle as O

RNG = np.random.default_rng(20150128)


def rnd(*shape):
    return RNG.standard_normal(shape)


# ---------------------------------------------------------------------------------------------
# brute force written independently, in pure Python, straight from Eq. 1
# ---------------------------------------------------------------------------------------------

def brute_conv(x, w, b, ph, pw, sh=1, sw=1):
    n_, c_, h_, w_ = x.shape
    k_, _, r_, s_ = w.shape
    oh_, ow_ = (h_ + 2 * ph - r_) // sh + 1, (w_ + 2 * pw - s_) // sw + 1
    y = np.zeros((n_, k_, oh_, ow_))
    for n, k, oh, ow in itertools.product(range(n_), range(k_), range(oh_), range(ow_)):
        acc = b[k]
        for c, r, s in itertools.product(range(c_), range(r_), range(s_)):
            ih, iw = oh * sh + r - ph, ow * sw + s - pw
            if 0 <= ih < h_ and 0 <= iw < w_:
                acc += w[k, c, r, s] * x[n, c, ih, iw]
        y[n, k, oh, ow] = acc
    return y


@pytest.mark.parametrize("c,k,r,s,ph,pw", [(1, 1, 2, 2, 0, 0), (1, 3, 2, 2, 0, 0), (3, 2, 3, 3, 1, 1),
                                            (2, 2, 3, 1, 0, 2), (2, 3, 1, 4, 1, 0), (2, 1, 5, 5, 2, 2)])
def test_conv_fwd_brute_force(c, k, r, s, ph, pw):
    x, w, b = rnd(2, c, 5, 5), rnd(k, c, r, s), rnd(k)
    np.testing.assert_allclose(O.conv_fwd(x, w, b, pad=(ph, pw)), brute_conv(x, w, b, ph, pw), rtol=0, atol=1e-13)


def test_conv_fwd_brute_force_strided():
    x, w, b = rnd(1, 2, 7, 6), rnd(2, 2, 3, 2), rnd(2)
    np.testing.assert_allclose(O.conv_fwd(x, w, b, pad=(1, 0), stride=(2, 3)), brute_conv(x, w, b, 1, 0, 2, 3),
                               atol=1e-13)


def test_paper_fig2_shapes():
    """Fig. 2: a 3x3 image and three 2x2 kernels give three 2x2 maps; the patch matrix has 4 patches of
    4 elements; with a batch of 2 (Fig. 5) the two patch matrices sit side by side."""
    x, w = rnd(1, 1, 3, 3), rnd(3, 1, 2, 2)
    assert O.conv_fwd(x, w).shape == (1, 3, 2, 2)
    col = O.im2col(x, (2, 2))
    assert col.shape == (4, 4)
    x2 = np.concatenate([x, rnd(1, 1, 3, 3)])
    col2 = O.im2col(x2, (2, 2))
    assert col2.shape == (4, 8)
    np.testing.assert_array_equal(col2[:, :4], col)
    # the first patch (column 0) is the top-left 2x2 block, row-major
    np.testing.assert_array_equal(col[:, 0], x[0, 0, :2, :2].ravel())
    # product of the kernel matrix (one kernel per row) with the patch matrix: one feature map per row
    y = O.conv_fwd(x2, w)
    prod = w.reshape(3, 4) @ col2
    np.testing.assert_allclose(prod.reshape(3, 2, 2, 2).transpose(1, 0, 2, 3), y, atol=1e-14)


def test_paper_fig3_multichannel_rows():
    """Fig. 3: a 3x3x3 feature map unrolled once has Cin*kh*kw rows."""
    assert O.im2col(rnd(1, 3, 3, 3), (2, 2)).shape == (12, 4)


def test_conv_is_cross_correlation_scipy():
    x, w = rnd(1, 1, 9, 8), rnd(1, 1, 4, 3)
    ref = scipy.signal.correlate2d(x[0, 0], w[0, 0], mode="valid")
    np.testing.assert_allclose(O.conv_fwd(x, w)[0, 0], ref, atol=1e-13)
    # and it is not the flipped (true convolution) variant
    assert not np.allclose(O.conv_fwd(x, w)[0, 0], scipy.signal.convolve2d(x[0, 0], w[0, 0], mode="valid"))


@pytest.mark.parametrize("pad", [(0, 0), (2, 2), (1, 3)])
def test_conv_fwd_torch_cpu(pad):
    x, w, b = rnd(3, 4, 11, 10), rnd(5, 4, 5, 3), rnd(5)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(w), torch.from_numpy(b), padding=pad)
    np.testing.assert_allclose(O.conv_fwd(x, w, b, pad=pad), ref.numpy(), atol=1e-12)
    np.testing.assert_allclose(O.conv_fwd(x, w, b, pad=pad, relu=True), ref.clamp_min(0).numpy(), atol=1e-12)


def test_conv_delta_kernel_identity_and_shift():
    x = rnd(2, 1, 6, 6)
    w = np.zeros((1, 1, 3, 3))
    w[0, 0, 1, 1] = 1.0
    np.testing.assert_array_equal(O.conv_fwd(x, w, pad=(1, 1)), x)
    w[:] = 0
    w[0, 0, 0, 2] = 1.0  # tap (r=0,s=2): y[oh,ow] = x[oh-1, ow+1]
    y = O.conv_fwd(x, w, pad=(1, 1))
    np.testing.assert_array_equal(y[:, :, 1:, :-1], x[:, :, :-1, 1:])
    assert np.all(y[:, :, 0, :] == 0) and np.all(y[:, :, :, -1] == 0)


def test_conv_1x1_is_matmul():
    x, w, b = rnd(2, 7, 4, 5), rnd(3, 7, 1, 1), rnd(3)
    ref = np.einsum("kc,nchw->nkhw", w[:, :, 0, 0], x) + b[None, :, None, None]
    np.testing.assert_allclose(O.conv_fwd(x, w, b), ref, atol=1e-13)


def test_conv_linearity():
    x1, x2, w = rnd(1, 2, 6, 6), rnd(1, 2, 6, 6), rnd(3, 2, 3, 3)
    lhs = O.conv_fwd(2.0 * x1 - 3.0 * x2, w, pad=(1, 1))
    rhs = 2.0 * O.conv_fwd(x1, w, pad=(1, 1)) - 3.0 * O.conv_fwd(x2, w, pad=(1, 1))
    np.testing.assert_allclose(lhs, rhs, atol=1e-12)


# ---------------------------------------------------------------------------------------------
# im2col / col2im
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("c,r,s,ph,pw", [(1, 2, 2, 0, 0), (3, 3, 3, 1, 1), (2, 5, 1, 0, 0), (2, 1, 4, 0, 2)])
def test_im2col_matmul_equals_direct_conv(c, r, s, ph, pw):
    x, w, b = rnd(3, c, 7, 6), rnd(4, c, r, s), rnd(4)
    col = O.im2col(x, (r, s), pad=(ph, pw))
    oh, ow = O.conv_out_hw(7, 6, r, s, ph, pw)
    y = (w.reshape(4, -1) @ col + b[:, None]).reshape(4, 3, oh, ow).transpose(1, 0, 2, 3)
    np.testing.assert_allclose(y, O.conv_fwd(x, w, b, pad=(ph, pw)), atol=1e-12)


def brute_im2col(x, r_, s_, ph, pw):
    n_, c_, h_, w_ = x.shape
    oh_, ow_ = h_ + 2 * ph - r_ + 1, w_ + 2 * pw - s_ + 1
    col = np.zeros((c_ * r_ * s_, n_ * oh_ * ow_))
    for c, r, s, n, oh, ow in itertools.product(range(c_), range(r_), range(s_), range(n_), range(oh_), range(ow_)):
        ih, iw = oh + r - ph, ow + s - pw
        if 0 <= ih < h_ and 0 <= iw < w_:
            col[(c * r_ + r) * s_ + s, (n * oh_ + oh) * ow_ + ow] = x[n, c, ih, iw]
    return col


def test_im2col_brute_force():
    x = rnd(2, 2, 4, 5)
    np.testing.assert_array_equal(O.im2col(x, (3, 2), pad=(1, 0)), brute_im2col(x, 3, 2, 1, 0))


@pytest.mark.parametrize("c,r,s,ph,pw", [(1, 2, 2, 0, 0), (3, 3, 3, 1, 1), (2, 5, 3, 2, 0)])
def test_unroll_adjoint_identity(c, r, s, ph, pw):
    """<im2col(x), y> = <x, col2im(y)>: col2im is the transpose of the (linear) unroll."""
    x = rnd(2, c, 7, 8)
    col = O.im2col(x, (r, s), pad=(ph, pw))
    yy = rnd(*col.shape)
    lhs = float(np.sum(col * yy))
    rhs = float(np.sum(x * O.col2im(yy, x.shape, (r, s), pad=(ph, pw))))
    assert abs(lhs - rhs) <= 1e-11 * max(1.0, abs(lhs))


def test_col2im_multiplicity_closed_form():
    """col2im(im2col(x)) = x * (number of patches containing the pixel); for a valid unroll that count
    is min(h, R-1, H-1-h, H-R)+1 per axis, R*S in the interior."""
    x = rnd(1, 2, 9, 8)
    r, s = 3, 2
    back = O.col2im(O.im2col(x, (r, s)), x.shape, (r, s))
    cnt_h = np.array([min(h, r - 1, 9 - 1 - h, 9 - r) + 1 for h in range(9)])
    cnt_w = np.array([min(w, s - 1, 8 - 1 - w, 8 - s) + 1 for w in range(8)])
    np.testing.assert_allclose(back, x * np.outer(cnt_h, cnt_w)[None, None], atol=1e-13)
    assert cnt_h[4] * cnt_w[4] == r * s


# ---------------------------------------------------------------------------------------------
# gradients: finite differences, bilinear identities, autograd as library third opinion
# ---------------------------------------------------------------------------------------------

def central_diff(f, a, h=1e-6):
    g = np.zeros_like(a)
    flat, gf = a.reshape(-1), g.reshape(-1)
    for i in range(flat.size):
        old = flat[i]
        flat[i] = old + h
        fp = f()
        flat[i] = old - h
        fm = f()
        flat[i] = old
        gf[i] = (fp - fm) / (2 * h)
    return g


@pytest.mark.parametrize("pad", [(0, 0), (1, 2)])
def test_conv_gradients_finite_differences(pad):
    x, w, b = rnd(2, 2, 5, 6), rnd(3, 2, 3, 2), rnd(3)
    dy = rnd(*O.conv_fwd(x, w, b, pad=pad).shape)

    def loss():
        return float(np.sum(O.conv_fwd(x, w, b, pad=pad) * dy))

    dw, db = O.conv_bwd_filter(x, dy, (3, 2), pad=pad)
    dx = O.conv_bwd_data(w, dy, (5, 6), pad=pad)
    np.testing.assert_allclose(dw, central_diff(loss, w), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(db, central_diff(loss, b), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(dx, central_diff(loss, x), rtol=1e-6, atol=1e-7)


def test_conv_gradients_strided_finite_differences():
    x, w = rnd(1, 2, 7, 7), rnd(2, 2, 3, 3)
    kw = dict(pad=(1, 1), stride=(2, 2))
    dy = rnd(*O.conv_fwd(x, w, **kw).shape)

    def loss():
        return float(np.sum(O.conv_fwd(x, w, **kw) * dy))

    np.testing.assert_allclose(O.conv_bwd_filter(x, dy, (3, 3), **kw)[0], central_diff(loss, w), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(O.conv_bwd_data(w, dy, (7, 7), **kw), central_diff(loss, x), rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("pad", [(0, 0), (2, 2), (0, 3)])
def test_conv_bilinear_identities(pad):
    """<dy, conv(x,w)> = <dw(x,dy), w> = <dx(w,dy), x> for the bias-free layer."""
    x, w = rnd(3, 4, 9, 10), rnd(5, 4, 5, 4)
    y = O.conv_fwd(x, w, pad=pad)
    dy = rnd(*y.shape)
    ref = float(np.sum(dy * y))
    dw, db = O.conv_bwd_filter(x, dy, (5, 4), pad=pad)
    dx = O.conv_bwd_data(w, dy, (9, 10), pad=pad)
    assert abs(float(np.sum(dw * w)) - ref) <= 1e-11 * abs(ref)
    assert abs(float(np.sum(dx * x)) - ref) <= 1e-11 * abs(ref)
    np.testing.assert_allclose(db, dy.sum(axis=(0, 2, 3)), atol=1e-12)


def test_conv_gradients_autograd():
    x, w, b = rnd(2, 3, 8, 7), rnd(4, 3, 3, 5), rnd(4)
    xt, wt, bt = (torch.from_numpy(a).requires_grad_() for a in (x, w, b))
    yt = torch.nn.functional.conv2d(xt, wt, bt, padding=(1, 2))
    dy = rnd(*yt.shape)
    yt.backward(torch.from_numpy(dy))
    dw, db = O.conv_bwd_filter(x, dy, (3, 5), pad=(1, 2))
    np.testing.assert_allclose(dw, wt.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(db, bt.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(O.conv_bwd_data(w, dy, (8, 7), pad=(1, 2)), xt.grad.numpy(), atol=1e-12)


def test_bwd_data_is_col2im_of_transposed_product():
    """The paper's backward route: multiply by the transposed kernel matrix, then phi_c^{-1}."""
    x, w = rnd(2, 3, 6, 6), rnd(4, 3, 3, 3)
    dy = rnd(2, 4, 6, 6)
    dcol = w.reshape(4, -1).T @ dy.transpose(1, 0, 2, 3).reshape(4, -1)
    np.testing.assert_allclose(O.col2im(dcol, x.shape, (3, 3), pad=(1, 1)), O.conv_bwd_data(w, dy, (6, 6), pad=(1, 1)),
                               atol=1e-12)


# ---------------------------------------------------------------------------------------------
# probes (single-output numpy definitions) agree with the full C loops
# ---------------------------------------------------------------------------------------------

def test_probes_match_full():
    x, w, b = rnd(2, 3, 7, 8), rnd(4, 3, 3, 2), rnd(4)
    pad = (1, 1)
    y = O.conv_fwd(x, w, b, pad=pad, relu=True)
    dy = rnd(*y.shape)
    dw, _ = O.conv_bwd_filter(x, dy, (3, 2), pad=pad)
    dx = O.conv_bwd_data(w, dy, (7, 8), pad=pad)
    iy = [tuple(int(RNG.integers(0, d)) for d in y.shape) for _ in range(20)] + [(0, 0, 0, 0), (1, 3, 6, 8)]
    np.testing.assert_allclose(O.conv_fwd_at(x, w, b, pad, iy, relu=True), [y[i] for i in iy], atol=1e-13)
    iw = [tuple(int(RNG.integers(0, d)) for d in dw.shape) for _ in range(20)]
    np.testing.assert_allclose(O.conv_bwd_filter_at(x, dy, (3, 2), pad, iw), [dw[i] for i in iw], atol=1e-12)
    ix = [tuple(int(RNG.integers(0, d)) for d in dx.shape) for _ in range(20)] + [(0, 0, 0, 0), (1, 2, 6, 7)]
    np.testing.assert_allclose(O.conv_bwd_data_at(w, dy, pad, ix), [dx[i] for i in ix], atol=1e-12)


@pytest.mark.parametrize("hw,rs,pad", [((7, 8), (3, 2), (1, 1)), ((6, 6), (4, 4), (0, 0)), ((5, 9), (5, 3), (2, 1)),
                                       ((9, 4), (1, 4), (0, 3)), ((8, 8), (8, 8), (0, 0)), ((4, 5), (3, 3), (2, 2))])
def test_input_gradient_probe_matches_full_at_every_pixel(hw, rs, pad):
    """The single-pixel input-gradient probe sums a rectangle of existing taps at once; every pixel of small
    layers - interior, borders, corners, 'valid' and padded, taps wider than the output - against the C loops."""
    w = rnd(3, 2, *rs)
    oh, ow = O.conv_out_hw(hw[0], hw[1], rs[0], rs[1], pad[0], pad[1])
    dy = rnd(2, 3, oh, ow)
    dx = O.conv_bwd_data(w, dy, hw, pad=pad)
    ix = list(np.ndindex(*dx.shape))
    np.testing.assert_allclose(O.conv_bwd_data_at(w, dy, pad, ix), dx.reshape(-1), atol=1e-12)


# ---------------------------------------------------------------------------------------------
# pooling
# ---------------------------------------------------------------------------------------------

def brute_pool(x, win, st):
    n_, c_, h_, w_ = x.shape
    oh_, ow_ = (h_ - win) // st + 1, (w_ - win) // st + 1
    y = np.zeros((n_, c_, oh_, ow_))
    am = np.zeros((n_, c_, oh_, ow_), dtype=np.int32)
    for n, c, oh, ow in itertools.product(range(n_), range(c_), range(oh_), range(ow_)):
        cands = [(x[n, c, oh * st + i, ow * st + j], (oh * st + i) * w_ + ow * st + j)
                 for i in range(win) for j in range(win)]
        best = max(v for v, _ in cands)
        y[n, c, oh, ow] = best
        am[n, c, oh, ow] = min(i for v, i in cands if v == best)
    return y, am


@pytest.mark.parametrize("h,w,win,st", [(4, 4, 2, 2), (7, 8, 3, 2), (32, 32, 3, 2), (5, 5, 2, 1)])
def test_maxpool_brute_force_with_ties(h, w, win, st):
    x = RNG.integers(0, 3, size=(2, 3, h, w)).astype(np.float64)  # few distinct values: many ties
    y, am = O.maxpool_fwd(x, (win, win), (st, st))
    yb, amb = brute_pool(x, win, st)
    np.testing.assert_array_equal(y, yb)
    np.testing.assert_array_equal(am, amb)


def test_maxpool_paper_fig4_shape_and_output_size():
    y, am = O.maxpool_fwd(rnd(1, 1, 4, 4), (2, 2), (2, 2))
    assert y.shape == (1, 1, 2, 2) and am.dtype == np.int32
    assert O.maxpool_fwd(rnd(1, 1, 32, 32), (3, 3), (2, 2))[0].shape == (1, 1, 15, 15)  # floor mode: 32->15->7->3
    assert O.maxpool_fwd(rnd(1, 1, 15, 15), (3, 3), (2, 2))[0].shape == (1, 1, 7, 7)


def test_maxpool_constant_input_picks_window_origin():
    x = np.full((1, 2, 7, 7), 0.5)
    _, am = O.maxpool_fwd(x, (3, 3), (2, 2))
    oh, ow = np.meshgrid(range(3), range(3), indexing="ij")
    np.testing.assert_array_equal(am[0, 0], (2 * oh) * 7 + 2 * ow)


def test_maxpool_torch_cpu():
    x = rnd(2, 3, 9, 9)
    yt, it = torch.nn.functional.max_pool2d(torch.from_numpy(x), 3, 2, return_indices=True)
    y, am = O.maxpool_fwd(x, (3, 3), (2, 2))
    np.testing.assert_array_equal(y, yt.numpy())
    np.testing.assert_array_equal(am, it.numpy().astype(np.int32))


def test_maxpool_bwd_sum_and_finite_differences():
    x = rnd(2, 2, 7, 7)  # distinct values: the max is differentiable
    y, am = O.maxpool_fwd(x, (3, 3), (2, 2))
    dy = rnd(*y.shape)
    dx = O.maxpool_bwd(dy, am, (7, 7))
    assert abs(dx.sum() - dy.sum()) < 1e-12

    def loss():
        return float(np.sum(O.maxpool_fwd(x, (3, 3), (2, 2))[0] * dy))

    np.testing.assert_allclose(dx, central_diff(loss, x, h=1e-7), rtol=1e-5, atol=1e-6)


def test_maxpool_bwd_overlap_accumulates():
    x = np.zeros((1, 1, 5, 5))
    x[0, 0, 2, 2] = 1.0  # the centre is the max of all four 3x3 stride-2 windows
    y, am = O.maxpool_fwd(x, (3, 3), (2, 2))
    assert np.all(am == 12)
    dx = O.maxpool_bwd(np.array([[[[1.0, 2.0], [3.0, 4.0]]]]), am, (5, 5))
    assert dx[0, 0, 2, 2] == 10.0 and dx.sum() == 10.0


# ---------------------------------------------------------------------------------------------
# ReLU, fully connected, losses, SGD
# ---------------------------------------------------------------------------------------------

def test_relu():
    x = np.array([-2.0, -0.0, 0.0, 1e-300, 3.0])
    np.testing.assert_array_equal(O.relu_fwd(x), [0, 0, 0, 1e-300, 3.0])
    np.testing.assert_array_equal(O.relu_bwd(x, np.full(5, 7.0)), [0, 0, 0, 7.0, 7.0])


def test_fc_matches_matmul_and_autograd():
    x, w, b = rnd(6, 9), rnd(4, 9), rnd(4)
    np.testing.assert_allclose(O.fc_fwd(x, w, b), x @ w.T + b, atol=1e-13)
    np.testing.assert_allclose(O.fc_fwd(x, w, b, relu=True), np.maximum(x @ w.T + b, 0), atol=1e-13)
    dy = rnd(6, 4)
    dw, db, dx = O.fc_bwd(x, w, dy)
    xt, wt, bt = (torch.from_numpy(a).requires_grad_() for a in (x, w, b))
    torch.nn.functional.linear(xt, wt, bt).backward(torch.from_numpy(dy))
    np.testing.assert_allclose(dw, wt.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(db, bt.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(dx, xt.grad.numpy(), atol=1e-13)


def test_fc_finite_differences():
    x, w, b = rnd(3, 5), rnd(2, 5), rnd(2)
    dy = rnd(3, 2)

    def loss():
        return float(np.sum(O.fc_fwd(x, w, b) * dy))

    dw, db, dx = O.fc_bwd(x, w, dy)
    np.testing.assert_allclose(dw, central_diff(loss, w), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(db, central_diff(loss, b), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(dx, central_diff(loss, x), rtol=1e-6, atol=1e-8)


def test_softmax_loss_closed_forms():
    z = np.full((7, 10), 3.25)
    labels = np.arange(7, dtype=np.int32)
    loss, dz = O.softmax_loss(z, labels)
    assert abs(loss - math.log(10.0)) < 1e-14  # uniform logits: loss = ln(classes)
    np.testing.assert_allclose(dz.sum(axis=1), 0.0, atol=1e-16)
    z = rnd(5, 10) * 4
    labels = RNG.integers(0, 10, size=5).astype(np.int32)
    loss, dz = O.softmax_loss(z, labels)
    ref = np.mean(scipy.special.logsumexp(z, axis=1) - z[np.arange(5), labels])
    assert abs(loss - ref) < 1e-13
    np.testing.assert_allclose(dz.sum(axis=1), 0.0, atol=1e-15)
    onehot = np.eye(10)[labels]
    np.testing.assert_allclose(dz, (scipy.special.softmax(z, axis=1) - onehot) / 5, atol=1e-15)
    # shift invariance and large logits (max subtraction)
    assert abs(O.softmax_loss(z + 1000.0, labels)[0] - loss) < 1e-10


def test_softmax_loss_finite_differences():
    z = rnd(3, 4)
    labels = np.array([1, 3, 0], dtype=np.int32)
    _, dz = O.softmax_loss(z, labels)
    np.testing.assert_allclose(dz, central_diff(lambda: O.softmax_loss(z, labels)[0], z), rtol=1e-6, atol=1e-9)


def test_l2_loss_and_sgd():
    y, t = rnd(4, 1, 3, 3), rnd(4, 1, 3, 3)
    loss, dy = O.l2_loss(y, t)
    assert abs(loss - np.sum((y - t) ** 2) / 8.0) < 1e-13
    np.testing.assert_allclose(dy, (y - t) / 4.0, atol=1e-15)
    np.testing.assert_allclose(dy, central_diff(lambda: O.l2_loss(y, t)[0], y), rtol=1e-6, atol=1e-9)
    w, dw = rnd(10), rnd(10)
    np.testing.assert_allclose(O.sgd_update(w, dw, 0.01), w - 0.01 * dw, atol=1e-16)


# ---------------------------------------------------------------------------------------------
# whole chain
# ---------------------------------------------------------------------------------------------

def test_chain_gradient_finite_differences_and_descent():
    """A tiny conv-ReLU-pool-fc chain: the chained backward equals the finite-difference gradient of
    the loss, and one SGD step lowers the loss."""
    from oracle.net import train_step
    from paper_1501_07338_amd import workloads as wl

    net = wl.Net("tiny", 9, 3, (2, 8, 8), [wl.Conv(3, 3, 3, 1, 1, relu=True), wl.Pool(3, 2), wl.FC(5, relu=True), wl.FC(4)],
                 "softmax", classes=4, lr=0.05)
    params = [None if p is None else (p[0].astype(np.float64), p[1].astype(np.float64) + 0.1) for p in wl.make_params(net)]
    inputs = {"x": rnd(3, 2, 8, 8), "labels": np.array([0, 3, 1], dtype=np.int32)}
    res = train_step(net, inputs, params)

    def loss():
        return train_step(net, inputs, params)["loss"]

    for li in (0, 2, 3):
        np.testing.assert_allclose(res["grads"][li][0], central_diff(loss, params[li][0]), rtol=2e-5, atol=1e-8)
        np.testing.assert_allclose(res["grads"][li][1], central_diff(loss, params[li][1]), rtol=2e-5, atol=1e-8)
    np.testing.assert_allclose(res["dacts"][0], central_diff(loss, inputs["x"]), rtol=2e-5, atol=1e-8)
    assert train_step(net, inputs, res["new_params"])["loss"] < res["loss"]


# ---- the other sigma functions Eq. 1 names, and average pooling ("Vectorizing Pooling") --------------------
def test_tanh_and_sigmoid_closed_forms_and_symmetries():
    # exact rational values: tanh(ln 2) = (2 - 1/2)/(2 + 1/2) = 3/5, sigmoid(ln 3) = 3/4, sigmoid(0) = 1/2, tanh(0) = 0
    np.testing.assert_allclose(O.tanh_fwd(np.array([np.log(2.0), 0.0, -np.log(2.0)])), [0.6, 0.0, -0.6], atol=1e-15)
    np.testing.assert_allclose(O.sigmoid_fwd(np.array([np.log(3.0), 0.0, -np.log(3.0)])), [0.75, 0.5, 0.25], atol=1e-15)
    x = np.random.default_rng(40).normal(size=257) * 3.0
    np.testing.assert_allclose(O.tanh_fwd(-x), -O.tanh_fwd(x), atol=1e-15)           # odd
    np.testing.assert_allclose(O.sigmoid_fwd(x) + O.sigmoid_fwd(-x), 1.0, atol=1e-15)  # sigma(x) + sigma(-x) = 1
    np.testing.assert_allclose(O.tanh_fwd(x), 2.0 * O.sigmoid_fwd(2.0 * x) - 1.0, atol=1e-14)  # ties the two together
    # library third opinion
    from scipy.special import expit
    np.testing.assert_allclose(O.sigmoid_fwd(x), expit(x), atol=1e-15)
    np.testing.assert_allclose(O.tanh_fwd(x), torch.tanh(torch.from_numpy(x)).numpy(), atol=1e-15)
    # saturation keeps its sign and stays inside the open interval's closure
    assert O.tanh_fwd(np.array([40.0]))[0] == 1.0 and O.sigmoid_fwd(np.array([-800.0]))[0] == 0.0


@pytest.mark.parametrize("name", ["tanh", "sigmoid"])
def test_tanh_sigmoid_backward_is_the_derivative(name):
    fwd, bwd = (O.tanh_fwd, O.tanh_bwd) if name == "tanh" else (O.sigmoid_fwd, O.sigmoid_bwd)
    rng = np.random.default_rng(41)
    x, dy = rng.normal(size=64) * 2.0, rng.normal(size=64)
    got = bwd(fwd(x), dy)  # the backward pass is written in terms of the forward output
    eps = 1e-6
    fd = (fwd(x + eps) - fwd(x - eps)) / (2 * eps) * dy
    np.testing.assert_allclose(got, fd, rtol=1e-8, atol=1e-10)
    # autograd as an independent derivative
    xt = torch.from_numpy(x).requires_grad_(True)
    (torch.tanh(xt) if name == "tanh" else torch.sigmoid(xt)).backward(torch.from_numpy(dy))
    np.testing.assert_allclose(got, xt.grad.numpy(), atol=1e-14)


def _avgpool_brute(x, win, stride):
    n, c, h, w = x.shape
    oh, ow = (h - win[0]) // stride[0] + 1, (w - win[1]) // stride[1] + 1
    y = np.zeros((n, c, oh, ow))
    for a in range(n):
        for b in range(c):
            for i in range(oh):
                for j in range(ow):
                    vals = [x[a, b, i * stride[0] + p, j * stride[1] + q] for p in range(win[0]) for q in range(win[1])]
                    y[a, b, i, j] = sum(vals) / len(vals)
    return y


@pytest.mark.parametrize("shape,win,stride", [((2, 3, 4, 4), (2, 2), (2, 2)), ((1, 2, 7, 9), (3, 3), (2, 2)),
                                              ((2, 1, 5, 6), (2, 3), (1, 2)), ((1, 1, 3, 3), (3, 3), (3, 3))])
def test_avgpool_brute_force_library_and_adjoint(shape, win, stride):
    rng = np.random.default_rng(42)
    x = rng.normal(size=shape)
    y = O.avgpool_fwd(x, win, stride)
    np.testing.assert_allclose(y, _avgpool_brute(x, win, stride), atol=1e-14)
    ref = torch.nn.functional.avg_pool2d(torch.from_numpy(x), win, stride).numpy()  # floor mode, no padding
    assert y.shape == ref.shape
    np.testing.assert_allclose(y, ref, atol=1e-14)
    # the gradient is the transpose of a linear map: <avgpool(x), dy> = <x, avgpool_bwd(dy)> exactly
    dy = rng.normal(size=y.shape)
    dx = O.avgpool_bwd(dy, shape[2:], win, stride)
    assert abs(np.sum(y * dy) - np.sum(x * dx)) <= 1e-12 * max(1.0, abs(np.sum(y * dy)))
    # and autograd agrees element by element (also on the rows / columns no window covers: zero)
    xt = torch.from_numpy(x).requires_grad_(True)
    torch.nn.functional.avg_pool2d(xt, win, stride).backward(torch.from_numpy(dy))
    np.testing.assert_allclose(dx, xt.grad.numpy(), atol=1e-14)


def test_avgpool_tiling_windows_reduce_to_block_means_and_upscaling():
    """stride = window: the forward pass is a reshape-mean and the backward pass is the nearest-neighbour
    upscaling of dy (the paper's back-propagation through pooling) divided by the window size."""
    rng = np.random.default_rng(43)
    x = rng.normal(size=(2, 3, 6, 8))
    y = O.avgpool_fwd(x, (2, 2), (2, 2))
    np.testing.assert_allclose(y, x.reshape(2, 3, 3, 2, 4, 2).mean(axis=(3, 5)), atol=1e-15)
    dy = rng.normal(size=y.shape)
    up = np.repeat(np.repeat(dy, 2, axis=2), 2, axis=3) / 4.0
    np.testing.assert_allclose(O.avgpool_bwd(dy, (6, 8), (2, 2), (2, 2)), up, atol=1e-15)
    # constant input -> the same constant; mass conservation of the gradient
    np.testing.assert_allclose(O.avgpool_fwd(np.full((1, 1, 5, 5), 2.5), (3, 3), (2, 2)), 2.5, atol=1e-15)
    assert abs(O.avgpool_bwd(dy, (6, 8), (2, 2), (2, 2)).sum() - dy.sum()) < 1e-12


# ---- the pooling layer with bias and sigma (Eq. 3) -------------------------------------------------------
@pytest.mark.parametrize("mode", ["max", "avg"])
@pytest.mark.parametrize("act", ["none", "relu", "tanh", "sigmoid"])
def test_pool_layer_matches_library_composition_and_finite_differences(mode, act):
    """Eq. 3, y = sigma(phi_p(x) + b): forward against torch's CPU pooling + broadcast bias + activation in fp64;
    backward (dx, dbias) against central differences of a random linear functional of y."""
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    rng = np.random.default_rng(4100)
    n, c, h, w, win, st = 2, 3, 7, 8, 3, 2
    x = rng.standard_normal((n, c, h, w))
    bias = rng.standard_normal(c)
    g = rng.standard_normal((n, c, (h - win) // st + 1, (w - win) // st + 1))
    y, am = O.pool_layer_fwd(x, bias, (win, win), (st, st), mode, act)
    xt = torch.from_numpy(x)
    pooled = F.max_pool2d(xt, win, st) if mode == "max" else F.avg_pool2d(xt, win, st)
    z = pooled + torch.from_numpy(bias)[None, :, None, None]
    want = {"none": z, "relu": torch.relu(z), "tanh": torch.tanh(z), "sigmoid": torch.sigmoid(z)}[act]
    np.testing.assert_allclose(y, want.numpy(), rtol=1e-13, atol=1e-15)

    dx, db, delta = O.pool_layer_bwd(y, g, am, (h, w), (win, win), (st, st), mode, act)
    assert delta.shape == y.shape

    def loss():  # central_diff perturbs x / bias in place
        return float(np.sum(O.pool_layer_fwd(x, bias, (win, win), (st, st), mode, act)[0] * g))

    # random x: no ties, and no pre-activation within the step of the ReLU kink
    np.testing.assert_allclose(dx, central_diff(loss, x), rtol=2e-6, atol=1e-8)
    np.testing.assert_allclose(db, central_diff(loss, bias), rtol=2e-6, atol=1e-8)


def test_pool_layer_without_bias_and_sigma_is_plain_pooling():
    rng = np.random.default_rng(4101)
    x = rng.standard_normal((2, 2, 6, 6))
    y, am = O.pool_layer_fwd(x, None, (2, 2), (2, 2))
    ry, ram = O.maxpool_fwd(x, (2, 2), (2, 2))
    np.testing.assert_array_equal(y, ry)
    np.testing.assert_array_equal(am, ram)
    g = rng.standard_normal(y.shape)
    dx, db, delta = O.pool_layer_bwd(y, g, am, (6, 6), (2, 2), (2, 2))
    np.testing.assert_array_equal(dx, O.maxpool_bwd(g, ram, (6, 6)))
    np.testing.assert_array_equal(delta, g)
    np.testing.assert_allclose(db, g.sum(axis=(0, 2, 3)))
    # a constant shift of one map's bias shifts exactly that map's output (max and mean commute with it)
    y2 = O.pool_layer_fwd(x, np.array([0.0, 1.5]), (2, 2), (2, 2))[0]
    np.testing.assert_allclose(y2[:, 1], ry[:, 1] + 1.5)
    np.testing.assert_array_equal(y2[:, 0], ry[:, 0])


# ---- the chain's handling of discrete decisions ------------------------------------------------------------
def test_chain_store_hook_and_decision_overrides():
    """`store` = identity and `decisions` = the chain's own decisions change nothing; a stored activation is what
    the next layer reads; an overridden pooling choice or ReLU side moves the gradient by exactly the routed
    amount (checked on a two-layer chain by hand)."""
    from oracle.net import train_step
    from paper_1501_07338_amd import workloads as wl
    net = wl.make_net("cfg2", 3)
    inputs, params = wl.make_inputs(net), wl.make_params(net)
    ref = train_step(net, inputs, params)
    same = train_step(net, inputs, params, store=lambda a: a)
    relu_own = {li: ref["acts"][li + 1] > 0 for li, L in enumerate(net.layers) if getattr(L, "relu", False)}
    own = train_step(net, inputs, params, decisions={"argmax": ref["argmax"], "relu": relu_own})
    for a, b, c in zip(ref["dacts"], same["dacts"], own["dacts"]):
        np.testing.assert_array_equal(a, b)
        np.testing.assert_array_equal(a, c)
    # a coarser storage type: every stored activation is on its grid, and layer li+1 is computed from it
    grid = lambda a: np.round(np.asarray(a) * 64.0) / 64.0
    q = train_step(net, inputs, params, store=grid)
    for a in q["acts"][1:]:
        np.testing.assert_array_equal(a, grid(a))
    L0 = net.layers[0]
    np.testing.assert_array_equal(q["acts"][1], grid(O.conv_fwd(q["acts"][0], params[0][0], params[0][1], relu=L0.relu)))
    np.testing.assert_array_equal(q["acts"][2], grid(O.maxpool_fwd(q["acts"][1], (2, 2), (2, 2))[0]))
    # by hand: conv (1x1 kernel, weight 1) -> ReLU -> 2x2 pool, upstream gradient g
    tiny = wl.Net("tiny", 9, 1, (1, 2, 2), [wl.Conv(1, 1, 1, relu=True), wl.Pool(2, 2)], "upstream")
    x = np.array([[[[1.0, 3.0], [2.0, -1.0]]]])
    g = np.array([[[[5.0]]]])
    p = [(np.ones((1, 1, 1, 1)), np.zeros(1)), None]
    r0 = train_step(tiny, {"x": x, "upstream": g}, p)
    np.testing.assert_array_equal(r0["dacts"][0], [[[[0.0, 5.0], [0.0, 0.0]]]])       # the maximum is the 3
    r1 = train_step(tiny, {"x": x, "upstream": g}, p, decisions={"argmax": {1: np.array([[[[2]]]], dtype=np.int32)}})
    np.testing.assert_array_equal(r1["dacts"][0], [[[[0.0, 0.0], [5.0, 0.0]]]])       # routed to flat index 2 instead
    r2 = train_step(tiny, {"x": x, "upstream": g}, p, decisions={"relu": {0: np.zeros((1, 1, 2, 2), dtype=bool)}})
    np.testing.assert_array_equal(r2["dacts"][0], np.zeros((1, 1, 2, 2)))             # every ReLU input taken as <= 0
    np.testing.assert_array_equal(r2["acts"][1], r0["acts"][1])                       # forward tensors untouched


def _golden_shape_cases():
    from pathlib import Path
    cases = []
    for line in (Path(__file__).parent / "golden" / "paper_shapes.txt").read_text().splitlines():
        if line.strip() and not line.startswith("#"):
            kind, cite, args, want = (f.strip() for f in line.split("|"))
            cases.append(pytest.param(kind, args.split(), tuple(int(v) for v in want.split("x")), id=f"{kind}: {cite[:50]}"))
    return cases


@pytest.mark.parametrize("kind,args,want", _golden_shape_cases())
def test_paper_shapes_fixture(kind, args, want):
    """The shapes the paper states (tests/golden/paper_shapes.txt, each with its passage) come out of the oracle."""
    dims = lambda t: tuple(int(v) for v in t.split("x"))
    if kind == "conv":
        (c, h, w), (k, r, s), ph, pw = dims(args[0]), dims(args[1]), int(args[2]), int(args[3])
        if c * r * s * k * h * w > 2e8:  # the large layers: the output-shape rule alone (no arithmetic)
            assert (k, h + 2 * ph - r + 1, w + 2 * pw - s + 1) == want
        else:
            assert O.conv_fwd(np.zeros((1, c, h, w)), np.zeros((k, c, r, s)), pad=(ph, pw)).shape[1:] == want
    elif kind == "unroll":
        (c, h, w), (r, s), batch = dims(args[0]), dims(args[1]), int(args[2])
        assert O.im2col(np.zeros((batch, c, h, w)), (r, s)).shape == want
    else:
        (h, w), win, stride = dims(args[0]), int(args[1]), int(args[2])
        assert O.maxpool_fwd(np.zeros((1, 1, h, w)), (win, win), (stride, stride))[0].shape[2:] == want
