"""Per-operator parity of the HIP path (through the C ABI) against the fp64 oracle, on seeded inputs
whose sizes span several tiles and leave ragged tails."""
import numpy as np
import pytest
import torch

import oracle as O
from paper_1501_07338_amd import vcnn
from paper_1501_07338_amd.workloads import random_tensor
from util import TOL_F32, assert_close, rel_err, to_dev, to_np

pytestmark = pytest.mark.gpu

DEV = "cuda:0"

# (n, c, h, w, k, r, s, ph, pw): ragged everything; M below / at / above one MFMA tile; K and N not
# multiples of the tile sizes; odd N (scalar store path); 1x1; tall and wide kernels.
CONV_SHAPES = [
    (2, 1, 9, 9, 3, 2, 2, 0, 0),
    (3, 5, 19, 23, 37, 3, 5, 1, 2),
    (8, 1, 28, 28, 6, 5, 5, 0, 0),
    (5, 3, 17, 15, 1, 5, 5, 2, 2),
    (3, 7, 13, 11, 130, 3, 3, 1, 1),
    (2, 20, 12, 12, 50, 5, 5, 0, 0),
    (4, 33, 10, 10, 40, 1, 1, 0, 0),
    (1, 2, 40, 9, 5, 21, 1, 0, 0),
    (1, 3, 9, 40, 5, 1, 21, 0, 0),
    (2, 4, 20, 20, 64, 9, 9, 4, 4),
    (3, 2, 6, 7, 4, 1, 1, 1, 1),
    (1, 1, 5, 5, 1, 5, 5, 0, 0),
    (3, 19, 21, 22, 1, 8, 8, 0, 0),     # one output map, many channels (channel slices)
    (2, 9, 30, 13, 3, 5, 4, 2, 1),      # three output maps
    (2, 2, 33, 70, 21, 3, 9, 1, 4),     # two input channels, wide rows
    (5, 4, 12, 12, 9, 16, 16, 8, 8),    # kernel larger than the image interior
    (2, 1, 70, 70, 7, 21, 1, 0, 0),     # tall single-column kernel
    (65, 3, 63, 65, 8, 3, 3, 1, 1),     # at most 32 maps on many large images: the 512-pixel tile
    (2, 6, 40, 40, 48, 5, 5, 2, 2),     # 33..48 output maps: 16-row matrix-core tiles, wide pixel tile
    (3, 38, 14, 14, 38, 3, 3, 1, 1),    # ... in both directions (the input gradient has 38 maps too), small image
    (2, 40, 9, 30, 44, 2, 3, 0, 1),     # ... ragged everything
    (3, 6, 9, 11, 7, 4, 3, 2, 0),       # small layer (fused input gradient): ragged channel group, odd map count, 3 pixel tiles
    (2, 9, 6, 14, 33, 1, 1, 1, 0),      # ... one tap with padding, 4 pixel tiles, two batches of maps
    (2, 8, 6, 6, 40, 5, 6, 4, 5),       # ... 'full' padding, 30 taps, large LDS tile
    (2, 6, 8, 8, 70, 3, 3, 1, 1),       # ... more than 64 maps: the kernel-matrix entries come in two batches
    (200, 16, 7, 7, 8, 3, 3, 1, 1),     # ... more blocks than are resident at once (the tighter register budget)
    (3, 20, 7, 7, 40, 1, 1, 0, 0),      # 1 x 1 with an odd pixel count: groups of four run over the end of a sample
    (5, 130, 5, 5, 70, 1, 1, 0, 0),     # ... two column tiles of the kernel matrix, three row tiles, 125 columns in all
    (2, 33, 3, 1, 64, 1, 1, 0, 0),      # ... fewer pixels per sample than one group of four
    (2, 64, 12, 12, 1, 4, 4, 0, 0),     # one map over 32 and more channels: the taps as rows of a matrix-core product
    (3, 32, 13, 10, 1, 5, 5, 2, 2),     # ... the fewest channels that take this route (the denoising network's last layer)
    (3, 70, 9, 11, 1, 5, 5, 2, 2),      # ... padded ('same'), odd pixel counts
    (2, 130, 14, 9, 1, 8, 3, 0, 1),     # ... rectangular kernel, padded along one axis only
    (2, 136, 11, 9, 1, 7, 7, 3, 3),     # ... 49 taps (an odd count on two row tiles) on an odd plane, 128 and more channels: the streaming product
    (2, 1, 150, 200, 38, 121, 1, 0, 0), # tall kernel on a wide plane: tiles are strips of rows x columns (16-row matrix-core tiles)
    (2, 2, 100, 230, 20, 90, 1, 3, 0),  # ... 32-row tiles, padded rows, two channels
    (1, 1, 140, 190, 64, 100, 2, 0, 1), # ... 64 maps, two-column kernel, padded columns
    (2, 1, 130, 210, 40, 60, 2, 0, 0),  # ... kernel gradient with the whole 120-column kernel matrix per block
]


@pytest.fixture(params=["auto", "explicit", "implicit"])
def algo(request):
    """Runs a test with the per-shape kernel choice, with the unroll forced explicit (phi_c as its own
    kernel + matrix product) and with the implicit matrix-core kernel preferred wherever it applies, so
    every realisation stays covered."""
    vcnn.set_conv_algo({"auto": vcnn.ALGO_AUTO, "explicit": vcnn.ALGO_EXPLICIT, "implicit": vcnn.ALGO_IMPLICIT}[request.param])
    yield request.param
    vcnn.set_conv_algo(vcnn.ALGO_AUTO)


def ws_for(d, which):
    need = vcnn.conv_workspace_bytes(d, which)
    return torch.empty(max(need, 256), dtype=torch.uint8, device=DEV)


def conv_case(shape, seed):
    n, c, h, w, k, r, s, ph, pw = shape
    x = random_tensor(seed, (n, c, h, w))
    wt = random_tensor(seed + 1, (k, c, r, s), scale=(2.0 / (c * r * s)) ** 0.5)
    b = random_tensor(seed + 2, (k,), scale=0.1)
    oh, ow = h + 2 * ph - r + 1, w + 2 * pw - s + 1
    dy = random_tensor(seed + 3, (n, k, oh, ow))
    return x, wt, b, dy


@pytest.mark.parametrize("shape", CONV_SHAPES)
def test_im2col_bit_exact(shape):
    n, c, h, w, k, r, s, ph, pw = shape
    x, *_ = conv_case(shape, 100)
    d = vcnn.conv_desc(n, c, h, w, k, r, s, ph, pw)
    oh, ow = vcnn.conv_out_shape(d)
    col = torch.full((c * r * s, n * oh * ow), float("nan"), device=DEV)
    vcnn.im2col(d, to_dev(x), col)
    ref = O.im2col(x, (r, s), pad=(ph, pw)).astype(np.float32)
    np.testing.assert_array_equal(to_np(col), ref)


@pytest.mark.parametrize("shape", CONV_SHAPES)
def test_col2im(shape):
    n, c, h, w, k, r, s, ph, pw = shape
    d = vcnn.conv_desc(n, c, h, w, k, r, s, ph, pw)
    oh, ow = vcnn.conv_out_shape(d)
    col = random_tensor(200, (c * r * s, n * oh * ow))
    dx = torch.full((n, c, h, w), float("nan"), device=DEV)
    vcnn.col2im(d, to_dev(col), dx)
    assert_close(to_np(dx), O.col2im(col, (n, c, h, w), (r, s), pad=(ph, pw)), 1e-6, "col2im")


def test_unroll_adjoint_identity_on_gpu():
    """<im2col(x), y> = <x, col2im(y)> with both operators from the HIP path."""
    n, c, h, w, r, s, ph, pw = 3, 4, 14, 13, 5, 3, 2, 1
    d = vcnn.conv_desc(n, c, h, w, 1, r, s, ph, pw)
    oh, ow = vcnn.conv_out_shape(d)
    x = random_tensor(300, (n, c, h, w))
    yy = random_tensor(301, (c * r * s, n * oh * ow))
    col = torch.empty((c * r * s, n * oh * ow), device=DEV)
    back = torch.empty((n, c, h, w), device=DEV)
    vcnn.im2col(d, to_dev(x), col)
    vcnn.col2im(d, to_dev(yy), back)
    lhs = float(np.sum(to_np(col).astype(np.float64) * yy))
    rhs = float(np.sum(x.astype(np.float64) * to_np(back)))
    assert abs(lhs - rhs) <= 1e-5 * abs(lhs)


@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("shape", CONV_SHAPES)
def test_conv_fwd(shape, relu, algo):
    n, c, h, w, k, r, s, ph, pw = shape
    x, wt, b, _ = conv_case(shape, 400)
    d = vcnn.conv_desc(n, c, h, w, k, r, s, ph, pw, act=vcnn.ACT_RELU if relu else vcnn.ACT_NONE)
    oh, ow = vcnn.conv_out_shape(d)
    y = torch.full((n, k, oh, ow), float("nan"), device=DEV)
    vcnn.conv_fwd(d, to_dev(x), to_dev(wt), to_dev(b), y, ws_for(d, vcnn.PASS_FWD))
    assert_close(to_np(y), O.conv_fwd(x, wt, b, pad=(ph, pw), relu=relu), TOL_F32, "conv_fwd")
    if not relu:  # bias is optional
        vcnn.conv_fwd(d, to_dev(x), to_dev(wt), None, y, ws_for(d, vcnn.PASS_FWD))
        assert_close(to_np(y), O.conv_fwd(x, wt, None, pad=(ph, pw)), TOL_F32, "conv_fwd without bias")


@pytest.mark.parametrize("shape", CONV_SHAPES)
def test_conv_bwd_filter(shape, algo):
    n, c, h, w, k, r, s, ph, pw = shape
    x, _, _, dy = conv_case(shape, 500)
    d = vcnn.conv_desc(n, c, h, w, k, r, s, ph, pw)
    dw = torch.full((k, c, r, s), float("nan"), device=DEV)
    db = torch.full((k,), float("nan"), device=DEV)
    ws = ws_for(d, vcnn.PASS_BWD_FILTER)
    vcnn.conv_bwd_filter(d, to_dev(x), to_dev(dy), dw, db, ws)
    rdw, rdb = O.conv_bwd_filter(x, dy, (r, s), pad=(ph, pw))
    assert_close(to_np(dw), rdw, TOL_F32, "dw")
    assert_close(to_np(db), rdb, TOL_F32, "db")
    # run-to-run bit identity (no floating-point atomics, fixed reduction order)
    first = to_np(dw).copy()
    dw.fill_(float("nan"))
    vcnn.conv_bwd_filter(d, to_dev(x), to_dev(dy), dw, None, ws)
    np.testing.assert_array_equal(to_np(dw), first)


@pytest.mark.parametrize("shape", CONV_SHAPES)
def test_conv_bwd_data(shape, algo):
    n, c, h, w, k, r, s, ph, pw = shape
    _, wt, _, dy = conv_case(shape, 600)
    d = vcnn.conv_desc(n, c, h, w, k, r, s, ph, pw)
    dx = torch.full((n, c, h, w), float("nan"), device=DEV)
    ws = ws_for(d, vcnn.PASS_BWD_DATA)
    vcnn.conv_bwd_data(d, to_dev(wt), to_dev(dy), dx, ws)
    assert_close(to_np(dx), O.conv_bwd_data(wt, dy, (h, w), pad=(ph, pw)), TOL_F32, "dx")
    # run-to-run bit identity (fixed summation order on every route)
    first = to_np(dx).copy()
    dx.fill_(float("nan"))
    vcnn.conv_bwd_data(d, to_dev(wt), to_dev(dy), dx, ws)
    np.testing.assert_array_equal(to_np(dx), first)


def _act_output(act, x):
    """A tensor that can be the forward output of `act`: the input of the layer above."""
    if act == vcnn.ACT_RELU:
        return np.maximum(x, 0).astype(np.float32)
    if act == vcnn.ACT_TANH:
        return np.tanh(x).astype(np.float32)
    return (np.tanh(x) * 0.5 + 0.5).astype(np.float32)


def _act_bwd_oracle(act, y, g):
    if act == vcnn.ACT_RELU:
        return O.relu_bwd(y, g)
    return O.tanh_bwd(y, g) if act == vcnn.ACT_TANH else O.sigmoid_bwd(y, g)


@pytest.mark.parametrize("shape", CONV_SHAPES)
def test_conv_bwd_data_with_activation_derivative_folded(shape, algo):
    """conv_bwd_data_act = conv_bwd_data followed by act_bwd against the layer's input (an activation's output), on
    every route: fused into the store where the route has it, as a pass over dx in place elsewhere."""
    n, c, h, w, k, r, s, ph, pw = shape
    x, wt, _, dy = conv_case(shape, 640)
    d = vcnn.conv_desc(n, c, h, w, k, r, s, ph, pw)
    ws = ws_for(d, vcnn.PASS_BWD_DATA)
    plain = O.conv_bwd_data(wt, dy, (h, w), pad=(ph, pw))
    acts = [vcnn.ACT_RELU] if (n * c * h * w) % 3 else [vcnn.ACT_RELU, vcnn.ACT_TANH, vcnn.ACT_SIGMOID]
    for act in acts:
        xin = _act_output(act, x)
        dx = torch.full((n, c, h, w), float("nan"), device=DEV)
        vcnn.conv_bwd_data_act(d, act, to_dev(xin), to_dev(wt), to_dev(dy), dx, ws)
        assert_close(to_np(dx), _act_bwd_oracle(act, xin.astype(np.float64), plain), TOL_F32, f"dx * sigma' (act {act})")
        if act == vcnn.ACT_RELU:  # the mask is exact: zero wherever the input is not positive
            assert not np.any(to_np(dx)[xin <= 0])
    # no activation below: the plain call, x not read
    dx = torch.full((n, c, h, w), float("nan"), device=DEV)
    vcnn.conv_bwd_data_act(d, vcnn.ACT_NONE, None, to_dev(wt), to_dev(dy), dx, ws)
    ref = torch.empty_like(dx)
    vcnn.conv_bwd_data(d, to_dev(wt), to_dev(dy), ref, ws)
    np.testing.assert_array_equal(to_np(dx), to_np(ref))


def test_bwd_filter_split_contraction_many_columns():
    """Long contraction (N = 8*61*67 columns) so the filter gradient is split into several partial sums."""
    shape = (8, 3, 63, 69, 10, 3, 3, 0, 0)
    n, c, h, w, k, r, s, ph, pw = shape
    x, _, _, dy = conv_case(shape, 700)
    d = vcnn.conv_desc(n, c, h, w, k, r, s, ph, pw)
    dw = torch.empty((k, c, r, s), device=DEV)
    db = torch.empty((k,), device=DEV)
    vcnn.conv_bwd_filter(d, to_dev(x), to_dev(dy), dw, db, ws_for(d, vcnn.PASS_BWD_FILTER))
    rdw, rdb = O.conv_bwd_filter(x, dy, (r, s))
    assert_close(to_np(dw), rdw, TOL_F32, "dw")
    assert_close(to_np(db), rdb, TOL_F32, "db")


# layers the fused route of the input gradient (transposed product + phi_c^{-1} per tile on chip) accepts: at least
# 64 output maps, and the input pixels one 128 x 128 tile of the patch-matrix gradient touches fit a small LDS region
FOLD_SHAPES = [
    (2, 2, 70, 70, 130, 16, 16, 0, 0),   # one channel per row tile (256 taps), 24 column tiles, contraction tail (130 maps)
    (3, 5, 14, 18, 64, 16, 16, 8, 8),    # padded: region rows and columns outside the image are dropped
    (2, 3, 20, 20, 70, 8, 8, 0, 0),      # 64 taps per channel: a row tile spans two channels, the last one is short
    (1, 7, 9, 9, 64, 3, 3, 1, 1),        # K = 63: one ragged row tile over all channels, scalar kernel-matrix loads
    (2, 1, 40, 33, 96, 11, 12, 3, 0),    # one channel, 132 taps: the second row tile holds 4 rows
    (4, 38, 20, 20, 72, 16, 16, 0, 0),   # the shape family of the deconvolution network's third layer (5 x 5 outputs)
    (1, 3, 20, 20, 256, 8, 8, 0, 0),     # 128 maps and more: the bf16 variant contracts on the bf16 matrix cores
    (2, 5, 14, 18, 136, 16, 16, 8, 8),   # ... padded, contraction tail (136 = 17 words of 8)
    (3, 2, 40, 40, 200, 16, 16, 0, 0),   # ... 625 pixels per sample: five column tiles of 128, the last one short
]


@pytest.mark.parametrize("dtype", [vcnn.F32, vcnn.BF16])
@pytest.mark.parametrize("shape", FOLD_SHAPES)
def test_conv_bwd_data_fused_fold_route(shape, dtype):
    n, c, h, w, k, r, s, ph, pw = shape
    x, wt, b, dy = conv_case(shape, 1900)
    tol = TOL_F32
    cast = lambda t: t
    if dtype == vcnn.BF16:
        from paper_1501_07338_amd.workloads import bf16_round
        from util import TOL_BF16
        wt, dy, tol = bf16_round(wt), bf16_round(dy), TOL_BF16
        cast = lambda t: t.to(torch.bfloat16)
    d = vcnn.conv_desc(n, c, h, w, k, r, s, ph, pw, dtype=dtype)
    want = O.conv_bwd_data(wt, dy, (h, w), pad=(ph, pw))
    wd, dyd = cast(to_dev(wt)), cast(to_dev(dy))
    try:
        other = []
        for a in (vcnn.ALGO_EXPLICIT, vcnn.ALGO_IMPLICIT):
            vcnn.set_conv_algo(a)
            other.append(vcnn.conv_workspace_bytes(d, vcnn.PASS_BWD_DATA))
        vcnn.set_conv_algo(vcnn.ALGO_FOLD)
        need = vcnn.conv_workspace_bytes(d, vcnn.PASS_BWD_DATA)
        # its workspace holds the folded regions only: not the patch-matrix gradient, not a flipped kernel matrix
        assert 0 < need < other[0] and need != other[1], "the fused route was not taken"
        ws = torch.empty(need, dtype=torch.uint8, device=DEV)
        ws.fill_(0xFF)  # NaN patterns: nothing may be read before it is written
        dx = cast(torch.full((n, c, h, w), float("nan"), device=DEV))
        vcnn.conv_bwd_data(d, wd, dyd, dx, ws)
        assert_close(to_np(dx.float()), want, tol, "fused fold dx")
        dx2 = cast(torch.full((n, c, h, w), float("nan"), device=DEV))
        vcnn.conv_bwd_data(d, wd, dyd, dx2, ws)
        torch.cuda.synchronize()
        assert torch.equal(dx, dx2), "not bit-identical from run to run"
    finally:
        vcnn.set_conv_algo(vcnn.ALGO_AUTO)


# layers with one-dimensional kernels, for the Fourier-domain forward pass (the paper's related-work comparison)
FFT_SHAPES = [
    (2, 3, 9, 40, 5, 1, 21, 0, 0),       # 1 x 21 on rows of 40: transform length 64
    (1, 2, 40, 9, 5, 21, 1, 0, 0),       # 21 x 1 on columns
    (3, 5, 7, 33, 20, 1, 9, 0, 4),       # padded along the kernel: 'same' rows
    (2, 4, 33, 7, 3, 9, 1, 4, 0),        # ... columns
    (2, 1, 70, 70, 7, 21, 1, 0, 0),      # one channel, transform length 128
    (2, 38, 6, 184, 38, 1, 121, 0, 0),   # the deconvolution network's second layer on a few rows (length 256)
    (1, 1, 184, 20, 38, 121, 1, 0, 0),   # ... its first layer on a few columns
    (1, 2, 3, 600, 2, 1, 100, 0, 0),     # transform length 1024
    (2, 3, 5, 16, 4, 1, 16, 0, 0),       # kernel as long as the line: one output per line
    (1, 17, 4, 50, 33, 1, 8, 0, 7),      # 'full' padding, more maps than one batch of the contraction
]


@pytest.mark.parametrize("dtype", [vcnn.F32, vcnn.BF16])
@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("shape", FFT_SHAPES)
def test_conv_fwd_fourier_route(shape, relu, dtype):
    n, c, h, w, k, r, s, ph, pw = shape
    x, wt, b, _ = conv_case(shape, 2900)
    tol = TOL_F32
    cast = lambda t: t
    if dtype == vcnn.BF16:
        from paper_1501_07338_amd.workloads import bf16_round
        from util import TOL_BF16
        x, wt, tol = bf16_round(x), bf16_round(wt), TOL_BF16
        cast = lambda t: t.to(torch.bfloat16)
    d = vcnn.conv_desc(n, c, h, w, k, r, s, ph, pw, dtype=dtype, act=vcnn.ACT_RELU if relu else vcnn.ACT_NONE)
    oh, ow = vcnn.conv_out_shape(d)
    want = O.conv_fwd(x, wt, b, pad=(ph, pw), relu=relu)
    try:
        vcnn.set_conv_algo(vcnn.ALGO_AUTO)
        plain = vcnn.conv_workspace_bytes(d, vcnn.PASS_FWD)
        vcnn.set_conv_algo(vcnn.ALGO_FFT)
        need = vcnn.conv_workspace_bytes(d, vcnn.PASS_FWD)
        assert need > plain and need >= 8 * (c + k) * n * (h if r == 1 else w) * 17, "the Fourier route was not taken"
        ws = torch.empty(need, dtype=torch.uint8, device=DEV)
        ws.fill_(0xFF)  # NaN patterns: nothing may be read before it is written
        y = cast(torch.full((n, k, oh, ow), float("nan"), device=DEV))
        vcnn.conv_fwd(d, cast(to_dev(x)), cast(to_dev(wt)), to_dev(b), y, ws)
        assert_close(to_np(y.float()), want, tol, "Fourier-domain forward")
    finally:
        vcnn.set_conv_algo(vcnn.ALGO_AUTO)


POOL_SHAPES = [(2, 3, 4, 4, 2, 2), (3, 5, 24, 24, 2, 2), (2, 7, 32, 32, 3, 2), (3, 4, 15, 15, 3, 2), (2, 2, 7, 7, 3, 2),
               (1, 3, 9, 11, 2, 1), (2, 2, 5, 6, 5, 1), (1, 1, 3, 3, 3, 3)]


@pytest.mark.parametrize("ties", [False, True])
@pytest.mark.parametrize("shape", POOL_SHAPES)
def test_pool_fwd_bwd(shape, ties):
    n, c, h, w, win, st = shape
    x = random_tensor(800, (n, c, h, w))
    if ties:  # few distinct values (as after a ReLU): equal maxima must resolve to the lowest index
        x = np.maximum(np.round(x * 2) / 2, 0).astype(np.float32)
    d = vcnn.pool_desc(n, c, h, w, win, win, st, st)
    oh, ow = vcnn.pool_out_shape(d)
    y = torch.full((n, c, oh, ow), float("nan"), device=DEV)
    am = torch.full((n, c, oh, ow), -7, dtype=torch.int32, device=DEV)
    vcnn.pool_fwd(d, to_dev(x), y, am)
    ry, ram = O.maxpool_fwd(x, (win, win), (st, st))
    np.testing.assert_array_equal(to_np(am), ram)
    np.testing.assert_array_equal(to_np(y), ry.astype(np.float32))
    dy = random_tensor(801, (n, c, oh, ow))
    dx = torch.full((n, c, h, w), float("nan"), device=DEV)
    vcnn.pool_bwd(d, to_dev(dy), am, dx)
    assert_close(to_np(dx), O.maxpool_bwd(dy, ram, (h, w)), 1e-6, "pool dx")


# (n, c, h, w, (win_h, win_w), (stride_h, stride_w)): windows and strides that differ between the two axes
RECT_POOL_SHAPES = [(2, 3, 9, 11, (2, 3), (1, 2)), (3, 4, 16, 12, (3, 2), (2, 1)), (2, 5, 32, 32, (3, 2), (2, 2)),
                    (1, 2, 7, 20, (1, 4), (1, 3)), (2, 2, 13, 6, (5, 1), (2, 1)), (130, 6, 12, 10, (2, 3), (2, 3)),
                    (1, 1, 4, 9, (4, 2), (3, 5))]


@pytest.mark.parametrize("ties", [False, True])
@pytest.mark.parametrize("shape", RECT_POOL_SHAPES)
def test_pool_rectangular_windows_and_strides(shape, ties):
    """win_h != win_w and stride_h != stride_w through every pooling call: max forward (values, argmax), its
    routing gradient alone and with an activation derivative folded in, the mean and its transpose, and the
    pooling layer of Eq. 3 with bias and sigma."""
    n, c, h, w, win, st = shape
    x = random_tensor(830, (n, c, h, w))
    if ties:
        x = np.maximum(np.round(x * 2) / 2, 0).astype(np.float32)
    d = vcnn.pool_desc(n, c, h, w, win[0], win[1], st[0], st[1])
    oh, ow = vcnn.pool_out_shape(d)
    assert (oh, ow) == ((h - win[0]) // st[0] + 1, (w - win[1]) // st[1] + 1)
    y = torch.full((n, c, oh, ow), float("nan"), device=DEV)
    am = torch.full((n, c, oh, ow), -7, dtype=torch.int32, device=DEV)
    vcnn.pool_fwd(d, to_dev(x), y, am)
    ry, ram = O.maxpool_fwd(x, win, st)
    np.testing.assert_array_equal(to_np(am), ram)
    np.testing.assert_array_equal(to_np(y), ry.astype(np.float32))
    dy = random_tensor(831, (n, c, oh, ow))
    dx = torch.full((n, c, h, w), float("nan"), device=DEV)
    vcnn.pool_bwd(d, to_dev(dy), am, dx)
    rdx = O.maxpool_bwd(dy, ram, (h, w))
    assert_close(to_np(dx), rdx, 1e-6, "pool dx")
    xr = np.maximum(x, 0).astype(np.float32)  # as the output of a ReLU below
    vcnn.pool_fwd(d, to_dev(xr), y, am)
    ram_r = O.maxpool_fwd(xr, win, st)[1]
    np.testing.assert_array_equal(to_np(am), ram_r)
    vcnn.pool_bwd_act(d, vcnn.ACT_RELU, to_dev(xr), to_dev(dy), am, dx)
    assert_close(to_np(dx), O.relu_bwd(xr, O.maxpool_bwd(dy, ram_r, (h, w))), 1e-6, "pool dx * relu'")
    # the mean and its transpose
    da = vcnn.pool_desc(n, c, h, w, win[0], win[1], st[0], st[1], mode=vcnn.POOL_AVG)
    vcnn.pool_fwd(da, to_dev(x), y, None)
    assert_close(to_np(y), O.avgpool_fwd(x, win, st), 1e-6, "avgpool y")
    vcnn.pool_bwd(da, to_dev(dy), None, dx)
    assert_close(to_np(dx), O.avgpool_bwd(dy, (h, w), win, st), 1e-6, "avgpool dx")
    # Eq. 3: sigma(pool + b), and its gradients
    bias = random_tensor(832, (c,))
    for mode, desc in (("max", d), ("avg", da)):
        amx = am if mode == "max" else None
        vcnn.pool_layer_fwd(desc, vcnn.ACT_TANH, to_dev(x), to_dev(bias), y, amx)
        ly, lam = O.pool_layer_fwd(x, bias, win, st, mode, "tanh")
        assert_close(to_np(y), ly, 1e-6, f"{mode} pool layer y")
        if mode == "max":
            np.testing.assert_array_equal(to_np(am), lam)
        y32 = to_np(y)
        db = torch.full((c,), float("nan"), device=DEV)
        ws = torch.empty(max(vcnn.pool_layer_workspace_bytes(desc), 16), dtype=torch.uint8, device=DEV)
        vcnn.pool_layer_bwd(desc, vcnn.ACT_TANH, y, to_dev(dy), amx, db, dx, ws)
        ldx, ldb, _ = O.pool_layer_bwd(y32, dy, lam, (h, w), win, st, mode, "tanh")
        assert_close(to_np(dx), ldx, 1e-6, f"{mode} pool layer dx")
        assert_close(to_np(db), ldb, TOL_F32, f"{mode} pool layer dbias")


def _sigma_bwd(act, y, g):
    return {vcnn.ACT_RELU: O.relu_bwd, vcnn.ACT_TANH: O.tanh_bwd, vcnn.ACT_SIGMOID: O.sigmoid_bwd}[act](y, g)


@pytest.mark.parametrize("act", [vcnn.ACT_RELU, vcnn.ACT_TANH, vcnn.ACT_SIGMOID])
@pytest.mark.parametrize("shape", POOL_SHAPES)
def test_pool_bwd_with_activation_derivative_folded(shape, act):
    """pool_bwd_act = pool_bwd followed by act_bwd against the pooling input (an activation's output)."""
    n, c, h, w, win, st = shape
    x = random_tensor(810, (n, c, h, w))
    x = np.maximum(x, 0).astype(np.float32) if act == vcnn.ACT_RELU else np.tanh(x).astype(np.float32) * 0.5 + 0.5
    d = vcnn.pool_desc(n, c, h, w, win, win, st, st)
    oh, ow = vcnn.pool_out_shape(d)
    y = torch.empty((n, c, oh, ow), device=DEV)
    am = torch.empty((n, c, oh, ow), dtype=torch.int32, device=DEV)
    vcnn.pool_fwd(d, to_dev(x), y, am)
    ram = O.maxpool_fwd(x, (win, win), (st, st))[1]
    np.testing.assert_array_equal(to_np(am), ram)
    dy = random_tensor(811, (n, c, oh, ow))
    dx = torch.full((n, c, h, w), float("nan"), device=DEV)
    vcnn.pool_bwd_act(d, act, to_dev(x), to_dev(dy), am, dx)
    assert_close(to_np(dx), _sigma_bwd(act, x, O.maxpool_bwd(dy, ram, (h, w))), 1e-6, "pool dx * sigma'")
    # no activation below: the plain call, x not read
    vcnn.pool_bwd_act(d, vcnn.ACT_NONE, None, to_dev(dy), am, dx)
    assert_close(to_np(dx), O.maxpool_bwd(dy, ram, (h, w)), 1e-6, "pool dx")
    # average pooling takes the same call
    da = vcnn.pool_desc(n, c, h, w, win, win, st, st, mode=vcnn.POOL_AVG)
    vcnn.pool_bwd_act(da, act, to_dev(x), to_dev(dy), None, dx)
    assert_close(to_np(dx), _sigma_bwd(act, x, O.avgpool_bwd(dy, (h, w), (win, win), (st, st))), 1e-6, "avgpool dx * sigma'")


_ACT_NAME = {vcnn.ACT_NONE: "none", vcnn.ACT_RELU: "relu", vcnn.ACT_TANH: "tanh", vcnn.ACT_SIGMOID: "sigmoid"}


@pytest.mark.parametrize("mode", ["max", "avg"])
@pytest.mark.parametrize("act", [vcnn.ACT_NONE, vcnn.ACT_RELU, vcnn.ACT_TANH, vcnn.ACT_SIGMOID])
@pytest.mark.parametrize("shape", [(3, 5, 24, 24, 2, 2), (2, 7, 32, 32, 3, 2), (130, 20, 9, 11, 2, 1), (1, 1, 3, 3, 3, 3)])
def test_pool_layer_bias_sigma(shape, act, mode):
    """The pooling layer of Eq. 3, y = sigma(pool(x) + b), and its gradients (dx, dbias) against the oracle."""
    n, c, h, w, win, st = shape
    x, bias = random_tensor(820, (n, c, h, w)), random_tensor(821, (c,))
    d = vcnn.pool_desc(n, c, h, w, win, win, st, st, mode=vcnn.POOL_MAX if mode == "max" else vcnn.POOL_AVG)
    oh, ow = vcnn.pool_out_shape(d)
    y = torch.full((n, c, oh, ow), float("nan"), device=DEV)
    am = torch.full((n, c, oh, ow), -7, dtype=torch.int32, device=DEV) if mode == "max" else None
    vcnn.pool_layer_fwd(d, act, to_dev(x), to_dev(bias), y, am)
    ry, ram = O.pool_layer_fwd(x, bias, (win, win), (st, st), mode, _ACT_NAME[act])
    assert_close(to_np(y), ry, 1e-6, "pool layer y")
    if mode == "max":
        np.testing.assert_array_equal(to_np(am), ram)
    # backward from the GPU's own fp32 output, so both sides evaluate sigma' at the same point
    y32 = to_np(y)
    dy = random_tensor(822, (n, c, oh, ow))
    dx = torch.full((n, c, h, w), float("nan"), device=DEV)
    db = torch.full((c,), float("nan"), device=DEV)
    ws = torch.empty(max(vcnn.pool_layer_workspace_bytes(d), 16), dtype=torch.uint8, device=DEV)
    vcnn.pool_layer_bwd(d, act, y, to_dev(dy), am, db, dx, ws)
    rdx, rdb, _ = O.pool_layer_bwd(y32, dy, ram, (h, w), (win, win), (st, st), mode, _ACT_NAME[act])
    assert_close(to_np(dx), rdx, 1e-6, "pool layer dx")
    assert_close(to_np(db), rdb, TOL_F32, "pool layer dbias")
    # without the bias gradient; a workspace that is too small is refused before any launch
    dx2 = torch.full((n, c, h, w), float("nan"), device=DEV)
    vcnn.pool_layer_bwd(d, act, y, to_dev(dy), am, None, dx2, ws)
    assert torch.equal(dx, dx2)
    if act != vcnn.ACT_NONE:
        with pytest.raises(vcnn.VcnnError):
            vcnn.pool_layer_bwd(d, act, y, to_dev(dy), am, db, dx2, ws[:8])


@pytest.mark.parametrize("act", [vcnn.ACT_RELU, vcnn.ACT_TANH, vcnn.ACT_SIGMOID])
@pytest.mark.parametrize("b,i,o", [(128, 800, 500), (128, 500, 10), (7, 33, 5), (256, 2048, 1000)])
def test_fc_bwd_with_activation_derivative_folded(b, i, o, act):
    """fc_bwd_act = fc_bwd with act_bwd against the layer's input applied to dx (small and large product kernels)."""
    x = random_tensor(1010, (b, i))
    x = np.maximum(x, 0).astype(np.float32) if act == vcnn.ACT_RELU else np.tanh(x).astype(np.float32) * 0.5 + 0.5
    w, dy = random_tensor(1011, (o, i), scale=(2.0 / i) ** 0.5), random_tensor(1012, (b, o))
    dx = torch.full((b, i), float("nan"), device=DEV)
    dw, db = torch.full((o, i), float("nan"), device=DEV), torch.full((o,), float("nan"), device=DEV)
    vcnn.fc_bwd_act(vcnn.F32, b, i, o, act, to_dev(x), to_dev(w), to_dev(dy), dw, db, dx)
    rdw, rdb, rdx = O.fc_bwd(x, w, dy)
    assert_close(to_np(dx), _sigma_bwd(act, x, rdx), TOL_F32, "fc dx * sigma'")
    assert_close(to_np(dw), rdw, TOL_F32, "fc dw")
    assert_close(to_np(db), rdb, TOL_F32, "fc db")
    # the input gradient alone gives the same bits; without an activation below it is the plain call
    dx2 = torch.full((b, i), float("nan"), device=DEV)
    vcnn.fc_bwd_act(vcnn.F32, b, i, o, act, to_dev(x), to_dev(w), to_dev(dy), None, None, dx2)
    assert torch.equal(dx, dx2)
    plain = torch.full((b, i), float("nan"), device=DEV)
    vcnn.fc_bwd(vcnn.F32, b, i, o, None, to_dev(w), to_dev(dy), None, None, plain)
    vcnn.fc_bwd_act(vcnn.F32, b, i, o, vcnn.ACT_NONE, None, to_dev(w), to_dev(dy), None, None, dx)
    assert torch.equal(dx, plain)


@pytest.mark.parametrize("count", [1, 3, 4, 1023, 4099])
def test_act(count):
    x = random_tensor(900, (count,))
    x[::5] = 0.0
    dy = random_tensor(901, (count,))
    y = torch.full((count,), float("nan"), device=DEV)
    vcnn.act_fwd(vcnn.ACT_RELU, vcnn.F32, count, to_dev(x), y)
    np.testing.assert_array_equal(to_np(y), O.relu_fwd(x).astype(np.float32))
    dx = torch.full((count,), float("nan"), device=DEV)
    vcnn.act_bwd(vcnn.ACT_RELU, vcnn.F32, count, to_dev(x), to_dev(dy), dx)
    np.testing.assert_array_equal(to_np(dx), O.relu_bwd(x, dy).astype(np.float32))
    # in place, with the forward output as reference
    g = to_dev(dy)
    vcnn.act_bwd(vcnn.ACT_RELU, vcnn.F32, count, y, g, g)
    np.testing.assert_array_equal(to_np(g), O.relu_bwd(x, dy).astype(np.float32))
    xin = to_dev(x)
    vcnn.act_fwd(vcnn.ACT_RELU, vcnn.F32, count, xin, xin)
    np.testing.assert_array_equal(to_np(xin), O.relu_fwd(x).astype(np.float32))


@pytest.mark.parametrize("b,i,o", [(128, 800, 500), (128, 500, 10), (7, 33, 5), (1, 1, 1), (130, 70, 131), (128, 576, 64), (40, 100, 48)])
@pytest.mark.parametrize("relu", [False, True])
def test_fc(b, i, o, relu):
    x, w, bias = random_tensor(1000, (b, i)), random_tensor(1001, (o, i), scale=(2.0 / i) ** 0.5), random_tensor(1002, (o,))
    dy = random_tensor(1003, (b, o))
    y = torch.full((b, o), float("nan"), device=DEV)
    vcnn.fc_fwd(vcnn.F32, b, i, o, vcnn.ACT_RELU if relu else vcnn.ACT_NONE, to_dev(x), to_dev(w), to_dev(bias), y)
    assert_close(to_np(y), O.fc_fwd(x, w, bias, relu=relu), TOL_F32, "fc y")
    dw = torch.full((o, i), float("nan"), device=DEV)
    db = torch.full((o,), float("nan"), device=DEV)
    dx = torch.full((b, i), float("nan"), device=DEV)
    vcnn.fc_bwd(vcnn.F32, b, i, o, to_dev(x), to_dev(w), to_dev(dy), dw, db, dx)
    rdw, rdb, rdx = O.fc_bwd(x, w, dy)
    assert_close(to_np(dw), rdw, TOL_F32, "fc dw")
    assert_close(to_np(db), rdb, TOL_F32, "fc db")
    assert_close(to_np(dx), rdx, TOL_F32, "fc dx")
    # the two strands issued separately (parameter gradients / input gradient) give the same bits
    dw2, db2, dx2 = torch.full_like(dw, float("nan")), torch.full_like(db, float("nan")), torch.full_like(dx, float("nan"))
    vcnn.fc_bwd(vcnn.F32, b, i, o, to_dev(x), None, to_dev(dy), dw2, db2, None)
    vcnn.fc_bwd(vcnn.F32, b, i, o, None, to_dev(w), to_dev(dy), None, None, dx2)
    assert torch.equal(dw, dw2) and torch.equal(db, db2) and torch.equal(dx, dx2)


@pytest.mark.parametrize("act,fwd,bwd", [(vcnn.ACT_TANH, O.tanh_fwd, O.tanh_bwd), (vcnn.ACT_SIGMOID, O.sigmoid_fwd, O.sigmoid_bwd)])
@pytest.mark.parametrize("count", [1, 255, 4099])
def test_tanh_sigmoid_fwd_bwd(act, fwd, bwd, count):
    x = random_tensor(1700, (count,), scale=3.0)
    x[0] = 30.0  # saturation
    dy = random_tensor(1701, (count,))
    y = torch.full((count,), float("nan"), device=DEV)
    vcnn.act_fwd(act, vcnn.F32, count, to_dev(x), y)
    assert_close(to_np(y), fwd(x), 1e-6, "sigma fwd")
    # backward from the forward output: feed both sides the same fp32 output
    yh = to_np(y)
    dx = torch.full((count,), float("nan"), device=DEV)
    vcnn.act_bwd(act, vcnn.F32, count, y, to_dev(dy), dx)
    assert_close(to_np(dx), bwd(yh, dy), 1e-6, "sigma bwd")
    # in place
    z = to_dev(x)
    vcnn.act_fwd(act, vcnn.F32, count, z, z)
    assert torch.equal(z, y)


@pytest.mark.parametrize("act,fwd", [(vcnn.ACT_TANH, O.tanh_fwd), (vcnn.ACT_SIGMOID, O.sigmoid_fwd)])
def test_conv_and_fc_forward_with_smooth_sigma(act, fwd):
    n, c, h, w, k, r, s, ph, pw = 3, 5, 9, 11, 7, 3, 3, 1, 1
    x, wt, b = random_tensor(1710, (n, c, h, w)), random_tensor(1711, (k, c, r, s), scale=0.3), random_tensor(1712, (k,))
    d = vcnn.conv_desc(n, c, h, w, k, r, s, ph, pw, act=act)
    y = torch.full((n, k, h, w), float("nan"), device=DEV)
    vcnn.conv_fwd(d, to_dev(x), to_dev(wt), to_dev(b), y, ws_for(d, vcnn.PASS_FWD))
    assert_close(to_np(y), fwd(O.conv_fwd(x, wt, b, pad=(ph, pw))), TOL_F32, "conv + sigma")
    bsz, i, o = 9, 33, 12
    xf, wf, bf = random_tensor(1713, (bsz, i)), random_tensor(1714, (o, i), scale=0.3), random_tensor(1715, (o,))
    yf = torch.full((bsz, o), float("nan"), device=DEV)
    vcnn.fc_fwd(vcnn.F32, bsz, i, o, act, to_dev(xf), to_dev(wf), to_dev(bf), yf)
    assert_close(to_np(yf), fwd(O.fc_fwd(xf, wf, bf)), TOL_F32, "fc + sigma")


AVG_SHAPES = [(2, 3, 4, 4, 2, 2), (3, 5, 24, 24, 2, 2), (2, 7, 32, 32, 3, 2), (3, 4, 15, 15, 3, 2), (1, 3, 9, 11, 2, 1),
              (2, 2, 5, 6, 5, 1), (1, 1, 3, 3, 3, 3)]


@pytest.mark.parametrize("shape", AVG_SHAPES)
def test_avgpool_fwd_bwd(shape):
    n, c, h, w, win, st = shape
    x = random_tensor(1720, (n, c, h, w))
    d = vcnn.pool_desc(n, c, h, w, win, win, st, st, mode=vcnn.POOL_AVG)
    oh, ow = vcnn.pool_out_shape(d)
    y = torch.full((n, c, oh, ow), float("nan"), device=DEV)
    vcnn.pool_fwd(d, to_dev(x), y, None)  # no argmax record for the average
    assert_close(to_np(y), O.avgpool_fwd(x, (win, win), (st, st)), 1e-6, "avgpool y")
    dy = random_tensor(1721, (n, c, oh, ow))
    dx = torch.full((n, c, h, w), float("nan"), device=DEV)
    vcnn.pool_bwd(d, to_dev(dy), None, dx)
    assert_close(to_np(dx), O.avgpool_bwd(dy, (h, w), (win, win), (st, st)), 1e-6, "avgpool dx")


@pytest.mark.parametrize("b,c", [(128, 10), (1, 10), (300, 7), (5, 1), (70, 16), (33, 17), (9, 100)])
def test_softmax_loss(b, c):
    z = random_tensor(1100, (b, c), scale=3.0)
    labels = (np.arange(b) * 7 % c).astype(np.int32)
    loss = torch.full((), float("nan"), device=DEV)
    dz = torch.full((b, c), float("nan"), device=DEV)
    vcnn.softmax_loss(b, c, to_dev(z), to_dev(labels), loss, dz)
    rl, rdz = O.softmax_loss(z, labels)
    assert abs(float(to_np(loss)) - rl) <= TOL_F32 * max(abs(rl), 1e-3)
    if c > 1:
        assert_close(to_np(dz), rdz, TOL_F32, "dlogits")
    else:
        assert np.max(np.abs(to_np(dz))) < 1e-7


@pytest.mark.parametrize("c", [10, 16, 40])
@pytest.mark.parametrize("bad", [-1, -2147483648, 2147483647, None])
def test_softmax_loss_label_out_of_range_is_flagged_not_dereferenced(c, bad):
    """A label outside [0, classes) must not be used as an index: the call completes, the loss is NaN and so is
    that sample's gradient row; every other row is the ordinary result."""
    b = 37
    bad = c if bad is None else bad
    z = random_tensor(1110, (b, c), scale=2.0)
    labels = (np.arange(b) * 3 % c).astype(np.int32)
    good = labels.copy()
    labels[[4, 20]] = bad
    loss = torch.zeros((), device=DEV)
    dz = torch.zeros((b, c), device=DEV)
    vcnn.softmax_loss(b, c, to_dev(z), to_dev(labels), loss, dz)
    got = to_np(dz)
    assert np.isnan(float(to_np(loss)))
    assert np.all(np.isnan(got[[4, 20]]))
    rows = np.setdiff1d(np.arange(b), [4, 20])
    assert_close(got[rows], O.softmax_loss(z, good)[1][rows], TOL_F32, "dlogits of the rows with valid labels")


def test_softmax_loss_uniform_logits_is_log_classes():
    z = np.full((64, 10), 1.5, dtype=np.float32)
    loss = torch.empty((), device=DEV)
    vcnn.softmax_loss(64, 10, to_dev(z), to_dev(np.zeros(64, dtype=np.int32)), loss, None)
    assert abs(float(to_np(loss)) - np.log(10.0)) < 1e-6


@pytest.mark.parametrize("shape", [(4, 1, 5, 7), (64, 1, 64, 64), (16, 1, 42, 42)])
def test_l2_loss_and_sgd(shape):
    y, t = random_tensor(1200, shape), random_tensor(1201, shape)
    loss = torch.full((), float("nan"), device=DEV)
    dy = torch.full(shape, float("nan"), device=DEV)
    vcnn.l2_loss(vcnn.F32, y.size, shape[0], to_dev(y), to_dev(t), loss, dy)
    rl, rdy = O.l2_loss(y, t)
    assert abs(float(to_np(loss)) - rl) <= TOL_F32 * abs(rl)
    assert_close(to_np(dy), rdy, 1e-6, "l2 dy")
    w = to_dev(y)
    vcnn.sgd_update(y.size, 0.01, w, to_dev(t))
    assert_close(to_np(w), O.sgd_update(y, t, 0.01), 1e-6, "sgd")


def test_sgd_update_multi_matches_oracle_per_tensor():
    """Several parameter tensors of ragged sizes in one launch (one of them empty), with and without the
    bfloat16 working copy."""
    shapes = [(500, 800), (500,), (1,), (0,), (50, 20, 5, 5), (257,), (10, 500), (3, 3)]
    ws = [random_tensor(1300 + k, sh) for k, sh in enumerate(shapes)]
    gs = [random_tensor(1400 + k, sh) for k, sh in enumerate(shapes)]
    wd, gd = [to_dev(w) for w in ws], [to_dev(g) for g in gs]
    w16 = [torch.full(sh, float("nan"), dtype=torch.bfloat16, device=DEV) if k % 2 == 0 else None
           for k, sh in enumerate(shapes)]
    vcnn.sgd_update_multi(0.01, wd, gd, w16)
    for k, (w, g) in enumerate(zip(ws, gs)):
        if w.size == 0:
            continue
        ref = O.sgd_update(w, g, 0.01)
        assert_close(to_np(wd[k]), ref, 1e-6, f"sgd tensor {k}")
        if w16[k] is not None:  # the copy is the rounding of the updated fp32 value: bit-exact against torch's rounding
            torch.cuda.synchronize()
            assert torch.equal(w16[k], wd[k].to(torch.bfloat16))
    # more tensors than one launch holds
    many = [to_dev(random_tensor(1500 + k, (33 + k,))) for k in range(40)]
    grads = [to_dev(random_tensor(1600 + k, (33 + k,))) for k in range(40)]
    before = [to_np(t).copy() for t in many]
    vcnn.sgd_update_multi(0.5, many, grads)
    for k in range(40):
        assert_close(to_np(many[k]), O.sgd_update(before[k], to_np(grads[k]), 0.5), 1e-6, f"sgd many {k}")


@pytest.mark.parametrize("empty", [(0,), (0, 5, 17), (15, 16, 31, 32), tuple(range(0, 40, 2)), tuple(range(39))])
def test_sgd_update_multi_with_empty_tensors_among_many(empty):
    """More tensors than one launch holds, some of them empty: every non-empty tensor is updated exactly once
    (an empty tensor takes no slot of a launch, so the launches' tensor ranges must follow the slots, not the
    positions)."""
    sizes = [0 if k in empty else 33 + 7 * k for k in range(40)]
    many = [to_dev(random_tensor(1500 + k, (sizes[k],))) for k in range(40)]
    grads = [to_dev(random_tensor(1600 + k, (sizes[k],))) for k in range(40)]
    before = [to_np(t).copy() for t in many]
    vcnn.sgd_update_multi(0.5, many, grads)
    for k in range(40):
        if sizes[k]:
            assert_close(to_np(many[k]), O.sgd_update(before[k], to_np(grads[k]), 0.5), 1e-6, f"sgd tensor {k} of 40")


SPLIT_SHAPES = [
    (3, 12, 19, 23, 37, 3, 5, 1, 2),    # ragged everything, 33..48 maps
    (2, 20, 12, 12, 50, 5, 5, 0, 0),
    (4, 33, 10, 10, 40, 1, 1, 0, 0),    # 1 x 1
    (3, 7, 13, 11, 130, 3, 3, 1, 1),    # many maps
    (9, 16, 16, 16, 64, 5, 5, 2, 2),    # a batch that is not a multiple of the 8-image groups of the kernel gradient
    (2, 38, 30, 30, 96, 16, 16, 0, 0),  # the shape class of the deconvolution network's large layer
]


@pytest.mark.parametrize("shape", SPLIT_SHAPES)
def test_conv_split_products_route(shape):
    """VCNN_ALGO_SPLIT: the float products of the forward pass and of the kernel gradient as six bfloat16 products each.
    The result must hold the float tolerance - and by a wide margin, the dropped terms lying below float rounding."""
    n, c, h, w, k, r, s, ph, pw = shape
    x = random_tensor(2600, (n, c, h, w))
    wt = random_tensor(2601, (k, c, r, s), scale=(2.0 / (c * r * s)) ** 0.5)
    b = random_tensor(2602, (k,), scale=0.1)
    oh, ow = h + 2 * ph - r + 1, w + 2 * pw - s + 1
    dy = random_tensor(2603, (n, k, oh, ow))
    xd, wd, bd, dyd = (torch.from_numpy(a).to(DEV) for a in (x, wt, b, dy))
    d = vcnn.conv_desc(n, c, h, w, k, r, s, ph, pw, act=vcnn.ACT_RELU)
    sizes = {}
    try:
        for name, algo in (("auto", vcnn.ALGO_AUTO), ("split", vcnn.ALGO_SPLIT)):
            vcnn.set_conv_algo(algo)
            sizes[name] = [vcnn.conv_workspace_bytes(d, p) for p in range(3)]
        assert sizes["split"][0] != sizes["auto"][0] and sizes["split"][1] != sizes["auto"][1]  # the route is taken
        assert sizes["split"][2] == sizes["auto"][2]  # the input gradient is not re-routed
        ws = torch.empty(max(256, *sizes["split"]), dtype=torch.uint8, device=DEV)
        y = torch.full((n, k, oh, ow), float("nan"), device=DEV)
        vcnn.conv_fwd(d, xd, wd, bd, y, ws)
        want = O.conv_fwd(x, wt, b, pad=(ph, pw), relu=True)
        assert_close(to_np(y), want, 2e-6, "split-product conv_fwd")
        dw = torch.full((k, c, r, s), float("nan"), device=DEV)
        db = torch.full((k,), float("nan"), device=DEV)
        vcnn.conv_bwd_filter(d, xd, dyd, dw, db, ws)
        rdw, rdb = O.conv_bwd_filter(x, dy, (r, s), pad=(ph, pw))
        assert_close(to_np(dw), rdw, 2e-6, "split-product dw")
        assert_close(to_np(db), rdb, TOL_F32, "split-product db")
        dw2 = torch.empty_like(dw)  # fixed order of the six products and of their slices: the same bits again
        vcnn.conv_bwd_filter(d, xd, dyd, dw2, db, ws)
        y2 = torch.empty_like(y)
        vcnn.conv_fwd(d, xd, wd, bd, y2, ws)
        assert torch.equal(dw, dw2) and torch.equal(y, y2)
    finally:
        vcnn.set_conv_algo(vcnn.ALGO_AUTO)


@pytest.mark.parametrize("bf16,per_instr", [(False, 4096.0), (True, 32768.0)])
def test_benchaid_mfma_counts_its_flops_and_runs(bf16, per_instr):
    """The benchmark's register-only matrix-core loop (a measurement aid outside the layer library)."""
    from paper_1501_07338_amd import benchaid
    blocks, iters = 8, 10
    sink = torch.full((blocks * 256,), float("nan"), device=DEV)
    flop = benchaid.mfma(bf16, blocks, iters, sink)
    assert flop == blocks * 4 * iters * 4 * per_instr
    assert np.all(np.isfinite(to_np(sink)))
    if not bf16:
        # thread 0 holds column 0, rows 8*(q/4) + q%4 of the 32x32 product; lane l supplies A[l%32][l/32] and B[l/32][l%32]
        fa = lambda t: np.float32(1.0) + np.float32(0.001) * np.float32(t % 61)
        fb = lambda t: np.float32(0.5) + np.float32(0.002) * np.float32(t % 53)
        rows = [8 * (q // 4) + q % 4 for q in range(16)]
        want = 4 * iters * sum(float(fa(r)) * float(fb(0)) + float(fa(r + 32)) * float(fb(32)) for r in rows)
        assert abs(float(to_np(sink)[0]) - want) <= 1e-4 * want
    # the variant with operands that change from instruction to instruction: same count, finite sums
    sink.fill_(float("nan"))
    assert benchaid.mfma(bf16, blocks, 16, sink, toggle=True) == blocks * 4 * 16 * 4 * per_instr
    assert np.all(np.isfinite(to_np(sink)))
    with pytest.raises(RuntimeError):
        benchaid.mfma(bf16, blocks, 10, sink, toggle=True)  # not a multiple of eight


@pytest.mark.parametrize("staged", [False, True])
def test_benchaid_mfma_lds_counts_its_flops_and_runs(staged):
    """The LDS-fed matrix-core loop of the benchmark's yardsticks: its flop count, a finite result, bad arguments."""
    from paper_1501_07338_amd import benchaid
    blocks, iters = 16, 24
    sink = torch.full((blocks * 256,), float("nan"), device=DEV)
    words = torch.ones(8192 * 4, device=DEV)
    assert benchaid.mfma_lds(staged, blocks, iters, sink, words) == blocks * 4 * iters * 16 * 4096.0
    assert np.all(np.isfinite(to_np(sink)))
    with pytest.raises(RuntimeError):
        benchaid.mfma_lds(staged, blocks, 10, sink, words)  # not a multiple of eight
    if staged:
        with pytest.raises(RuntimeError):
            benchaid.mfma_lds(True, blocks, iters, sink, torch.ones(64, device=DEV))  # too few words to fetch from


def test_benchaid_copy_copies():
    from paper_1501_07338_amd import benchaid
    src = torch.arange(1 << 20, dtype=torch.float32, device=DEV)
    dst = torch.zeros_like(src)
    assert benchaid.copy(src, dst) == 4 << 20
    torch.cuda.synchronize()
    assert torch.equal(src, dst)


def test_gpu_launch_of_bad_arguments_is_rejected_cleanly():
    d = vcnn.conv_desc(2, 3, 8, 8, 4, 3, 3)
    x = torch.zeros((2, 3, 8, 8), device=DEV)
    w = torch.zeros((4, 3, 3, 3), device=DEV)
    y = torch.zeros((2, 4, 6, 6), device=DEV)
    if vcnn.conv_workspace_bytes(d, vcnn.PASS_FWD):
        with pytest.raises(vcnn.VcnnError) as e:
            vcnn.conv_fwd(d, x, w, None, y, None)
        assert e.value.status == vcnn.ERR_WORKSPACE
    with pytest.raises(vcnn.VcnnError) as e:
        vcnn.conv_fwd(vcnn.conv_desc(2, 3, 8, 8, 4, 3, 3, dtype=5), x, w, None, y, None)
    assert e.value.status == vcnn.ERR_UNSUPPORTED
