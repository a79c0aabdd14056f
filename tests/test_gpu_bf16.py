"""The bfloat16 variant: x, w, y, dy, dx stored as bf16, accumulation / bias / dW / db / loss in fp32.
Per pass the oracle is fp64 arithmetic on the same bf16-rounded operands; tolerance is 2e-2 max-norm relative for
bf16 tensors and the fp32 bar for tensors the path keeps in fp32.  In the whole-chain test the oracle additionally
rounds each stored activation to bf16, so that both sides take the ReLU / pooling decisions in the storage type."""
import numpy as np
import pytest
import torch

import oracle as O
from oracle.net import train_step as oracle_step
from paper_1501_07338_amd import vcnn
from paper_1501_07338_amd import workloads as wl
from paper_1501_07338_amd.net import TrainStep
from util import TOL_BF16, TOL_F32, assert_close, to_dev, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

SHAPES = [
    (2, 136, 11, 9, 1, 7, 7, 3, 3),     # one map, 49 taps, 136 channels: the streaming taps-as-rows product on bfloat16 storage
    (2, 1, 150, 200, 38, 121, 1, 0, 0), # tall kernel on a wide plane, one channel: strip tiles with bfloat16 storage
    (3, 5, 19, 23, 37, 3, 5, 1, 2),
    (2, 20, 12, 12, 50, 5, 5, 0, 0),
    (4, 33, 10, 10, 40, 1, 1, 0, 0),
    (3, 7, 13, 11, 130, 3, 3, 1, 1),
    (5, 3, 17, 15, 1, 5, 5, 2, 2),
    (3, 19, 21, 22, 1, 8, 8, 0, 0),
    (2, 2, 33, 70, 21, 3, 9, 1, 4),
    (2, 16, 16, 16, 64, 5, 5, 2, 2),
    (3, 9, 14, 15, 20, 3, 3, 1, 1),     # at most 32 maps: one 32-row tile per wave in every pass
    (2, 64, 12, 12, 1, 4, 4, 0, 0),     # a single map over many channels goes to the matrix cores as well
    (2, 40, 9, 11, 1, 4, 4, 1, 1),      # ... 32 to 63 channels: forward and kernel gradient as taps-as-rows products
    (2, 16, 40, 40, 48, 5, 5, 2, 2),    # 33..48 maps: three 16-row tiles per wave, wide pixel tile
    (3, 38, 14, 14, 38, 3, 3, 1, 1),    # ... forward and input gradient alike, small image
    (2, 40, 9, 30, 44, 2, 3, 0, 1),     # ... ragged
    (600, 8, 10, 10, 200, 3, 3, 1, 1),  # many maps, many small images: the four waves of a block take different maps
                                        # (large images: different pixels, test_conv_bf16_wide_pixel_tiles with 200 maps)
]


def b16(a):
    """bf16-rounded fp32 host array and its device bf16 tensor (the conversion is exact)."""
    r = wl.bf16_round(a)
    return r, torch.from_numpy(r).to(DEV).to(torch.bfloat16)


def f32_of(t):
    torch.cuda.synchronize()
    return t.float().cpu().numpy()


@pytest.fixture(params=["auto", "explicit", "implicit"])
def algo(request):
    vcnn.set_conv_algo({"auto": vcnn.ALGO_AUTO, "explicit": vcnn.ALGO_EXPLICIT, "implicit": vcnn.ALGO_IMPLICIT}[request.param])
    yield request.param
    vcnn.set_conv_algo(vcnn.ALGO_AUTO)


@pytest.mark.parametrize("shape", SHAPES)
def test_conv_bf16(shape, algo):
    n, c, h, w, k, r, s, ph, pw = shape
    x, xd = b16(wl.random_tensor(2000, (n, c, h, w)))
    wt, wd = b16(wl.random_tensor(2001, (k, c, r, s), scale=(2.0 / (c * r * s)) ** 0.5))
    b = wl.random_tensor(2002, (k,), scale=0.1)
    oh, ow = h + 2 * ph - r + 1, w + 2 * pw - s + 1
    dy, dyd = b16(wl.random_tensor(2003, (n, k, oh, ow)))
    d = vcnn.conv_desc(n, c, h, w, k, r, s, ph, pw, dtype=vcnn.BF16, act=vcnn.ACT_RELU)
    ws = torch.empty(max(256, *(vcnn.conv_workspace_bytes(d, p) for p in range(3))), dtype=torch.uint8, device=DEV)
    y = torch.full((n, k, oh, ow), float("nan"), dtype=torch.bfloat16, device=DEV)
    vcnn.conv_fwd(d, xd, wd, torch.from_numpy(b).to(DEV), y, ws)
    assert_close(f32_of(y), O.conv_fwd(x, wt, b, pad=(ph, pw), relu=True), TOL_BF16, "bf16 conv_fwd")
    # the stored value is the correctly rounded bf16 of an fp32-accurate result: error at most half a bf16 ulp
    want = O.conv_fwd(x, wt, b, pad=(ph, pw), relu=True)
    assert np.max(np.abs(f32_of(y) - want) / np.maximum(np.abs(want), 1e-3 * np.max(want))) <= 2.0 ** -8

    dw = torch.full((k, c, r, s), float("nan"), device=DEV)
    db = torch.full((k,), float("nan"), device=DEV)
    vcnn.conv_bwd_filter(d, xd, dyd, dw, db, ws)
    rdw, rdb = O.conv_bwd_filter(x, dy, (r, s), pad=(ph, pw))
    assert_close(to_np(dw), rdw, TOL_F32, "bf16 dw (fp32 result)")
    assert_close(to_np(db), rdb, TOL_F32, "bf16 db (fp32 result)")

    dx = torch.full((n, c, h, w), float("nan"), dtype=torch.bfloat16, device=DEV)
    vcnn.conv_bwd_data(d, wd, dyd, dx, ws)
    assert_close(f32_of(dx), O.conv_bwd_data(wt, dy, (h, w), pad=(ph, pw)), TOL_BF16, "bf16 dx")
    # the same with the ReLU derivative of the layer below folded into the store (x read as that ReLU's output)
    xr, xrd = b16(np.maximum(x, 0))
    dx.fill_(float("nan"))
    vcnn.conv_bwd_data_act(d, vcnn.ACT_RELU, xrd, wd, dyd, dx, ws)
    assert_close(f32_of(dx), O.relu_bwd(xr.astype(np.float64), O.conv_bwd_data(wt, dy, (h, w), pad=(ph, pw))), TOL_BF16,
                 "bf16 dx * relu'")
    assert not np.any(f32_of(dx)[xr <= 0])


def _check_bf16_layer(n, c, h, w, k, r, s, ph, pw, seed):
    x, xd = b16(wl.random_tensor(seed, (n, c, h, w)))
    wt, wd = b16(wl.random_tensor(seed + 1, (k, c, r, s), scale=(2.0 / (c * r * s)) ** 0.5))
    b = wl.random_tensor(seed + 2, (k,), scale=0.1)
    oh, ow = h + 2 * ph - r + 1, w + 2 * pw - s + 1
    dy, dyd = b16(wl.random_tensor(seed + 3, (n, k, oh, ow)))
    d = vcnn.conv_desc(n, c, h, w, k, r, s, ph, pw, dtype=vcnn.BF16, act=vcnn.ACT_NONE)
    ws = torch.empty(max(256, *(vcnn.conv_workspace_bytes(d, p) for p in range(3))), dtype=torch.uint8, device=DEV)
    y = torch.full((n, k, oh, ow), float("nan"), dtype=torch.bfloat16, device=DEV)
    vcnn.conv_fwd(d, xd, wd, torch.from_numpy(b).to(DEV), y, ws)
    assert_close(f32_of(y), O.conv_fwd(x, wt, b, pad=(ph, pw)), TOL_BF16, "bf16 conv_fwd")
    dw = torch.full((k, c, r, s), float("nan"), device=DEV)
    db = torch.full((k,), float("nan"), device=DEV)
    vcnn.conv_bwd_filter(d, xd, dyd, dw, db, ws)
    rdw, rdb = O.conv_bwd_filter(x, dy, (r, s), pad=(ph, pw))
    assert_close(to_np(dw), rdw, TOL_F32, "bf16 dw (fp32 result)")
    assert_close(to_np(db), rdb, TOL_F32, "bf16 db (fp32 result)")
    dx = torch.full((n, c, h, w), float("nan"), dtype=torch.bfloat16, device=DEV)
    vcnn.conv_bwd_data(d, wd, dyd, dx, ws)
    assert_close(f32_of(dx), O.conv_bwd_data(wt, dy, (h, w), pad=(ph, pw)), TOL_BF16, "bf16 dx")
    # the same with the ReLU derivative of the layer below folded into the store (x read as that ReLU's output)
    xr, xrd = b16(np.maximum(x, 0))
    dx.fill_(float("nan"))
    vcnn.conv_bwd_data_act(d, vcnn.ACT_RELU, xrd, wd, dyd, dx, ws)
    assert_close(f32_of(dx), O.relu_bwd(xr.astype(np.float64), O.conv_bwd_data(wt, dy, (h, w), pad=(ph, pw))), TOL_BF16,
                 "bf16 dx * relu'")
    assert not np.any(f32_of(dx)[xr <= 0])


POINTWISE_SHAPES = [
    (3, 64, 7, 7, 96),      # odd plane size (rows start on odd elements), one ragged 128-row tile
    (2, 72, 13, 11, 40),    # contraction not a multiple of the 64-deep slab, 64-row tile
    (5, 136, 9, 15, 200),   # two row tiles, two pixel tiles, three slabs
    (2, 32, 20, 20, 32),    # even plane size, the smallest row count
    (3, 40, 5, 3, 64),      # 15 pixels: a last pixel group of three
    (4, 48, 2, 3, 56),      # 6 pixels: below one group of eight (the kernel gradient falls back)
    (2, 512, 17, 9, 512),   # the shape class of the deconvolution network's 1 x 1 layer: whole slabs, a second pixel
                            # tile that overlaps the first
    (3, 128, 13, 11, 192),  # odd plane of 143 pixels, two and three whole slabs
    (2, 64, 16, 9, 64),     # even plane of 144 pixels, a single slab
    (1, 64, 16, 16, 320),   # exactly two pixel tiles, three row tiles
]


# (the element offset is only used where all three passes take the products of this test: their loads are written
# for rows at any 2-byte boundary; other realisations are given tensors as an allocator returns them)
@pytest.mark.parametrize("shape,offset", [(sh, off) for sh in POINTWISE_SHAPES for off in (0, 1) if off == 0 or sh[2] * sh[3] >= 8])
def test_conv_bf16_pointwise(shape, offset):
    """Unpadded 1 x 1 layers of the bf16 variant: the three plain bf16 products on the tensors as stored.  offset = 1
    places x, dy, y and dx one element into their buffers, so that every row parity occurs also for even planes."""
    n, c, h, w, k = shape

    def placed(a):
        r = wl.bf16_round(a)
        buf = torch.zeros(r.size + 8, dtype=torch.bfloat16, device=DEV)
        view = buf[offset:offset + r.size].view(r.shape)
        view.copy_(torch.from_numpy(r).to(DEV))
        return r, view

    def blank(shape_):
        buf = torch.full((int(np.prod(shape_)) + 8,), float("nan"), dtype=torch.bfloat16, device=DEV)
        return buf, buf[offset:offset + int(np.prod(shape_))].view(shape_)

    x, xd = placed(wl.random_tensor(2500, (n, c, h, w)))
    wt, wd = b16(wl.random_tensor(2501, (k, c, 1, 1), scale=(2.0 / c) ** 0.5))
    b = wl.random_tensor(2502, (k,), scale=0.1)
    dy, dyd = placed(wl.random_tensor(2503, (n, k, h, w)))
    for act, relu in ((vcnn.ACT_NONE, False), (vcnn.ACT_RELU, True)):
        d = vcnn.conv_desc(n, c, h, w, k, 1, 1, 0, 0, dtype=vcnn.BF16, act=act)
        ws = torch.empty(max(256, *(vcnn.conv_workspace_bytes(d, p) for p in range(3))), dtype=torch.uint8, device=DEV)
        ybuf, y = blank((n, k, h, w))
        vcnn.conv_fwd(d, xd, wd, torch.from_numpy(b).to(DEV), y, ws)
        assert_close(f32_of(y), O.conv_fwd(x, wt, b, pad=(0, 0), relu=relu), TOL_BF16, "bf16 1x1 conv_fwd")
        # nothing is written outside the tensor
        assert torch.isnan(ybuf[:offset]).all() and torch.isnan(ybuf[offset + y.numel():]).all()
    dw = torch.full((k, c, 1, 1), float("nan"), device=DEV)
    db = torch.full((k,), float("nan"), device=DEV)
    vcnn.conv_bwd_filter(d, xd, dyd, dw, db, ws)
    rdw, rdb = O.conv_bwd_filter(x, dy, (1, 1), pad=(0, 0))
    assert_close(to_np(dw), rdw, TOL_F32, "bf16 1x1 dw (fp32 result)")
    assert_close(to_np(db), rdb, TOL_F32, "bf16 1x1 db (fp32 result)")
    dxbuf, dx = blank((n, c, h, w))
    vcnn.conv_bwd_data(d, wd, dyd, dx, ws)
    assert_close(f32_of(dx), O.conv_bwd_data(wt, dy, (h, w), pad=(0, 0)), TOL_BF16, "bf16 1x1 dx")
    assert torch.isnan(dxbuf[:offset]).all() and torch.isnan(dxbuf[offset + dx.numel():]).all()
    if offset:  # a kernel matrix that is not 16-byte aligned takes the generic product: same result within the bar
        _, wd_off = placed(wt)
        ybuf, y = blank((n, k, h, w))
        vcnn.conv_fwd(d, xd, wd_off, torch.from_numpy(b).to(DEV), y, ws)
        assert_close(f32_of(y), O.conv_fwd(x, wt, b, pad=(0, 0), relu=True), TOL_BF16, "bf16 1x1 conv_fwd, offset kernel matrix")
    # run to run the kernel gradient's ordered partial sums give the same bits
    dw2 = torch.empty_like(dw)
    vcnn.conv_bwd_filter(d, xd, dyd, dw2, db, ws)
    assert torch.equal(dw, dw2)


@pytest.mark.parametrize("k", [40, 100, 200])           # waves of a block: all on the contraction, 2 x 2, all on the maps
@pytest.mark.parametrize("hw", [(40, 64), (64, 80)])    # pixel tiles of 128 and of 160 win the tile choice
def test_conv_bf16_wide_pixel_tiles(k, hw):
    """Shapes large enough that the bf16 matrix-core kernel picks its 128- and 160-pixel wave tiles, for each
    arrangement of the four waves; 12 channels = one full and one half-empty group of 8."""
    _check_bf16_layer(16, 12, hw[0], hw[1], k, 3, 3, 1, 1, seed=2300 + k)


@pytest.mark.parametrize("k", [40, 100, 200])
@pytest.mark.parametrize("c", [7, 13, 17])              # kernel-matrix widths 63, 117, 153: column tiles of 64, 128, 160
def test_filter_grad_bf16_column_tiles(k, c):
    """Filter gradient of the bf16 variant for each column-tile width and wave arrangement, with a batch that
    is not a multiple of the 8-image interleave and several pixel runs per image."""
    _check_bf16_layer(11, c, 30, 26, k, 3, 3, 1, 1, seed=2400 + 10 * c + k)


def test_unroll_bf16_bit_exact():
    n, c, h, w, r, s, ph, pw = 3, 5, 14, 13, 5, 3, 2, 1
    d = vcnn.conv_desc(n, c, h, w, 1, r, s, ph, pw, dtype=vcnn.BF16)
    oh, ow = vcnn.conv_out_shape(d)
    x, xd = b16(wl.random_tensor(2100, (n, c, h, w)))
    col = torch.full((c * r * s, n * oh * ow), float("nan"), dtype=torch.bfloat16, device=DEV)
    vcnn.im2col(d, xd, col)
    np.testing.assert_array_equal(f32_of(col), O.im2col(x, (r, s), pad=(ph, pw)).astype(np.float32))
    cf = wl.random_tensor(2101, (c * r * s, n * oh * ow))
    dx = torch.full((n, c, h, w), float("nan"), dtype=torch.bfloat16, device=DEV)
    vcnn.col2im(d, torch.from_numpy(cf).to(DEV), dx)
    assert_close(f32_of(dx), O.col2im(cf, (n, c, h, w), (r, s), pad=(ph, pw)), TOL_BF16, "bf16 col2im")


def test_pool_act_l2_bf16():
    x, xd = b16(np.maximum(wl.random_tensor(2200, (3, 4, 15, 15)), 0))
    d = vcnn.pool_desc(3, 4, 15, 15, 3, 3, 2, 2, dtype=vcnn.BF16)
    y = torch.empty((3, 4, 7, 7), dtype=torch.bfloat16, device=DEV)
    am = torch.empty((3, 4, 7, 7), dtype=torch.int32, device=DEV)
    vcnn.pool_fwd(d, xd, y, am)
    ry, ram = O.maxpool_fwd(x, (3, 3), (2, 2))
    np.testing.assert_array_equal(to_np(am), ram)  # bit-exact argmax on identical (bf16) inputs
    np.testing.assert_array_equal(f32_of(y), ry.astype(np.float32))
    dy, dyd = b16(wl.random_tensor(2201, (3, 4, 7, 7)))
    dx = torch.empty((3, 4, 15, 15), dtype=torch.bfloat16, device=DEV)
    vcnn.pool_bwd(d, dyd, am, dx)
    assert_close(f32_of(dx), O.maxpool_bwd(dy, ram, (15, 15)), TOL_BF16, "bf16 pool dx")

    g, gd = b16(wl.random_tensor(2202, (3 * 4 * 15 * 15 + 3,)))
    r, rd = b16(wl.random_tensor(2203, g.shape))
    out = torch.empty(g.shape, dtype=torch.bfloat16, device=DEV)
    vcnn.act_fwd(vcnn.ACT_RELU, vcnn.BF16, g.size, gd, out)
    np.testing.assert_array_equal(f32_of(out), O.relu_fwd(g).astype(np.float32))
    vcnn.act_bwd(vcnn.ACT_RELU, vcnn.BF16, g.size, rd, gd, out)
    np.testing.assert_array_equal(f32_of(out), O.relu_bwd(r, g).astype(np.float32))

    yv, yd = b16(wl.random_tensor(2204, (4, 1, 9, 9)))
    t = wl.random_tensor(2205, (4, 1, 9, 9))
    loss = torch.empty((), device=DEV)
    dyo = torch.empty((4, 1, 9, 9), dtype=torch.bfloat16, device=DEV)
    vcnn.l2_loss(vcnn.BF16, yv.size, 4, yd, torch.from_numpy(t).to(DEV), loss, dyo)
    rl, rdy = O.l2_loss(yv, t)
    assert abs(float(to_np(loss)) - rl) <= TOL_F32 * abs(rl)
    assert_close(f32_of(dyo), rdy, TOL_BF16, "bf16 l2 dy")


def test_fc_bf16():
    b, i, o = 33, 70, 45
    x, xd = b16(wl.random_tensor(2300, (b, i)))
    w, wd = b16(wl.random_tensor(2301, (o, i), scale=(2.0 / i) ** 0.5))
    bias = wl.random_tensor(2302, (o,))
    dy, dyd = b16(wl.random_tensor(2303, (b, o)))
    y = torch.empty((b, o), dtype=torch.bfloat16, device=DEV)
    vcnn.fc_fwd(vcnn.BF16, b, i, o, vcnn.ACT_NONE, xd, wd, torch.from_numpy(bias).to(DEV), y)
    assert_close(f32_of(y), O.fc_fwd(x, w, bias), TOL_BF16, "bf16 fc y")
    dw = torch.empty((o, i), device=DEV)
    db = torch.empty((o,), device=DEV)
    dx = torch.empty((b, i), dtype=torch.bfloat16, device=DEV)
    vcnn.fc_bwd(vcnn.BF16, b, i, o, xd, wd, dyd, dw, db, dx)
    rdw, rdb, rdx = O.fc_bwd(x, w, dy)
    assert_close(to_np(dw), rdw, TOL_F32, "bf16 fc dw")
    assert_close(to_np(db), rdb, TOL_F32, "bf16 fc db")
    assert_close(f32_of(dx), rdx, TOL_BF16, "bf16 fc dx")


def reference(name, batch, chain=True):
    net = wl.make_net(name, batch)
    inputs, params = wl.make_inputs(net), wl.make_params(net)
    inputs = dict(inputs, x=wl.bf16_round(inputs["x"]))
    params = [None if p is None else (wl.bf16_round(p[0]), p[1]) for p in params]
    return net, inputs, params, oracle_step(net, inputs, params) if chain else None


@pytest.mark.parametrize("name,batch", [("cfg5", 1), ("cfg4", 2)])
def test_bf16_layerwise_parity(name, batch):
    """Layer-wise protocol in the bf16 variant: every HIP layer pass is fed the bf16 rounding of the
    ORACLE's tensors for that layer (so no rounding or ReLU decision of an earlier layer leaks in) and
    must meet the 2e-2 bar (fp32 bar for dW, db, which the path keeps in fp32) against the oracle
    evaluated on those same rounded tensors."""
    net, inputs, params, ref = reference(name, batch)
    for li, L in enumerate(net.layers):
        assert isinstance(L, wl.Conv)
        a_in, a_in_d = b16(ref["acts"][li].astype(np.float32))
        w, wd = b16(params[li][0])
        b = params[li][1]
        pad = (L.pad_h, L.pad_w)
        n, c, h, wdt = a_in.shape
        d = vcnn.conv_desc(n, c, h, wdt, L.cout, L.kh, L.kw, L.pad_h, L.pad_w, dtype=vcnn.BF16,
                           act=vcnn.ACT_RELU if L.relu else vcnn.ACT_NONE)
        ws = torch.empty(max(256, *(vcnn.conv_workspace_bytes(d, p) for p in range(3))), dtype=torch.uint8, device=DEV)
        y = torch.full(ref["acts"][li + 1].shape, float("nan"), dtype=torch.bfloat16, device=DEV)
        vcnn.conv_fwd(d, a_in_d, wd, torch.from_numpy(b).to(DEV), y, ws)
        want = O.conv_fwd(a_in, w, b, pad=pad, relu=L.relu)
        assert_close(f32_of(y), want, TOL_BF16, f"{name} bf16 layer {li} fwd")
        # gradient w.r.t. the pre-activation, from the oracle's tensors, rounded to bf16
        dpre = O.relu_bwd(ref["acts"][li + 1], ref["dacts"][li + 1]) if L.relu else ref["dacts"][li + 1]
        dpre, dpre_d = b16(dpre.astype(np.float32))
        dw = torch.full(w.shape, float("nan"), device=DEV)
        db = torch.full(b.shape, float("nan"), device=DEV)
        vcnn.conv_bwd_filter(d, a_in_d, dpre_d, dw, db, ws)
        rdw, rdb = O.conv_bwd_filter(a_in, dpre, (L.kh, L.kw), pad=pad)
        assert_close(to_np(dw), rdw, TOL_F32, f"{name} bf16 layer {li} dw")
        assert_close(to_np(db), rdb, TOL_F32, f"{name} bf16 layer {li} db")
        dx = torch.full(a_in.shape, float("nan"), dtype=torch.bfloat16, device=DEV)
        vcnn.conv_bwd_data(d, wd, dpre_d, dx, ws)
        assert_close(f32_of(dx), O.conv_bwd_data(w, dpre, (h, wdt), pad=pad), TOL_BF16, f"{name} bf16 layer {li} dx")


def stored_bf16(a):
    """What a layer of the bf16 variant leaves in memory: the value rounded to bfloat16 (nearest even)."""
    return wl.bf16_round(np.asarray(a, dtype=np.float32)).astype(np.float64)


@pytest.mark.parametrize("name,batch", [("cfg5", 1), ("cfg4", 2), ("cfg2", 16), ("cfg3", 8)])
def test_bf16_training_step(name, batch):
    """Whole step in the bf16 variant, every tensor of the chain element-wise against the fp64 oracle started from
    the same bf16-rounded input and weights.  Both sides take the chain's discrete decisions (ReLU side, pooling
    maximum) in the same precision, the storage type's: the oracle rounds every activation to bfloat16 as it is
    stored and computes each layer in fp64 from the stored values.  Decisions that still differ must be ties within
    one bf16 step of the oracle's own values (the two sides' fp32 / fp64 sums can round to neighbouring bf16
    values); the oracle's backward pass then takes those validated choices, and activations, input gradients and
    parameter gradients all meet the 2e-2 bar."""
    net, inputs, params, _ = reference(name, batch, chain=False)
    ref = oracle_step(net, inputs, params, store=stored_bf16)
    ts = TrainStep(net, params, inputs, device=DEV, first_layer_dx=True, dtype=vcnn.BF16)
    ts.step()
    flips = 0
    step16 = 2.0 ** -7  # two neighbouring bfloat16 values differ by at most 2^-7 relative
    for li, L in enumerate(net.layers):
        got, want = f32_of(ts.acts[li + 1]).astype(np.float64), ref["acts"][li + 1]
        assert_close(got, want, TOL_BF16, f"{name} bf16 act {li}")
        if isinstance(L, wl.Pool):
            gam, ram, x_ref = ts.argmax[li].cpu().numpy(), ref["argmax"][li], ref["acts"][li]
            for n, c, oh, ow in np.argwhere(gam != ram):
                plane = x_ref[n, c].reshape(-1)
                a, b = plane[ram[n, c, oh, ow]], plane[gam[n, c, oh, ow]]
                assert abs(a - b) <= 2 * step16 * max(abs(a), abs(b)), f"{name} bf16 argmax {(li, n, c, oh, ow)} is not a near-tie"
                flips += 1
        elif L.relu:
            differ = (got > 0) != (want > 0)
            assert np.all(np.maximum(np.abs(got), np.abs(want))[differ] <= 1e-3 * np.max(np.abs(want))), \
                f"{name} bf16 layer {li}: a ReLU decision differs away from zero"
            flips += int(np.count_nonzero(differ))
    print(f"{name} bf16 batch {batch}: {flips} near-tie decisions differ")
    relu_side = {li: ref["acts"][li + 1] > 0 for li, L in enumerate(net.layers) if getattr(L, "relu", False)}
    if flips:
        relu_side = {li: f32_of(ts.acts[li + 1]) > 0 for li in relu_side}
        ref = oracle_step(net, inputs, params, store=stored_bf16, decisions={
            "argmax": {li: am.cpu().numpy() for li, am in ts.argmax.items()}, "relu": relu_side})
    if net.loss != "upstream":
        assert abs(float(to_np(ts.loss)) - ref["loss"]) <= TOL_BF16 * abs(ref["loss"])
    for li in range(len(net.layers) - 1, -1, -1):
        if ts.folds(li):  # stored with the ReLU derivative of the layer below already applied
            assert_close(f32_of(ts.dpre[li - 1]), O.relu_bwd(relu_side[li - 1].astype(np.float64), ref["dacts"][li]),
                         TOL_BF16, f"{name} bf16 dpre {li - 1}")
        else:
            assert_close(f32_of(ts.dacts[li]), ref["dacts"][li], TOL_BF16, f"{name} bf16 dact {li}")
        if ts.grads[li] is not None:
            # products of bf16-stored tensors that carry their own rounding: the chain's bar, not the 1e-4 that holds
            # for a single pass on identical operands (test_bf16_layerwise_parity)
            assert_close(to_np(ts.grads[li][0]), ref["grads"][li][0], TOL_BF16, f"{name} bf16 dw {li}")
            assert_close(to_np(ts.grads[li][1]), ref["grads"][li][1], TOL_BF16, f"{name} bf16 db {li}")
            # the update moved the master weights by -lr * dw
            moved = to_np(ts.params[li][0]).astype(np.float64) - params[li][0]
            want = -net.lr * to_np(ts.grads[li][0]).astype(np.float64)
            assert np.max(np.abs(moved - want)) <= 1e-2 * np.max(np.abs(want)) + 2.0 ** -23 * np.max(np.abs(params[li][0]))
            # and the bf16 copy the next step reads is the rounding of the new master weights
            np.testing.assert_array_equal(f32_of(ts.params16[li]), wl.bf16_round(to_np(ts.params[li][0])))


def test_smooth_sigma_and_avgpool_bf16():
    """tanh / sigmoid and average pooling on bf16 tensors: fp32 arithmetic on the bf16-rounded inputs, result
    rounded once."""
    x, xd = b16(wl.random_tensor(2500, (3 * 4 * 15 * 15,), scale=2.0))
    dy, dyd = b16(wl.random_tensor(2501, x.shape))
    for act, fwd, bwd in ((vcnn.ACT_TANH, O.tanh_fwd, O.tanh_bwd), (vcnn.ACT_SIGMOID, O.sigmoid_fwd, O.sigmoid_bwd)):
        y = torch.empty(x.shape, dtype=torch.bfloat16, device=DEV)
        vcnn.act_fwd(act, vcnn.BF16, x.size, xd, y)
        assert_close(f32_of(y), fwd(x), TOL_BF16, "bf16 sigma fwd")
        dx = torch.empty(x.shape, dtype=torch.bfloat16, device=DEV)
        vcnn.act_bwd(act, vcnn.BF16, x.size, y, dyd, dx)
        assert_close(f32_of(dx), bwd(f32_of(y), dy), TOL_BF16, "bf16 sigma bwd")
    xp, xpd = b16(wl.random_tensor(2502, (3, 4, 15, 15)))
    d = vcnn.pool_desc(3, 4, 15, 15, 3, 3, 2, 2, dtype=vcnn.BF16, mode=vcnn.POOL_AVG)
    yp = torch.empty((3, 4, 7, 7), dtype=torch.bfloat16, device=DEV)
    vcnn.pool_fwd(d, xpd, yp, None)
    assert_close(f32_of(yp), O.avgpool_fwd(xp, (3, 3), (2, 2)), TOL_BF16, "bf16 avgpool y")
    g, gd = b16(wl.random_tensor(2503, (3, 4, 7, 7)))
    dxp = torch.empty((3, 4, 15, 15), dtype=torch.bfloat16, device=DEV)
    vcnn.pool_bwd(d, gd, None, dxp)
    assert_close(f32_of(dxp), O.avgpool_bwd(g, (15, 15), (3, 3), (2, 2)), TOL_BF16, "bf16 avgpool dx")


@pytest.mark.parametrize("mode", ["max", "avg"])
def test_pool_layer_bias_sigma_bf16(mode):
    """Eq. 3's pooling layer on bf16 tensors (tanh); the fused input gradients of pool_bwd_act / fc_bwd_act on bf16."""
    n, c, h, w = 4, 6, 14, 14
    x, xd = b16(wl.random_tensor(2600, (n, c, h, w)))
    bias = wl.random_tensor(2601, (c,))
    d = vcnn.pool_desc(n, c, h, w, 2, 2, 2, 2, dtype=vcnn.BF16, mode=vcnn.POOL_MAX if mode == "max" else vcnn.POOL_AVG)
    y = torch.empty((n, c, 7, 7), dtype=torch.bfloat16, device=DEV)
    am = torch.empty((n, c, 7, 7), dtype=torch.int32, device=DEV) if mode == "max" else None
    vcnn.pool_layer_fwd(d, vcnn.ACT_TANH, xd, to_dev(bias), y, am)
    ry, ram = O.pool_layer_fwd(x, bias, (2, 2), (2, 2), mode, "tanh")
    assert_close(f32_of(y), ry, TOL_BF16, "bf16 pool layer y")
    if mode == "max":
        np.testing.assert_array_equal(am.cpu().numpy(), ram)
    dy, dyd = b16(wl.random_tensor(2602, (n, c, 7, 7)))
    dx = torch.empty((n, c, h, w), dtype=torch.bfloat16, device=DEV)
    db = torch.empty((c,), device=DEV)
    ws = torch.empty(vcnn.pool_layer_workspace_bytes(d), dtype=torch.uint8, device=DEV)
    vcnn.pool_layer_bwd(d, vcnn.ACT_TANH, y, dyd, am, db, dx, ws)
    rdx, rdb, _ = O.pool_layer_bwd(f32_of(y), dy, ram, (h, w), (2, 2), (2, 2), mode, "tanh")
    assert_close(f32_of(dx), rdx, TOL_BF16, "bf16 pool layer dx")
    assert_close(db.cpu().numpy(), rdb, TOL_BF16, "bf16 pool layer dbias")
    # ReLU derivative of the layer below folded into the pooling / fully connected input gradients
    xr, xrd = b16(np.maximum(x, 0))
    dx2 = torch.empty_like(dx)
    vcnn.pool_bwd_act(d, vcnn.ACT_RELU, xrd, dyd, am, dx2)
    plain = O.maxpool_bwd(dy, ram, (h, w)) if mode == "max" else O.avgpool_bwd(dy, (h, w), (2, 2), (2, 2))
    assert_close(f32_of(dx2), O.relu_bwd(xr, plain), TOL_BF16, "bf16 pool dx * relu'")
    b, i, o = 32, 96, 40
    xf, xfd = b16(np.maximum(wl.random_tensor(2603, (b, i)), 0))
    wf, wfd = b16(wl.random_tensor(2604, (o, i), scale=0.2))
    gf, gfd = b16(wl.random_tensor(2605, (b, o)))
    dxf = torch.empty((b, i), dtype=torch.bfloat16, device=DEV)
    dwf, dbf = torch.empty((o, i), device=DEV), torch.empty((o,), device=DEV)
    vcnn.fc_bwd_act(vcnn.BF16, b, i, o, vcnn.ACT_RELU, xfd, wfd, gfd, dwf, dbf, dxf)
    rdw, rdbf, rdxf = O.fc_bwd(xf, wf, gf)
    assert_close(f32_of(dxf), O.relu_bwd(xf, rdxf), TOL_BF16, "bf16 fc dx * relu'")
    assert_close(dwf.cpu().numpy(), rdw, TOL_BF16, "bf16 fc dw")
    assert_close(dbf.cpu().numpy(), rdbf, TOL_BF16, "bf16 fc db")
