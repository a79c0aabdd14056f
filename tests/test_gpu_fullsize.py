"""Full-size parity of the big layers (workloads cfg4 and cfg5 at their stated batch), in the launch
configuration the benchmark times.  The nested-loop oracle would need minutes for these, so each pass
is checked at sampled output positions that the oracle's single-output probes evaluate straight from
the definition, plus size-independent properties (bias-gradient sum, determinism)."""
import numpy as np
import pytest
import torch

import oracle as O
from paper_1501_07338_amd import vcnn
from paper_1501_07338_amd import workloads as wl
from util import TOL_F32, to_dev, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
SAMPLES = 40


def conv_layers(name):
    net = wl.make_net(name)
    return [(li, L, net.in_shape(li)) for li, L in enumerate(net.layers) if isinstance(L, wl.Conv)]


CASES = [(name, li) for name in ("cfg4", "cfg5") for li, _, _ in conv_layers(name)]


def sample_idx(rng, shape, extra=()):
    idx = [tuple(int(rng.integers(0, d)) for d in shape) for _ in range(SAMPLES)]
    corners = [tuple(0 for _ in shape), tuple(d - 1 for d in shape)]
    return idx + corners + list(extra)


def check_samples(got, want, what):
    want = np.asarray(want, dtype=np.float64)
    err = np.max(np.abs(np.asarray(got, dtype=np.float64) - want)) / max(np.max(np.abs(want)), 1e-30)
    assert err <= TOL_F32, f"{what}: sampled max-norm relative error {err:.3e}"


@pytest.mark.parametrize("name,li", CASES)
def test_conv_layer_full_size_sampled(name, li):
    net = wl.make_net(name)
    L = net.layers[li]
    n, c, h, w = net.in_shape(li)
    _, k, oh, ow = net.shapes[li]
    pad = (L.pad_h, L.pad_w)
    seed = 5000 + 100 * net.index + li
    x = np.abs(wl.random_tensor(seed, (n, c, h, w))) if li > 0 else wl.random_tensor(seed, (n, c, h, w))
    wt = wl.random_tensor(seed + 1, (k, c, L.kh, L.kw), scale=(2.0 / (c * L.kh * L.kw)) ** 0.5)
    b = wl.random_tensor(seed + 2, (k,), scale=0.1)
    dy = wl.random_tensor(seed + 3, (n, k, oh, ow))
    rng = np.random.default_rng(seed)

    d = vcnn.conv_desc(n, c, h, w, k, L.kh, L.kw, L.pad_h, L.pad_w, act=vcnn.ACT_RELU if L.relu else vcnn.ACT_NONE)
    ws = torch.empty(max(256, *(vcnn.conv_workspace_bytes(d, p) for p in range(3))), dtype=torch.uint8, device=DEV)
    xd, wd, bd, dyd = to_dev(x), to_dev(wt), to_dev(b), to_dev(dy)

    y = torch.full((n, k, oh, ow), float("nan"), device=DEV)
    vcnn.conv_fwd(d, xd, wd, bd, y, ws)
    yh = to_np(y)
    assert np.all(np.isfinite(yh))
    idx = sample_idx(rng, yh.shape)
    check_samples([yh[i] for i in idx], O.conv_fwd_at(x, wt, b, pad, idx, relu=L.relu), f"{name} conv{li} fwd")

    dw = torch.full(wt.shape, float("nan"), device=DEV)
    db = torch.full((k,), float("nan"), device=DEV)
    vcnn.conv_bwd_filter(d, xd, dyd, dw, db, ws)
    dwh = to_np(dw)
    assert np.all(np.isfinite(dwh))
    idx = sample_idx(rng, dwh.shape)
    check_samples([dwh[i] for i in idx], O.conv_bwd_filter_at(x, dy, (L.kh, L.kw), pad, idx), f"{name} conv{li} dw")
    check_samples(to_np(db), dy.astype(np.float64).sum(axis=(0, 2, 3)), f"{name} conv{li} db")
    # run-to-run bit identity at full size
    dw2 = torch.empty_like(dw)
    vcnn.conv_bwd_filter(d, xd, dyd, dw2, None, ws)
    assert torch.equal(dw, dw2)

    dx = torch.full((n, c, h, w), float("nan"), device=DEV)
    vcnn.conv_bwd_data(d, wd, dyd, dx, ws)
    dxh = to_np(dx)
    assert np.all(np.isfinite(dxh))
    border = [(0, 0, 0, w - 1), (n - 1, c - 1, h - 1, 0), (n // 2, c // 2, h // 2, w // 2)]
    idx = sample_idx(rng, dxh.shape, border)
    check_samples([dxh[i] for i in idx], O.conv_bwd_data_at(wt, dy, pad, idx), f"{name} conv{li} dx")


def test_unroll_full_size_properties():
    """phi_c and phi_c^{-1} at a large layer (cfg4 c2: 1600 x 262144 patch matrix): sampled entries
    are exact copies, and the adjoint identity holds."""
    n, c, h, w, r, s, ph, pw = 64, 64, 64, 64, 5, 5, 2, 2
    d = vcnn.conv_desc(n, c, h, w, 32, r, s, ph, pw)
    x = wl.random_tensor(7001, (n, c, h, w))
    xd = to_dev(x)
    col = torch.empty((c * r * s, n * h * w), device=DEV)
    vcnn.im2col(d, xd, col)
    rng = np.random.default_rng(7)
    rows = rng.integers(0, c * r * s, size=200)
    cols = rng.integers(0, n * h * w, size=200)
    got = col[torch.from_numpy(rows).to(DEV), torch.from_numpy(cols).to(DEV)].cpu().numpy()
    for g, rr, cc in zip(got, rows, cols):
        ci, q = divmod(int(rr), r * s)
        ri, si = divmod(q, s)
        ni, p = divmod(int(cc), h * w)
        ohh, oww = divmod(p, w)
        ih, iw = ohh + ri - ph, oww + si - pw
        want = x[ni, ci, ih, iw] if 0 <= ih < h and 0 <= iw < w else 0.0
        assert g == want
    # <phi_c(x), y> = <x, phi_c^{-1}(y)> with y = phi_c(x) itself: both sides on the GPU tensors, fp64 on the host
    back = torch.empty((n, c, h, w), device=DEV)
    vcnn.col2im(d, col, back)
    lhs = float(torch.sum(col.double() * col.double()))
    rhs = float(torch.sum(xd.double() * back.double()))
    assert abs(lhs - rhs) <= 1e-6 * abs(lhs)


@pytest.mark.parametrize("li", [li for li, _, _ in conv_layers("cfg5")])
def test_cfg5_layer_full_size_bf16_sampled(li):
    """The bf16 variant at cfg5's full batch (the configuration the benchmark times): bf16 matrix-core
    kernels for the forward pass and both gradients, sampled against the oracle's probes evaluated on
    the same bf16-rounded tensors."""
    from util import TOL_BF16
    net = wl.make_net("cfg5")
    L = net.layers[li]
    n, c, h, w = net.in_shape(li)
    _, k, oh, ow = net.shapes[li]
    pad = (L.pad_h, L.pad_w)
    seed = 6000 + li
    x = wl.bf16_round(np.abs(wl.random_tensor(seed, (n, c, h, w))) if li > 0 else wl.random_tensor(seed, (n, c, h, w)))
    wt = wl.bf16_round(wl.random_tensor(seed + 1, (k, c, L.kh, L.kw), scale=(2.0 / (c * L.kh * L.kw)) ** 0.5))
    b = wl.random_tensor(seed + 2, (k,), scale=0.1)
    dy = wl.bf16_round(wl.random_tensor(seed + 3, (n, k, oh, ow)))
    rng = np.random.default_rng(seed)
    dev16 = lambda a: torch.from_numpy(a).to(DEV).to(torch.bfloat16)
    host = lambda t: (torch.cuda.synchronize(), t.float().cpu().numpy())[1]

    d = vcnn.conv_desc(n, c, h, w, k, L.kh, L.kw, L.pad_h, L.pad_w, dtype=vcnn.BF16,
                       act=vcnn.ACT_RELU if L.relu else vcnn.ACT_NONE)
    ws = torch.empty(max(256, *(vcnn.conv_workspace_bytes(d, p) for p in range(3))), dtype=torch.uint8, device=DEV)
    xd, wd, bd, dyd = dev16(x), dev16(wt), to_dev(b), dev16(dy)

    def check(got, want, tol, what):
        want = np.asarray(want, dtype=np.float64)
        err = np.max(np.abs(np.asarray(got, dtype=np.float64) - want)) / max(np.max(np.abs(want)), 1e-30)
        assert err <= tol, f"{what}: sampled max-norm relative error {err:.3e}"

    y = torch.full((n, k, oh, ow), float("nan"), dtype=torch.bfloat16, device=DEV)
    vcnn.conv_fwd(d, xd, wd, bd, y, ws)
    yh = host(y)
    assert np.all(np.isfinite(yh))
    idx = sample_idx(rng, yh.shape)
    check([yh[i] for i in idx], O.conv_fwd_at(x, wt, b, pad, idx, relu=L.relu), TOL_BF16, f"cfg5 bf16 conv{li} fwd")

    dw = torch.full(wt.shape, float("nan"), device=DEV)
    db = torch.full((k,), float("nan"), device=DEV)
    vcnn.conv_bwd_filter(d, xd, dyd, dw, db, ws)
    dwh = to_np(dw)
    assert np.all(np.isfinite(dwh))
    idx = sample_idx(rng, dwh.shape)
    check([dwh[i] for i in idx], O.conv_bwd_filter_at(x, dy, (L.kh, L.kw), pad, idx), TOL_F32, f"cfg5 bf16 conv{li} dw")
    check(to_np(db), dy.astype(np.float64).sum(axis=(0, 2, 3)), TOL_F32, f"cfg5 bf16 conv{li} db")

    dx = torch.full((n, c, h, w), float("nan"), dtype=torch.bfloat16, device=DEV)
    vcnn.conv_bwd_data(d, wd, dyd, dx, ws)
    dxh = host(dx)
    assert np.all(np.isfinite(dxh))
    idx = sample_idx(rng, dxh.shape, [(0, 0, 0, w - 1), (n - 1, c - 1, h - 1, 0)])
    check([dxh[i] for i in idx], O.conv_bwd_data_at(wt, dy, pad, idx), TOL_BF16, f"cfg5 bf16 conv{li} dx")
