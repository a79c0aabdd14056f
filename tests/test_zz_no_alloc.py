"""The kernel-gradient entry point that allocates nothing (its partial sums live in a fixed array inside the
library) against the ordinary entry point with a caller workspace: same bits, on calls in a row that share the
array, the later ones with smaller inputs; a layer that needs more than the array holds is rejected."""
import ctypes

import pytest
import torch

from paper_1501_07338_amd import vcnn
from paper_1501_07338_amd import workloads as wl
from util import to_dev

DEV = "cuda:0"

# (n, c, h, w, k, r, s, pad_h, pad_w), in call order: each later layer needs less scratch memory than the first
SEQUENCE = [(128, 32, 7, 7, 64, 5, 5, 2, 2),     # cfg3 c3: 25 MiB of partial sums
            (128, 20, 12, 12, 50, 5, 5, 0, 0),   # cfg2 c2: 12 MiB
            (8, 1, 28, 28, 6, 5, 5, 0, 0),       # cfg1: a few KiB
            (3, 5, 9, 11, 7, 3, 2, 1, 0)]


def run_pair(shape, dtype, seed):
    n, c, h, w, k, r, s, ph, pw = shape
    d = vcnn.conv_desc(n, c, h, w, k, r, s, ph, pw, dtype=dtype)
    oh, ow = vcnn.conv_out_shape(d)
    x, dy = wl.random_tensor(seed, (n, c, h, w)), wl.random_tensor(seed + 1, (n, k, oh, ow))
    xd, dyd = to_dev(x), to_dev(dy)
    if dtype == vcnn.BF16:
        xd, dyd = xd.to(torch.bfloat16), dyd.to(torch.bfloat16)
    need = vcnn.conv_workspace_bytes(d, vcnn.PASS_BWD_FILTER)
    assert need <= vcnn.conv_bwd_filter_noalloc_limit()
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=DEV)
    dw_ref = torch.full((k, c, r, s), float("nan"), device=DEV)
    db_ref = torch.full((k,), float("nan"), device=DEV)
    vcnn.conv_bwd_filter(d, xd, dyd, dw_ref, db_ref, ws)
    dw = torch.full((k, c, r, s), float("nan"), device=DEV)
    db = torch.full((k,), float("nan"), device=DEV)
    vcnn.conv_bwd_filter_noalloc(d, xd, dyd, dw, db)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(dw).all()) and bool(torch.isfinite(db).all())
    assert torch.equal(dw, dw_ref), f"{shape}: dw differs from the workspace entry point"
    assert torch.equal(db, db_ref), f"{shape}: dbias differs from the workspace entry point"
    # without the bias gradient
    dw2 = torch.full((k, c, r, s), float("nan"), device=DEV)
    vcnn.conv_bwd_filter_noalloc(d, xd, dyd, dw2, None)
    torch.cuda.synchronize()
    assert torch.equal(dw2, dw_ref)


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [vcnn.F32, vcnn.BF16])
def test_noalloc_kernel_gradient_matches_workspace_entry_point_on_calls_in_a_row(dtype):
    for i, shape in enumerate(SEQUENCE):
        run_pair(shape, dtype, 9000 + 10 * i)
    run_pair(SEQUENCE[0], dtype, 9100)  # and a large one again after the small ones


@pytest.mark.gpu
def test_noalloc_kernel_gradient_allocates_nothing():
    shape = SEQUENCE[1]
    n, c, h, w, k, r, s, ph, pw = shape
    d = vcnn.conv_desc(n, c, h, w, k, r, s, ph, pw)
    oh, ow = vcnn.conv_out_shape(d)
    xd, dyd = to_dev(wl.random_tensor(9200, (n, c, h, w))), to_dev(wl.random_tensor(9201, (n, k, oh, ow)))
    dw, db = torch.empty((k, c, r, s), device=DEV), torch.empty((k,), device=DEV)
    vcnn.conv_bwd_filter_noalloc(d, xd, dyd, dw, db)  # first use on the device: looks the array up
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for _ in range(5):
        vcnn.conv_bwd_filter_noalloc(d, xd, dyd, dw, db)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 == free0, "device memory in use changed across allocation-free calls"


def test_noalloc_kernel_gradient_rejects_layers_beyond_the_array():
    """No GPU needed: the size check comes before anything touches the device."""
    d = vcnn.conv_desc(16, 512, 49, 49, 512, 1, 1)  # cfg5 c4: 107 MiB of partial sums
    assert vcnn.conv_workspace_bytes(d, vcnn.PASS_BWD_FILTER) > vcnn.conv_bwd_filter_noalloc_limit() == 32 << 20
    with pytest.raises(vcnn.VcnnError) as e:
        st = vcnn.lib().vcnn_conv_bwd_filter_noalloc(ctypes.byref(d), 8, 8, 8, None, None)  # dummy non-NULL pointers
        vcnn._check(st)
    assert e.value.status == vcnn.ERR_WORKSPACE
    assert "scratch" in vcnn.last_error()
    with pytest.raises(vcnn.VcnnError) as e:
        vcnn._check(vcnn.lib().vcnn_conv_bwd_filter_noalloc(ctypes.byref(d), None, 8, 8, None, None))
    assert e.value.status == vcnn.ERR_NULL
