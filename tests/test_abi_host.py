"""Host-side checks of the C-ABI library: it loads, exports every symbol the public header declares,
and rejects bad arguments before touching the GPU.  No compute call is made here."""
import ctypes
import re
from pathlib import Path

import pytest

from paper_1501_07338_amd import vcnn

ROOT = Path(__file__).resolve().parents[1]


def declared_symbols():
    text = (ROOT / "include" / "vcnn.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vcnn_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert len(names) >= 20
    handle = ctypes.CDLL(str(vcnn.LIB_PATH))
    for n in names:
        assert hasattr(handle, n), f"{n} declared in vcnn.h but not exported"
    assert sorted(vcnn.EXPORTS) == names, "python binding and header disagree on the entry points"


def test_version_and_status_strings():
    assert vcnn.version() >= 100
    assert vcnn.status_string(vcnn.OK) == "ok"
    assert "workspace" in vcnn.status_string(vcnn.ERR_WORKSPACE)


def test_conv_shape_algebra():
    d = vcnn.conv_desc(16, 38, 64, 64, 512, 16, 16)
    assert vcnn.conv_out_shape(d) == (49, 49)
    d = vcnn.conv_desc(64, 64, 64, 64, 32, 5, 5, 2, 2)
    assert vcnn.conv_out_shape(d) == (64, 64)
    need = vcnn.conv_workspace_bytes(d, vcnn.PASS_FWD)
    assert need >= 1600 * 262144 * 4 or need == 0  # either the explicit patch matrix or nothing (implicit)
    assert vcnn.conv_workspace_bytes(vcnn.conv_desc(2, 8, 5, 5, 4, 1, 1), vcnn.PASS_FWD) == 0
    p = vcnn.pool_desc(128, 32, 32, 32, 3, 3, 2, 2)
    assert vcnn.pool_out_shape(p) == (15, 15)


@pytest.mark.parametrize("kwargs,status", [
    (dict(n=0), vcnn.ERR_SHAPE), (dict(c=-1), vcnn.ERR_SHAPE), (dict(r=9), vcnn.ERR_SHAPE),
    (dict(pad_h=-1), vcnn.ERR_SHAPE), (dict(stride_h=2), vcnn.ERR_UNSUPPORTED), (dict(dtype=7), vcnn.ERR_UNSUPPORTED),
    (dict(act=5), vcnn.ERR_UNSUPPORTED), (dict(stride_w=0), vcnn.ERR_SHAPE)])
def test_conv_desc_validation(kwargs, status):
    base = dict(n=2, c=3, h=8, w=8, k=4, r=3, s=3)
    base.update(kwargs)
    with pytest.raises(vcnn.VcnnError) as e:
        vcnn.conv_out_shape(vcnn.conv_desc(**base))
    assert e.value.status == status
    assert vcnn.last_error()


def test_null_and_workspace_errors_need_no_gpu():
    d = vcnn.conv_desc(2, 3, 8, 8, 4, 3, 3)
    lib = vcnn.lib()
    assert lib.vcnn_conv_fwd(ctypes.byref(d), None, None, None, None, None, 0, None) == vcnn.ERR_NULL
    need = vcnn.conv_workspace_bytes(d, vcnn.PASS_BWD_DATA)
    if need:
        fake = 0x1000  # never dereferenced: validation fails first
        assert lib.vcnn_conv_bwd_data(ctypes.byref(d), fake, fake, fake, None, 0, None) == vcnn.ERR_WORKSPACE
        assert lib.vcnn_conv_bwd_data(ctypes.byref(d), fake, fake, fake, 0x1010, need, None) == vcnn.ERR_WORKSPACE
        assert lib.vcnn_conv_bwd_data(ctypes.byref(d), fake, fake, fake, 0x1100, need - 1, None) == vcnn.ERR_WORKSPACE
    assert lib.vcnn_conv_out_shape(None, None, None) == vcnn.ERR_NULL
    p = vcnn.pool_desc(1, 1, 2, 2, 3, 3, 1, 1)
    with pytest.raises(vcnn.VcnnError) as e:
        vcnn.pool_out_shape(p)
    assert e.value.status == vcnn.ERR_SHAPE
    assert lib.vcnn_pool_fwd(ctypes.byref(vcnn.pool_desc(1, 1, 4, 4, 2, 2, 2, 2)), None, None, None, None) == vcnn.ERR_NULL
    assert lib.vcnn_fc_fwd(vcnn.F32, 0, 4, 4, 0, None, None, None, None, None) == vcnn.ERR_SHAPE
    assert lib.vcnn_fc_fwd(vcnn.F32, 2, 4, 4, 0, None, None, None, None, None) == vcnn.ERR_NULL
    assert lib.vcnn_softmax_loss(4, 10, None, None, None, None, None) == vcnn.ERR_NULL
    assert lib.vcnn_act_fwd(7, vcnn.F32, 4, None, None, None) == vcnn.ERR_UNSUPPORTED
    assert lib.vcnn_set_conv_algo(99) == vcnn.ERR_UNSUPPORTED
    assert lib.vcnn_set_conv_algo(vcnn.ALGO_AUTO) == vcnn.OK


def test_fused_and_layer_entry_points_validate_before_launch():
    """The calls that fold an activation derivative, and the pooling layer of Eq. 3: unknown activation ids,
    NULL tensors and a workspace that is too small are refused on the host."""
    lib = vcnn.lib()
    p = vcnn.pool_desc(2, 3, 8, 8, 2, 2, 2, 2)
    fake = 0x1000  # never dereferenced: validation fails first
    assert lib.vcnn_pool_bwd_act(ctypes.byref(p), 9, fake, fake, fake, fake, None) == vcnn.ERR_UNSUPPORTED
    assert lib.vcnn_pool_bwd_act(ctypes.byref(p), vcnn.ACT_RELU, None, fake, fake, fake, None) == vcnn.ERR_NULL
    cd = vcnn.conv_desc(2, 3, 8, 8, 4, 3, 3)
    need_dx = vcnn.conv_workspace_bytes(cd, vcnn.PASS_BWD_DATA)
    assert lib.vcnn_conv_bwd_data_act(ctypes.byref(cd), 9, fake, fake, fake, fake, 0x1100, need_dx, None) == vcnn.ERR_UNSUPPORTED
    assert lib.vcnn_conv_bwd_data_act(ctypes.byref(cd), vcnn.ACT_RELU, None, fake, fake, fake, 0x1100, need_dx, None) == vcnn.ERR_NULL
    assert lib.vcnn_conv_bwd_data_act(ctypes.byref(cd), vcnn.ACT_NONE, None, fake, fake, None, 0x1100, need_dx, None) == vcnn.ERR_NULL
    if need_dx:
        assert lib.vcnn_conv_bwd_data_act(ctypes.byref(cd), vcnn.ACT_RELU, fake, fake, fake, fake, None, 0, None) == vcnn.ERR_WORKSPACE
    assert lib.vcnn_pool_layer_fwd(ctypes.byref(p), 9, fake, None, fake, fake, None) == vcnn.ERR_UNSUPPORTED
    assert lib.vcnn_pool_layer_fwd(ctypes.byref(p), vcnn.ACT_TANH, None, None, fake, fake, None) == vcnn.ERR_NULL
    assert lib.vcnn_pool_layer_workspace_bytes(ctypes.byref(p), None) == vcnn.ERR_NULL
    need = vcnn.pool_layer_workspace_bytes(p)
    assert need >= 2 * 3 * 4 * 4 * 4  # at least the delta tensor
    assert lib.vcnn_pool_layer_bwd(ctypes.byref(p), vcnn.ACT_TANH, fake, fake, fake, fake, fake, fake, need - 1,
                                   None) == vcnn.ERR_WORKSPACE
    assert lib.vcnn_pool_layer_bwd(ctypes.byref(p), vcnn.ACT_TANH, None, fake, fake, None, fake, fake, need,
                                   None) == vcnn.ERR_NULL  # y is needed for sigma'
    assert lib.vcnn_pool_layer_bwd(ctypes.byref(p), 9, fake, fake, fake, None, fake, fake, need, None) == vcnn.ERR_UNSUPPORTED
    assert lib.vcnn_fc_bwd_act(vcnn.F32, 4, 8, 2, 9, fake, fake, fake, None, None, fake, None) == vcnn.ERR_UNSUPPORTED
    # with an activation below, x is read for dx as well
    assert lib.vcnn_fc_bwd_act(vcnn.F32, 4, 8, 2, vcnn.ACT_RELU, None, fake, fake, None, None, fake, None) == vcnn.ERR_NULL
    assert lib.vcnn_fc_bwd_act(vcnn.F32, 0, 8, 2, vcnn.ACT_NONE, fake, fake, fake, None, None, fake, None) == vcnn.ERR_SHAPE


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
def test_workspace_queries_of_every_workload_layer(name):
    """Route planning runs on the host: for every convolution of the five workloads, every pass, both storage types
    and every forced route the query succeeds, agrees with itself, and stays below the explicit patch matrix plus its
    partial sums (the largest realisation there is)."""
    from paper_1501_07338_amd import workloads as wl
    net = wl.make_net(name)
    try:
        for li, L in enumerate(net.layers):
            if not isinstance(L, wl.Conv):
                continue
            n, c, h, w = net.in_shape(li)
            _, k, oh, ow = net.shapes[li]
            for dtype in (vcnn.F32, vcnn.BF16):
                d = vcnn.conv_desc(n, c, h, w, k, L.kh, L.kw, L.pad_h, L.pad_w, dtype=dtype)
                patch_matrix = 4 * c * L.kh * L.kw * n * oh * ow
                for algo in (vcnn.ALGO_AUTO, vcnn.ALGO_EXPLICIT, vcnn.ALGO_IMPLICIT, vcnn.ALGO_FOLD, vcnn.ALGO_FFT, vcnn.ALGO_SPLIT):
                    vcnn.set_conv_algo(algo)
                    for p in (vcnn.PASS_FWD, vcnn.PASS_BWD_FILTER, vcnn.PASS_BWD_DATA):
                        need = vcnn.conv_workspace_bytes(d, p)
                        assert need == vcnn.conv_workspace_bytes(d, p)
                        assert 0 <= need <= 3 * patch_matrix + (1 << 29), (name, li, dtype, algo, p, need)
    finally:
        vcnn.set_conv_algo(vcnn.ALGO_AUTO)
