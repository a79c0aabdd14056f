"""Host logic: the five synthetic networks have the shapes the benchmark table states, and the
generators are deterministic."""
import numpy as np
import pytest

from paper_1501_07338_amd import workloads as wl


def test_shapes():
    assert wl.make_net("cfg1").shapes == [(8, 6, 24, 24), (8, 6, 12, 12)]
    assert wl.make_net("cfg2").shapes == [(128, 20, 24, 24), (128, 20, 12, 12), (128, 50, 8, 8), (128, 50, 4, 4),
                                         (128, 500), (128, 10)]
    s3 = wl.make_net("cfg3").shapes
    assert s3[1] == (128, 32, 15, 15) and s3[3] == (128, 32, 7, 7) and s3[5] == (128, 64, 3, 3)
    assert wl.make_net("cfg4").shapes == [(64, 64, 64, 64), (64, 32, 64, 64), (64, 1, 64, 64)]
    assert wl.make_net("cfg5").shapes == [(16, 38, 64, 184), (16, 38, 64, 64), (16, 512, 49, 49), (16, 512, 49, 49),
                                         (16, 1, 42, 42)]


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg4"])
def test_generators_deterministic_and_distributed(name):
    net = wl.make_net(name, batch=4)
    a, b = wl.make_inputs(net), wl.make_inputs(net)
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])
    assert a["x"].dtype == np.float32 and a["x"].shape == (4,) + net.in_chw
    pa, pb = wl.make_params(net), wl.make_params(net)
    for p, q in zip(pa, pb):
        if p is not None:
            np.testing.assert_array_equal(p[0], q[0])
    w0 = pa[0][0]
    fan_in = w0[0].size
    assert abs(w0.std() - np.sqrt(2.0 / fan_in)) < 0.35 * np.sqrt(2.0 / fan_in)


def test_cfg5_inputs():
    net = wl.make_net("cfg5", batch=1)
    d = wl.make_inputs(net)
    assert d["x"].shape == (1, 1, 184, 184) and d["target"].shape == (1, 1, 42, 42)
    assert 0.3 < d["x"].mean() < 0.7  # blur kernel sums to one


def test_bf16_round():
    a = np.array([1.0, 1.00390625, 1.01171875, -3.1415927, 0.0], dtype=np.float32)
    r = wl.bf16_round(a)
    assert np.all((r.view(np.uint32) & 0xFFFF) == 0)
    assert r[1] == 1.0 and r[2] == np.float32(1.015625)  # ties to even, both directions
    assert abs(r[3] + 3.140625) < 1e-6
