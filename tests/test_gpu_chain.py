"""Parity of whole training steps on the five synthetic networks.

Two protocols:
  * layer-wise: every HIP layer call is fed the fp32 rounding of the ORACLE's input to that layer, so
    pooling sees bit-identical inputs and its argmax indices must match exactly;
  * end-to-end: the HIP chain runs on its own intermediates; tensors must match within tolerance and
    any argmax mismatch must be a near-tie in the oracle's own values.
cfg1-cfg3 run at their stated sizes, the two recognition networks also at the mini-batch sizes of the paper's
batch experiments (Tables 3 and 4: 1, 100, 300, 400; 200 lies between tested sizes on the same routes), where the
library picks other kernels; cfg4 and cfg5 run the same layer stack on a smaller batch so the nested-loop oracle
finishes in seconds (their layers at the stated batch are covered layer by layer in test_gpu_fullsize.py).
"""
import functools

import numpy as np
import pytest
import torch

import oracle as O
from oracle.net import train_step as oracle_step
from paper_1501_07338_amd import vcnn
from paper_1501_07338_amd import workloads as wl
from paper_1501_07338_amd.net import TrainStep
from util import TOL_F32, assert_close, to_dev, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
CASES = [("cfg1", None), ("cfg2", None), ("cfg3", None), ("cfg4", 4), ("cfg5", 1),
         ("cfg2", 1), ("cfg2", 100), ("cfg2", 300), ("cfg2", 400), ("cfg3", 1), ("cfg3", 100), ("cfg3", 300), ("cfg3", 400)]


@functools.lru_cache(maxsize=None)
def reference(name, batch):
    net = wl.make_net(name, batch)
    inputs, params = wl.make_inputs(net), wl.make_params(net)
    return net, inputs, params, oracle_step(net, inputs, params)


def f32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float32))


@pytest.mark.parametrize("name,batch", CASES)
def test_layerwise_parity(name, batch):
    net, inputs, params, ref = reference(name, batch)
    for li, L in enumerate(net.layers):
        a_in, a_out = f32(ref["acts"][li]), ref["acts"][li + 1]
        d_out = ref["dacts"][li + 1]
        tag = f"{name} layer {li} {L}"
        if isinstance(L, wl.Conv):
            w, b = params[li]
            n, c, h, wd = a_in.shape
            d = vcnn.conv_desc(n, c, h, wd, L.cout, L.kh, L.kw, L.pad_h, L.pad_w, act=vcnn.ACT_RELU if L.relu else 0)
            ws = torch.empty(max(256, *(vcnn.conv_workspace_bytes(d, p) for p in range(3))), dtype=torch.uint8, device=DEV)
            y = torch.full(a_out.shape, float("nan"), device=DEV)
            vcnn.conv_fwd(d, to_dev(a_in), to_dev(w), to_dev(b), y, ws)
            assert_close(to_np(y), a_out, TOL_F32, tag + " fwd")
            dpre = O.relu_bwd(a_out, d_out) if L.relu else d_out
            if L.relu:
                g = torch.full(a_out.shape, float("nan"), device=DEV)
                vcnn.act_bwd(vcnn.ACT_RELU, vcnn.F32, g.numel(), to_dev(f32(a_out)), to_dev(f32(d_out)), g)
                np.testing.assert_array_equal(to_np(g), f32(dpre))
            dw = torch.full(w.shape, float("nan"), device=DEV)
            db = torch.full(b.shape, float("nan"), device=DEV)
            vcnn.conv_bwd_filter(d, to_dev(a_in), to_dev(f32(dpre)), dw, db, ws)
            assert_close(to_np(dw), ref["grads"][li][0], TOL_F32, tag + " dw")
            assert_close(to_np(db), ref["grads"][li][1], TOL_F32, tag + " db")
            dx = torch.full(a_in.shape, float("nan"), device=DEV)
            vcnn.conv_bwd_data(d, to_dev(w), to_dev(f32(dpre)), dx, ws)
            assert_close(to_np(dx), ref["dacts"][li], TOL_F32, tag + " dx")
        elif isinstance(L, wl.Pool):
            n, c, h, wd = a_in.shape
            d = vcnn.pool_desc(n, c, h, wd, L.win, L.win, L.stride, L.stride)
            y = torch.full(a_out.shape, float("nan"), device=DEV)
            am = torch.full(a_out.shape, -1, dtype=torch.int32, device=DEV)
            vcnn.pool_fwd(d, to_dev(a_in), y, am)
            # the oracle's pooling input is already fp32-exact?  Not in general: compare against the
            # oracle run on the rounded input, which is what the HIP kernel saw.
            ry, ram = O.maxpool_fwd(a_in, (L.win, L.win), (L.stride, L.stride))
            np.testing.assert_array_equal(to_np(am), ram, err_msg=tag + " argmax")
            np.testing.assert_array_equal(to_np(y), f32(ry))
            dx = torch.full(a_in.shape, float("nan"), device=DEV)
            vcnn.pool_bwd(d, to_dev(f32(d_out)), am, dx)
            assert_close(to_np(dx), O.maxpool_bwd(f32(d_out), ram, (h, wd)), 1e-6, tag + " dx")
        else:
            w, b = params[li]
            x2 = a_in.reshape(a_in.shape[0], -1)
            bsz, in_f = x2.shape
            y = torch.full(a_out.shape, float("nan"), device=DEV)
            vcnn.fc_fwd(vcnn.F32, bsz, in_f, L.out, vcnn.ACT_RELU if L.relu else 0, to_dev(x2), to_dev(w), to_dev(b), y)
            assert_close(to_np(y), a_out, TOL_F32, tag + " fwd")
            dpre = O.relu_bwd(a_out, d_out) if L.relu else d_out
            dw = torch.full(w.shape, float("nan"), device=DEV)
            db = torch.full(b.shape, float("nan"), device=DEV)
            dx = torch.full(x2.shape, float("nan"), device=DEV)
            vcnn.fc_bwd(vcnn.F32, bsz, in_f, L.out, to_dev(x2), to_dev(w), to_dev(f32(dpre)), dw, db, dx)
            assert_close(to_np(dw), ref["grads"][li][0], TOL_F32, tag + " dw")
            assert_close(to_np(db), ref["grads"][li][1], TOL_F32, tag + " db")
            assert_close(to_np(dx), ref["dacts"][li].reshape(x2.shape), TOL_F32, tag + " dx")
    # cost
    out = f32(ref["acts"][-1])
    loss = torch.full((), float("nan"), device=DEV)
    dout = torch.full(out.shape, float("nan"), device=DEV)
    if net.loss == "softmax":
        vcnn.softmax_loss(out.shape[0], out.shape[1], to_dev(out), to_dev(inputs["labels"]), loss, dout)
    elif net.loss == "l2":
        vcnn.l2_loss(vcnn.F32, out.size, out.shape[0], to_dev(out), to_dev(inputs["target"]), loss, dout)
    if net.loss != "upstream":
        assert abs(float(to_np(loss)) - ref["loss"]) <= TOL_F32 * abs(ref["loss"])
        assert_close(to_np(dout), ref["dacts"][-1], TOL_F32, name + " dloss")


def argmax_mismatches_are_near_ties(gpu_am, ref_am, x_ref):
    """Every position where the HIP chain picked another index must be a near-tie in the oracle's
    own input (gap <= 1e-5 * max|x|)."""
    bad = np.argwhere(gpu_am != ref_am)
    scale = float(np.max(np.abs(x_ref)))
    for n, c, oh, ow in bad:
        plane = x_ref[n, c].reshape(-1)
        gap = abs(plane[ref_am[n, c, oh, ow]] - plane[gpu_am[n, c, oh, ow]])
        assert gap <= 1e-5 * scale, f"argmax mismatch at {(n, c, oh, ow)} is not a near-tie (gap {gap:.3e})"
    return len(bad)


# cfg5's 16 x 16 x 512 layer and cfg4's 512-map layer as six bfloat16 products per float product (VCNN_ALGO_SPLIT)
SPLIT_CASES = [("cfg5", 1, {2: vcnn.ALGO_SPLIT}), ("cfg4", 4, {1: vcnn.ALGO_SPLIT})]


@pytest.mark.parametrize("name,batch,algos", [(n, b, None) for n, b in CASES] + SPLIT_CASES)
def test_end_to_end_training_step(name, batch, algos):
    net, inputs, params, ref = reference(name, batch)
    ts = TrainStep(net, params, inputs, device=DEV, first_layer_dx=True, algos=algos)
    for li in algos or {}:  # the named layers really are planned under that route: its workspace need is another
        query = lambda: vcnn.conv_workspace_bytes(ts.descs[li], vcnn.PASS_FWD)
        assert ts._routed(li, query) != query()
    before = [None if p is None else (to_np(p[0]).copy(), to_np(p[1]).copy()) for p in ts.params]
    ts.step()
    torch.cuda.synchronize()
    flips = 0
    for li, L in enumerate(net.layers):
        got = to_np(ts.acts[li + 1])
        assert_close(got, ref["acts"][li + 1], TOL_F32, f"{name} act {li}")
        if isinstance(L, wl.Pool):
            flips += argmax_mismatches_are_near_ties(to_np(ts.argmax[li]), ref["argmax"][li], ref["acts"][li])
        elif L.relu:
            # a pre-activation within rounding of zero may land on the other side of the ReLU
            want = ref["acts"][li + 1]
            differ = (got > 0) != (want > 0)
            assert np.all(np.maximum(np.abs(got), np.abs(want))[differ] <= 1e-5 * np.max(np.abs(want)))
            flips += int(np.count_nonzero(differ))
    # A flipped near-tie (pool argmax or ReLU sign) legitimately moves one gradient element, which the max-norm
    # measure sees at full size and which spreads over a receptive field further down.  Each differing decision has
    # just been checked to be a tie within rounding of the oracle's own values, i.e. an equally valid choice; the
    # oracle's backward pass is then evaluated with those choices, and the gradients are held to the strict bar.
    print(f"{name} batch {net.batch}: {flips} near-tie decisions differ")
    relu_side = {li: ref["acts"][li + 1] > 0 for li, L in enumerate(net.layers) if getattr(L, "relu", False)}
    if flips:
        relu_side = {li: to_np(ts.acts[li + 1]) > 0 for li in relu_side}
        ref = oracle_step(net, inputs, params, decisions={
            "argmax": {li: to_np(am) for li, am in ts.argmax.items()}, "relu": relu_side})

    def check(got, want, what):
        assert_close(got, want, TOL_F32, what)

    for li in range(len(net.layers)):
        if ts.folds(li):  # stored with the ReLU derivative of the layer below already applied
            check(to_np(ts.dpre[li - 1]), O.relu_bwd(relu_side[li - 1].astype(np.float64), ref["dacts"][li]),
                  f"{name} dpre {li - 1}")
        else:
            check(to_np(ts.dacts[li]), ref["dacts"][li], f"{name} dact {li}")
        if ts.grads[li] is not None:
            check(to_np(ts.grads[li][0]), ref["grads"][li][0], f"{name} dw {li}")
            check(to_np(ts.grads[li][1]), ref["grads"][li][1], f"{name} db {li}")
            check(to_np(ts.params[li][0]), ref["new_params"][li][0], f"{name} w' {li}")
            check(to_np(ts.params[li][1]), ref["new_params"][li][1], f"{name} b' {li}")
            # the update changed the weights by -lr*dw (to fp32 rounding of w)
            step_gpu = to_np(ts.params[li][0]).astype(np.float64) - before[li][0]
            step_ref = -net.lr * ref["grads"][li][0]
            slack = 1e-3 * np.max(np.abs(step_ref)) + 2.0 ** -23 * np.max(np.abs(before[li][0]))
            assert np.max(np.abs(step_gpu - step_ref)) <= slack, f"{name} sgd step {li}"
    if net.loss != "upstream":
        assert abs(float(to_np(ts.loss)) - ref["loss"]) <= TOL_F32 * abs(ref["loss"])
    # run-to-run bit identity of a full step from the same state
    ts2 = TrainStep(net, params, inputs, device=DEV, first_layer_dx=True, algos=algos)
    ts2.step()
    assert vcnn.conv_algo() == vcnn.ALGO_AUTO  # a per-layer route choice leaves the process-wide one alone
    for li in range(len(net.layers)):
        if ts.grads[li] is not None:
            np.testing.assert_array_equal(to_np(ts.grads[li][0]), to_np(ts2.grads[li][0]))
        if ts.folds(li):
            np.testing.assert_array_equal(to_np(ts.dpre[li - 1]), to_np(ts2.dpre[li - 1]))
        else:
            np.testing.assert_array_equal(to_np(ts.dacts[li]), to_np(ts2.dacts[li]))


@pytest.mark.parametrize("name,batch", [("cfg2", 32), ("cfg3", 16)])
def test_hip_graph_replay_matches_eager(name, batch):
    """The benchmark replays a recorded step; every replay must leave exactly the state the eager
    call sequence leaves, with other work and synchronisations between the replays."""
    net = wl.make_net(name, batch)
    inputs, params = wl.make_inputs(net), wl.make_params(net)
    eager = TrainStep(net, params, inputs, device=DEV)
    graphed = TrainStep(net, params, inputs, device=DEV)
    graph = graphed.capture()  # runs one eager step, then records (and thereby runs) nothing more
    eager.step()
    torch.cuda.synchronize()
    for replay in range(4):
        eager.step()
        graph.replay()
        torch.cuda.synchronize()
        scratch = torch.randn(1 << 16, device=DEV).sum().item()  # unrelated eager work between replays
        assert np.isfinite(scratch)
        for li in range(len(net.layers)):
            if eager.grads[li] is not None:
                np.testing.assert_array_equal(to_np(graphed.grads[li][0]), to_np(eager.grads[li][0]),
                                              err_msg=f"replay {replay} dw {li}")
                np.testing.assert_array_equal(to_np(graphed.params[li][0]), to_np(eager.params[li][0]),
                                              err_msg=f"replay {replay} w {li}")
        assert float(to_np(graphed.loss)) == float(to_np(eager.loss))


@pytest.mark.parametrize("name,batch", [("cfg2", 32), ("cfg3", 16)])
def test_one_stream_step_matches_two_stream_step(name, batch):
    """The benchmark also times the step with every kernel on one stream; the schedule must not change a bit."""
    net = wl.make_net(name, batch)
    inputs, params = wl.make_inputs(net), wl.make_params(net)
    two = TrainStep(net, params, inputs, device=DEV)
    one = TrainStep(net, params, inputs, device=DEV, overlap=False)
    assert one.side is None and two.side is not None
    for _ in range(3):
        two.step()
        one.step()
    torch.cuda.synchronize()
    for li in range(len(net.layers)):
        if two.grads[li] is not None:
            np.testing.assert_array_equal(to_np(one.grads[li][0]), to_np(two.grads[li][0]), err_msg=f"dw {li}")
            np.testing.assert_array_equal(to_np(one.params[li][0]), to_np(two.params[li][0]), err_msg=f"w {li}")
    assert float(to_np(one.loss)) == float(to_np(two.loss))


@pytest.mark.parametrize("name,batch", [("cfg2", 1), ("cfg2", 100), ("cfg2", 200), ("cfg2", 400), ("cfg2", 600),
                                        ("cfg3", 1), ("cfg3", 200), ("cfg3", 400)])
def test_forward_only_pass(name, batch):
    """The test-time path the mini-batch sweep times (the paper's Table 4): TrainStep.forward alone, on a state
    whose gradient buffers were never written, against the oracle's forward tensors and pooling choices."""
    net = wl.make_net(name, batch)
    inputs, params = wl.make_inputs(net), wl.make_params(net)
    ts = TrainStep(net, params, inputs, device=DEV)
    for t in ts.acts[1:]:
        t.fill_(float("nan"))
    ts.forward()
    a = np.asarray(inputs["x"], dtype=np.float64)
    for li, L in enumerate(net.layers):
        if isinstance(L, wl.Conv):
            a = O.conv_fwd(a, params[li][0], params[li][1], pad=(L.pad_h, L.pad_w), relu=L.relu)
        elif isinstance(L, wl.Pool):
            ref_in = a
            a, am = O.maxpool_fwd(a, (L.win, L.win), (L.stride, L.stride))
            argmax_mismatches_are_near_ties(to_np(ts.argmax[li]), am, ref_in)
        else:
            a = O.fc_fwd(a.reshape(a.shape[0], -1), params[li][0], params[li][1], relu=L.relu)
        assert_close(to_np(ts.acts[li + 1]), a, TOL_F32, f"{name} batch {batch} forward-only act {li}")


@pytest.mark.parametrize("name,bf16", [("cfg4", False), ("cfg5", False), ("cfg5", True)])
def test_launch_schedules_agree_bit_for_bit_at_full_size(name, bf16):
    """The three ways the benchmark issues a step (two streams, one stream, HIP-graph replay) at the workloads'
    stated batch: one step each from the same seeded parameters must leave identical bits, the replay repeatedly
    (parameters restored in between, with other work and synchronisations between the replays)."""
    net = wl.make_net(name)
    inputs, params = wl.make_inputs(net), wl.make_params(net)
    dt = vcnn.BF16 if bf16 else vcnn.F32
    two = TrainStep(net, params, inputs, device=DEV, dtype=dt)
    one = TrainStep(net, params, inputs, device=DEV, dtype=dt, overlap=False)
    rep = TrainStep(net, params, inputs, device=DEV, dtype=dt)
    two.step()
    one.step()
    rep.snapshot()
    graph = rep.capture()  # one eager step, then the recording
    torch.cuda.synchronize()
    assert np.isfinite(float(to_np(two.loss)))

    def same(a, b, what):
        for li in range(len(net.layers)):
            if a.grads[li] is not None:
                assert torch.equal(a.grads[li][0], b.grads[li][0]), f"{what}: dw {li}"
                assert torch.equal(a.grads[li][1], b.grads[li][1]), f"{what}: db {li}"
                assert torch.equal(a.params[li][0], b.params[li][0]), f"{what}: w {li}"
            assert torch.equal(a.acts[li + 1], b.acts[li + 1]), f"{what}: act {li}"
        assert float(to_np(a.loss)) == float(to_np(b.loss)), what

    same(one, two, "one stream vs two streams")
    same(rep, two, "eager step of the recorded state vs two streams")
    for replay in range(3):
        rep.restore()
        graph.replay()
        torch.cuda.synchronize()
        assert np.isfinite(torch.randn(1 << 16, device=DEV).sum().item())  # unrelated eager work between replays
        same(rep, two, f"replay {replay} vs two streams")


def test_step_with_split_products_on_the_large_layer():
    """cfg5 at its stated batch with VCNN_ALGO_SPLIT on the 16 x 16 x 512 layer only (the per-layer route choice of
    TrainStep) beside the step on the float kernels: every activation and the loss within a tenth of the fp32 bar, the
    HIP-graph replay bit-identical to the eager step, and the process-wide route choice untouched.  (Gradients are
    held to the oracle's at batch 1 by the end-to-end test: at this size each passes through ReLU and max-pooling
    decisions that a last-bit change of an activation may flip, so two valid steps need not agree element by element.)"""
    net = wl.make_net("cfg5")
    inputs, params = wl.make_inputs(net), wl.make_params(net)
    base = TrainStep(net, params, inputs, device=DEV)
    split = TrainStep(net, params, inputs, device=DEV, algos={2: vcnn.ALGO_SPLIT})
    assert split.workspace.numel() > base.workspace.numel()  # the route is planned for that layer
    base.step()
    split.snapshot()
    graph = split.capture()  # one eager step, then the recording
    torch.cuda.synchronize()
    assert vcnn.conv_algo() == vcnn.ALGO_AUTO
    for li in range(len(net.layers)):
        a, b = split.acts[li + 1].double(), base.acts[li + 1].double()
        assert float((a - b).abs().max() / b.abs().max()) <= 0.1 * TOL_F32, f"act {li}"
    assert abs(float(split.loss) - float(base.loss)) <= 0.1 * TOL_F32 * abs(float(base.loss))
    eager = [t.clone() for pair in split.grads if pair is not None for t in pair] + [split.loss.clone()]
    split.restore()
    graph.replay()
    torch.cuda.synchronize()
    again = [t for pair in split.grads if pair is not None for t in pair] + [split.loss]
    assert all(torch.equal(a, b) for a, b in zip(eager, again))
