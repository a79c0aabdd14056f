#!/usr/bin/env python3
"""Benchmark of the vectorized CNN layer path on one MI355X.

A "step" is one full training step (forward, cost, backward, SGD update) of a synthetic network whose
inputs and weights are already resident in HBM; every arithmetic step runs in libvcnn's HIP kernels.
The headline is the largest of the five workloads, the deconvolution CNN cfg5 in fp32 (1.29 TFLOP per
step): images/s of the training step, GFLOP/s of its convolution passes against the fp32 matrix-core
peak, and the roofline record of the pass that takes the most time.  cfg5 with bf16 storage and
cfg1-cfg4 ride along as compact summaries; the long per-layer tables, the bandwidth-bound kernels and
the mini-batch sweep go to a side file (--detail).

Every timed step starts from the same seeded parameters: the squared-error networks (cfg4, cfg5) leave
the range of finite floats within three plain-SGD steps at the stated learning rate, so the initial
parameters are restored before each step, outside the step's event pair, and the per-layer timings run
on the tensors of exactly one step.  Each step is bracketed by its own pair of events on the stream it
is issued on; ms_per_step is the mean over the K timed steps.  A non-finite loss aborts the run.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5] [--others cfg5_bf16,cfg1,...]
"""
from __future__ import annotations

import argparse
import json
import math
import os
import statistics
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

METRIC = "conv fwd+bwd GFLOP/s (% MFMA peak) and images/sec per training step, 1 GPU"  # the benchmark's
HBM_PEAK_GBS = 8000.0
MFMA_F32_PEAK_TFLOPS = 157.3
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 -> fp32 accumulate
WORKLOAD_TEXT = {
    "cfg1": "cfg1: single conv block 8x1x28x28 -> conv5x5x6 -> ReLU -> maxpool2, fwd + bwd from an upstream gradient",
    "cfg2": "cfg2: small recognition CNN, batch 128x1x28x28, conv5x5x20-pool-conv5x5x50-pool-fc500-fc10, "
            "full training step (fwd + softmax-CE + bwd + SGD)",
    "cfg3": "cfg3: colour recognition CNN, batch 128x3x32x32, three conv5x5 (32,32,64) + 3x3/2 pools + fc64 + fc10, "
            "full training step",
    "cfg4": "cfg4: denoising CNN, batch 64x1x64x64, conv9x9x64-conv5x5x32-conv5x5x1 'same', L2 loss, full training step",
    "cfg5": "cfg5: deconvolution CNN, batch 16x1x184x184, conv121x1x38-conv1x121x38-conv16x16x512-conv1x1x512-conv8x8x1 "
            "valid, L2 loss, full training step (fwd + cost + bwd + SGD)",
}
LAUNCH_TEXT = {"graph": "one HIP-graph replay per step (parameter gradients on a second branch)",
               "two_streams": "eager: one C call per layer pass, parameter gradients on a second stream",
               "one_stream": "eager: one C call per layer pass, one stream"}


def conv_geom(net, li):
    from paper_1501_07338_amd.workloads import Conv
    L = net.layers[li]
    assert isinstance(L, Conv)
    n, c, h, w = net.in_shape(li)
    _, k, oh, ow = net.shapes[li]
    return dict(n=n, c=c, h=h, w=w, k=k, r=L.kh, s=L.kw, oh=oh, ow=ow, M=k, K=c * L.kh * L.kw, N=n * oh * ow)


def time_calls(fn, iters, stream):
    """Average duration in ms of `fn` over `iters` back-to-back enqueues, measured with events on
    the stream the kernels are launched on (one untimed call first)."""
    import torch
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    fn()
    stream.synchronize()
    start.record(stream)
    for _ in range(iters):
        fn()
    stop.record(stream)
    stop.synchronize()
    return start.elapsed_time(stop) / iters


def timed_steps(fn, steps, stream, before=None):
    """Times exactly `steps` calls of fn, each between its own pair of events on `stream`, synchronised on
    both sides of the whole region; `before` (the parameter restore) runs ahead of each step outside its
    event pair.  Returns (mean ms per step, median ms per step, wall ms per step including `before`)."""
    import torch
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b in pairs:
        if before is not None:
            before()
        a.record(stream)
        fn()
        b.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    ms = [a.elapsed_time(b) for a, b in pairs]
    return sum(ms) / steps, statistics.median(ms), wall_ms


def finite_or_die(name, loss):
    if not math.isfinite(loss):
        sys.exit(f"bench.py: {name}: the loss is not finite ({loss}); refusing to report timings of non-finite tensors")
    return loss


MARKERS: dict = {}  # marker id -> name of the phase it precedes (filled only with --markers)


def mark(name):
    """With --markers: launches an empty kernel whose grid size numbers the phase `name` in a kernel trace."""
    if MARKERS is not None and mark.enabled:
        from paper_1501_07338_amd import benchaid
        ident = len(MARKERS) + 1
        MARKERS[ident] = name
        benchaid.marker(ident)


mark.enabled = False


def run_workload(name, steps, warmup, layer_iters=10, algos=None, phase_prefix=None):
    """`name` is a workload, optionally suffixed `_bf16` for the bfloat16-storage variant; algos: per-layer route
    choices ({layer index: vcnn.ALGO_*}) for the step and the per-layer timings; phase_prefix: the name the per-layer
    phases carry in a kernel trace (--markers) when it is not the workload's."""
    import torch
    from paper_1501_07338_amd import vcnn, workloads as wl
    from paper_1501_07338_amd.net import TrainStep

    bf16 = name.endswith("_bf16")
    net = wl.make_net(name[:-5] if bf16 else name)
    inputs, params = wl.make_inputs(net), wl.make_params(net)
    ts = TrainStep(net, params, inputs, device="cuda:0", first_layer_dx=False, dtype=vcnn.BF16 if bf16 else vcnn.F32,
                   algos=algos)
    ts.snapshot()
    esize = 2.0 if bf16 else 4.0
    stream = torch.cuda.current_stream()
    losses = []

    def timed(fn):
        for _ in range(warmup):
            ts.restore()
            fn()
        res = timed_steps(fn, steps, stream, before=ts.restore)
        losses.append(finite_or_die(name, float(ts.loss.item())))  # the loss of a first step, every time
        return res

    # The same step, issued three ways; the fastest is the workload's figure.  On the small networks every kernel
    # is a few microseconds, the fork / join between the two streams costs more than the overlap returns and a
    # plain in-order launch wins; on the large ones the parameter-gradient strand on a second stream pays, eagerly
    # or as a replayed graph.
    modes = {}
    modes["two_streams"] = timed(ts.step)
    side, ts.side = ts.side, None  # the same step with every kernel on one stream (no fork / join events)
    modes["one_stream"] = timed(ts.step)
    ts.side = side
    ts.restore()
    graph = ts.capture()
    modes["graph"] = timed(graph.replay)
    assert max(losses) - min(losses) <= 1e-6 * abs(losses[0]), f"{name}: the three launch modes disagree on the loss {losses}"
    launch = min(modes, key=lambda m: modes[m][0])
    best_ms = modes[launch][0]
    res = {"workload": name, "batch": net.batch, "storage_dtype": "bf16" if bf16 else "f32", "ms_per_step": best_ms,
           "ms_per_step_median": modes[launch][1], "wall_ms_per_step_with_restore": modes[launch][2],
           "launch": launch, "ms_per_step_by_launch": {m: v[0] for m, v in modes.items()},
           "images_per_s": net.batch / (best_ms * 1e-3), "loss_first_step": losses[0]}

    # Per-layer passes on the tensors of exactly one step from the seeded parameters (no update applied)
    ts.restore()
    ts.forward()
    ts.cost()
    ts.backward()
    torch.cuda.synchronize()
    finite_or_die(name, float(ts.loss.item()))
    for t in ts.acts + [g for pair in ts.grads if pair is not None for g in pair]:
        if not bool(torch.isfinite(t.float()).all()):
            sys.exit(f"bench.py: {name}: non-finite tensor ahead of the per-layer timings")
    layers = []
    conv_flops = conv_ms = 0.0
    for li, L in enumerate(net.layers):
        if not isinstance(L, wl.Conv):
            continue
        g = conv_geom(net, li)
        d = ts.descs[li]
        w, b = ts.weights(li), ts.params[li][1]
        dw, db = ts.grads[li]
        a_in, a_out = ts.acts[li], ts.acts[li + 1]
        dy = ts.dpre.get(li, ts.dacts[li + 1])  # the gradient w.r.t. the pre-activation, as the step passes it
        flops = 2.0 * g["M"] * g["K"] * g["N"]
        dx_buf = ts.dacts[li] if li > 0 else torch.empty_like(a_in)
        y_buf = torch.empty_like(a_out)  # the forward pass is re-run into a spare buffer: the step's tensors stay as they are
        routed = lambda call, li=li: ts._routed(li, call)  # the layer's own route choice, if it has one
        passes = {
            "fwd": lambda: routed(lambda: vcnn.conv_fwd(d, a_in, w, b, y_buf, ts.workspace)),
            "bwd_filter": lambda: routed(lambda: vcnn.conv_bwd_filter(d, a_in, dy, dw, db, ts.workspace_side)),
            "bwd_data": lambda: routed(lambda: vcnn.conv_bwd_data(d, w, dy, dx_buf, ts.workspace)),
        }
        in_b = esize * g["n"] * g["c"] * g["h"] * g["w"]
        out_b = esize * g["M"] * g["N"]
        w_b = esize * g["M"] * g["K"]
        ws_need = routed(lambda: max(vcnn.conv_workspace_bytes(d, p) for p in (vcnn.PASS_FWD, vcnn.PASS_BWD_DATA)))
        assert ts.workspace.numel() >= ws_need
        for pname, fn in passes.items():
            mark(f"{phase_prefix or name}.conv{li}.{pname}")
            t = time_calls(fn, layer_iters, stream)
            mark("-")
            peak = MFMA_BF16_PEAK_TFLOPS if bf16 else MFMA_F32_PEAK_TFLOPS
            layers.append({"layer": f"conv{li}", "pass": pname, "M": g["M"], "K": g["K"], "N": g["N"], "ms": t,
                           "gflops": flops / (t * 1e6),
                           # the bf16 variant contracts on the bf16 matrix-core instructions: priced against their peak
                           "pct_mfma_peak": 100.0 * flops / (t * 1e9) / peak,
                           "algorithmic_bytes": in_b + out_b + w_b, "gbs": (in_b + out_b + w_b) / (t * 1e6),
                           "in_step": not (li == 0 and pname == "bwd_data")})
            if not (li == 0 and pname == "bwd_data"):
                conv_flops += flops
                conv_ms += t
        del y_buf, dx_buf
    res["conv_layers"] = layers
    res["conv_gflops_fwd_bwd"] = conv_flops / (conv_ms * 1e6) if conv_ms else None
    peak = MFMA_BF16_PEAK_TFLOPS if bf16 else MFMA_F32_PEAK_TFLOPS
    res["conv_pct_mfma_peak"] = 100.0 * res["conv_gflops_fwd_bwd"] / (peak * 1e3) if conv_ms else None
    res["roofline"] = dominant_roofline(res)
    del graph, ts
    torch.cuda.empty_cache()
    return res


def measured_traffic(name):
    """HBM bytes per launch of the named pass from the tracked counter summary (profiles/traffic.json, written by
    `python -m paper_1501_07338_amd.benchaid.profile_summary` from two rocprofv3 --pmc runs); None if not covered."""
    path = ROOT / "profiles" / "traffic.json"
    if not path.exists():
        return None
    try:
        rec = json.loads(path.read_text()).get("passes", {}).get(name)
    except (ValueError, OSError):
        return None
    return None if rec is None else rec.get("hbm_bytes")


def dominant_roofline(res):
    """Roofline record of the convolution pass that takes the most time inside the step.  A pass whose
    arithmetic intensity (flops over input + output + kernel bytes) is above the machine balance
    (matrix-core peak over 8 TB/s) is priced against the matrix-core peak of the instructions it contracts
    on (fp32: 157.3 TFLOP/s; bf16 variant: 2.5 PFLOP/s), else against HBM."""
    layers = [l for l in res.get("conv_layers") or [] if l["in_step"]]
    if not layers:
        return None
    top = max(layers, key=lambda r: r["ms"])
    flops = 2.0 * top["M"] * top["K"] * top["N"]
    name = f"{res['workload']}.{top['layer']}.{top['pass']}"
    peak = MFMA_BF16_PEAK_TFLOPS if res.get("storage_dtype") == "bf16" else MFMA_F32_PEAK_TFLOPS
    if flops / top["algorithmic_bytes"] >= peak * 1e3 / HBM_PEAK_GBS:
        ach = flops / (top["ms"] * 1e9)
        return {"kernel": name, "bound": "mfma", "achieved": ach, "peak": peak, "unit": "TFLOP/s",
                "frac": ach / peak, "traffic": measured_traffic(name), "ms": top["ms"], "flops": flops}
    ach = top["algorithmic_bytes"] / (top["ms"] * 1e6)
    return {"kernel": name, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": ach / HBM_PEAK_GBS, "traffic": measured_traffic(name), "ms": top["ms"],
            "bytes": top["algorithmic_bytes"]}


def hbm_kernels(stream):
    """Achieved GB/s of the bandwidth-bound kernels at the largest shapes of the workloads: the explicit
    unroll phi_c / phi_c^{-1} (cfg4 c2: 1.68 GB patch matrix; cfg5 c5: 3.7 GB), max pooling (cfg3 p1 at the
    workload's batch 128, and at batch 2048, which is NOT a workload of the benchmark: it only shows the
    kernel's bandwidth once the tensor is no longer launch-latency sized) and ReLU (cfg4 c1 output).
    Algorithmic bytes over the median of three timing loops."""
    import torch
    from paper_1501_07338_amd import vcnn
    out = []

    def timed(fn):
        ts = sorted(time_calls(fn, 10, stream) for _ in range(3))
        return ts[1]

    def rec(kernel, shape, nbytes, ms, note=None):
        r = {"kernel": kernel, "shape": shape, "algorithmic_bytes": nbytes, "ms": ms, "gbs": nbytes / (ms * 1e6),
             "frac_hbm_peak": nbytes / (ms * 1e6) / HBM_PEAK_GBS}
        if note:
            r["note"] = note
        out.append(r)

    for name, (n, c, h, w, k, r, s, ph, pw) in {"cfg4.c2": (64, 64, 64, 64, 32, 5, 5, 2, 2),
                                                 "cfg5.c5": (16, 512, 49, 49, 1, 8, 8, 0, 0)}.items():
        d = vcnn.conv_desc(n, c, h, w, k, r, s, ph, pw)
        oh, ow = vcnn.conv_out_shape(d)
        K, N = c * r * s, n * oh * ow
        x = torch.randn(n, c, h, w, device="cuda")
        col = torch.empty(K, N, device="cuda")
        dx = torch.empty_like(x)
        nbytes = 4.0 * (K * N + x.numel())
        rec("im2col", name, nbytes, timed(lambda: vcnn.im2col(d, x, col)))
        rec("col2im", name, nbytes, timed(lambda: vcnn.col2im(d, col, dx)))
        del x, col, dx
    for name, n, note in (("cfg3.p1", 128, None),
                          ("cfg3.p1 at batch 2048", 2048, "not a BASELINE config: the layer at 16x the workload's batch")):
        c, h, w = 32, 32, 32
        d = vcnn.pool_desc(n, c, h, w, 3, 3, 2, 2)
        oh, ow = vcnn.pool_out_shape(d)
        x = torch.randn(n, c, h, w, device="cuda")
        y = torch.empty(n, c, oh, ow, device="cuda")
        am = torch.empty(n, c, oh, ow, dtype=torch.int32, device="cuda")
        dy, dx = torch.randn_like(y), torch.empty_like(x)
        rec("pool_fwd", name, 4.0 * (x.numel() + 2 * y.numel()), timed(lambda: vcnn.pool_fwd(d, x, y, am)), note)
        rec("pool_bwd", name, 4.0 * (x.numel() + 2 * y.numel()), timed(lambda: vcnn.pool_bwd(d, dy, am, dx)), note)
        del x, y, am, dy, dx
    t = torch.randn(64, 64, 64, 64, device="cuda")  # cfg4 c1 output
    g, o = torch.randn_like(t), torch.empty_like(t)
    mark("relu_bwd on 3 x 67 MB")
    rec("relu_bwd", "cfg4.c1 output", 12.0 * t.numel(), timed(lambda: vcnn.act_bwd(vcnn.ACT_RELU, vcnn.F32, t.numel(), t, g, o)))
    mark("-")
    del t, g, o
    torch.cuda.empty_cache()
    return out


def fourier_comparison(stream):
    """Forward pass of the deconvolution network's two layers with one-dimensional kernels (121 x 1 and 1 x 121) on
    the unroll + matrix-core route and through the Fourier domain - the alternative the paper's related-work
    paragraph names.  A comparison only: the default route never takes the transform."""
    import torch
    from paper_1501_07338_amd import vcnn
    rows = []
    for name, (n, c, h, w, k, r, s) in {"cfg5.c1 (121x1, 1->38 maps)": (16, 1, 184, 184, 38, 121, 1),
                                        "cfg5.c2 (1x121, 38->38 maps)": (16, 38, 64, 184, 38, 1, 121)}.items():
        x = torch.rand(n, c, h, w, device="cuda")
        wt = torch.randn(k, c, r, s, device="cuda") * (2.0 / (c * r * s)) ** 0.5
        b = torch.zeros(k, device="cuda")
        d = vcnn.conv_desc(n, c, h, w, k, r, s)
        oh, ow = vcnn.conv_out_shape(d)
        y = torch.empty(n, k, oh, ow, device="cuda")
        row = {"layer": name, "gflop": 2.0 * k * c * r * s * n * oh * ow / 1e9}
        try:
            for key, algo in (("unroll_ms", vcnn.ALGO_AUTO), ("fourier_ms", vcnn.ALGO_FFT)):
                vcnn.set_conv_algo(algo)
                ws = torch.empty(max(256, vcnn.conv_workspace_bytes(d, vcnn.PASS_FWD)), dtype=torch.uint8, device="cuda")
                row[key] = sorted(time_calls(lambda: vcnn.conv_fwd(d, x, wt, b, y, ws), 10, stream) for _ in range(3))[1]
                del ws
        finally:
            vcnn.set_conv_algo(vcnn.ALGO_AUTO)
        rows.append(row)
    torch.cuda.empty_cache()
    return rows


def split_products_comparison(steps, warmup, default_res):
    """The same cfg5 training step with VCNN_ALGO_SPLIT: the float products of the forward pass and of the kernel
    gradient as sums of six bfloat16 products each (every float operand is exactly a sum of three bfloat16 terms; the
    three smallest term products lie below float rounding).  On request only - the headline is the float
    matrix-core path; this row shows what the chip's bfloat16 rate buys at float accuracy."""
    from paper_1501_07338_amd import vcnn
    # the large layer only (c3: 383 GFLOP per pass, contraction 9728): on the smaller layers six passes of the bf16
    # kernels cost more than one of the float kernel
    res = run_workload("cfg5", steps, warmup, layer_iters=5, algos={2: vcnn.ALGO_SPLIT}, phase_prefix="cfg5_split_products")
    passes = {(l["layer"], l["pass"]): l["ms"] for l in res["conv_layers"]}
    base = {(l["layer"], l["pass"]): l["ms"] for l in default_res["conv_layers"]}
    return {"what": "cfg5 step with VCNN_ALGO_SPLIT on the 16x16x512 layer (opt-in): its fp32 forward and kernel-gradient "
                    "products as six bf16 matrix-core products each, fp32 accumulate; everything else as in the headline",
            "ms_per_step": res["ms_per_step"], "images_per_s": res["images_per_s"], "launch": res["launch"],
            "loss_first_step": res["loss_first_step"],
            "loss_rel_diff_to_default": abs(res["loss_first_step"] - default_res["loss_first_step"]) / abs(default_res["loss_first_step"]),
            "conv_ms_split_vs_default": {f"{k[0]}.{k[1]}": [passes[k], base[k]] for k in passes
                                         if k in base and abs(passes[k] - base[k]) > 0.1 * base[k]}}


def aids(stream):
    """The benchmark's own yardsticks (outside the layer library): the matrix-core rate with register operands
    only - what the chip sustains under MFMA load, beside the data-sheet peaks the roofline fractions are quoted
    against - and a plain streaming copy of 1 GiB, the kernel of known size that the HBM traffic counters of a
    profiler run are scaled by."""
    import torch
    from paper_1501_07338_amd import benchaid
    blocks, out = 512, {}
    sink = torch.empty(blocks * 256, device="cuda")
    for name, bf16, iters, peak in (("f32", False, 20000, MFMA_F32_PEAK_TFLOPS), ("bf16", True, 40000, MFMA_BF16_PEAK_TFLOPS)):
        flop = benchaid.mfma(bf16, blocks, iters, sink)
        ms = sorted(time_calls(lambda: benchaid.mfma(bf16, blocks, iters, sink), 3, stream) for _ in range(3))[1]
        out["mfma_" + name] = {"sustained_tflops": flop / (ms * 1e9), "data_sheet_tflops": peak, "ms": ms}
        # the same loop with operands whose bits change from instruction to instruction, as a layer's do: the
        # clock the chip holds depends on the power the matrix cores draw
        ms = sorted(time_calls(lambda: benchaid.mfma(bf16, blocks, iters, sink, toggle=True), 3, stream) for _ in range(3))[1]
        out["mfma_" + name]["sustained_tflops_changing_operands"] = flop / (ms * 1e9)
    # the matrix-core loop of a 128 x 128 fp32 tile fed from LDS as the layer kernels feed it, three blocks per compute
    # unit: alone, and with the fetch of new operand words from the L2 into LDS between the barriers
    words = torch.empty(8 << 20 >> 2, device="cuda").normal_()  # 8 MB
    sink3 = torch.empty(768 * 256, device="cuda")
    for key, staged in (("lds_fed_tflops", False), ("lds_fed_with_staging_tflops", True)):
        flop = benchaid.mfma_lds(staged, 768, 4000, sink3, words)
        ms = sorted(time_calls(lambda: benchaid.mfma_lds(staged, 768, 4000, sink3, words), 3, stream) for _ in range(3))[1]
        out["mfma_f32"][key] = flop / (ms * 1e9)
    del words, sink3
    src = torch.empty(1 << 28, device="cuda").normal_()
    dst = torch.empty_like(src)
    mark("copy of 1 GiB")
    ms = sorted(time_calls(lambda: benchaid.copy(src, dst), 5, stream) for _ in range(3))[1]
    mark("-")
    out["copy_1GiB"] = {"bytes_moved": 2.0 * src.numel() * 4, "ms": ms, "gbs": 2.0 * src.numel() * 4 / (ms * 1e6)}
    del src, dst, sink
    torch.cuda.empty_cache()
    return out


def batch_sweep(stream, steps=50):
    """Training and forward-only images/s of the two recognition networks over the mini-batch sizes of the
    paper's batch experiments (Tables 3 and 4: 1, 100, 200, 300, 400).  These softmax networks stay finite
    under repeated updates (checked), so their steps run back to back."""
    import torch
    from paper_1501_07338_amd import workloads as wl
    from paper_1501_07338_amd.net import TrainStep
    rows = []
    for name in ("cfg2", "cfg3"):
        for b in (1, 100, 200, 300, 400):
            net = wl.make_net(name, b)
            ts = TrainStep(net, wl.make_params(net), wl.make_inputs(net), device="cuda:0")
            ts.snapshot()
            for _ in range(5):
                ts.step()
            graph = ts.capture()
            for _ in range(5):
                graph.replay()
            train_ms = timed_steps(graph.replay, steps, stream, before=ts.restore)[0]
            finite_or_die(f"{name} batch {b}", float(ts.loss.item()))
            fwd_ms = timed_steps(ts.forward, steps, stream)[0]
            rows.append({"workload": name, "batch": b, "train_ms_per_step": train_ms, "train_images_per_s": b / (train_ms * 1e-3),
                         "forward_ms": fwd_ms, "forward_images_per_s": b / (fwd_ms * 1e-3)})
            del ts, graph
    torch.cuda.empty_cache()
    return rows


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(name, budget_s=30.0):
    """The fp64 oracle, as it stands, timed on this host's cores on a bounded sample of the same workload: whole
    training steps of the network at a mini-batch small enough for about 10-30 s of CPU work (cfg5: one sample of
    the 16, every layer at its full spatial size; the oracle's loops are per sample, so images/s carries over)."""
    import oracle
    from oracle.net import train_step
    from paper_1501_07338_amd import workloads as wl
    base = name[:-5] if name.endswith("_bf16") else name
    full = wl.make_net(base)
    batch = {"cfg5": 1, "cfg4": 8}.get(base, full.batch)
    net = wl.make_net(base, batch)
    inputs, params = wl.make_inputs(net), wl.make_params(net)
    times = []
    t_all = time.perf_counter()
    while not times or (time.perf_counter() - t_all < 0.5 * budget_s and len(times) < 15):
        t0 = time.perf_counter()
        train_step(net, inputs, params)
        times.append(time.perf_counter() - t0)
    med = statistics.median(times)
    return {"value": batch / med, "unit": "images/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"{len(times)} full training step(s) of {base} at batch {batch} of {full.batch} "
                      f"(all layers at full spatial size), median; fp64 nested loops",
            "s_per_step": med, "cpu_model": cpu_model()}


def summary(r):
    """The compact per-workload record of the JSON line."""
    out = {k: r[k] for k in ("batch", "storage_dtype", "ms_per_step", "images_per_s", "launch", "loss_first_step")}
    out["conv_tflops_fwd_bwd"] = None if r["conv_gflops_fwd_bwd"] is None else r["conv_gflops_fwd_bwd"] / 1e3
    out["conv_pct_mfma_peak"] = r["conv_pct_mfma_peak"]
    rf = r.get("roofline")
    if rf:
        out["roofline"] = {k: rf[k] for k in ("kernel", "bound", "achieved", "peak", "unit", "frac", "traffic")}
    return out


def rounded(o, digits=5):
    if isinstance(o, float):
        return float(f"{o:.{digits}g}")
    if isinstance(o, dict):
        return {k: rounded(v, digits) for k, v in o.items()}
    if isinstance(o, (list, tuple)):
        return [rounded(v, digits) for v in o]
    return o


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg5")
    ap.add_argument("--others", default="cfg5_bf16,cfg4,cfg3,cfg2,cfg1", help="comma list of further workloads to report ('' for none)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--no-sweep", action="store_true", help="skip the mini-batch sweep of cfg2 / cfg3")
    ap.add_argument("--no-hbm", action="store_true", help="skip the bandwidth-bound kernels and the benchmark's yardsticks")
    ap.add_argument("--markers", action="store_true", help="number the per-layer timing phases with empty marker kernels "
                    "(for rocprofv3 traces; the map goes to the detail file)")
    ap.add_argument("--detail", default=str(ROOT / "gpurun_out" / "bench_detail.json"), help="where the long tables go")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the layer path is single-GPU); use --gpus 1")

    import torch
    from paper_1501_07338_amd import vcnn
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    vcnn.lib()  # raises if the HIP library has not been built: there is no fallback path

    mark.enabled = args.markers
    main_res = run_workload(args.workload, args.steps, args.warmup)
    others = {}
    for name in [s for s in args.others.split(",") if s and s != args.workload]:
        small = name in ("cfg1", "cfg2", "cfg3")
        others[name] = run_workload(name, max(args.steps, 100) if small else args.steps, args.warmup,
                                    layer_iters=10 if small else 5)

    detail = {"main": main_res, "other_workloads": others, "markers": MARKERS}
    stream = torch.cuda.current_stream()
    if not args.no_hbm:
        detail["hbm_kernels"] = hbm_kernels(stream)
        detail["yardsticks"] = aids(stream)
        detail["fourier_comparison"] = fourier_comparison(stream)
        if args.workload == "cfg5":
            detail["split_products"] = split_products_comparison(args.steps, args.warmup, main_res)
    if not args.no_sweep:
        detail["batch_sweep"] = batch_sweep(stream)

    base = args.workload[:-5] if args.workload.endswith("_bf16") else args.workload
    out = {
        "metric": METRIC,
        "value": main_res["images_per_s"], "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": main_res["storage_dtype"], "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT.get(base, base) + (" [bf16 storage, fp32 accumulation]" if base != args.workload else ""),
                   "launch": LAUNCH_TEXT[main_res["launch"]], "ms_per_step_by_launch": main_res["ms_per_step_by_launch"],
                   "ms_per_step_median": main_res["ms_per_step_median"],
                   "timing": "each step between its own event pair on the launch stream, mean of the K steps; the seeded "
                             "parameters are restored before every step outside the pair",
                   "loss_first_step": main_res["loss_first_step"]},
        "conv_gflops_fwd_bwd": main_res["conv_gflops_fwd_bwd"],
        "conv_pct_mfma_peak": main_res["conv_pct_mfma_peak"],
        "roofline": {k: main_res["roofline"][k] for k in ("kernel", "bound", "achieved", "peak", "unit", "frac", "traffic")},
        # [layer, pass, ms, TFLOP/s, % of the matrix-core peak]
        "conv_layers": [[l["layer"], l["pass"], l["ms"], l["gflops"] / 1e3, l["pct_mfma_peak"]] for l in main_res["conv_layers"]],
        "other_workloads": {k: summary(v) for k, v in others.items()},
    }
    if "hbm_kernels" in detail:
        out["hbm_kernels"] = [[h["kernel"], h["shape"], h["gbs"], h["frac_hbm_peak"]] for h in detail["hbm_kernels"]]
        out["yardsticks"] = {"mfma_f32_sustained_tflops": detail["yardsticks"]["mfma_f32"]["sustained_tflops"],
                             "mfma_bf16_sustained_tflops": detail["yardsticks"]["mfma_bf16"]["sustained_tflops"],
                             "mfma_f32_changing_operands_tflops": detail["yardsticks"]["mfma_f32"]["sustained_tflops_changing_operands"],
                             "mfma_f32_lds_fed_tflops": detail["yardsticks"]["mfma_f32"]["lds_fed_tflops"],
                             "mfma_f32_lds_fed_with_staging_tflops": detail["yardsticks"]["mfma_f32"]["lds_fed_with_staging_tflops"],
                             "mfma_bf16_changing_operands_tflops": detail["yardsticks"]["mfma_bf16"]["sustained_tflops_changing_operands"],
                             "copy_1GiB_gbs": detail["yardsticks"]["copy_1GiB"]["gbs"]}
        out["fourier_comparison"] = [[r["layer"], r["unroll_ms"], r["fourier_ms"]] for r in detail["fourier_comparison"]]
    if "split_products" in detail:
        out["split_products"] = detail["split_products"]
    if "batch_sweep" in detail:  # [workload, batch, training images/s, forward-only images/s]
        out["batch_sweep"] = [[r["workload"], r["batch"], r["train_images_per_s"], r["forward_images_per_s"]]
                              for r in detail["batch_sweep"]]
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(args.workload)
        detail["cpu_baseline"] = out["cpu_baseline"]
    try:
        os.makedirs(os.path.dirname(args.detail), exist_ok=True)
        with open(args.detail, "w") as f:
            json.dump(detail, f, allow_nan=False, indent=1)
        out["detail_file"] = os.path.relpath(args.detail, ROOT)
    except (OSError, ValueError) as e:
        out["detail_file"] = f"not written: {e}"
    print(json.dumps(rounded(out), allow_nan=False))


if __name__ == "__main__":
    main()
