#!/usr/bin/env python3
"""Benchmark of the vectorized CNN layer path on one MI355X.

A "step" is one full training step (forward, cost, backward, SGD update) of a synthetic network whose
inputs and weights are already resident in HBM; every arithmetic step runs in libvcnn's HIP kernels.
The headline line reports images/s on the small recognition CNN (workload cfg2: every operator of
the path - unrolled convolutions, ReLU, max pooling, fully connected layers, softmax cost - is in
it).  The step is timed three ways - issued eagerly (one C call per layer pass) on one stream, eagerly with the
parameter gradients on a second stream, and replayed from a HIP graph recorded once - and the fastest is the
figure, the others riding along (`config.launch` says which was used).  Per-layer GFLOP/s of every convolution pass, the roofline figure of the dominant call,
the other four workloads and the CPU-oracle baseline ride along in the same JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2] [--others cfg1,cfg3,cfg4,cfg5]
"""
from __future__ import annotations

import argparse
import json
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

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
            "valid, L2 loss, full training step",
}


def conv_geom(net, li):
    from paper_1501_07338_amd.workloads import Conv
    L = net.layers[li]
    assert isinstance(L, Conv)
    n, c, h, w = net.in_shape(li)
    _, k, oh, ow = net.shapes[li]
    return dict(n=n, c=c, h=h, w=w, k=k, r=L.kh, s=L.kw, oh=oh, ow=ow, M=k, K=c * L.kh * L.kw, N=n * oh * ow)


def time_calls(fn, iters, stream):
    """Average duration in ms of `fn` over `iters` back-to-back enqueues, measured with events on
    the stream the kernels are launched on."""
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


def timed_steps(fn, steps, stream):
    """Wall-clock and GPU-event time per step of `steps` calls of fn, synchronised on both sides."""
    import torch
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(steps):
        fn()
    ev1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    return max(wall_ms, ev0.elapsed_time(ev1) / steps)


def run_workload(name, steps, warmup, layer_iters=10):
    """`name` is a workload, optionally suffixed `_bf16` for the bfloat16-storage variant."""
    import torch
    from paper_1501_07338_amd import vcnn, workloads as wl
    from paper_1501_07338_amd.net import TrainStep

    bf16 = name.endswith("_bf16")
    net = wl.make_net(name[:-5] if bf16 else name)
    inputs, params = wl.make_inputs(net), wl.make_params(net)
    ts = TrainStep(net, params, inputs, device="cuda:0", first_layer_dx=False, dtype=vcnn.BF16 if bf16 else vcnn.F32)
    esize = 2.0 if bf16 else 4.0
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        ts.step()
    eager_ms = timed_steps(ts.step, steps, stream)
    side, ts.side = ts.side, None  # the same step with every kernel on one stream (no fork / join events)
    for _ in range(warmup):
        ts.step()
    single_ms = timed_steps(ts.step, steps, stream)
    ts.side = side
    graph = ts.capture()
    for _ in range(warmup):
        graph.replay()
    graph_ms = timed_steps(graph.replay, steps, stream)
    # The same step, issued three ways; the fastest is the workload's figure.  On the small networks every kernel
    # is a few microseconds, the fork / join between the two streams costs more than the overlap returns and a
    # plain in-order launch wins; on the large ones the parameter-gradient strand on a second stream pays, eagerly
    # or as a replayed graph.
    modes = {"one HIP-graph replay per step (parameter gradients on a second branch)": graph_ms,
             "eager: one C call per layer pass, parameter gradients on a second stream": eager_ms,
             "eager: one C call per layer pass, one stream": single_ms}
    launch = min(modes, key=modes.get)
    best_ms = modes[launch]
    res = {"workload": name, "batch": net.batch, "storage_dtype": "bf16" if bf16 else "f32", "ms_per_step": best_ms,
           "launch": launch,
           "ms_per_step_graph": graph_ms, "ms_per_step_eager": eager_ms, "ms_per_step_eager_one_stream": single_ms,
           "images_per_s": net.batch / (best_ms * 1e-3), "images_per_s_graph": net.batch / (graph_ms * 1e-3),
           "images_per_s_eager": net.batch / (eager_ms * 1e-3),
           "images_per_s_eager_one_stream": net.batch / (single_ms * 1e-3),
           "loss_after_timed_steps": float(ts.loss.item())}

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
        passes = {
            "fwd": lambda: vcnn.conv_fwd(d, a_in, w, b, a_out, ts.workspace),
            "bwd_filter": lambda: vcnn.conv_bwd_filter(d, a_in, dy, dw, db, ts.workspace_side),
            "bwd_data": lambda: vcnn.conv_bwd_data(d, w, dy, ts.dacts[li], ts.workspace),
        }
        in_b = esize * g["n"] * g["c"] * g["h"] * g["w"]
        out_b = esize * g["M"] * g["N"]
        w_b = esize * g["M"] * g["K"]
        for pname, fn in passes.items():
            t = time_calls(fn, layer_iters, stream)
            layers.append({"layer": f"conv{li}", "pass": pname, "M": g["M"], "K": g["K"], "N": g["N"], "ms": t,
                           "gflops": flops / (t * 1e6),
                           "pct_mfma_f32_peak": 100.0 * flops / (t * 1e9) / MFMA_F32_PEAK_TFLOPS,
                           # the bf16 variant contracts on the bf16 matrix-core instructions: price it against their peak
                           "pct_mfma_peak": 100.0 * flops / (t * 1e9) / (MFMA_BF16_PEAK_TFLOPS if bf16 else MFMA_F32_PEAK_TFLOPS),
                           "algorithmic_bytes": in_b + out_b + w_b, "gbs": (in_b + out_b + w_b) / (t * 1e6),
                           "in_step": not (li == 0 and pname == "bwd_data")})
            if not (li == 0 and pname == "bwd_data"):
                conv_flops += flops
                conv_ms += t
    res["conv_layers"] = layers
    res["conv_gflops_fwd_bwd"] = conv_flops / (conv_ms * 1e6) if conv_ms else None
    res["conv_pct_mfma_f32_peak"] = 100.0 * res["conv_gflops_fwd_bwd"] / (MFMA_F32_PEAK_TFLOPS * 1e3) if conv_ms else None
    res["roofline"] = dominant_roofline(res)
    return res


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
                "frac": ach / peak, "traffic": MEASURED_TRAFFIC.get(name)}
    ach = top["algorithmic_bytes"] / (top["ms"] * 1e6)
    return {"kernel": name, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": ach / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC.get(name)}


def hbm_kernels(stream):
    """Achieved GB/s of the bandwidth-bound kernels at the largest shapes of the workloads: the explicit
    unroll phi_c / phi_c^{-1} (cfg4 c2: 1.68 GB patch matrix; cfg5 c5: 3.7 GB), max pooling (cfg3 p1)
    and ReLU (cfg4 c1 output).  Algorithmic bytes over the median of three timing loops."""
    import torch
    from paper_1501_07338_amd import vcnn
    out = []

    def timed(fn):
        ts = sorted(time_calls(fn, 10, stream) for _ in range(3))
        return ts[1]

    def rec(kernel, shape, nbytes, ms):
        out.append({"kernel": kernel, "shape": shape, "algorithmic_bytes": nbytes, "ms": ms, "gbs": nbytes / (ms * 1e6),
                    "frac_hbm_peak": nbytes / (ms * 1e6) / HBM_PEAK_GBS})

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
    # cfg3 p1 (3x3 stride 2, 24 MB: launch-latency sized) and the same layer at 16x the batch, where the
    # tensor is large enough for the bandwidth to show
    for name, n in {"cfg3.p1": 128, "cfg3.p1 at batch 2048": 2048}.items():
        c, h, w = 32, 32, 32
        d = vcnn.pool_desc(n, c, h, w, 3, 3, 2, 2)
        oh, ow = vcnn.pool_out_shape(d)
        x = torch.randn(n, c, h, w, device="cuda")
        y = torch.empty(n, c, oh, ow, device="cuda")
        am = torch.empty(n, c, oh, ow, dtype=torch.int32, device="cuda")
        dy, dx = torch.randn_like(y), torch.empty_like(x)
        rec("pool_fwd", name, 4.0 * (x.numel() + 2 * y.numel()), timed(lambda: vcnn.pool_fwd(d, x, y, am)))
        rec("pool_bwd", name, 4.0 * (x.numel() + 2 * y.numel()), timed(lambda: vcnn.pool_bwd(d, dy, am, dx)))
        del x, y, am, dy, dx
    t = torch.randn(64, 64, 64, 64, device="cuda")  # cfg4 c1 output
    g, o = torch.randn_like(t), torch.empty_like(t)
    rec("relu_bwd", "cfg4.c1 output", 12.0 * t.numel(), timed(lambda: vcnn.act_bwd(vcnn.ACT_RELU, vcnn.F32, t.numel(), t, g, o)))
    torch.cuda.empty_cache()
    return out


def mfma_sustained(stream):
    """Matrix-core rate with register operands only (no memory traffic): what the chip sustains under MFMA
    load, reported beside the data-sheet peaks the roofline fractions are quoted against."""
    import torch
    from paper_1501_07338_amd import vcnn
    blocks, out = 512, {}
    sink = torch.empty(blocks * 256, device="cuda")
    for name, dtype, iters, peak in (("f32", vcnn.F32, 20000, MFMA_F32_PEAK_TFLOPS), ("bf16", vcnn.BF16, 40000, 2500.0)):
        flop = vcnn.probe_mfma(dtype, blocks, iters, sink)
        ms = sorted(time_calls(lambda: vcnn.probe_mfma(dtype, blocks, iters, sink), 3, stream) for _ in range(3))[1]
        out[name] = {"sustained_tflops": flop / (ms * 1e9), "data_sheet_tflops": peak, "ms": ms}
    return out


def batch_sweep(stream, steps=50):
    """Training and forward-only images/s of the two recognition networks over the mini-batch sizes of the
    paper's batch experiments (Tables 3 and 4: 1, 100, 200, 300, 400)."""
    import torch
    from paper_1501_07338_amd import workloads as wl
    from paper_1501_07338_amd.net import TrainStep
    rows = []
    for name in ("cfg2", "cfg3"):
        for b in (1, 100, 200, 300, 400):
            net = wl.make_net(name, b)
            ts = TrainStep(net, wl.make_params(net), wl.make_inputs(net), device="cuda:0")
            for _ in range(5):
                ts.step()
            graph = ts.capture()
            for _ in range(5):
                graph.replay()
            train_ms = timed_steps(graph.replay, steps, stream)
            fwd_ms = timed_steps(ts.forward, steps, stream)
            rows.append({"workload": name, "batch": b, "train_ms_per_step": train_ms, "train_images_per_s": b / (train_ms * 1e-3),
                         "forward_ms": fwd_ms, "forward_images_per_s": b / (fwd_ms * 1e-3)})
            del ts, graph
    torch.cuda.empty_cache()
    return rows


# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (see profiles/); filled in
# from the committed summaries, None where no counter run covers the kernel.
MEASURED_TRAFFIC: dict = {
    # (2 x FETCH_SIZE + WRITE_SIZE) x 1024 of the call's main kernel, profiles/cfg5_cfg4_cfg2_hbm_traffic_pmc.txt
    "cfg2.conv2.fwd": 7.2e6,         # conv_small_kernel: 2699 KiB fetched (x2), 1600 KiB written
    "cfg2.conv2.bwd_filter": 19.6e6,   # conv_halo_filter_kernel<64, 256, ...> on 256 blocks: 2494 KiB fetched (x2),
                                       # 14146 KiB of partial products written (then added by sum_slices_split)
    "cfg2.conv2.bwd_data": 4.1e6,      # conv_small_bwd_kernel<2, 3>: 1294 KiB fetched (x2), 1440 KiB written (the
                                       # patch-matrix gradient stays on chip)
    "cfg5.conv2.fwd": 356.1e6,       # conv_halo_kernel<128, 128, ...>
    "cfg5.conv2.bwd_filter": 479.9e6,  # conv_halo_filter_kernel<128, 128, ...> (without the slice sum)
    "cfg5.conv2.bwd_data": 7937.3e6,   # gemm_f32_kernel<128, 128, 16, ...> of the explicit route (without col2im)
    "cfg5_bf16.conv2.fwd": 199.9e6,    # conv_halo_bf16_kernel<4, 1, 2, 5> (without the two re-layout passes)
    "cfg5_bf16.conv2.bwd_filter": 425.8e6,  # filter_grad_bf16_kernel<4, 1, 2, 4>
    "cfg5_bf16.conv2.bwd_data": 635.2e6,    # conv_halo_bf16_kernel<1, 4, 3, 8, true>: the kernel matrix is re-fetched past L2
}


def cpu_baseline(name, budget_s=20.0):
    """The fp64 oracle, as it stands, timed on this host's cores on the same workload."""
    import oracle
    from oracle.net import train_step
    from paper_1501_07338_amd import workloads as wl
    net = wl.make_net(name)
    inputs, params = wl.make_inputs(net), wl.make_params(net)
    train_step(net, inputs, params)  # warm-up (loads the library, touches memory)
    times = []
    t_all = time.perf_counter()
    while len(times) < 3 or (time.perf_counter() - t_all < 0.5 * budget_s and len(times) < 15):
        t0 = time.perf_counter()
        train_step(net, inputs, params)
        times.append(time.perf_counter() - t0)
        if time.perf_counter() - t_all > budget_s:
            break
    times.sort()
    med = times[len(times) // 2]
    return {"value": net.batch / med, "unit": "images/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"{len(times)} full training steps of {name} (batch {net.batch}), median", "s_per_step": med}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--others", default="cfg1,cfg3,cfg4,cfg5,cfg5_bf16", help="comma list of further workloads to report ('' for none)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--no-sweep", action="store_true", help="skip the mini-batch sweep of cfg2 / cfg3")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the layer path is single-GPU); use --gpus 1")

    import torch
    from paper_1501_07338_amd import vcnn
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    vcnn.lib()  # raises if the HIP library has not been built: there is no fallback path

    main_res = run_workload(args.workload, args.steps, args.warmup)
    others = {}
    for name in [s for s in args.others.split(",") if s and s != args.workload]:
        big = name.startswith(("cfg4", "cfg5"))
        others[name] = run_workload(name, max(3, min(args.steps, 20)) if big else args.steps,
                                    max(2, min(args.warmup, 3)) if big else args.warmup, layer_iters=5 if big else 10)
        torch.cuda.empty_cache()

    out = {
        "metric": "images/sec per training step (conv fwd+bwd GFLOP/s and % of fp32 MFMA peak alongside)",
        "value": main_res["images_per_s"], "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT.get(args.workload, args.workload), "launch": main_res["launch"],
                   "graph_ms_per_step": main_res["ms_per_step_graph"], "eager_ms_per_step": main_res["ms_per_step_eager"],
                   "eager_one_stream_ms_per_step": main_res["ms_per_step_eager_one_stream"]},
        "conv_gflops_fwd_bwd": main_res.get("conv_gflops_fwd_bwd"),
        "conv_pct_mfma_f32_peak": main_res.get("conv_pct_mfma_f32_peak"),
        "roofline": main_res["roofline"],
        "conv_layers": main_res.get("conv_layers"),
        "hbm_kernels": hbm_kernels(torch.cuda.current_stream()),
        "mfma_sustained": mfma_sustained(torch.cuda.current_stream()),
        "other_workloads": others,
    }
    if not args.no_sweep:
        out["batch_sweep"] = batch_sweep(torch.cuda.current_stream())
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(args.workload)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
