"""Sequences the C-ABI layer calls into one training step of a layer chain (forward, cost, backward,
SGD) on one GPU.  This module only owns buffers (torch device tensors), streams and call order; every
arithmetic step runs inside libvcnn's kernels.

The backward pass has two independent strands per layer: the input gradient, which the next layer
down waits for, and the parameter gradients, which only the update at the end of the step needs.
With `overlap=True` the parameter gradients are issued on a second stream (own workspace), forked
after each layer's pre-activation gradient is ready and joined before the update, so the small layers'
launch-bound kernels run side by side.  Captured into a HIP graph the fork/join become graph edges.
"""
from __future__ import annotations

from typing import List, Optional

import numpy as np
import torch

from . import vcnn
from .workloads import FC, Conv, Net, Pool


class TrainStep:
    """Device-resident state of one network: parameters, activations, gradients, workspace."""

    def __init__(self, net: Net, params: list, inputs: dict, device: str = "cuda:0", first_layer_dx: bool = False,
                 dtype: int = vcnn.F32, overlap: bool = True, algos: Optional[dict] = None, fold_conv_act: bool = True):
        """algos: {layer index: vcnn.ALGO_*} - convolutions named there are planned and launched under that route
        choice, the others under the process-wide one.  fold_conv_act=False: convolutions store their plain input
        gradient and the ReLU derivative of the layer below is a pass of its own (for comparisons)."""
        self.net, self.dev, self.dtype = net, torch.device(device), dtype
        self.fold_conv_act = fold_conv_act
        self.algos = dict(algos or {})
        self.first_layer_dx = first_layer_dx
        self.side = torch.cuda.Stream(self.dev) if overlap else None  # default priority
        f32 = dict(dtype=torch.float32, device=self.dev)
        # element type of activations and their gradients; parameters, their gradients and the loss stay fp32
        act = dict(dtype=torch.bfloat16 if dtype == vcnn.BF16 else torch.float32, device=self.dev)
        self.x = torch.from_numpy(np.ascontiguousarray(inputs["x"])).to(self.dev)
        if dtype == vcnn.BF16:  # a storage-format change of the given input, done by the library's own kernel
            x16 = torch.empty(self.x.shape, **act)
            vcnn.f32_to_bf16(self.x.numel(), self.x, x16)
            self.x = x16
        self.labels = torch.from_numpy(inputs["labels"]).to(self.dev) if "labels" in inputs else None
        self.target = torch.from_numpy(inputs["target"]).to(self.dev) if "target" in inputs else None
        self.upstream = torch.from_numpy(inputs["upstream"]).to(self.dev) if "upstream" in inputs else None
        self.params: List[Optional[tuple]] = [
            None if p is None else (torch.from_numpy(p[0]).to(self.dev), torch.from_numpy(p[1]).to(self.dev))
            for p in params]
        self.grads = [None if p is None else (torch.empty_like(p[0]), torch.empty_like(p[1])) for p in self.params]
        # bf16 variant: fp32 master weights plus a bf16 copy refreshed after every update
        self.params16 = [None if p is None or dtype != vcnn.BF16 else torch.empty(p[0].shape, **act) for p in self.params]
        self.acts = [self.x] + [torch.empty(s, **act) for s in net.shapes]
        self.dacts = [torch.empty_like(a) for a in self.acts]
        self.argmax = {li: torch.empty(net.shapes[li], dtype=torch.int32, device=self.dev)
                       for li, L in enumerate(net.layers) if isinstance(L, Pool)}
        self.loss = torch.zeros((), **f32)
        self.descs = {}
        ws_bytes, ws_side_bytes = 0, 0
        self.dpre, self.forked = {}, {}
        for li, L in enumerate(net.layers):
            ishape = net.in_shape(li)
            if isinstance(L, Conv):
                d = vcnn.conv_desc(ishape[0], ishape[1], ishape[2], ishape[3], L.cout, L.kh, L.kw, L.pad_h, L.pad_w,
                                   dtype=dtype, act=vcnn.ACT_RELU if L.relu else vcnn.ACT_NONE)
                self.descs[li] = d
                # (a first layer's filter gradient has no input gradient to overlap with and runs on the main stream)
                need = self._routed(li, lambda: [vcnn.conv_workspace_bytes(d, p)
                                                 for p in (vcnn.PASS_FWD, vcnn.PASS_BWD_DATA, vcnn.PASS_BWD_FILTER)])
                ws_bytes = max(ws_bytes, *need)
                ws_side_bytes = max(ws_side_bytes, need[2])
            elif isinstance(L, Pool):
                self.descs[li] = vcnn.pool_desc(ishape[0], ishape[1], ishape[2], ishape[3], L.win, L.win, L.stride,
                                                L.stride, dtype=dtype)
            if getattr(L, "relu", False):  # gradient w.r.t. the pre-activation, read by both strands
                self.dpre[li] = torch.empty(net.shapes[li], **act)
            if isinstance(L, (Conv, FC)):
                self.forked[li] = torch.cuda.Event()
        self.workspace = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=self.dev)
        self.workspace_side = torch.empty(max(ws_side_bytes, 256), dtype=torch.uint8, device=self.dev)
        if dtype == vcnn.BF16 and net.loss == "softmax":  # the cost works on float logits
            self.logits32 = torch.empty(net.out_shape, **f32)
            self.dlogits32 = torch.empty(net.out_shape, **f32)
        self.refresh_weights()

    def weights(self, li):
        """The weight tensor the layer kernels read: the fp32 parameters, or their bf16 copy."""
        return self.params16[li] if self.dtype == vcnn.BF16 else self.params[li][0]

    def refresh_weights(self, stream=None):
        if self.dtype == vcnn.BF16:
            for p, p16 in zip(self.params, self.params16):
                if p is not None:
                    vcnn.f32_to_bf16(p[0].numel(), p[0], p16, stream)

    def snapshot(self):
        """Keeps a device copy of the current parameters for restore()."""
        self._saved = [None if p is None else (p[0].clone(), p[1].clone()) for p in self.params]

    def restore(self, stream=None):
        """Puts the parameters of the last snapshot() back (device-to-device copies, no arithmetic) and refreshes the
        bf16 working copies, so that the next step starts from the same state again."""
        for p, q in zip(self.params, self._saved):
            if p is not None:
                p[0].copy_(q[0], non_blocking=True)
                p[1].copy_(q[1], non_blocking=True)
        self.refresh_weights(stream)

    def folds(self, li):
        """True if layer li's input gradient is stored with the ReLU derivative of layer li-1 folded in,
        i.e. it is written to dpre[li-1] (w.r.t. that layer's pre-activation) and dacts[li] stays unused."""
        L = self.net.layers[li]
        kinds = (Pool, FC, Conv) if self.fold_conv_act else (Pool, FC)
        return li > 0 and getattr(self.net.layers[li - 1], "relu", False) and isinstance(L, kinds)

    def _routed(self, li, call):
        """call() under the route choice given for layer li (the process-wide choice is put back afterwards)."""
        algo = self.algos.get(li)
        if algo is None:
            return call()
        before = vcnn.conv_algo()
        vcnn.set_conv_algo(algo)
        try:
            return call()
        finally:
            vcnn.set_conv_algo(before)

    # ---- one pass each ---------------------------------------------------------------------------
    def forward(self, stream=None):
        net = self.net
        for li, L in enumerate(net.layers):
            a_in, a_out = self.acts[li], self.acts[li + 1]
            if isinstance(L, Conv):
                w, b = self.weights(li), self.params[li][1]
                self._routed(li, lambda: vcnn.conv_fwd(self.descs[li], a_in, w, b, a_out, self.workspace, stream))
            elif isinstance(L, Pool):
                vcnn.pool_fwd(self.descs[li], a_in, a_out, self.argmax[li], stream)
            else:
                w, b = self.weights(li), self.params[li][1]
                bsz = a_in.shape[0]
                vcnn.fc_fwd(self.dtype, bsz, a_in.numel() // bsz, L.out, vcnn.ACT_RELU if L.relu else vcnn.ACT_NONE,
                            a_in, w, b, a_out, stream)

    def cost(self, stream=None):
        net, out, dout = self.net, self.acts[-1], self.dacts[-1]
        if net.loss == "softmax" and self.dtype == vcnn.BF16:
            vcnn.bf16_to_f32(out.numel(), out, self.logits32, stream)
            vcnn.softmax_loss(out.shape[0], out.shape[1], self.logits32, self.labels, self.loss, self.dlogits32, stream)
            vcnn.f32_to_bf16(out.numel(), self.dlogits32, dout, stream)
        elif net.loss == "softmax":
            vcnn.softmax_loss(out.shape[0], out.shape[1], out, self.labels, self.loss, dout, stream)
        elif net.loss == "l2":
            vcnn.l2_loss(self.dtype, out.numel(), out.shape[0], out, self.target, self.loss, dout, stream)
        elif net.loss == "upstream":
            if self.dtype == vcnn.BF16:
                vcnn.f32_to_bf16(dout.numel(), self.upstream, dout, stream)
            else:
                dout.copy_(self.upstream)  # a device-to-device copy of the given gradient, no arithmetic
        else:
            raise ValueError(net.loss)

    def backward(self, stream=None):
        net = self.net
        main = stream if stream is not None else torch.cuda.current_stream()
        side = self.side if self.side is not None else main
        folded = False  # the layer above already applied this layer's ReLU derivative and wrote dpre[li]
        for li in range(len(net.layers) - 1, -1, -1):
            L = net.layers[li]
            a_in, a_out, d = self.acts[li], self.acts[li + 1], self.dacts[li + 1]
            need_dx = li > 0 or self.first_layer_dx
            if getattr(L, "relu", False):
                if not folded:
                    vcnn.act_bwd(vcnn.ACT_RELU, self.dtype, d.numel(), a_out, d, self.dpre[li], main)
                d = self.dpre[li]
            # every layer folds the ReLU derivative of the layer below into its input-gradient store: it lands in
            # that layer's dpre directly
            folded = self.folds(li)
            dx_out = self.dpre[li - 1] if folded else self.dacts[li]
            act_below = vcnn.ACT_RELU if folded else vcnn.ACT_NONE
            if isinstance(L, Pool):
                if need_dx:
                    vcnn.pool_bwd_act(self.descs[li], act_below, a_in, d, self.argmax[li], dx_out, main)
                continue
            w = self.weights(li)
            dw, db = self.grads[li]
            if isinstance(L, FC):  # one call: at these sizes both products and the bias gradient share a launch
                bsz = a_in.shape[0]
                vcnn.fc_bwd_act(self.dtype, bsz, a_in.numel() // bsz, L.out, act_below, a_in, w, d, dw, db,
                                dx_out if need_dx else None, main)
                continue
            if not need_dx:  # nothing to overlap with
                self._routed(li, lambda: vcnn.conv_bwd_filter(self.descs[li], a_in, d, dw, db, self.workspace, main))
                continue
            if side is not main:  # fork: the parameter-gradient strand starts once d is complete
                self.forked[li].record(main)
                side.wait_event(self.forked[li])
            # the input gradient first: the chain below waits for it, and a kernel-gradient block that is already
            # resident can leave no LDS for it
            self._routed(li, lambda: vcnn.conv_bwd_data_act(self.descs[li], act_below, a_in if folded else None, w, d,
                                                            dx_out, self.workspace, main))
            self._routed(li, lambda: vcnn.conv_bwd_filter(self.descs[li], a_in, d, dw, db, self.workspace_side, side))
        if side is not main:  # join before anything reads the parameter gradients
            main.wait_stream(side)

    def update(self, stream=None):
        ws = [t for p in self.params if p is not None for t in p]
        gs = [t for g in self.grads if g is not None for t in g]
        w16 = None
        if self.dtype == vcnn.BF16:  # the weights' bf16 working copies are refreshed by the same launch
            w16 = [t for p, h in zip(self.params, self.params16) if p is not None for t in (h, None)]
        vcnn.sgd_update_multi(self.net.lr, ws, gs, w16, stream)

    def step(self, stream=None):
        self.forward(stream)
        self.cost(stream)
        self.backward(stream)
        self.update(stream)

    # ---- HIP graph ---------------------------------------------------------------------------------
    def capture(self):
        """Records one full step (forward, cost, backward, SGD) into a HIP graph and returns the
        graph; `graph.replay()` then re-issues the whole launch sequence with one call.  The step
        is run eagerly once first so that one-time kernel attribute set-up happens outside the capture."""
        self.step()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.step()
        return graph
