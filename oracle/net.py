"""One training step of a layer chain in the fp64 oracle (test infrastructure only).

Takes a network description (a list of Conv / Pool / FC records with a loss kind), inputs and
weights, and applies the oracle's layer functions in order: forward, loss, backward, SGD.  All
intermediate tensors are kept so that each HIP layer can be checked in isolation on the oracle's
own input to that layer.

Two optional arguments concern the discrete decisions of the chain (which side of zero a ReLU input lies on,
which element of a pooling window is the maximum), which floating point takes and which a comparison of
whole chains must take alike on both sides:
  * `store`: a function applied to every activation as it is stored (e.g. rounding to the storage type of a
    reduced-precision variant), so that the decisions are taken on the values the layers above actually read;
    arithmetic inside each layer stays fp64.
  * `decisions`: {"argmax": {layer: int32 array}, "relu": {layer: bool array}} used by the backward pass in
    place of the chain's own.  A caller passes only alternatives it has checked to be ties within rounding of the
    oracle's own values; the forward tensors are never affected.
"""
from __future__ import annotations

import numpy as np

import oracle as O


def _kind(L) -> str:
    return type(L).__name__


def train_step(net, inputs: dict, params: list, store=None, decisions=None) -> dict:
    """Returns a dict with: acts (input of each layer, then the final output), argmax (per pool layer), loss,
    dacts (gradient w.r.t. each entry of acts), grads [(dw, db) | None], new_params [(w, b) | None]."""
    keep = (lambda a: a) if store is None else (lambda a: np.asarray(store(a), dtype=np.float64))
    decisions = decisions or {}
    acts = [np.asarray(inputs["x"], dtype=np.float64)]
    argmax = {}
    for li, L in enumerate(net.layers):
        a = acts[-1]
        if _kind(L) == "Conv":
            w, b = params[li]
            acts.append(keep(O.conv_fwd(a, w, b, pad=(L.pad_h, L.pad_w), relu=L.relu)))
        elif _kind(L) == "Pool":
            y, am = O.maxpool_fwd(a, (L.win, L.win), (L.stride, L.stride))
            argmax[li] = am
            acts.append(keep(y))
        elif _kind(L) == "FC":
            w, b = params[li]
            acts.append(keep(O.fc_fwd(a.reshape(a.shape[0], -1), w, b, relu=L.relu)))
        else:
            raise TypeError(L)

    out = acts[-1]
    if net.loss == "softmax":
        loss, dout = O.softmax_loss(out, inputs["labels"])
    elif net.loss == "l2":
        loss, dout = O.l2_loss(out, inputs["target"])
    elif net.loss == "upstream":
        loss, dout = float("nan"), np.asarray(inputs["upstream"], dtype=np.float64)
    else:
        raise ValueError(net.loss)

    def through_relu(li, a_out, d):
        mask = decisions.get("relu", {}).get(li)
        if mask is None:
            return O.relu_bwd(a_out, d)  # post-activation output is > 0 exactly where the pre-activation is
        return O.relu_bwd(np.asarray(mask, dtype=np.float64).reshape(d.shape), d)  # x > 0 <=> mask

    dacts = [None] * len(acts)
    dacts[-1] = dout
    grads = [None] * len(net.layers)
    for li in range(len(net.layers) - 1, -1, -1):
        L = net.layers[li]
        a_in, a_out, d = acts[li], acts[li + 1], dacts[li + 1]
        if _kind(L) == "Conv":
            w, _ = params[li]
            if L.relu:
                d = through_relu(li, a_out, d)
            dw, db = O.conv_bwd_filter(a_in, d, (L.kh, L.kw), pad=(L.pad_h, L.pad_w))
            grads[li] = (dw, db)
            dacts[li] = O.conv_bwd_data(w, d, a_in.shape[2:], pad=(L.pad_h, L.pad_w))
        elif _kind(L) == "Pool":
            dacts[li] = O.maxpool_bwd(d, decisions.get("argmax", {}).get(li, argmax[li]), a_in.shape[2:])
        elif _kind(L) == "FC":
            w, _ = params[li]
            if L.relu:
                d = through_relu(li, a_out, d)
            x2 = a_in.reshape(a_in.shape[0], -1)
            dw, db, dx = O.fc_bwd(x2, w, d)
            grads[li] = (dw, db)
            dacts[li] = dx.reshape(a_in.shape)

    new_params = [None if p is None else (O.sgd_update(p[0], g[0], net.lr), O.sgd_update(p[1], g[1], net.lr))
                  for p, g in zip(params, grads)]
    return {"acts": acts, "argmax": argmax, "loss": loss, "dacts": dacts, "grads": grads,
            "new_params": new_params}
