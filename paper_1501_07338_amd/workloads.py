"""Seeded synthetic workloads: network shapes and input/weight generators.

This module holds no arithmetic of the layer path itself; it only describes the five benchmark
networks and draws their inputs, labels, targets and initial weights from a counter-based generator
(numpy Philox), so that the CPU oracle and the HIP path can be fed the very same arrays.  Values
are drawn in fp64 and rounded once to fp32.

Seed convention: Philox key = 1000 * config index + tensor index (tensor 0 = input, 1 = labels /
target / upstream gradient, 10 + 2*l = weights of parametrised layer l, 11 + 2*l = its bias).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np


@dataclass(frozen=True)
class Conv:
    cout: int
    kh: int
    kw: int
    pad_h: int = 0
    pad_w: int = 0
    relu: bool = False


@dataclass(frozen=True)
class Pool:
    win: int
    stride: int


@dataclass(frozen=True)
class FC:
    out: int
    relu: bool = False


@dataclass
class Net:
    name: str
    index: int
    batch: int
    in_chw: Tuple[int, int, int]
    layers: list
    loss: str  # "softmax" | "l2" | "upstream"
    classes: int = 0
    bias_init: float = 0.0
    lr: float = 0.01
    shapes: List[Tuple[int, ...]] = field(default_factory=list)  # activation shape after each layer

    def __post_init__(self):
        c, h, w = self.in_chw
        cur: Tuple[int, ...] = (self.batch, c, h, w)
        self.shapes = []
        for L in self.layers:
            if isinstance(L, Conv):
                n, c, h, w = cur
                cur = (n, L.cout, h + 2 * L.pad_h - L.kh + 1, w + 2 * L.pad_w - L.kw + 1)
            elif isinstance(L, Pool):
                n, c, h, w = cur
                cur = (n, c, (h - L.win) // L.stride + 1, (w - L.win) // L.stride + 1)
            elif isinstance(L, FC):
                cur = (cur[0], L.out)
            self.shapes.append(cur)

    def in_shape(self, li: int) -> Tuple[int, ...]:
        return (self.batch,) + tuple(self.in_chw) if li == 0 else self.shapes[li - 1]

    @property
    def out_shape(self) -> Tuple[int, ...]:
        return self.shapes[-1]


def make_net(name: str, batch: Optional[int] = None) -> Net:
    """The five benchmark networks.  `batch` overrides the stated mini-batch size (used by parity
    tests that need a chain the CPU oracle finishes quickly)."""
    if name == "cfg1":  # single conv block with an upstream gradient
        return Net(name, 1, batch or 8, (1, 28, 28), [Conv(6, 5, 5, relu=True), Pool(2, 2)], "upstream",
                   bias_init=0.01)
    if name == "cfg2":  # small recognition CNN
        return Net(name, 2, batch or 128, (1, 28, 28),
                   [Conv(20, 5, 5, relu=True), Pool(2, 2), Conv(50, 5, 5, relu=True), Pool(2, 2),
                    FC(500, relu=True), FC(10)], "softmax", classes=10)
    if name == "cfg3":  # colour recognition CNN
        return Net(name, 3, batch or 128, (3, 32, 32),
                   [Conv(32, 5, 5, 2, 2, relu=True), Pool(3, 2), Conv(32, 5, 5, 2, 2, relu=True), Pool(3, 2),
                    Conv(64, 5, 5, 2, 2, relu=True), Pool(3, 2), FC(64), FC(10)], "softmax", classes=10)
    if name == "cfg4":  # denoising CNN, 'same' padding, L2 loss
        return Net(name, 4, batch or 64, (1, 64, 64),
                   [Conv(64, 9, 9, 4, 4, relu=True), Conv(32, 5, 5, 2, 2, relu=True), Conv(1, 5, 5, 2, 2)], "l2")
    if name == "cfg5":  # deconvolution CNN with large separable kernels, valid padding, L2 loss
        return Net(name, 5, batch or 16, (1, 184, 184),
                   [Conv(38, 121, 1), Conv(38, 1, 121, relu=True), Conv(512, 16, 16, relu=True),
                    Conv(512, 1, 1, relu=True), Conv(1, 8, 8)], "l2")
    raise ValueError(f"unknown workload {name!r}")


NET_NAMES = ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5")


def _rng(net_index: int, tensor: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=1000 * net_index + tensor))


def _f32(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a.astype(np.float32))


def _valid_filter(img: np.ndarray, ker: np.ndarray) -> np.ndarray:
    """Input synthesis only (blur / smoothing of the synthetic images): valid sliding-window sum of
    the last two axes of `img` with `ker`, in fp64."""
    kh, kw = ker.shape
    oh, ow = img.shape[-2] - kh + 1, img.shape[-1] - kw + 1
    out = np.zeros(img.shape[:-2] + (oh, ow))
    for i in range(kh):
        for j in range(kw):
            if ker[i, j] != 0.0:
                out += ker[i, j] * img[..., i:i + oh, j:j + ow]
    return out


def _motion_kernel(rng: np.random.Generator, size: int = 15, steps: int = 64) -> np.ndarray:
    """Random-walk motion-blur kernel: visit counts of a lattice walk from the centre, sum 1."""
    ker = np.zeros((size, size))
    i = j = size // 2
    ker[i, j] += 1.0
    moves = rng.integers(0, 4, size=steps)
    for m in moves:
        di, dj = ((-1, 0), (1, 0), (0, -1), (0, 1))[int(m)]
        i = min(max(i + di, 0), size - 1)
        j = min(max(j + dj, 0), size - 1)
        ker[i, j] += 1.0
    return ker / ker.sum()


def make_inputs(net: Net) -> dict:
    """Returns {"x": fp32 input, and one of "labels" (int32), "target" (fp32), "upstream" (fp32)}."""
    b = net.batch
    c, h, w = net.in_chw
    r0, r1 = _rng(net.index, 0), _rng(net.index, 1)
    out = {}
    if net.name in ("cfg1", "cfg2"):
        out["x"] = _f32(r0.random((b, c, h, w)))
    elif net.name == "cfg3":
        out["x"] = _f32(r0.standard_normal((b, c, h, w)))
    elif net.name == "cfg4":
        raw = r0.random((b, c, h + 4, w + 4))
        clean = _valid_filter(raw, np.full((5, 5), 1.0 / 25.0))
        noisy = clean + (25.0 / 255.0) * r1.standard_normal(clean.shape)
        out["x"] = _f32(noisy)
        out["target"] = _f32(clean)
    elif net.name == "cfg5":
        sharp = r0.random((b, c, h + 14, w + 14))
        ker = _motion_kernel(r1)
        out["x"] = _f32(_valid_filter(sharp, ker))
        oh, ow = net.out_shape[2:]
        top, left = 7 + (h - oh) // 2, 7 + (w - ow) // 2
        out["target"] = _f32(sharp[:, :, top:top + oh, left:left + ow])
    else:
        raise ValueError(net.name)
    if net.loss == "softmax":
        out["labels"] = r1.integers(0, net.classes, size=(b,)).astype(np.int32)
    elif net.loss == "upstream":
        out["upstream"] = _f32(r1.standard_normal(net.out_shape))
    return out


def make_params(net: Net) -> list:
    """He-normal weights (variance 2 / fan-in) and constant biases, one (w, b) pair per parametrised
    layer (None for pooling layers), fp32."""
    params = []
    pl = 0
    for li, L in enumerate(net.layers):
        ishape = net.in_shape(li)
        if isinstance(L, Conv):
            fan_in = ishape[1] * L.kh * L.kw
            wshape = (L.cout, ishape[1], L.kh, L.kw)
            nout = L.cout
        elif isinstance(L, FC):
            fan_in = int(np.prod(ishape[1:]))
            wshape = (L.out, fan_in)
            nout = L.out
        else:
            params.append(None)
            continue
        wgt = _rng(net.index, 10 + 2 * pl).standard_normal(wshape) * np.sqrt(2.0 / fan_in)
        params.append((_f32(wgt), np.full((nout,), net.bias_init, dtype=np.float32)))
        pl += 1
    return params


def random_tensor(seed: int, shape, dist: str = "normal", scale: float = 1.0) -> np.ndarray:
    """Free-standing seeded fp32 tensor for per-layer parity cases."""
    g = np.random.Generator(np.random.Philox(key=seed))
    a = g.standard_normal(shape) if dist == "normal" else g.random(shape)
    return _f32(a * scale)


def bf16_round(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bfloat16 (ties to even), returned as fp32.  Input synthesis
    for the reduced-precision variant: both the oracle and the HIP path start from these values."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    rounded = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return rounded.astype(np.uint32).view(np.float32).reshape(a.shape)
