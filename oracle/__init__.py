"""fp64 CPU oracle for the vectorized CNN layer path (Ren & Xu, AAAI 2015).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's CPU-baseline
leg.  The product package never imports it, and it never imports the product package.

`vcnn_oracle.c` holds the plain nested-loop definitions (Eq. 1-4 of the paper and their exact
derivatives); this module builds it with gcc, binds it with ctypes and adds single-output "probe"
functions in numpy that evaluate one output element of a layer straight from its definition, for
checking full-size workloads at sampled positions.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "vcnn_oracle.c"
_LIB = _HERE / "libvcnn_oracle.so"
_lib = None

_D = ctypes.POINTER(ctypes.c_double)
_I = ctypes.POINTER(ctypes.c_int32)


def build(force: bool = False) -> Path:
    """Compile the C oracle into a shared library next to its source."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".so.tmp{os.getpid()}")
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", str(tmp), str(_SRC), "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(str(_LIB))
        _lib.oracle_softmax_loss.restype = ctypes.c_double
        _lib.oracle_l2_loss.restype = ctypes.c_double
    return _lib


def threads() -> int:
    """Number of OpenMP threads the C loops will use."""
    n = os.environ.get("OMP_NUM_THREADS")
    avail = len(os.sched_getaffinity(0))
    return min(int(n), avail) if n and n.isdigit() and int(n) > 0 else avail


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a: np.ndarray):
    return a.ctypes.data_as(_D)


def conv_out_hw(h, w, r, s, ph, pw, sh=1, sw=1):
    return (h + 2 * ph - r) // sh + 1, (w + 2 * pw - s) // sw + 1


def conv_fwd(x, w, b=None, pad=(0, 0), stride=(1, 1), relu=False):
    """Eq. 1 of the paper evaluated directly; x [N,C,H,W], w [K,C,R,S], b [K] or None."""
    x, w = _f64(x), _f64(w)
    n, c, h, wd = x.shape
    k, c2, r, s = w.shape
    assert c == c2
    oh, ow = conv_out_hw(h, wd, r, s, pad[0], pad[1], stride[0], stride[1])
    y = np.empty((n, k, oh, ow), dtype=np.float64)
    bb = _f64(b) if b is not None else None
    _load().oracle_conv_fwd(_p(x), _p(w), _p(bb) if bb is not None else None, _p(y), n, c, h, wd, k, r, s,
                            pad[0], pad[1], stride[0], stride[1], int(relu))
    return y


def conv_bwd_filter(x, dy, rs, pad=(0, 0), stride=(1, 1)):
    """Gradient of Eq. 1's linear part w.r.t. kernels and biases; returns (dw, db)."""
    x, dy = _f64(x), _f64(dy)
    n, c, h, wd = x.shape
    k = dy.shape[1]
    r, s = rs
    assert dy.shape == (n, k) + conv_out_hw(h, wd, r, s, pad[0], pad[1], stride[0], stride[1])
    dw = np.empty((k, c, r, s), dtype=np.float64)
    db = np.empty((k,), dtype=np.float64)
    _load().oracle_conv_bwd_filter(_p(x), _p(dy), _p(dw), _p(db), n, c, h, wd, k, r, s, pad[0], pad[1],
                                   stride[0], stride[1])
    return dw, db


def conv_bwd_data(w, dy, hw, pad=(0, 0), stride=(1, 1)):
    """Gradient w.r.t. the layer input (phi_c^{-1} applied to the kernel-transposed product)."""
    w, dy = _f64(w), _f64(dy)
    k, c, r, s = w.shape
    n = dy.shape[0]
    h, wd = hw
    assert dy.shape == (n, k) + conv_out_hw(h, wd, r, s, pad[0], pad[1], stride[0], stride[1])
    dx = np.empty((n, c, h, wd), dtype=np.float64)
    _load().oracle_conv_bwd_data(_p(w), _p(dy), _p(dx), n, c, h, wd, k, r, s, pad[0], pad[1], stride[0],
                                 stride[1])
    return dx


def im2col(x, rs, pad=(0, 0), stride=(1, 1)):
    """phi_c of Eq. 2/4: [C*R*S, N*OH*OW] patch matrix."""
    x = _f64(x)
    n, c, h, wd = x.shape
    r, s = rs
    oh, ow = conv_out_hw(h, wd, r, s, pad[0], pad[1], stride[0], stride[1])
    col = np.empty((c * r * s, n * oh * ow), dtype=np.float64)
    _load().oracle_im2col(_p(x), _p(col), n, c, h, wd, r, s, pad[0], pad[1], stride[0], stride[1])
    return col


def col2im(col, xshape, rs, pad=(0, 0), stride=(1, 1)):
    """phi_c^{-1}: sum the entries of the patch matrix that are copies of one pixel."""
    col = _f64(col)
    n, c, h, wd = xshape
    r, s = rs
    oh, ow = conv_out_hw(h, wd, r, s, pad[0], pad[1], stride[0], stride[1])
    assert col.shape == (c * r * s, n * oh * ow)
    dx = np.empty(xshape, dtype=np.float64)
    _load().oracle_col2im(_p(col), _p(dx), n, c, h, wd, r, s, pad[0], pad[1], stride[0], stride[1])
    return dx


def maxpool_fwd(x, win, stride):
    """Max pooling; returns (y, argmax) with argmax the int32 flat index h*W+w in the input plane."""
    x = _f64(x)
    n, c, h, wd = x.shape
    oh, ow = (h - win[0]) // stride[0] + 1, (wd - win[1]) // stride[1] + 1
    y = np.empty((n, c, oh, ow), dtype=np.float64)
    am = np.empty((n, c, oh, ow), dtype=np.int32)
    _load().oracle_maxpool_fwd(_p(x), _p(y), am.ctypes.data_as(_I), n, c, h, wd, win[0], win[1], stride[0],
                               stride[1])
    return y, am


def maxpool_bwd(dy, argmax, hw):
    dy = _f64(dy)
    am = np.ascontiguousarray(argmax, dtype=np.int32)
    n, c, oh, ow = dy.shape
    dx = np.empty((n, c, hw[0], hw[1]), dtype=np.float64)
    _load().oracle_maxpool_bwd(_p(dy), am.ctypes.data_as(_I), _p(dx), n, c, hw[0], hw[1], oh, ow)
    return dx


def relu_fwd(x):
    x = _f64(x)
    y = np.empty_like(x)
    _load().oracle_relu_fwd(_p(x), _p(y), ctypes.c_int64(x.size))
    return y


def relu_bwd(x, dy):
    x, dy = _f64(x), _f64(dy)
    dx = np.empty_like(x)
    _load().oracle_relu_bwd(_p(x), _p(dy), _p(dx), ctypes.c_int64(x.size))
    return dx


def _elementwise(name, *arrays):
    arrays = [_f64(a) for a in arrays]
    out = np.empty_like(arrays[0])
    getattr(_load(), name)(*[_p(a) for a in arrays], _p(out), ctypes.c_int64(out.size))
    return out


def tanh_fwd(x):
    return _elementwise("oracle_tanh_fwd", x)


def tanh_bwd(y, dy):
    """dx from the forward OUTPUT y = tanh(x)."""
    return _elementwise("oracle_tanh_bwd", y, dy)


def sigmoid_fwd(x):
    return _elementwise("oracle_sigmoid_fwd", x)


def sigmoid_bwd(y, dy):
    """dx from the forward OUTPUT y = sigmoid(x)."""
    return _elementwise("oracle_sigmoid_bwd", y, dy)


def avgpool_fwd(x, win, stride):
    x = _f64(x)
    n, c, h, wd = x.shape
    oh, ow = (h - win[0]) // stride[0] + 1, (wd - win[1]) // stride[1] + 1
    y = np.empty((n, c, oh, ow), dtype=np.float64)
    _load().oracle_avgpool_fwd(_p(x), _p(y), n, c, h, wd, win[0], win[1], stride[0], stride[1])
    return y


def avgpool_bwd(dy, hw, win, stride):
    dy = _f64(dy)
    n, c, oh, ow = dy.shape
    dx = np.empty((n, c, hw[0], hw[1]), dtype=np.float64)
    _load().oracle_avgpool_bwd(_p(dy), _p(dx), n, c, hw[0], hw[1], win[0], win[1], stride[0], stride[1])
    return dx


_SIGMA = {"none": (lambda z: _f64(z).copy(), lambda y, g: _f64(g).copy()), "relu": (relu_fwd, relu_bwd),
          "tanh": (tanh_fwd, tanh_bwd), "sigmoid": (sigmoid_fwd, sigmoid_bwd)}


def pool_layer_fwd(x, bias, win, stride, mode="max", act="none"):
    """The pooling layer of Eq. 3, "Vectorizing Pooling": y = sigma(phi_p(x) + b), one bias per feature map,
    phi_p the max or the mean of each window.  Returns (y, argmax); argmax is None for average pooling."""
    if mode == "max":
        pooled, am = maxpool_fwd(x, win, stride)
    else:
        pooled, am = avgpool_fwd(x, win, stride), None
    z = pooled + (0.0 if bias is None else _f64(bias)[None, :, None, None])
    return _SIGMA[act][0](z), am


def pool_layer_bwd(y, dy, argmax, hw, win, stride, mode="max", act="none"):
    """Gradients of the layer above from its output y and dL/dy: through sigma (delta = dy * sigma'(.), from y),
    then dbias[c] = sum of delta over samples and pixels, and dx = delta routed back through phi_p (to the
    recorded maximum, or spread evenly over the window).  Returns (dx, dbias, delta)."""
    delta = _SIGMA[act][1](y, dy)
    dbias = delta.sum(axis=(0, 2, 3))
    dx = maxpool_bwd(delta, argmax, hw) if mode == "max" else avgpool_bwd(delta, hw, win, stride)
    return dx, dbias, delta


def fc_fwd(x, w, b=None, relu=False):
    x, w = _f64(x), _f64(w)
    bsz, i = x.shape
    o = w.shape[0]
    assert w.shape == (o, i)
    y = np.empty((bsz, o), dtype=np.float64)
    bb = _f64(b) if b is not None else None
    _load().oracle_fc_fwd(_p(x), _p(w), _p(bb) if bb is not None else None, _p(y), bsz, i, o, int(relu))
    return y


def fc_bwd(x, w, dy, need_dx=True):
    x, w, dy = _f64(x), _f64(w), _f64(dy)
    bsz, i = x.shape
    o = w.shape[0]
    dw = np.empty((o, i), dtype=np.float64)
    db = np.empty((o,), dtype=np.float64)
    dx = np.empty((bsz, i), dtype=np.float64) if need_dx else None
    _load().oracle_fc_bwd(_p(x), _p(w), _p(dy), _p(dw), _p(db), _p(dx) if need_dx else None, bsz, i, o)
    return dw, db, dx


def softmax_loss(z, labels):
    z = _f64(z)
    lab = np.ascontiguousarray(labels, dtype=np.int32)
    bsz, cn = z.shape
    dz = np.empty_like(z)
    loss = _load().oracle_softmax_loss(_p(z), lab.ctypes.data_as(_I), _p(dz), bsz, cn)
    return float(loss), dz


def l2_loss(y, t):
    y, t = _f64(y), _f64(t)
    assert y.shape == t.shape
    dy = np.empty_like(y)
    loss = _load().oracle_l2_loss(_p(y), _p(t), _p(dy), ctypes.c_int64(y.size), y.shape[0])
    return float(loss), dy


def sgd_update(w, dw, lr):
    w = _f64(w).copy()
    dw = _f64(dw)
    _load().oracle_sgd_update(_p(w), _p(dw), ctypes.c_double(lr), ctypes.c_int64(w.size))
    return w


# --------------------------------------------------------------------------------------------------
# Single-output probes (numpy, fp64): one element of a layer's result straight from its definition,
# for full-size workloads where computing every output on the CPU would take minutes.
# --------------------------------------------------------------------------------------------------

def _padded(x, pad):
    return np.pad(_f64(x), ((0, 0), (0, 0), (pad[0], pad[0]), (pad[1], pad[1])))


def conv_fwd_at(x, w, b, pad, idx, relu=False):
    """Eq. 1 at output positions idx = [(n,k,oh,ow), ...], stride 1."""
    xp, w = _padded(x, pad), _f64(w)
    r, s = w.shape[2:]
    out = np.empty(len(idx))
    for t, (n, k, oh, ow) in enumerate(idx):
        v = float(np.sum(w[k] * xp[n, :, oh:oh + r, ow:ow + s])) + (float(b[k]) if b is not None else 0.0)
        out[t] = max(v, 0.0) if relu else v
    return out


def conv_bwd_filter_at(x, dy, rs, pad, idx):
    """dw at positions idx = [(k,c,r,s), ...], stride 1."""
    xp, dy = _padded(x, pad), _f64(dy)
    oh, ow = dy.shape[2:]
    return np.array([float(np.sum(dy[:, k] * xp[:, c, r:r + oh, s:s + ow])) for (k, c, r, s) in idx])


def conv_bwd_data_at(w, dy, pad, idx):
    """dx at positions idx = [(n,c,h,w), ...], stride 1: sum over kernels and taps of
    w[k,c,r,s] * dy[n,k,h+ph-r,w+pw-s] for the taps whose output position exists (the terms phi_c^{-1} adds up
    for that pixel).  The existing taps of a pixel form one rectangle r0..r1 x s0..s1; the sum runs over it at once."""
    w, dy = _f64(w), _f64(dy)
    _, _, r, s = w.shape
    oh, ow = dy.shape[2:]
    out = np.empty(len(idx))
    for t, (n, c, h, wi) in enumerate(idx):
        # tap rr exists iff 0 <= h + ph - rr < oh
        r0, r1 = max(0, h + pad[0] - oh + 1), min(r - 1, h + pad[0])
        s0, s1 = max(0, wi + pad[1] - ow + 1), min(s - 1, wi + pad[1])
        if r0 > r1 or s0 > s1:
            out[t] = 0.0
            continue
        taps = w[:, c, r0:r1 + 1, s0:s1 + 1]
        # output rows h+ph-rr for rr = r0..r1, i.e. descending: reverse the window to line it up with the taps
        win = dy[n, :, h + pad[0] - r1:h + pad[0] - r0 + 1, wi + pad[1] - s1:wi + pad[1] - s0 + 1][:, ::-1, ::-1]
        out[t] = float(np.sum(taps * win))
    return out
