"""ctypes binding of libvcnn.so: one Python function per C entry point, same names, argument
marshalling only.  Tensors are torch tensors on the GPU (torch supplies device memory and the
stream, nothing else); every computation happens inside the library's HIP kernels.

The library must have been built (`python -m paper_1501_07338_amd.build` or `__graft_entry__.build()`);
there is no fallback path: a missing library raises.
"""
from __future__ import annotations

import ctypes
from ctypes import POINTER, Structure, byref, c_char_p, c_float, c_int32, c_size_t, c_void_p
from pathlib import Path

LIB_PATH = Path(__file__).resolve().parent / "libvcnn.so"

OK, ERR_NULL, ERR_SHAPE, ERR_WORKSPACE, ERR_UNSUPPORTED, ERR_HIP = 0, -1, -2, -3, -4, -5
F32, BF16 = 0, 1
ACT_NONE, ACT_RELU, ACT_TANH, ACT_SIGMOID = 0, 1, 2, 3
POOL_MAX, POOL_AVG = 0, 1
PASS_FWD, PASS_BWD_FILTER, PASS_BWD_DATA = 0, 1, 2
ALGO_AUTO, ALGO_EXPLICIT, ALGO_IMPLICIT, ALGO_FOLD, ALGO_FFT, ALGO_SPLIT = 0, 1, 2, 3, 4, 5


class ConvDesc(Structure):
    _fields_ = [(n, c_int32) for n in ("n", "c", "h", "w", "k", "r", "s", "pad_h", "pad_w", "stride_h", "stride_w",
                                        "dtype", "act")]


class PoolDesc(Structure):
    _fields_ = [(n, c_int32) for n in ("n", "c", "h", "w", "win_h", "win_w", "stride_h", "stride_w", "dtype", "mode")]


class VcnnError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"vcnn status {status}: {message}")
        self.status = status


_SIGNATURES = {
    "vcnn_status_string": (c_char_p, [c_int32]),
    "vcnn_last_error": (c_char_p, []),
    "vcnn_version": (c_int32, []),
    "vcnn_set_conv_algo": (c_int32, [c_int32]),
    "vcnn_conv_out_shape": (c_int32, [POINTER(ConvDesc), POINTER(c_int32), POINTER(c_int32)]),
    "vcnn_conv_workspace_bytes": (c_int32, [POINTER(ConvDesc), c_int32, POINTER(c_size_t)]),
    "vcnn_im2col": (c_int32, [POINTER(ConvDesc), c_void_p, c_void_p, c_void_p]),
    "vcnn_col2im": (c_int32, [POINTER(ConvDesc), c_void_p, c_void_p, c_void_p]),
    "vcnn_conv_fwd": (c_int32, [POINTER(ConvDesc), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    "vcnn_conv_bwd_filter": (c_int32, [POINTER(ConvDesc), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t,
                                       c_void_p]),
    "vcnn_conv_bwd_filter_noalloc_limit": (c_size_t, []),
    "vcnn_conv_bwd_filter_noalloc": (c_int32, [POINTER(ConvDesc), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]),
    "vcnn_conv_bwd_data": (c_int32, [POINTER(ConvDesc), c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    "vcnn_conv_bwd_data_act": (c_int32, [POINTER(ConvDesc), c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                         c_size_t, c_void_p]),
    "vcnn_pool_out_shape": (c_int32, [POINTER(PoolDesc), POINTER(c_int32), POINTER(c_int32)]),
    "vcnn_pool_fwd": (c_int32, [POINTER(PoolDesc), c_void_p, c_void_p, c_void_p, c_void_p]),
    "vcnn_pool_bwd": (c_int32, [POINTER(PoolDesc), c_void_p, c_void_p, c_void_p, c_void_p]),
    "vcnn_pool_layer_fwd": (c_int32, [POINTER(PoolDesc), c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]),
    "vcnn_pool_layer_workspace_bytes": (c_int32, [POINTER(PoolDesc), POINTER(c_size_t)]),
    "vcnn_pool_layer_bwd": (c_int32, [POINTER(PoolDesc), c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                      c_void_p, c_size_t, c_void_p]),
    "vcnn_pool_bwd_act": (c_int32, [POINTER(PoolDesc), c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]),
    "vcnn_fc_bwd_act": (c_int32, [c_int32, c_int32, c_int32, c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_void_p,
                                  c_void_p, c_void_p, c_void_p]),
    "vcnn_act_fwd": (c_int32, [c_int32, c_int32, c_size_t, c_void_p, c_void_p, c_void_p]),
    "vcnn_act_bwd": (c_int32, [c_int32, c_int32, c_size_t, c_void_p, c_void_p, c_void_p, c_void_p]),
    "vcnn_fc_fwd": (c_int32, [c_int32, c_int32, c_int32, c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_void_p,
                              c_void_p]),
    "vcnn_fc_bwd": (c_int32, [c_int32, c_int32, c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                              c_void_p, c_void_p]),
    "vcnn_softmax_loss": (c_int32, [c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]),
    "vcnn_l2_loss": (c_int32, [c_int32, c_size_t, c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]),
    "vcnn_sgd_update": (c_int32, [c_size_t, c_float, c_void_p, c_void_p, c_void_p]),
    "vcnn_sgd_update_multi": (c_int32, [c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_float, c_void_p]),
    "vcnn_f32_to_bf16": (c_int32, [c_size_t, c_void_p, c_void_p, c_void_p]),
    "vcnn_bf16_to_f32": (c_int32, [c_size_t, c_void_p, c_void_p, c_void_p]),
}

EXPORTS = tuple(_SIGNATURES)
_lib = None


def lib() -> ctypes.CDLL:
    """Loads libvcnn.so on first use; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_1501_07338_amd.build); "
                               "there is no fallback path")
        # torch first: the device pointers and streams passed in belong to the HIP runtime torch loads, and the
        # library must resolve its HIP symbols against that same copy (a second runtime sees no device)
        import torch  # noqa: F401
        handle = ctypes.CDLL(str(LIB_PATH))
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def _check(status: int) -> None:
    if status != OK:
        raise VcnnError(status, lib().vcnn_last_error().decode())


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def conv_desc(n, c, h, w, k, r, s, pad_h=0, pad_w=0, stride_h=1, stride_w=1, dtype=F32, act=ACT_NONE) -> ConvDesc:
    return ConvDesc(n, c, h, w, k, r, s, pad_h, pad_w, stride_h, stride_w, dtype, act)


def pool_desc(n, c, h, w, win_h, win_w, stride_h, stride_w, dtype=F32, mode=POOL_MAX) -> PoolDesc:
    return PoolDesc(n, c, h, w, win_h, win_w, stride_h, stride_w, dtype, mode)


def version() -> int:
    return lib().vcnn_version()


def status_string(status: int) -> str:
    return lib().vcnn_status_string(status).decode()


def last_error() -> str:
    return lib().vcnn_last_error().decode()


_conv_algo = ALGO_AUTO  # what this binding last set (the library keeps the choice process-wide and has no getter)


def set_conv_algo(algo: int) -> None:
    global _conv_algo
    _check(lib().vcnn_set_conv_algo(algo))
    _conv_algo = algo


def conv_algo() -> int:
    """The route choice last made through set_conv_algo (AUTO at start)."""
    return _conv_algo


def conv_out_shape(d: ConvDesc):
    oh, ow = c_int32(), c_int32()
    _check(lib().vcnn_conv_out_shape(byref(d), byref(oh), byref(ow)))
    return oh.value, ow.value


def conv_workspace_bytes(d: ConvDesc, which: int) -> int:
    b = c_size_t()
    _check(lib().vcnn_conv_workspace_bytes(byref(d), which, byref(b)))
    return b.value


def im2col(d, x, col, stream=None):
    _check(lib().vcnn_im2col(byref(d), _ptr(x), _ptr(col), _stream(stream)))


def col2im(d, col, dx, stream=None):
    _check(lib().vcnn_col2im(byref(d), _ptr(col), _ptr(dx), _stream(stream)))


def _ws(ws):
    return (None, 0) if ws is None else (ws.data_ptr(), ws.numel() * ws.element_size())


def conv_fwd(d, x, w, bias, y, workspace=None, stream=None):
    p, nbytes = _ws(workspace)
    _check(lib().vcnn_conv_fwd(byref(d), _ptr(x), _ptr(w), _ptr(bias), _ptr(y), p, nbytes, _stream(stream)))


def conv_bwd_filter(d, x, dy, dw, dbias, workspace=None, stream=None):
    p, nbytes = _ws(workspace)
    _check(lib().vcnn_conv_bwd_filter(byref(d), _ptr(x), _ptr(dy), _ptr(dw), _ptr(dbias), p, nbytes, _stream(stream)))


def conv_bwd_filter_noalloc_limit() -> int:
    return lib().vcnn_conv_bwd_filter_noalloc_limit()


def conv_bwd_filter_noalloc(d, x, dy, dw, dbias, stream=None):
    _check(lib().vcnn_conv_bwd_filter_noalloc(byref(d), _ptr(x), _ptr(dy), _ptr(dw), _ptr(dbias), _stream(stream)))


def conv_bwd_data(d, w, dy, dx, workspace=None, stream=None):
    p, nbytes = _ws(workspace)
    _check(lib().vcnn_conv_bwd_data(byref(d), _ptr(w), _ptr(dy), _ptr(dx), p, nbytes, _stream(stream)))


def conv_bwd_data_act(d, act_below, x, w, dy, dx, workspace=None, stream=None):
    p, nbytes = _ws(workspace)
    _check(lib().vcnn_conv_bwd_data_act(byref(d), act_below, _ptr(x), _ptr(w), _ptr(dy), _ptr(dx), p, nbytes, _stream(stream)))


def pool_out_shape(d: PoolDesc):
    oh, ow = c_int32(), c_int32()
    _check(lib().vcnn_pool_out_shape(byref(d), byref(oh), byref(ow)))
    return oh.value, ow.value


def pool_fwd(d, x, y, argmax, stream=None):
    _check(lib().vcnn_pool_fwd(byref(d), _ptr(x), _ptr(y), _ptr(argmax), _stream(stream)))


def pool_bwd(d, dy, argmax, dx, stream=None):
    _check(lib().vcnn_pool_bwd(byref(d), _ptr(dy), _ptr(argmax), _ptr(dx), _stream(stream)))


def pool_layer_fwd(d, act, x, bias, y, argmax, stream=None):
    _check(lib().vcnn_pool_layer_fwd(byref(d), act, _ptr(x), _ptr(bias), _ptr(y), _ptr(argmax), _stream(stream)))


def pool_layer_workspace_bytes(d):
    n = c_size_t(0)
    _check(lib().vcnn_pool_layer_workspace_bytes(byref(d), byref(n)))
    return n.value


def pool_layer_bwd(d, act, y, dy, argmax, dbias, dx, workspace, stream=None):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().vcnn_pool_layer_bwd(byref(d), act, _ptr(y), _ptr(dy), _ptr(argmax), _ptr(dbias), _ptr(dx),
                                     _ptr(workspace), nbytes, _stream(stream)))


def pool_bwd_act(d, act_below, x, dy, argmax, dx, stream=None):
    _check(lib().vcnn_pool_bwd_act(byref(d), act_below, _ptr(x), _ptr(dy), _ptr(argmax), _ptr(dx), _stream(stream)))


def act_fwd(act, dtype, count, x, y, stream=None):
    _check(lib().vcnn_act_fwd(act, dtype, count, _ptr(x), _ptr(y), _stream(stream)))


def act_bwd(act, dtype, count, ref, dy, dx, stream=None):
    _check(lib().vcnn_act_bwd(act, dtype, count, _ptr(ref), _ptr(dy), _ptr(dx), _stream(stream)))


def fc_fwd(dtype, batch, in_f, out_f, act, x, w, bias, y, stream=None):
    _check(lib().vcnn_fc_fwd(dtype, batch, in_f, out_f, act, _ptr(x), _ptr(w), _ptr(bias), _ptr(y), _stream(stream)))


def fc_bwd(dtype, batch, in_f, out_f, x, w, dy, dw, dbias, dx, stream=None):
    _check(lib().vcnn_fc_bwd(dtype, batch, in_f, out_f, _ptr(x), _ptr(w), _ptr(dy), _ptr(dw), _ptr(dbias), _ptr(dx),
                             _stream(stream)))


def fc_bwd_act(dtype, batch, in_f, out_f, act_below, x, w, dy, dw, dbias, dx, stream=None):
    _check(lib().vcnn_fc_bwd_act(dtype, batch, in_f, out_f, act_below, _ptr(x), _ptr(w), _ptr(dy), _ptr(dw), _ptr(dbias),
                                 _ptr(dx), _stream(stream)))


def softmax_loss(batch, classes, logits, labels, loss, dlogits, stream=None):
    _check(lib().vcnn_softmax_loss(batch, classes, _ptr(logits), _ptr(labels), _ptr(loss), _ptr(dlogits),
                                   _stream(stream)))


def l2_loss(dtype, count, batch, y, target, loss, dy, stream=None):
    _check(lib().vcnn_l2_loss(dtype, count, batch, _ptr(y), _ptr(target), _ptr(loss), _ptr(dy), _stream(stream)))


def sgd_update(count, lr, w, dw, stream=None):
    _check(lib().vcnn_sgd_update(count, lr, _ptr(w), _ptr(dw), _stream(stream)))


def sgd_update_multi(lr, ws, dws, w16s=None, stream=None):
    """One launch for a list of parameter tensors; w16s (optional) are their bfloat16 working copies."""
    n = len(ws)
    counts = (c_size_t * n)(*[w.numel() for w in ws])
    wp = (c_void_p * n)(*[_ptr(w) for w in ws])
    dp = (c_void_p * n)(*[_ptr(g) for g in dws])
    hp = None if w16s is None else (c_void_p * n)(*[_ptr(h) for h in w16s])
    _check(lib().vcnn_sgd_update_multi(n, counts, wp, dp, hp, lr, _stream(stream)))


def f32_to_bf16(count, src, dst, stream=None):
    _check(lib().vcnn_f32_to_bf16(count, _ptr(src), _ptr(dst), _stream(stream)))


def bf16_to_f32(count, src, dst, stream=None):
    _check(lib().vcnn_bf16_to_f32(count, _ptr(src), _ptr(dst), _stream(stream)))
