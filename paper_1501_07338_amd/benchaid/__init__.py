"""ctypes loader of libvcnn_benchaid.so: measurement aids the benchmark uses (a register-only matrix-core
loop and a plain streaming copy).  Not part of the layer library; nothing in the layer path imports this."""
from __future__ import annotations

import ctypes
from ctypes import byref, c_double, c_int, c_size_t, c_void_p
from pathlib import Path

LIB_PATH = Path(__file__).resolve().parents[1] / "libvcnn_benchaid.so"
_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_1501_07338_amd.build)")
        import torch  # noqa: F401  (one HIP runtime per process: torch's)
        h = ctypes.CDLL(str(LIB_PATH))
        h.benchaid_mfma.restype, h.benchaid_mfma.argtypes = c_int, [c_int, c_int, c_int, c_int, c_void_p, c_void_p, c_void_p]
        h.benchaid_mfma_lds.restype, h.benchaid_mfma_lds.argtypes = c_int, [c_int, c_int, c_int, c_void_p, c_void_p, c_int, c_void_p, c_void_p]
        h.benchaid_copy.restype, h.benchaid_copy.argtypes = c_int, [c_void_p, c_void_p, c_size_t, c_void_p]
        h.benchaid_marker.restype, h.benchaid_marker.argtypes = c_int, [c_int, c_void_p]
        _lib = h
    return _lib


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def mfma(bf16: bool, blocks: int, iters: int, sink, stream=None, toggle: bool = False) -> float:
    """Launches the register-only matrix-core loop (toggle: operands that change from instruction to instruction);
    returns the flop count of the launch."""
    flop = c_double()
    err = lib().benchaid_mfma(int(bf16), int(toggle), blocks, iters, sink.data_ptr(), byref(flop), _stream(stream))
    if err:
        raise RuntimeError(f"benchaid_mfma: HIP error {err}")
    return flop.value


def mfma_lds(staged: bool, blocks: int, iters: int, sink, src=None, stream=None) -> float:
    """Launches the fp32 matrix-core loop of a 128 x 128 tile fed from LDS (staged: with the fetch of new operand
    words from the device tensor src into LDS every 64 instructions); returns the flop count of the launch."""
    flop = c_double()
    count4 = 0 if src is None else src.numel() * src.element_size() // 16
    err = lib().benchaid_mfma_lds(int(staged), blocks, iters, sink.data_ptr(), None if src is None else src.data_ptr(),
                                  count4, byref(flop), _stream(stream))
    if err:
        raise RuntimeError(f"benchaid_mfma_lds: HIP error {err}")
    return flop.value


def copy(src, dst, stream=None) -> int:
    """dst <- src with one streaming kernel; returns the bytes copied."""
    nbytes = src.numel() * src.element_size()
    err = lib().benchaid_copy(src.data_ptr(), dst.data_ptr(), nbytes, _stream(stream))
    if err:
        raise RuntimeError(f"benchaid_copy: HIP error {err}")
    return nbytes


def marker(ident: int, stream=None) -> None:
    """An empty kernel of `ident` blocks: marks the start of a phase in a kernel trace."""
    err = lib().benchaid_marker(ident, _stream(stream))
    if err:
        raise RuntimeError(f"benchaid_marker: HIP error {err}")
