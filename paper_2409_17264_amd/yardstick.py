"""ctypes binding over libmedha_yardstick.so: the two measurement yardsticks of the
benchmark harness (an MFMA-only loop and an HBM -> LDS streaming read).  They are
not part of the attention path and live in their own shared library."""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmedha_yardstick.so")
_LIB = None

EXPORTS = ("medha_yardstick_mfma_bf16", "medha_yardstick_stream_lds")


def load_library():
    global _LIB
    if _LIB is not None:
        return _LIB
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2409_17264_amd.build`")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    lib.medha_yardstick_mfma_bf16.restype = ctypes.c_int
    lib.medha_yardstick_mfma_bf16.argtypes = [vp, sz, i32, i32, vp, sz, vp]
    lib.medha_yardstick_stream_lds.restype = ctypes.c_int
    lib.medha_yardstick_stream_lds.argtypes = [vp, sz, i32, vp, sz, vp]
    _LIB = lib
    return lib


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def mfma_bf16(operands: torch.Tensor, blocks: int, iters: int, sink: torch.Tensor) -> float:
    """Enqueue the matrix-instruction yardstick; returns the flop it performs."""
    assert operands.is_cuda and operands.dtype == torch.bfloat16 and operands.is_contiguous()
    assert sink.is_cuda and sink.dtype == torch.float32 and sink.is_contiguous()
    rc = load_library().medha_yardstick_mfma_bf16(
        operands.data_ptr(), operands.numel() * 2, blocks, iters, sink.data_ptr(), sink.numel(),
        _stream())
    if rc != 0:
        raise RuntimeError(f"medha_yardstick_mfma_bf16 failed: {rc}")
    return float(blocks) * 8 * iters * 4 * 32768


def stream_lds(src: torch.Tensor, blocks: int, sink: torch.Tensor) -> float:
    """Enqueue the HBM -> LDS streaming yardstick; returns the bytes it reads."""
    assert src.is_cuda and src.is_contiguous()
    assert sink.is_cuda and sink.is_contiguous() and sink.dtype == torch.int32
    nbytes = src.numel() * src.element_size()
    rc = load_library().medha_yardstick_stream_lds(src.data_ptr(), nbytes, blocks,
                                                   sink.data_ptr(), sink.numel(), _stream())
    if rc != 0:
        raise RuntimeError(f"medha_yardstick_stream_lds failed: {rc}")
    return float(nbytes)
