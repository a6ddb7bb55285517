"""ctypes binding of libfdprobes.so: the benchmark's bandwidth probes (a plain streaming copy and
the attention kernel's staged read over a contiguous buffer).  Not part of the product library."""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfdprobes.so")
STREAM_READ_SUMS = 512 * 256
_lib = None


def load() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python paper_2605_20022_amd/build.py`")
        lib = C.CDLL(LIB_PATH)
        lib.fdp_stream_copy.restype = C.c_int
        lib.fdp_stream_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        lib.fdp_stream_read.restype = C.c_int
        lib.fdp_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        _lib = lib
    return _lib


def _stream(stream):
    return C.c_void_p((stream or torch.cuda.current_stream()).cuda_stream)


def stream_copy(src: torch.Tensor, dst: torch.Tensor, stream=None) -> None:
    rc = load().fdp_stream_copy(src.data_ptr(), dst.data_ptr(), src.numel() * src.element_size(), _stream(stream))
    if rc:
        raise RuntimeError(f"fdp_stream_copy failed ({rc})")


def stream_read(src: torch.Tensor, sums: torch.Tensor, nbytes=None, stream=None) -> None:
    """Staged read of `src` (bytes a multiple of 32768); sums: 512 * 256 32-bit words on the device."""
    if sums.numel() != STREAM_READ_SUMS or sums.element_size() != 4 or not sums.is_contiguous():
        raise ValueError("sums must be a contiguous tensor of 512 * 256 32-bit words")
    n = src.numel() * src.element_size() if nbytes is None else nbytes
    rc = load().fdp_stream_read(src.data_ptr(), n, sums.data_ptr(), _stream(stream))
    if rc:
        raise RuntimeError(f"fdp_stream_read failed ({rc})")
