"""ctypes binding of libspecprobe (include/spec_probe.h): the read-stream measurement aid that bench.py times
beside the attention kernels. Not part of the method; nothing in the hot path loads it."""
from __future__ import annotations

import ctypes
import os

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libspecprobe.so")
_lib = None


def load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} not found: build it with `python -m paper_2305_09781_amd.build`")
        _lib = ctypes.CDLL(_LIB_PATH)
        _lib.spec_probe_read_stream.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
        _lib.spec_probe_read_stream.restype = ctypes.c_int
    return _lib


def spec_probe_read_stream(buf: torch.Tensor, sink: torch.Tensor, stream=None):
    """One plain read pass over `buf` (device tensor); `sink` holds at least 16 device bytes."""
    if stream is None:
        stream = torch.cuda.current_stream()
    rc = load().spec_probe_read_stream(ctypes.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size(),
                                       ctypes.c_void_p(sink.data_ptr()), ctypes.c_void_p(stream.cuda_stream))
    if rc != 0:
        raise RuntimeError(f"spec_probe_read_stream failed (code {rc})")
