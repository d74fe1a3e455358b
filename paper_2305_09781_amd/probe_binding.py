"""ctypes binding of libspecprobe (include/spec_probe.h): the measurement aids that bench.py times beside the
attention kernels (a plain read stream; the memory requests of an attention launch without its arithmetic). Not
part of the method; nothing in the hot path loads it."""
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
        _lib.spec_probe_attention_traffic.argtypes = [ctypes.c_int] * 5 + [ctypes.c_void_p] * 6 + [ctypes.c_int, ctypes.c_void_p]
        _lib.spec_probe_attention_traffic.restype = ctypes.c_int
    return _lib


def spec_probe_read_stream(buf: torch.Tensor, sink: torch.Tensor, stream=None):
    """One plain read pass over `buf` (device tensor); `sink` holds at least 16 device bytes."""
    if stream is None:
        stream = torch.cuda.current_stream()
    rc = load().spec_probe_read_stream(ctypes.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size(),
                                       ctypes.c_void_p(sink.data_ptr()), ctypes.c_void_p(stream.cuda_stream))
    if rc != 0:
        raise RuntimeError(f"spec_probe_read_stream failed (code {rc})")


TRAFFIC_QUERIES, TRAFFIC_NEW_ROWS, TRAFFIC_APPEND, TRAFFIC_OUTPUTS = 1, 2, 4, 8
TRAFFIC_ALL = 15


def spec_probe_attention_traffic(k_cache, v_cache, q, k_new, v_new, out, prefix: int, flags: int = TRAFFIC_ALL, stream=None):
    """The memory requests of one fused append + attention launch without arithmetic (equal prefix lengths `prefix`).
    k_cache, v_cache: contiguous [B, H, S_cap, 128] bf16; q, k_new, v_new, out: contiguous [B, N, H, 128] bf16."""
    B, H, S_cap, D = k_cache.shape
    N = q.shape[1]
    for t in (k_cache, v_cache, q, k_new, v_new, out):
        if t.dtype != torch.bfloat16 or not t.is_contiguous() or t.shape[-1] != 128 or not t.is_cuda:
            raise ValueError("spec_probe_attention_traffic takes contiguous bf16 device tensors with 128 elements per row")
    if v_cache.shape != k_cache.shape or any(t.shape != (B, N, H, D) for t in (q, k_new, v_new, out)):
        raise ValueError("spec_probe_attention_traffic: shapes do not match [B,H,S_cap,128] / [B,N,H,128]")
    if stream is None:
        stream = torch.cuda.current_stream()
    vp = ctypes.c_void_p
    rc = load().spec_probe_attention_traffic(B, H, N, int(prefix), S_cap, vp(k_cache.data_ptr()), vp(v_cache.data_ptr()),
                                             vp(q.data_ptr()), vp(k_new.data_ptr()), vp(v_new.data_ptr()),
                                             vp(out.data_ptr()), int(flags), vp(stream.cuda_stream))
    if rc != 0:
        raise RuntimeError(f"spec_probe_attention_traffic failed (code {rc})")
