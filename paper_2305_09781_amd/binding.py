"""ctypes binding of libspectree (include/spec_tree.h): argument marshalling only.

Each function has the name of the C entry point it calls and passes device pointers of torch tensors
(torch is used for device memory and streams, nothing else). Every step of the hot path runs in the
HIP kernels of the library; there is no fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libspectree.so")
_lib = None

SPEC_F32, SPEC_BF16 = 0, 1
SPEC_MAX_TREE_NODES = 128
ST_BAD_TREE, ST_CAPACITY, ST_BAD_PATH, ST_ZERO_RESIDUAL, ST_BAD_BLOCK = 1, 2, 4, 8, 16
ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_CAPACITY, ERR_HIP, ERR_WORKSPACE = -1, -2, -3, -4, -5

EXPORTED = [
    "spec_kv_append", "spec_kv_append_rope", "spec_tree_attention", "spec_tree_attention_append", "spec_tree_attention_workspace_bytes",
    "spec_verify_greedy",
    "spec_verify_stochastic", "spec_verify_stochastic_workspace_bytes", "spec_verify_naive",
    "spec_verify_naive_workspace_bytes", "spec_tree_expand_topk", "spec_tree_merge", "spec_kv_commit", "spec_strerror",
    "spec_version",
    "spec_kv_append_paged", "spec_kv_append_rope_paged", "spec_tree_attention_paged", "spec_tree_attention_append_paged",
    "spec_tree_attention_paged_workspace_bytes", "spec_kv_commit_paged",
    "spec_lm_head_argmax", "spec_lm_head_argmax_workspace_bytes", "spec_verify_greedy_lm_head",
    "spec_qk_rope_append", "spec_qk_rope_append_paged", "spec_tree_attention_append_static",
    "spec_lm_head_logits_stats", "spec_lm_head_logits_stats_workspace_bytes", "spec_verify_stochastic_stats",
    "spec_verify_stochastic_stats_workspace_bytes",
    "spec_tree_attention_append_rope", "spec_tree_attention_append_rope_paged",
]
STATIC_SCRATCH_BYTES = 64 << 20


class SpecError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = load().spec_strerror(code).decode()
        super().__init__(f"{where}: {msg} (code {code})")


class AttnDesc(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("H", ctypes.c_int32), ("H_kv", ctypes.c_int32), ("D", ctypes.c_int32),
        ("N", ctypes.c_int32), ("S_cap", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("max_prefix_len", ctypes.c_int32),
        ("q_stride_b", ctypes.c_int64), ("q_stride_n", ctypes.c_int64), ("q_stride_h", ctypes.c_int64),
        ("kv_stride_b", ctypes.c_int64), ("kv_stride_h", ctypes.c_int64), ("kv_stride_s", ctypes.c_int64),
        ("new_stride_b", ctypes.c_int64), ("new_stride_n", ctypes.c_int64), ("new_stride_h", ctypes.c_int64),
        ("softmax_scale", ctypes.c_float), ("plan_chunk_keys", ctypes.c_int32), ("plan_balanced_wgs", ctypes.c_int32),
        ("plan_heads_per_wg", ctypes.c_int32),
    ]


class KvPages(ctypes.Structure):
    _fields_ = [("block_table", ctypes.c_void_p), ("max_blocks", ctypes.c_int32), ("block_tokens", ctypes.c_int32),
                ("n_blocks", ctypes.c_int32)]


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Loads libspectree.so built in-tree; raises if it is missing (there is no other code path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} not found: build it with `python -m paper_2305_09781_amd.build` "
                           "(the HIP library is the only implementation of the hot path)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
    dp = ctypes.POINTER(AttnDesc)
    lib.spec_kv_append.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp]
    lib.spec_kv_append.restype = ctypes.c_int
    lib.spec_kv_append_rope.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp]
    lib.spec_kv_append_rope.restype = ctypes.c_int
    lib.spec_tree_attention.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp, vp]
    lib.spec_tree_attention.restype = ctypes.c_int
    lib.spec_tree_attention_append.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp, vp]
    lib.spec_tree_attention_append.restype = ctypes.c_int
    lib.spec_tree_attention_append_static.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.spec_tree_attention_append_static.restype = ctypes.c_int
    lib.spec_tree_attention_append_rope.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, sz, vp, vp]
    lib.spec_tree_attention_append_rope.restype = ctypes.c_int
    lib.spec_tree_attention_workspace_bytes.argtypes = [dp]
    lib.spec_tree_attention_workspace_bytes.restype = sz
    lib.spec_verify_greedy.argtypes = [i32, i32, i32, i32, vp, vp, vp, i32, vp, vp, vp, vp, vp, sz, vp, vp]
    lib.spec_verify_greedy.restype = ctypes.c_int
    lib.spec_verify_stochastic.argtypes = [i32, i32, i32, i32, vp, vp, i32, vp, vp, vp, vp, vp, vp, f32, i32,
                                           vp, vp, vp, vp, sz, vp, vp]
    lib.spec_verify_stochastic.restype = ctypes.c_int
    lib.spec_verify_stochastic_workspace_bytes.argtypes = [i32, i32, i32]
    lib.spec_verify_stochastic_workspace_bytes.restype = sz
    lib.spec_verify_naive.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, f32, i32, vp, vp, vp, vp, vp, sz, vp, vp]
    lib.spec_verify_naive.restype = ctypes.c_int
    lib.spec_verify_naive_workspace_bytes.argtypes = [i32, i32, i32]
    lib.spec_verify_naive_workspace_bytes.restype = sz
    lib.spec_tree_expand_topk.argtypes = [i32, i32, i32, i32, vp, i32, vp, i32, vp, vp, vp]
    lib.spec_tree_expand_topk.restype = ctypes.c_int
    lib.spec_tree_merge.argtypes = [i32, i32, i32, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.spec_tree_merge.restype = ctypes.c_int
    lib.spec_kv_commit.argtypes = [dp, i32, ctypes.POINTER(vp), ctypes.POINTER(vp), vp, i32, vp, vp, vp, vp, vp]
    lib.spec_kv_commit.restype = ctypes.c_int
    pp = ctypes.POINTER(KvPages)
    lib.spec_kv_append_paged.argtypes = [dp, pp, vp, vp, vp, vp, vp, vp, vp]
    lib.spec_kv_append_paged.restype = ctypes.c_int
    lib.spec_kv_append_rope_paged.argtypes = [dp, pp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp]
    lib.spec_kv_append_rope_paged.restype = ctypes.c_int
    lib.spec_tree_attention_paged.argtypes = [dp, pp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp, vp]
    lib.spec_tree_attention_paged.restype = ctypes.c_int
    lib.spec_tree_attention_append_paged.argtypes = [dp, pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp, vp]
    lib.spec_tree_attention_append_paged.restype = ctypes.c_int
    lib.spec_tree_attention_append_rope_paged.argtypes = [dp, pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, sz,
                                                          vp, vp]
    lib.spec_tree_attention_append_rope_paged.restype = ctypes.c_int
    lib.spec_tree_attention_paged_workspace_bytes.argtypes = [dp, pp]
    lib.spec_tree_attention_paged_workspace_bytes.restype = sz
    lib.spec_kv_commit_paged.argtypes = [dp, pp, i32, ctypes.POINTER(vp), ctypes.POINTER(vp), vp, i32, vp, vp, vp, vp, vp]
    lib.spec_kv_commit_paged.restype = ctypes.c_int
    lib.spec_qk_rope_append.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp]
    lib.spec_qk_rope_append.restype = ctypes.c_int
    lib.spec_qk_rope_append_paged.argtypes = [dp, pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp]
    lib.spec_qk_rope_append_paged.restype = ctypes.c_int
    lib.spec_lm_head_argmax_workspace_bytes.argtypes = [i32, i32]
    lib.spec_lm_head_argmax_workspace_bytes.restype = sz
    lib.spec_lm_head_argmax.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.spec_lm_head_argmax.restype = ctypes.c_int
    lib.spec_verify_greedy_lm_head.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, sz, vp, vp]
    lib.spec_verify_greedy_lm_head.restype = ctypes.c_int
    lib.spec_lm_head_logits_stats_workspace_bytes.argtypes = [i32, i32]
    lib.spec_lm_head_logits_stats_workspace_bytes.restype = sz
    lib.spec_lm_head_logits_stats.argtypes = [i32, i32, i32, vp, vp, f32, vp, vp, vp, vp, vp, sz, vp]
    lib.spec_lm_head_logits_stats.restype = ctypes.c_int
    lib.spec_verify_stochastic_stats_workspace_bytes.argtypes = [i32, i32]
    lib.spec_verify_stochastic_stats_workspace_bytes.restype = sz
    lib.spec_verify_stochastic_stats.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, f32, i32,
                                                 vp, vp, vp, vp, sz, vp, vp]
    lib.spec_verify_stochastic_stats.restype = ctypes.c_int
    lib.spec_strerror.argtypes = [ctypes.c_int]
    lib.spec_strerror.restype = ctypes.c_char_p
    lib.spec_version.restype = ctypes.c_int
    _lib = lib
    return lib


# ------------------------------------------------------------------------------------------------
# marshalling helpers
# ------------------------------------------------------------------------------------------------

def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dtype_code(dt: torch.dtype) -> int:
    if dt == torch.float32:
        return SPEC_F32
    if dt == torch.bfloat16:
        return SPEC_BF16
    raise TypeError(f"unsupported dtype {dt}")


def _check(rc: int, where: str):
    if rc != 0:
        raise SpecError(rc, where)


def make_desc(q_like: torch.Tensor, k_cache: torch.Tensor, max_prefix_len: int = 0,
              softmax_scale: float = 0.0, k_new: Optional[torch.Tensor] = None,
              plan: Tuple[int, int, int] = (0, 0, 0)) -> AttnDesc:
    """Descriptor from a [B,N,H,D] tensor (q / out), a [B,H_kv,S_cap,D] cache and, for grouped-query heads,
    the [B,N,H_kv,D] k_new (its strides; without it k_new / v_new are taken to be laid out like q).
    plan = the descriptor's launch-plan hints (plan_chunk_keys, plan_balanced_wgs, plan_heads_per_wg)."""
    B, N, H, D = q_like.shape
    Bc, Hkv, S_cap, Dc = k_cache.shape
    if (Bc, Dc) != (B, D) or q_like.stride(3) != 1 or k_cache.stride(3) != 1:
        raise ValueError("q must be [B,N,H,D], cache [B,H_kv,S_cap,D], D contiguous")
    new = (0, 0, 0)
    if k_new is not None:
        if tuple(k_new.shape) != (B, N, Hkv, D) or k_new.stride(3) != 1:
            raise ValueError("k_new / v_new must be [B,N,H_kv,D], D contiguous")
        new = (k_new.stride(0), k_new.stride(1), k_new.stride(2))
    return AttnDesc(B, H, Hkv, D, N, S_cap, _dtype_code(q_like.dtype), int(max_prefix_len),
                    q_like.stride(0), q_like.stride(1), q_like.stride(2),
                    k_cache.stride(0), k_cache.stride(1), k_cache.stride(2), *new, float(softmax_scale),
                    int(plan[0]), int(plan[1]), int(plan[2]))


def _same_layout(a: torch.Tensor, b: torch.Tensor, what: str):
    if a.shape != b.shape or a.stride() != b.stride() or a.dtype != b.dtype:
        raise ValueError(f"{what} must share shape, strides and dtype")


# ------------------------------------------------------------------------------------------------
# entry points
# ------------------------------------------------------------------------------------------------

def spec_kv_append(k_new, v_new, k_cache, v_cache, prefix_len, status=None, stream=None, desc=None):
    _same_layout(k_new, v_new, "k_new and v_new")
    _same_layout(k_cache, v_cache, "k_cache and v_cache")
    d = desc if desc is not None else make_desc(k_new, k_cache)
    _check(load().spec_kv_append(ctypes.byref(d), _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache),
                                 _ptr(prefix_len), _ptr(status), _stream(stream)), "spec_kv_append")


def spec_kv_append_rope(k_new, v_new, k_cache, v_cache, tree_depth, prefix_len, rope_cos, rope_sin, status=None, stream=None):
    """KV append with the rotary embedding applied to K at position prefix_len + tree_depth (in place)."""
    _same_layout(k_cache, v_cache, "k_cache and v_cache")
    _same_layout(k_new, v_new, "k_new and v_new")
    D = k_new.shape[-1]
    for tab in (rope_cos, rope_sin):
        if tab.dtype != torch.float32 or tab.dim() != 2 or tab.shape[1] != D // 2 or not tab.is_contiguous():
            raise ValueError("rope tables must be contiguous float32 [rope_len, D/2]")
    d = make_desc(k_new, k_cache)
    _check(load().spec_kv_append_rope(ctypes.byref(d), _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache),
                                      _ptr(tree_depth), _ptr(prefix_len), _ptr(rope_cos), _ptr(rope_sin),
                                      rope_cos.shape[0], _ptr(status), _stream(stream)), "spec_kv_append_rope")


def spec_qk_rope_append(q, k_new, v_new, k_cache, v_cache, tree_depth, prefix_len, rope_cos, rope_sin, status=None,
                        stream=None, block_table=None):
    """Rotary embedding of q (in place) and of K on its way into the cache, V appended, in one launch. With
    block_table the caches are pools of blocks (paged)."""
    _same_layout(k_cache, v_cache, "k_cache and v_cache")
    _same_layout(k_new, v_new, "k_new and v_new")
    D = k_new.shape[-1]
    for tab in (rope_cos, rope_sin):
        if tab.dtype != torch.float32 or tab.dim() != 2 or tab.shape[1] != D // 2 or not tab.is_contiguous():
            raise ValueError("rope tables must be contiguous float32 [rope_len, D/2]")
    if block_table is None:
        d = make_desc(q, k_cache, k_new=k_new)
        _check(load().spec_qk_rope_append(ctypes.byref(d), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache),
                                          _ptr(tree_depth), _ptr(prefix_len), _ptr(rope_cos), _ptr(rope_sin),
                                          rope_cos.shape[0], _ptr(status), _stream(stream)), "spec_qk_rope_append")
    else:
        d, pg = make_paged_desc(q, k_cache, block_table, k_new=k_new)
        _check(load().spec_qk_rope_append_paged(ctypes.byref(d), ctypes.byref(pg), _ptr(q), _ptr(k_new), _ptr(v_new),
                                                _ptr(k_cache), _ptr(v_cache), _ptr(tree_depth), _ptr(prefix_len),
                                                _ptr(rope_cos), _ptr(rope_sin), rope_cos.shape[0], _ptr(status),
                                                _stream(stream)), "spec_qk_rope_append_paged")


def spec_tree_attention_workspace_bytes(desc: AttnDesc) -> int:
    return int(load().spec_tree_attention_workspace_bytes(ctypes.byref(desc)))


def spec_tree_attention(q, k_cache, v_cache, tree_parent, tree_depth, prefix_len, out=None, workspace=None,
                        status=None, max_prefix_len: int = 0, softmax_scale: float = 0.0, stream=None, desc=None,
                        plan=(0, 0, 0)):
    _same_layout(k_cache, v_cache, "k_cache and v_cache")
    if out is None:
        out = torch.empty_like(q)
    _same_layout(q, out, "q and out")
    d = desc if desc is not None else make_desc(q, k_cache, max_prefix_len, softmax_scale, plan=plan)
    need = spec_tree_attention_workspace_bytes(d)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().spec_tree_attention(ctypes.byref(d), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(tree_parent),
                                      _ptr(tree_depth), _ptr(prefix_len), _ptr(out), _ptr(workspace), ws_bytes,
                                      _ptr(status), _stream(stream)), "spec_tree_attention")
    return out


def spec_tree_attention_append(q, k_new, v_new, k_cache, v_cache, tree_parent, tree_depth, prefix_len, out=None,
                               workspace=None, status=None, max_prefix_len: int = 0, softmax_scale: float = 0.0,
                               stream=None, desc=None, plan=(0, 0, 0)):
    """KV append of the tree rows fused with the tree attention over them."""
    _same_layout(k_cache, v_cache, "k_cache and v_cache")
    _same_layout(k_new, v_new, "k_new and v_new")
    if out is None:
        out = torch.empty_like(q)
    _same_layout(q, out, "q and out")
    d = desc if desc is not None else make_desc(q, k_cache, max_prefix_len, softmax_scale, k_new=k_new, plan=plan)
    need = spec_tree_attention_workspace_bytes(d)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().spec_tree_attention_append(ctypes.byref(d), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache),
                                             _ptr(v_cache), _ptr(tree_parent), _ptr(tree_depth), _ptr(prefix_len),
                                             _ptr(out), _ptr(workspace), ws_bytes, _ptr(status), _stream(stream)),
           "spec_tree_attention_append")
    return out


def spec_tree_attention_append_rope(q, k_new, v_new, k_cache, v_cache, tree_parent, tree_depth, prefix_len, rope_cos,
                                    rope_sin, out=None, workspace=None, status=None, max_prefix_len: int = 0,
                                    softmax_scale: float = 0.0, stream=None, plan=(0, 0, 0), block_table=None):
    """Rotary embedding of q (in registers: q is not modified) and of the new K rows, KV append and tree attention
    in one launch. With block_table the caches are pools of blocks (paged)."""
    _same_layout(k_cache, v_cache, "k_cache and v_cache")
    _same_layout(k_new, v_new, "k_new and v_new")
    D = k_new.shape[-1]
    for tab in (rope_cos, rope_sin):
        if tab.dtype != torch.float32 or tab.dim() != 2 or tab.shape[1] != D // 2 or not tab.is_contiguous():
            raise ValueError("rope tables must be contiguous float32 [rope_len, D/2]")
    if out is None:
        out = torch.empty_like(q)
    _same_layout(q, out, "q and out")
    if block_table is None:
        d = make_desc(q, k_cache, max_prefix_len, softmax_scale, k_new=k_new, plan=plan)
        need = spec_tree_attention_workspace_bytes(d)
    else:
        d, pg = make_paged_desc(q, k_cache, block_table, max_prefix_len, softmax_scale, k_new=k_new, plan=plan)
        need = spec_tree_attention_paged_workspace_bytes(d, pg)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    if block_table is None:
        _check(load().spec_tree_attention_append_rope(ctypes.byref(d), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache),
                                                      _ptr(v_cache), _ptr(tree_parent), _ptr(tree_depth),
                                                      _ptr(prefix_len), _ptr(rope_cos), _ptr(rope_sin), rope_cos.shape[0],
                                                      _ptr(out), _ptr(workspace), ws_bytes, _ptr(status),
                                                      _stream(stream)), "spec_tree_attention_append_rope")
    else:
        _check(load().spec_tree_attention_append_rope_paged(ctypes.byref(d), ctypes.byref(pg), _ptr(q), _ptr(k_new),
                                                            _ptr(v_new), _ptr(k_cache), _ptr(v_cache), _ptr(tree_parent),
                                                            _ptr(tree_depth), _ptr(prefix_len), _ptr(rope_cos),
                                                            _ptr(rope_sin), rope_cos.shape[0], _ptr(out), _ptr(workspace),
                                                            ws_bytes, _ptr(status), _stream(stream)),
               "spec_tree_attention_append_rope_paged")
    return out


def spec_tree_attention_append_static(q, k_new, v_new, k_cache, v_cache, tree_parent, tree_depth, prefix_len, out,
                                      status=None, max_prefix_len: int = 0, softmax_scale: float = 0.0, stream=None,
                                      desc=None, plan=(0, 0, 0)):
    """spec_tree_attention_append on the library's own scratch array: no workspace, and nothing is allocated
    here either (the caller brings `out`)."""
    _same_layout(k_cache, v_cache, "k_cache and v_cache")
    _same_layout(k_new, v_new, "k_new and v_new")
    _same_layout(q, out, "q and out")
    d = desc if desc is not None else make_desc(q, k_cache, max_prefix_len, softmax_scale, k_new=k_new, plan=plan)
    _check(load().spec_tree_attention_append_static(ctypes.byref(d), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache),
                                                    _ptr(v_cache), _ptr(tree_parent), _ptr(tree_depth),
                                                    _ptr(prefix_len), _ptr(out), _ptr(status), _stream(stream)),
           "spec_tree_attention_append_static")
    return out


def spec_verify_greedy(logits, tree_token, tree_parent, Lmax: Optional[int] = None, status=None, stream=None,
                       out: Optional[Tuple[torch.Tensor, ...]] = None):
    """Returns (accepted_path [B,Lmax], accepted_len [B], out_tokens [B,Lmax], node_argmax [B,N])."""
    B, N, V = logits.shape
    Lmax = N if Lmax is None else Lmax
    dev = logits.device
    if out is None:
        out = (torch.empty((B, Lmax), dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int32, device=dev),
               torch.empty((B, Lmax), dtype=torch.int32, device=dev), torch.empty((B, N), dtype=torch.int32, device=dev))
    path, ln, toks, amax = out
    _check(load().spec_verify_greedy(B, N, V, _dtype_code(logits.dtype), _ptr(logits), _ptr(tree_token),
                                     _ptr(tree_parent), Lmax, _ptr(path), _ptr(ln), _ptr(toks), _ptr(amax), None, 0,
                                     _ptr(status), _stream(stream)), "spec_verify_greedy")
    return path, ln, toks, amax


def spec_verify_stochastic_workspace_bytes(B: int, N: int, V: int) -> int:
    return int(load().spec_verify_stochastic_workspace_bytes(B, N, V))


def spec_verify_stochastic(logits, probs_ssm, ssm_row, tree_token, tree_parent, u_accept, u_order, u_final,
                           temperature: float = 1.0, Lmax: Optional[int] = None, workspace=None, status=None,
                           stream=None, out: Optional[Tuple[torch.Tensor, ...]] = None):
    """Returns (accepted_path [B,Lmax], accepted_len [B], out_tokens [B,Lmax])."""
    B, N, V = logits.shape
    Lmax = N if Lmax is None else Lmax
    dev = logits.device
    if probs_ssm.dtype != torch.float32 or (probs_ssm.numel() and probs_ssm.shape[1] != V) or not probs_ssm.is_contiguous():
        raise ValueError("probs_ssm must be contiguous float32 [R,V]")
    need = spec_verify_stochastic_workspace_bytes(B, N, V)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    if out is None:
        out = (torch.empty((B, Lmax), dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int32, device=dev),
               torch.empty((B, Lmax), dtype=torch.int32, device=dev))
    path, ln, toks = out
    _check(load().spec_verify_stochastic(B, N, V, _dtype_code(logits.dtype), _ptr(logits), _ptr(probs_ssm),
                                         probs_ssm.shape[0], _ptr(ssm_row), _ptr(tree_token), _ptr(tree_parent),
                                         _ptr(u_accept), _ptr(u_order), _ptr(u_final), float(temperature), Lmax,
                                         _ptr(path), _ptr(ln), _ptr(toks), _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _ptr(status), _stream(stream)),
           "spec_verify_stochastic")
    return path, ln, toks


def spec_verify_naive_workspace_bytes(B: int, N: int, V: int) -> int:
    return int(load().spec_verify_naive_workspace_bytes(B, N, V))


def spec_verify_naive(logits, tree_token, tree_parent, u_sample, temperature: float = 1.0, Lmax: Optional[int] = None,
                      workspace=None, status=None, stream=None, out: Optional[Tuple[torch.Tensor, ...]] = None):
    """Returns (accepted_path [B,Lmax], accepted_len [B], out_tokens [B,Lmax], node_sample [B,N])."""
    B, N, V = logits.shape
    Lmax = N if Lmax is None else Lmax
    dev = logits.device
    if workspace is None:
        workspace = torch.empty(spec_verify_naive_workspace_bytes(B, N, V), dtype=torch.uint8, device=dev)
    if out is None:
        out = (torch.empty((B, Lmax), dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int32, device=dev),
               torch.empty((B, Lmax), dtype=torch.int32, device=dev), torch.empty((B, N), dtype=torch.int32, device=dev))
    path, ln, toks, samp = out
    _check(load().spec_verify_naive(B, N, V, _dtype_code(logits.dtype), _ptr(logits), _ptr(tree_token),
                                    _ptr(tree_parent), _ptr(u_sample), float(temperature), Lmax, _ptr(path), _ptr(ln),
                                    _ptr(toks), _ptr(samp), _ptr(workspace),
                                    workspace.numel() * workspace.element_size(), _ptr(status), _stream(stream)),
           "spec_verify_naive")
    return path, ln, toks, samp


def spec_tree_expand_topk(ssm_logits, k: int, child_slot, tree_token, status=None, stream=None):
    """tree_token[b, child_slot[f, j]] = j-th most likely token of ssm_logits[b, f, :] (in place)."""
    B, F, V = ssm_logits.shape
    N = tree_token.shape[1]
    if child_slot.dtype != torch.int32 or tuple(child_slot.shape) != (F, k) or not child_slot.is_contiguous():
        raise ValueError("child_slot must be contiguous int32 [F, k]")
    if not ssm_logits.is_contiguous() or not tree_token.is_contiguous() or tree_token.dtype != torch.int32:
        raise ValueError("ssm_logits and tree_token (int32) must be contiguous")
    _check(load().spec_tree_expand_topk(B, F, V, _dtype_code(ssm_logits.dtype), _ptr(ssm_logits), k, _ptr(child_slot), N,
                                        _ptr(tree_token), _ptr(status), _stream(stream)), "spec_tree_expand_topk")
    return tree_token


def spec_tree_merge(in_parent, in_token, in_size, Nout: int, status=None, stream=None, want_node_map: bool = True):
    """Returns (parent [B,Nout], depth, token, ssm, size [B], node_map [B,M,Nin] or None)."""
    B, M, Nin = in_parent.shape
    dev = in_parent.device
    for t in (in_parent, in_token, in_size):
        if t.dtype != torch.int32 or not t.is_contiguous():
            raise ValueError("tree_merge inputs must be contiguous int32")
    mk = lambda *shape: torch.empty(shape, dtype=torch.int32, device=dev)
    par, dep, tok, ssm, size = mk(B, Nout), mk(B, Nout), mk(B, Nout), mk(B, Nout), mk(B)
    node_map = mk(B, M, Nin) if want_node_map else None
    _check(load().spec_tree_merge(B, M, Nin, _ptr(in_parent), _ptr(in_token), _ptr(in_size), Nout, _ptr(par), _ptr(dep),
                                  _ptr(tok), _ptr(ssm), _ptr(size), _ptr(node_map), _ptr(status), _stream(stream)),
           "spec_tree_merge")
    return par, dep, tok, ssm, size, node_map


def spec_kv_commit(k_caches: Sequence[torch.Tensor], v_caches: Sequence[torch.Tensor], accepted_path, accepted_len,
                   prefix_len, N: int, prefix_len_out=None, status=None, stream=None):
    """Commits the accepted path in every layer's cache; returns prefix_len_out [B]."""
    L = len(k_caches)
    k0 = k_caches[0]
    for kc, vc in zip(k_caches, v_caches):
        _same_layout(kc, k0, "all layer caches")
        _same_layout(vc, k0, "all layer caches")
    B, H, S_cap, D = k0.shape
    d = AttnDesc(B, H, H, D, N, S_cap, _dtype_code(k0.dtype), 0, N * H * D, H * D, D,
                 k0.stride(0), k0.stride(1), k0.stride(2), 0, 0, 0, 0.0, 0, 0, 0)
    if prefix_len_out is None:
        prefix_len_out = torch.empty_like(prefix_len)
    arr_t = ctypes.c_void_p * L
    ks = arr_t(*[kc.data_ptr() for kc in k_caches])
    vs = arr_t(*[vc.data_ptr() for vc in v_caches])
    _check(load().spec_kv_commit(ctypes.byref(d), L, ks, vs, _ptr(accepted_path), accepted_path.shape[1],
                                 _ptr(accepted_len), _ptr(prefix_len), _ptr(prefix_len_out), _ptr(status),
                                 _stream(stream)), "spec_kv_commit")
    return prefix_len_out


# ------------------------------------------------------------------------------------------------
# paged caches: pools [n_blocks, H_kv, block_tokens, D] behind a block table [B, max_blocks]
# ------------------------------------------------------------------------------------------------

def make_paged_desc(q_like: torch.Tensor, k_pool: torch.Tensor, block_table: torch.Tensor, max_prefix_len: int = 0,
                    softmax_scale: float = 0.0, k_new: Optional[torch.Tensor] = None,
                    plan: Tuple[int, int, int] = (0, 0, 0)) -> Tuple[AttnDesc, KvPages]:
    """Descriptor and page description from a [B,N,H,D] tensor, a pool and the int32 block table (device).
    The logical capacity of a request is max_blocks * block_tokens rows."""
    B, N, H, D = q_like.shape
    n_blocks, Hkv, bt, Dc = k_pool.shape
    if Dc != D or q_like.stride(3) != 1 or k_pool.stride(3) != 1:
        raise ValueError("q must be [B,N,H,D], pool [n_blocks,H_kv,block_tokens,D], D contiguous")
    if block_table.dtype != torch.int32 or block_table.dim() != 2 or block_table.shape[0] != B or \
            not block_table.is_contiguous():
        raise ValueError("block_table must be contiguous int32 [B, max_blocks]")
    new = (0, 0, 0)
    if k_new is not None:
        if tuple(k_new.shape) != (B, N, Hkv, D) or k_new.stride(3) != 1:
            raise ValueError("k_new / v_new must be [B,N,H_kv,D], D contiguous")
        new = (k_new.stride(0), k_new.stride(1), k_new.stride(2))
    max_blocks = block_table.shape[1]
    d = AttnDesc(B, H, Hkv, D, N, max_blocks * bt, _dtype_code(q_like.dtype), int(max_prefix_len),
                 q_like.stride(0), q_like.stride(1), q_like.stride(2),
                 k_pool.stride(0), k_pool.stride(1), k_pool.stride(2), new[0], new[1], new[2], float(softmax_scale),
                 int(plan[0]), int(plan[1]), int(plan[2]))
    return d, KvPages(block_table.data_ptr(), max_blocks, bt, n_blocks)


def spec_tree_attention_paged_workspace_bytes(desc: AttnDesc, pages: KvPages) -> int:
    return int(load().spec_tree_attention_paged_workspace_bytes(ctypes.byref(desc), ctypes.byref(pages)))


def spec_kv_append_paged(k_new, v_new, k_pool, v_pool, block_table, prefix_len, status=None, stream=None):
    _same_layout(k_new, v_new, "k_new and v_new")
    _same_layout(k_pool, v_pool, "k_pool and v_pool")
    d, pg = make_paged_desc(k_new, k_pool, block_table, k_new=k_new if k_new.shape[2] == k_pool.shape[1] else None)
    _check(load().spec_kv_append_paged(ctypes.byref(d), ctypes.byref(pg), _ptr(k_new), _ptr(v_new), _ptr(k_pool),
                                       _ptr(v_pool), _ptr(prefix_len), _ptr(status), _stream(stream)),
           "spec_kv_append_paged")


def spec_kv_append_rope_paged(k_new, v_new, k_pool, v_pool, block_table, tree_depth, prefix_len, rope_cos, rope_sin,
                              status=None, stream=None):
    _same_layout(k_new, v_new, "k_new and v_new")
    _same_layout(k_pool, v_pool, "k_pool and v_pool")
    D = k_new.shape[-1]
    for tab in (rope_cos, rope_sin):
        if tab.dtype != torch.float32 or tab.dim() != 2 or tab.shape[1] != D // 2 or not tab.is_contiguous():
            raise ValueError("rope tables must be contiguous float32 [rope_len, D/2]")
    d, pg = make_paged_desc(k_new, k_pool, block_table, k_new=k_new)
    _check(load().spec_kv_append_rope_paged(ctypes.byref(d), ctypes.byref(pg), _ptr(k_new), _ptr(v_new), _ptr(k_pool),
                                            _ptr(v_pool), _ptr(tree_depth), _ptr(prefix_len), _ptr(rope_cos),
                                            _ptr(rope_sin), rope_cos.shape[0], _ptr(status), _stream(stream)),
           "spec_kv_append_rope_paged")


def spec_tree_attention_paged(q, k_pool, v_pool, block_table, tree_parent, tree_depth, prefix_len, out=None,
                              workspace=None, status=None, max_prefix_len: int = 0, softmax_scale: float = 0.0,
                              stream=None, k_new=None, v_new=None, plan=(0, 0, 0)):
    """Tree attention over paged caches; with k_new / v_new the KV append of the tree rows is fused in."""
    _same_layout(k_pool, v_pool, "k_pool and v_pool")
    if out is None:
        out = torch.empty_like(q)
    _same_layout(q, out, "q and out")
    d, pg = make_paged_desc(q, k_pool, block_table, max_prefix_len, softmax_scale, k_new=k_new, plan=plan)
    need = spec_tree_attention_paged_workspace_bytes(d, pg)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    if k_new is None:
        _check(load().spec_tree_attention_paged(ctypes.byref(d), ctypes.byref(pg), _ptr(q), _ptr(k_pool), _ptr(v_pool),
                                                _ptr(tree_parent), _ptr(tree_depth), _ptr(prefix_len), _ptr(out),
                                                _ptr(workspace), ws_bytes, _ptr(status), _stream(stream)),
               "spec_tree_attention_paged")
    else:
        _same_layout(k_new, v_new, "k_new and v_new")
        _check(load().spec_tree_attention_append_paged(ctypes.byref(d), ctypes.byref(pg), _ptr(q), _ptr(k_new),
                                                       _ptr(v_new), _ptr(k_pool), _ptr(v_pool), _ptr(tree_parent),
                                                       _ptr(tree_depth), _ptr(prefix_len), _ptr(out), _ptr(workspace),
                                                       ws_bytes, _ptr(status), _stream(stream)),
               "spec_tree_attention_append_paged")
    return out


def spec_tree_attention_append_paged(q, k_new, v_new, k_pool, v_pool, block_table, tree_parent, tree_depth, prefix_len,
                                     **kw):
    return spec_tree_attention_paged(q, k_pool, v_pool, block_table, tree_parent, tree_depth, prefix_len, k_new=k_new,
                                     v_new=v_new, **kw)


def spec_kv_commit_paged(k_pools: Sequence[torch.Tensor], v_pools: Sequence[torch.Tensor], block_table, accepted_path,
                         accepted_len, prefix_len, N: int, prefix_len_out=None, status=None, stream=None):
    """Commits the accepted path in every layer's paged cache; returns prefix_len_out [B]."""
    L = len(k_pools)
    k0 = k_pools[0]
    for kc, vc in zip(k_pools, v_pools):
        _same_layout(kc, k0, "all layer pools")
        _same_layout(vc, k0, "all layer pools")
    n_blocks, H, bt, D = k0.shape
    B, max_blocks = block_table.shape
    d = AttnDesc(B, H, H, D, N, max_blocks * bt, _dtype_code(k0.dtype), 0, N * H * D, H * D, D,
                 k0.stride(0), k0.stride(1), k0.stride(2), 0, 0, 0, 0.0, 0, 0, 0)
    pg = KvPages(block_table.data_ptr(), max_blocks, bt, n_blocks)
    if prefix_len_out is None:
        prefix_len_out = torch.empty_like(prefix_len)
    arr_t = ctypes.c_void_p * L
    ks = arr_t(*[kc.data_ptr() for kc in k_pools])
    vs = arr_t(*[vc.data_ptr() for vc in v_pools])
    _check(load().spec_kv_commit_paged(ctypes.byref(d), ctypes.byref(pg), L, ks, vs, _ptr(accepted_path),
                                       accepted_path.shape[1], _ptr(accepted_len), _ptr(prefix_len), _ptr(prefix_len_out),
                                       _ptr(status), _stream(stream)), "spec_kv_commit_paged")
    return prefix_len_out


# ------------------------------------------------------------------------------------------------
# LM head in front of the greedy verifier
# ------------------------------------------------------------------------------------------------

def spec_lm_head_argmax_workspace_bytes(M: int, V: int) -> int:
    return int(load().spec_lm_head_argmax_workspace_bytes(M, V))


def _lm_head_args(hidden, weight):
    if hidden.dtype != torch.bfloat16 or weight.dtype != torch.bfloat16 or hidden.dim() != 2 or weight.dim() != 2 or \
            hidden.shape[1] != weight.shape[1] or not hidden.is_contiguous() or not weight.is_contiguous():
        raise ValueError("hidden [M,K] and weight [V,K] must be contiguous bf16 with the same K")
    return hidden.shape[0], hidden.shape[1], weight.shape[0]


def spec_lm_head_argmax(hidden, weight, want_max: bool = False, workspace=None, stream=None):
    """(node_argmax [M] int32, node_max [M] float32 or None) of hidden . weight^T without the logits in memory."""
    M, K, V = _lm_head_args(hidden, weight)
    arg = torch.empty(M, dtype=torch.int32, device=hidden.device)
    mx = torch.empty(M, dtype=torch.float32, device=hidden.device) if want_max else None
    if workspace is None:
        workspace = torch.empty(max(spec_lm_head_argmax_workspace_bytes(M, V), 256), dtype=torch.uint8, device=hidden.device)
    _check(load().spec_lm_head_argmax(M, K, V, _ptr(hidden), _ptr(weight), _ptr(arg), _ptr(mx), _ptr(workspace),
                                      workspace.numel(), _stream(stream)), "spec_lm_head_argmax")
    return arg, mx


def spec_verify_greedy_lm_head(hidden, weight, tree_token, tree_parent, Lmax: Optional[int] = None, workspace=None,
                               status=None, stream=None, out=None):
    """Greedy verification from the LLM's last hidden states [B*N, K] and its output projection [V, K].
    Returns (accepted_path [B,Lmax], accepted_len [B], out_tokens [B,Lmax], node_argmax [B,N])."""
    M, K, V = _lm_head_args(hidden, weight)
    B, N = tree_token.shape
    if M != B * N:
        raise ValueError("hidden must have B*N rows")
    Lmax = N if Lmax is None else Lmax
    dev = hidden.device
    if out is None:
        out = (torch.empty((B, Lmax), dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int32, device=dev),
               torch.empty((B, Lmax), dtype=torch.int32, device=dev), torch.empty((B, N), dtype=torch.int32, device=dev))
    if workspace is None:
        workspace = torch.empty(max(spec_lm_head_argmax_workspace_bytes(M, V), 256), dtype=torch.uint8, device=dev)
    _check(load().spec_verify_greedy_lm_head(B, N, K, V, _ptr(hidden), _ptr(weight), _ptr(tree_token), _ptr(tree_parent),
                                             Lmax, _ptr(out[0]), _ptr(out[1]), _ptr(out[2]), _ptr(out[3]),
                                             _ptr(workspace), workspace.numel(), _ptr(status), _stream(stream)),
           "spec_verify_greedy_lm_head")
    return out


def spec_lm_head_logits_stats(hidden, weight, temperature: float = 1.0, workspace=None, stream=None, out=None):
    """One pass over the output projection: (logits [M,V] bf16, node_argmax [M] int32, node_max [M], node_sumexp [M]
    float32), the statistics being those of the rounded logits. `out`: those four tensors, brought by the caller."""
    M, K, V = _lm_head_args(hidden, weight)
    dev = hidden.device
    if out is not None:
        logits, arg, mx, se = out
    else:
        logits = torch.empty((M, V), dtype=torch.bfloat16, device=dev)
        arg = torch.empty(M, dtype=torch.int32, device=dev)
        mx, se = torch.empty(M, dtype=torch.float32, device=dev), torch.empty(M, dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = torch.empty(max(int(load().spec_lm_head_logits_stats_workspace_bytes(M, V)), 256), dtype=torch.uint8,
                                device=dev)
    _check(load().spec_lm_head_logits_stats(M, K, V, _ptr(hidden), _ptr(weight), float(temperature), _ptr(logits), _ptr(arg),
                                            _ptr(mx), _ptr(se), _ptr(workspace), workspace.numel(), _stream(stream)),
           "spec_lm_head_logits_stats")
    return logits, arg, mx, se


def spec_verify_stochastic_stats(logits, node_max, node_sumexp, probs_ssm, ssm_row, tree_token, tree_parent, u_accept,
                                 u_order, u_final, temperature: float = 1.0, Lmax: Optional[int] = None, workspace=None,
                                 status=None, stream=None, out: Optional[Tuple[torch.Tensor, ...]] = None):
    """spec_verify_stochastic from per-node (max, sum of exponentials) the caller already has.
    Returns (accepted_path [B,Lmax], accepted_len [B], out_tokens [B,Lmax])."""
    B, N, V = logits.shape
    Lmax = N if Lmax is None else Lmax
    dev = logits.device
    if probs_ssm.dtype != torch.float32 or (probs_ssm.numel() and probs_ssm.shape[1] != V) or not probs_ssm.is_contiguous():
        raise ValueError("probs_ssm must be contiguous float32 [R,V]")
    for t_ in (node_max, node_sumexp):
        if t_.dtype != torch.float32 or t_.numel() != B * N or not t_.is_contiguous():
            raise ValueError("node_max / node_sumexp must be contiguous float32 with B*N entries")
    if workspace is None:
        workspace = torch.empty(int(load().spec_verify_stochastic_stats_workspace_bytes(B, V)), dtype=torch.uint8, device=dev)
    if out is None:
        out = (torch.empty((B, Lmax), dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int32, device=dev),
               torch.empty((B, Lmax), dtype=torch.int32, device=dev))
    path, ln, toks = out
    _check(load().spec_verify_stochastic_stats(B, N, V, _dtype_code(logits.dtype), _ptr(logits), _ptr(node_max),
                                               _ptr(node_sumexp), _ptr(probs_ssm), probs_ssm.shape[0], _ptr(ssm_row),
                                               _ptr(tree_token), _ptr(tree_parent), _ptr(u_accept), _ptr(u_order),
                                               _ptr(u_final), float(temperature), Lmax, _ptr(path), _ptr(ln), _ptr(toks),
                                               _ptr(workspace), workspace.numel(), _ptr(status), _stream(stream)),
           "spec_verify_stochastic_stats")
    return path, ln, toks
