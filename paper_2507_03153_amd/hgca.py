"""Thin ctypes binding of libhgca.so (the C ABI declared in include/hgca.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  Tensors are torch tensors on the GPU; torch is used for device
memory and streams.  There is no CPU fallback: without the built library, or
with a tensor that is not on a GPU, the calls raise.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch  # noqa: F401  (loads the HIP runtime the library binds to; must precede CDLL)

F32, BF16 = 0, 1
OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_DEVICE = 0, -1, -2, -3, -4

# HGCA_LIB names another build of the same library (tuning experiments); the default is the in-tree one
_LIB_PATH = os.environ.get("HGCA_LIB") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "libhgca.so")

EXPORTS = ("hgca_status_string", "hgca_workspace_bytes", "hgca_dense_window_attn",
           "hgca_pool_scores", "hgca_select_salient", "hgca_sparse_attn", "hgca_lse_merge_splits", "hgca_lse_merge",
           "hgca_dense_window_attn_weights", "hgca_maw_update", "hgca_threshold_select", "hgca_select_topk",
           "hgca_kv_append", "hgca_kv_evict", "hgca_append_workspace_bytes", "hgca_append_attn",
           "hgca_append_tiers_workspace_bytes", "hgca_append_attn_tiers", "hgca_append_weights_tiers",
           "hgca_append_weights", "hgca_dense_window_attn_maw", "hgca_select_salient_grouped", "hgca_union_lists",
           "hgca_sparse_attn_grouped", "hgca_hybrid_decode_step", "hgca_ctx_compact",
           "hgca_managed_decode_step", "hgca_dense_window_attn_static", "hgca_hybrid_decode_step_selected", "hgca_kv_append_tokens",
           "hgca_managed_append_workspace_bytes", "hgca_managed_append_step")
STATIC_SCRATCH_BYTES = 16 << 20                  # HGCA_STATIC_SCRATCH_BYTES of include/hgca.h
CACHE_WINDOW_FULL, CACHE_CONTEXT_FULL, CACHE_LIST_FULL = 1, 2, 4


class Shape(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("sm_scale", ctypes.c_float)]


class KvView(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p), ("seq_lens", ctypes.c_void_p),
                ("block_table", ctypes.c_void_p), ("cap", ctypes.c_int32), ("block_size", ctypes.c_int32),
                ("max_blocks", ctypes.c_int32), ("first_block", ctypes.c_void_p)]


class CacheState(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("k_blocks", "v_blocks", "block_table", "first_win_block", "win_lens",
                                               "pool_lens", "a_maw", "ctx_idx", "ctx_cnt", "a_evicted", "plan",
                                               "status")] + \
               [(n, ctypes.c_int32) for n in ("block_size", "max_blocks", "win_blocks", "k_max", "pool_cap",
                                               "win_cap_blocks")]


class HgcaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built (python -m paper_2507_03153_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(f"{_LIB_PATH} is missing: build it with "
                                    "`python -m paper_2507_03153_amd.build`; there is no fallback path")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        ps, pk = ctypes.POINTER(Shape), ctypes.POINTER(KvView)
        L.hgca_status_string.restype = ctypes.c_char_p
        L.hgca_status_string.argtypes = [ctypes.c_int]
        L.hgca_workspace_bytes.restype = sz
        L.hgca_workspace_bytes.argtypes = [ps, i32, i32, i32]
        L.hgca_dense_window_attn.restype = ctypes.c_int
        L.hgca_dense_window_attn.argtypes = [ps, vp, pk, vp, vp, vp, sz, vp]
        L.hgca_dense_window_attn_static.restype = ctypes.c_int
        L.hgca_dense_window_attn_static.argtypes = [ps, vp, pk, vp, vp, vp]
        L.hgca_pool_scores.restype = ctypes.c_int
        L.hgca_pool_scores.argtypes = [ps, vp, pk, vp, vp]
        L.hgca_select_salient.restype = ctypes.c_int
        L.hgca_select_salient.argtypes = [ps, vp, pk, vp, i32, i32, vp, vp, vp, vp, sz, vp]
        L.hgca_sparse_attn.restype = ctypes.c_int
        L.hgca_sparse_attn.argtypes = [ps, vp, pk, vp, vp, i32, vp, vp, vp, vp, sz, vp]
        L.hgca_lse_merge_splits.restype = ctypes.c_int
        L.hgca_lse_merge_splits.argtypes = [ps, i32, vp, sz, i32, vp, sz, vp, i32, vp, vp]
        L.hgca_lse_merge.restype = ctypes.c_int
        L.hgca_lse_merge.argtypes = [ps, vp, vp, vp, vp, vp, i32, vp, vp]
        L.hgca_dense_window_attn_weights.restype = ctypes.c_int
        L.hgca_dense_window_attn_weights.argtypes = [ps, vp, pk, vp, vp, vp, vp, sz, vp]
        L.hgca_select_topk.restype = ctypes.c_int
        L.hgca_select_topk.argtypes = [ps, vp, vp, i32, vp, i32, i32, vp, vp, vp, vp]
        L.hgca_append_workspace_bytes.restype = sz
        L.hgca_append_workspace_bytes.argtypes = [ps, i32, i32]
        L.hgca_append_attn.restype = ctypes.c_int
        L.hgca_append_attn.argtypes = [ps, vp, i32, pk, i32, vp, vp, vp, sz, vp]
        L.hgca_append_weights_tiers.restype = ctypes.c_int
        L.hgca_append_weights_tiers.argtypes = [ps, vp, i32, pk, pk, i32, vp, vp, vp, vp, vp]
        L.hgca_append_tiers_workspace_bytes.restype = ctypes.c_size_t
        L.hgca_append_tiers_workspace_bytes.argtypes = [ps, i32, i32, i32]
        L.hgca_append_attn_tiers.restype = ctypes.c_int
        L.hgca_append_attn_tiers.argtypes = [ps, vp, i32, pk, pk, i32, vp, vp, vp, vp, vp, sz, vp]
        L.hgca_append_weights.restype = ctypes.c_int
        L.hgca_append_weights.argtypes = [ps, vp, i32, pk, i32, vp, vp, vp]
        L.hgca_kv_append.restype = ctypes.c_int
        L.hgca_kv_append.argtypes = [ps, ctypes.POINTER(CacheState), vp, vp, vp, vp]
        L.hgca_kv_append_tokens.restype = ctypes.c_int
        L.hgca_kv_append_tokens.argtypes = [ps, ctypes.POINTER(CacheState), vp, vp, i32, vp, vp]
        L.hgca_managed_append_workspace_bytes.restype = sz
        L.hgca_managed_append_workspace_bytes.argtypes = [ps, ctypes.POINTER(CacheState), i32]
        L.hgca_managed_append_step.restype = ctypes.c_int
        L.hgca_managed_append_step.argtypes = [ps, ctypes.POINTER(CacheState), vp, vp, vp, i32, ctypes.c_float,
                                               ctypes.c_double, i32, vp, vp, vp, vp, vp, sz, vp]
        L.hgca_kv_evict.restype = ctypes.c_int
        L.hgca_kv_evict.argtypes = [ps, ctypes.POINTER(CacheState), ctypes.c_double, vp]
        L.hgca_select_salient_grouped.restype = ctypes.c_int
        L.hgca_select_salient_grouped.argtypes = [ps, vp, pk, vp, i32, i32, vp, vp, vp, sz, vp]
        L.hgca_union_lists.restype = ctypes.c_int
        L.hgca_union_lists.argtypes = [ps, vp, vp, i32, i32, vp, vp, i32, vp, vp]
        L.hgca_sparse_attn_grouped.restype = ctypes.c_int
        L.hgca_sparse_attn_grouped.argtypes = [ps, vp, pk, vp, vp, i32, vp, vp, vp, sz, vp]
        L.hgca_managed_decode_step.restype = ctypes.c_int
        L.hgca_managed_decode_step.argtypes = [ps, ctypes.POINTER(CacheState), vp, vp, vp, ctypes.c_float,
                                               ctypes.c_double, vp, vp, i32, vp, vp, sz, vp, sz, vp]
        L.hgca_ctx_compact.restype = ctypes.c_int
        L.hgca_ctx_compact.argtypes = [ps, pk, vp, vp, i32, vp, vp, vp, i32, vp, vp]
        L.hgca_hybrid_decode_step.restype = ctypes.c_int
        L.hgca_hybrid_decode_step.argtypes = [ps, vp, pk, pk, vp, i32, i32, vp, vp, vp, i32, vp, vp, sz, vp, sz, vp]
        L.hgca_hybrid_decode_step_selected.restype = ctypes.c_int
        L.hgca_hybrid_decode_step_selected.argtypes = [ps, vp, pk, pk, vp, vp, i32, vp, vp, i32, vp, vp, sz, vp, sz, vp]
        L.hgca_dense_window_attn_maw.restype = ctypes.c_int
        L.hgca_dense_window_attn_maw.argtypes = [ps, vp, pk, vp, vp, vp, vp, i32, ctypes.c_float, vp, sz, vp]
        L.hgca_maw_update.restype = ctypes.c_int
        L.hgca_maw_update.argtypes = [ps, vp, vp, vp, i32, i32, ctypes.c_float, vp]
        L.hgca_threshold_select.restype = ctypes.c_int
        L.hgca_threshold_select.argtypes = [ps, vp, vp, i32, vp, i32, ctypes.c_double, i32, vp, vp, vp, vp]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().hgca_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != OK:
        raise HgcaError(status, where)


@dataclass
class Tier:
    """One KV tier on the GPU.  k/v: contiguous [B,Hkv,cap,d] or paged [n_blocks,Hkv,bs,d]."""
    k: torch.Tensor
    v: Optional[torch.Tensor]
    cap: int
    seq_lens: Optional[torch.Tensor] = None      # int32 [B]
    block_table: Optional[torch.Tensor] = None   # int32 [B,max_blocks]
    block_size: int = 0
    first_block: Optional[torch.Tensor] = None   # int32 [B]: the tier starts at this entry of its table row

    def view(self) -> KvView:
        for t in (self.k, self.v, self.seq_lens, self.block_table, self.first_block):
            if t is not None:
                _require_gpu(t)
        mb = 0 if self.block_table is None else int(self.block_table.shape[1])
        return KvView(_ptr(self.k), _ptr(self.v), _ptr(self.seq_lens), _ptr(self.block_table),
                      int(self.cap), int(self.block_size), mb, _ptr(self.first_block))


def _require_gpu(t: torch.Tensor) -> None:
    if not t.is_cuda:
        raise ValueError("libhgca takes GPU tensors only (no CPU path exists)")
    if not t.is_contiguous():
        raise ValueError("libhgca takes contiguous tensors")


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    return ctypes.c_void_p(t.data_ptr()) if t.numel() else ctypes.c_void_p(t.data_ptr() or 0)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"q/K/V must be float32 or bfloat16, got {t.dtype}")


def make_shape(q: torch.Tensor, n_kv_heads: int, sm_scale: float) -> Shape:
    _require_gpu(q)
    B, Hq, d = q.shape
    return Shape(_dtype_code(q), B, Hq, int(n_kv_heads), d, float(sm_scale))


def _stream(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def workspace_bytes(shape: Shape, max_window: int, max_pool: int, k_max: int) -> int:
    return int(lib().hgca_workspace_bytes(ctypes.byref(shape), int(max_window), int(max_pool), int(k_max)))


def alloc_workspace(shape: Shape, max_window: int, max_pool: int, k_max: int, device) -> torch.Tensor:
    n = workspace_bytes(shape, max_window, max_pool, k_max)
    if n == 0:
        raise HgcaError(ERR_INVALID_ARG, "hgca_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def dense_window_attn(shape: Shape, q, window: Tier, o_out, lse_out, ws, stream=None) -> None:
    """o_out = lse_out = None defers the result: the split partials stay in ws for lse_merge_splits."""
    for t in (q, ws) + (() if o_out is None else (o_out, lse_out)):
        _require_gpu(t)
    kv = window.view()
    _check(lib().hgca_dense_window_attn(ctypes.byref(shape), _ptr(q), ctypes.byref(kv), _ptr(o_out), _ptr(lse_out),
                                        _ptr(ws), ws.numel(), _stream(stream)), "hgca_dense_window_attn")


def dense_window_attn_static(shape: Shape, q, window: Tier, o_out, lse_out, stream=None) -> None:
    """dense_window_attn without a workspace: the split partials live in the library's own device array."""
    for t in (q, o_out, lse_out):
        _require_gpu(t)
    kv = window.view()
    _check(lib().hgca_dense_window_attn_static(ctypes.byref(shape), _ptr(q), ctypes.byref(kv), _ptr(o_out),
                                               _ptr(lse_out), _stream(stream)), "hgca_dense_window_attn_static")


def pool_scores(shape: Shape, q, pool: Tier, scores_out, stream=None) -> None:
    for t in (q, scores_out):
        _require_gpu(t)
    kv = pool.view()
    _check(lib().hgca_pool_scores(ctypes.byref(shape), _ptr(q), ctypes.byref(kv), _ptr(scores_out), _stream(stream)),
           "hgca_pool_scores")


def select_salient(shape: Shape, q, pool: Tier, k, k_max: int, idx_out, cnt_out, ws, stream=None,
                   sel_scores_out=None) -> None:
    """k: int (uniform budget) or int32 GPU tensor [B] (per-sequence budgets)."""
    for t in (q, idx_out, cnt_out, ws) + (() if sel_scores_out is None else (sel_scores_out,)):
        _require_gpu(t)
    kv = pool.view()
    if isinstance(k, torch.Tensor):
        _require_gpu(k)
        k_ptr, k_uni = _ptr(k), 0
    else:
        k_ptr, k_uni = None, int(k)
    _check(lib().hgca_select_salient(ctypes.byref(shape), _ptr(q), ctypes.byref(kv), k_ptr, k_uni, int(k_max),
                                     _ptr(idx_out), _ptr(cnt_out), _ptr(sel_scores_out), _ptr(ws), ws.numel(),
                                     _stream(stream)),
           "hgca_select_salient")


def sparse_attn(shape: Shape, q, pool: Tier, idx, cnt, k_max: int, o_out, lse_out, ws, stream=None,
                sel_scores=None) -> None:
    """sel_scores: scores of the listed entries for this q (from select_salient); K is then not re-read."""
    for t in (q, idx, cnt, ws) + (() if sel_scores is None else (sel_scores,)) + \
            (() if o_out is None else (o_out, lse_out)):
        _require_gpu(t)
    kv = pool.view()
    _check(lib().hgca_sparse_attn(ctypes.byref(shape), _ptr(q), ctypes.byref(kv), _ptr(idx), _ptr(cnt), int(k_max),
                                  _ptr(sel_scores), _ptr(o_out), _ptr(lse_out), _ptr(ws), ws.numel(), _stream(stream)),
           "hgca_sparse_attn")


def lse_merge_splits(shape: Shape, window_cap: int, ws_dense, k_max: int, ws_sparse, o_out, lse_out=None,
                     stream=None) -> None:
    """Folds the deferred split partials of a dense and a sparse call into the final O (and lse)."""
    for t in (o_out,) + tuple(x for x in (ws_dense, ws_sparse, lse_out) if x is not None):
        _require_gpu(t)
    nb = lambda w: 0 if w is None else w.numel()
    _check(lib().hgca_lse_merge_splits(ctypes.byref(shape), int(window_cap), _ptr(ws_dense), nb(ws_dense), int(k_max),
                                       _ptr(ws_sparse), nb(ws_sparse), _ptr(o_out), _dtype_code(o_out),
                                       _ptr(lse_out), _stream(stream)), "hgca_lse_merge_splits")


def lse_merge(shape: Shape, o_a, lse_a, o_b, lse_b, o_out, lse_out=None, stream=None) -> None:
    for t in (o_a, lse_a, o_b, lse_b, o_out):
        _require_gpu(t)
    _check(lib().hgca_lse_merge(ctypes.byref(shape), _ptr(o_a), _ptr(lse_a), _ptr(o_b), _ptr(lse_b), _ptr(o_out),
                                _dtype_code(o_out), _ptr(lse_out), _stream(stream)), "hgca_lse_merge")


def dense_window_attn_weights(shape: Shape, q, window: Tier, o_out, lse_out, a_out, ws, stream=None) -> None:
    """Dense window attention that also returns the window's softmax weights a_out [B,Hq,cap] (fp32)."""
    for t in (q, ws, o_out, lse_out, a_out):
        _require_gpu(t)
    kv = window.view()
    _check(lib().hgca_dense_window_attn_weights(ctypes.byref(shape), _ptr(q), ctypes.byref(kv), _ptr(o_out),
                                                _ptr(lse_out), _ptr(a_out), _ptr(ws), ws.numel(), _stream(stream)),
           "hgca_dense_window_attn_weights")


def maw_update(shape: Shape, a_maw, a_gpu, seq_lens, cap: int, n_new: int, alpha: float, stream=None) -> None:
    """a_maw <- (1 - alpha) a_maw + alpha a_gpu in place; the last n_new valid entries take a_gpu."""
    for t in (a_maw, a_gpu) + (() if seq_lens is None else (seq_lens,)):
        _require_gpu(t)
    _check(lib().hgca_maw_update(ctypes.byref(shape), _ptr(a_maw), _ptr(a_gpu), _ptr(seq_lens), int(cap), int(n_new),
                                 float(alpha), _stream(stream)), "hgca_maw_update")


def threshold_select(shape: Shape, weights, seq_lens, cap: int, size, beta: float, k_max: int, idx_out, cnt_out,
                     w_norm_out=None, stream=None) -> None:
    """size: int (uniform) or int32 GPU tensor [B]: the number of entries the weights were taken over."""
    for t in (weights, idx_out, cnt_out) + tuple(x for x in (seq_lens, w_norm_out) if x is not None):
        _require_gpu(t)
    if isinstance(size, torch.Tensor):
        _require_gpu(size)
        size_ptr, size_uni = _ptr(size), 0
    else:
        size_ptr, size_uni = None, int(size)
    _check(lib().hgca_threshold_select(ctypes.byref(shape), _ptr(weights), _ptr(seq_lens), int(cap), size_ptr,
                                       size_uni, float(beta), int(k_max), _ptr(idx_out), _ptr(cnt_out),
                                       _ptr(w_norm_out), _stream(stream)), "hgca_threshold_select")


def select_topk(shape: Shape, scores, seq_lens, cap: int, k, k_max: int, idx_out, cnt_out, sel_scores_out=None,
                stream=None) -> None:
    """Per-head top-k of caller-supplied fp32 scores [B,Hq,cap]; k: int or int32 GPU tensor [B]."""
    for t in (scores, idx_out, cnt_out) + tuple(x for x in (seq_lens, sel_scores_out) if x is not None):
        _require_gpu(t)
    if isinstance(k, torch.Tensor):
        _require_gpu(k)
        k_ptr, k_uni = _ptr(k), 0
    else:
        k_ptr, k_uni = None, int(k)
    _check(lib().hgca_select_topk(ctypes.byref(shape), _ptr(scores), _ptr(seq_lens), int(cap), k_ptr, k_uni, int(k_max),
                                  _ptr(idx_out), _ptr(cnt_out), _ptr(sel_scores_out), _stream(stream)),
           "hgca_select_topk")


def kv_append(shape: Shape, cache: CacheState, k_in, v_in, active=None, stream=None) -> None:
    """Writes the new token's K/V rows [B,Hkv,d] at the end of every (active) sequence's window."""
    for t in (k_in, v_in) + (() if active is None else (active,)):
        _require_gpu(t)
    _check(lib().hgca_kv_append(ctypes.byref(shape), ctypes.byref(cache), _ptr(k_in), _ptr(v_in), _ptr(active),
                                _stream(stream)), "hgca_kv_append")


def kv_append_tokens(shape: Shape, cache: CacheState, k_in, v_in, active=None, stream=None) -> None:
    """Writes a prompt's K/V rows [B,N,Hkv,d] behind every (active) sequence's window."""
    for t in (k_in, v_in) + (() if active is None else (active,)):
        _require_gpu(t)
    _check(lib().hgca_kv_append_tokens(ctypes.byref(shape), ctypes.byref(cache), _ptr(k_in), _ptr(v_in),
                                       int(k_in.shape[1]), _ptr(active), _stream(stream)), "hgca_kv_append_tokens")


def managed_append_workspace(shape: Shape, cache: CacheState, n_q: int, device) -> torch.Tensor:
    n = int(lib().hgca_managed_append_workspace_bytes(ctypes.byref(shape), ctypes.byref(cache), int(n_q)))
    if n == 0:
        raise HgcaError(ERR_INVALID_ARG, "hgca_managed_append_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def managed_append_step(shape: Shape, cache: CacheState, q, k_in, v_in, alpha: float, beta: float, a_gpu, a_cpu,
                        o_out, lse_out, ws, stream=None, one_part_p: bool = False) -> None:
    """One append turn over the managed cache (insert N tokens, attend to window and complete pool, merge, moving
    averages, re-evaluation of the salient lists, eviction) in one call.  q [B,N,Hq,d], k_in / v_in [B,N,Hkv,d]."""
    for t in (q, k_in, v_in, a_gpu, o_out, lse_out, ws) + (() if a_cpu is None else (a_cpu,)):
        _require_gpu(t)
    _check(lib().hgca_managed_append_step(ctypes.byref(shape), ctypes.byref(cache), _ptr(q), _ptr(k_in), _ptr(v_in),
                                          int(q.shape[1]), float(alpha), float(beta),
                                          APPEND_ONE_PART_P if one_part_p else 0, _ptr(a_gpu), _ptr(a_cpu), _ptr(o_out),
                                          _ptr(lse_out), _ptr(ws), ws.numel(), _stream(stream)),
           "hgca_managed_append_step")


def kv_evict(shape: Shape, cache: CacheState, beta: float, stream=None) -> None:
    """Sequences whose window reached l_max hand their oldest block(s) to the pool and sparsify them."""
    _check(lib().hgca_kv_evict(ctypes.byref(shape), ctypes.byref(cache), float(beta), _stream(stream)),
           "hgca_kv_evict")


def append_workspace(shape: Shape, n_q: int, max_tokens: int, device) -> torch.Tensor:
    n = int(lib().hgca_append_workspace_bytes(ctypes.byref(shape), int(n_q), int(max_tokens)))
    if n == 0:
        raise HgcaError(ERR_INVALID_ARG, "hgca_append_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


APPEND_CAUSAL_TAIL, APPEND_ONE_PART_P = 1, 2


def append_attn(shape: Shape, q, tier: Tier, causal_tail: bool, o_out, lse_out, ws, stream=None,
                one_part_p: bool = False) -> None:
    """q [B,N,Hq,d] bf16; o_out [B,N,Hq,d], lse_out [B,N,Hq] fp32."""
    for t in (q, o_out, lse_out, ws):
        _require_gpu(t)
    kv = tier.view()
    flags = (APPEND_CAUSAL_TAIL if causal_tail else 0) | (APPEND_ONE_PART_P if one_part_p else 0)
    _check(lib().hgca_append_attn(ctypes.byref(shape), _ptr(q), int(q.shape[1]), ctypes.byref(kv), flags,
                                  _ptr(o_out), _ptr(lse_out), _ptr(ws), ws.numel(), _stream(stream)),
           "hgca_append_attn")


def append_tiers_workspace(shape: Shape, n_q: int, window_cap: int, pool_cap: int, device) -> torch.Tensor:
    n = int(lib().hgca_append_tiers_workspace_bytes(ctypes.byref(shape), int(n_q), int(window_cap), int(pool_cap)))
    if n == 0:
        raise HgcaError(ERR_INVALID_ARG, "hgca_append_tiers_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def append_attn_tiers(shape: Shape, q, window: Tier, pool: Tier, o_out, lse_out, ws, lse_window_out=None,
                      lse_pool_out=None, causal_tail: bool = True, one_part_p: bool = False, stream=None) -> None:
    """Attention of q [B,N,Hq,d] bf16 over the window (causal among its last N tokens) and over the whole pool, merged:
    o_out [B,N,Hq,d], lse_out [B,N,Hq] fp32; the per-tier lse rows are optional outputs."""
    for t in (q, o_out, lse_out, ws):
        _require_gpu(t)
    for t in (lse_window_out, lse_pool_out):
        if t is not None:
            _require_gpu(t)
    kw, kp = window.view(), pool.view()
    flags = (APPEND_CAUSAL_TAIL if causal_tail else 0) | (APPEND_ONE_PART_P if one_part_p else 0)
    _check(lib().hgca_append_attn_tiers(ctypes.byref(shape), _ptr(q), int(q.shape[1]), ctypes.byref(kw), ctypes.byref(kp),
                                        flags, _ptr(o_out), _ptr(lse_out),
                                        _ptr(lse_window_out) if lse_window_out is not None else None,
                                        _ptr(lse_pool_out) if lse_pool_out is not None else None,
                                        _ptr(ws), ws.numel(), _stream(stream)), "hgca_append_attn_tiers")


def append_weights(shape: Shape, q, tier: Tier, causal_tail: bool, lse, a_out, stream=None) -> None:
    """Query-averaged softmax weights of the tier, a_out [B,Hq,cap] fp32; lse from append_attn on the same tier."""
    for t in (q, lse, a_out):
        _require_gpu(t)
    kv = tier.view()
    _check(lib().hgca_append_weights(ctypes.byref(shape), _ptr(q), int(q.shape[1]), ctypes.byref(kv), int(causal_tail),
                                     _ptr(lse), _ptr(a_out), _stream(stream)), "hgca_append_weights")


def append_weights_tiers(shape: Shape, q, window: Tier, pool: Tier, lse_window, lse_pool, a_gpu, a_cpu,
                         causal_tail: bool = True, stream=None) -> None:
    """Query-averaged weights of window and pool in one launch (bf16); the lse rows from append_attn_tiers."""
    for t in (q, lse_window, lse_pool, a_gpu, a_cpu):
        _require_gpu(t)
    kw, kp = window.view(), pool.view()
    _check(lib().hgca_append_weights_tiers(ctypes.byref(shape), _ptr(q), int(q.shape[1]), ctypes.byref(kw), ctypes.byref(kp),
                                           int(causal_tail), _ptr(lse_window), _ptr(lse_pool), _ptr(a_gpu), _ptr(a_cpu),
                                           _stream(stream)), "hgca_append_weights_tiers")


def dense_window_attn_maw(shape: Shape, q, window: Tier, o_out, lse_out, a_out, a_maw, n_new: int, alpha: float, ws,
                          stream=None) -> None:
    """dense_window_attn_weights and maw_update(a_maw, a_out, ...) in one call."""
    for t in (q, ws, o_out, lse_out, a_out, a_maw):
        _require_gpu(t)
    kv = window.view()
    _check(lib().hgca_dense_window_attn_maw(ctypes.byref(shape), _ptr(q), ctypes.byref(kv), _ptr(o_out), _ptr(lse_out),
                                            _ptr(a_out), _ptr(a_maw), int(n_new), float(alpha), _ptr(ws), ws.numel(),
                                            _stream(stream)), "hgca_dense_window_attn_maw")


def select_salient_grouped(shape: Shape, q, pool: Tier, k, k_max: int, idx_out, cnt_out, ws, stream=None) -> None:
    """One list per KV head (idx_out [B,Hkv,k_max], cnt_out [B,Hkv]): top-k of the maximum score over the group."""
    for t in (q, idx_out, cnt_out, ws):
        _require_gpu(t)
    kv = pool.view()
    if isinstance(k, torch.Tensor):
        _require_gpu(k)
        k_ptr, k_uni = _ptr(k), 0
    else:
        k_ptr, k_uni = None, int(k)
    _check(lib().hgca_select_salient_grouped(ctypes.byref(shape), _ptr(q), ctypes.byref(kv), k_ptr, k_uni, int(k_max),
                                             _ptr(idx_out), _ptr(cnt_out), _ptr(ws), ws.numel(), _stream(stream)),
           "hgca_select_salient_grouped")


def union_lists(shape: Shape, idx, cnt, k_max: int, n_positions: int, idx_out, cnt_out, k_max_out: int, status=None,
                stream=None) -> None:
    """Per KV head, the ascending union of its heads' lists."""
    for t in (idx, cnt, idx_out, cnt_out) + (() if status is None else (status,)):
        _require_gpu(t)
    _check(lib().hgca_union_lists(ctypes.byref(shape), _ptr(idx), _ptr(cnt), int(k_max), int(n_positions), _ptr(idx_out),
                                  _ptr(cnt_out), int(k_max_out), _ptr(status), _stream(stream)), "hgca_union_lists")


def sparse_attn_grouped(shape: Shape, q, pool: Tier, idx, cnt, k_max: int, o_out, lse_out, ws, stream=None) -> None:
    """sparse_attn with idx [B,Hkv,k_max], cnt [B,Hkv]: the heads of a group share the list."""
    for t in (q, idx, cnt, ws) + (() if o_out is None else (o_out, lse_out)):
        _require_gpu(t)
    kv = pool.view()
    _check(lib().hgca_sparse_attn_grouped(ctypes.byref(shape), _ptr(q), ctypes.byref(kv), _ptr(idx), _ptr(cnt), int(k_max),
                                          _ptr(o_out), _ptr(lse_out), _ptr(ws), ws.numel(), _stream(stream)),
           "hgca_sparse_attn_grouped")


def hybrid_decode_step(shape: Shape, q, window: Tier, pool: Tier, k, k_max: int, idx_out, cnt_out, o_out, lse_out,
                       ws_dense, ws_sparse, stream=None) -> None:
    """The whole decode step (dense, select, sparse, merge) in one library call."""
    for t in (q, idx_out, cnt_out, o_out, ws_dense, ws_sparse) + (() if lse_out is None else (lse_out,)):
        _require_gpu(t)
    kw, kp = window.view(), pool.view()
    if isinstance(k, torch.Tensor):
        _require_gpu(k)
        k_ptr, k_uni = _ptr(k), 0
    else:
        k_ptr, k_uni = None, int(k)
    _check(lib().hgca_hybrid_decode_step(ctypes.byref(shape), _ptr(q), ctypes.byref(kw), ctypes.byref(kp), k_ptr, k_uni,
                                         int(k_max), _ptr(idx_out), _ptr(cnt_out), _ptr(o_out), _dtype_code(o_out),
                                         _ptr(lse_out), _ptr(ws_dense), ws_dense.numel(), _ptr(ws_sparse),
                                         ws_sparse.numel(), _stream(stream)), "hgca_hybrid_decode_step")


def hybrid_decode_step_selected(shape: Shape, q, window: Tier, pool: Tier, idx, cnt, k_max: int, o_out, lse_out,
                                ws_dense, ws_sparse, stream=None, sel_scores=None) -> None:
    """The decode step over an existing selection (dense window part beside sparse part, merge) in one call."""
    for t in (q, idx, cnt, o_out, ws_dense, ws_sparse) + tuple(x for x in (lse_out, sel_scores) if x is not None):
        _require_gpu(t)
    kw, kp = window.view(), pool.view()
    _check(lib().hgca_hybrid_decode_step_selected(ctypes.byref(shape), _ptr(q), ctypes.byref(kw), ctypes.byref(kp),
                                                  _ptr(idx), _ptr(cnt), int(k_max), _ptr(sel_scores), _ptr(o_out),
                                                  _dtype_code(o_out), _ptr(lse_out), _ptr(ws_dense), ws_dense.numel(),
                                                  _ptr(ws_sparse), ws_sparse.numel(), _stream(stream)),
           "hgca_hybrid_decode_step_selected")


def ctx_compact(shape: Shape, pool: Tier, idx, cnt, k_max: int, k_ctx, v_ctx, ctx_cap: int, first_row=None,
                cnt_out=None, stream=None) -> None:
    """Copies the listed pool entries into per-head contiguous storage k_ctx / v_ctx [B,Hq,ctx_cap,d]."""
    for t in (idx, cnt, k_ctx, v_ctx) + tuple(x for x in (first_row, cnt_out) if x is not None):
        _require_gpu(t)
    kv = pool.view()
    _check(lib().hgca_ctx_compact(ctypes.byref(shape), ctypes.byref(kv), _ptr(idx), _ptr(cnt), int(k_max),
                                  _ptr(first_row), _ptr(k_ctx), _ptr(v_ctx), int(ctx_cap), _ptr(cnt_out),
                                  _stream(stream)), "hgca_ctx_compact")


def managed_decode_step(shape: Shape, state: "CacheState", q, k_in, v_in, alpha: float, beta: float, a_gpu, o_out,
                        lse_out, ws_dense, ws_sparse, stream=None) -> None:
    """One decode step over the managed cache (insert, attend, merge, moving average, eviction) in one call."""
    for t in (q, k_in, v_in, a_gpu, o_out, ws_dense, ws_sparse) + (() if lse_out is None else (lse_out,)):
        _require_gpu(t)
    _check(lib().hgca_managed_decode_step(ctypes.byref(shape), ctypes.byref(state), _ptr(q), _ptr(k_in), _ptr(v_in),
                                          float(alpha), float(beta), _ptr(a_gpu), _ptr(o_out),
                                          _dtype_code(o_out), _ptr(lse_out), _ptr(ws_dense), ws_dense.numel(),
                                          _ptr(ws_sparse), ws_sparse.numel(), _stream(stream)),
           "hgca_managed_decode_step")
