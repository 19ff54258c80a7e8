"""ctypes front end of the fp64 CPU oracle (hgca_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by the tests, the smoke check and the
benchmark's CPU-baseline leg, never by the HIP library or its binding.
Arrays are numpy; bf16 tensors are passed as uint16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hgca_oracle.c")
_LIB = os.path.join(_HERE, "libhgca_oracle.so")

F32, BF16 = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (portable x86-64 code, no FP contraction)."""
    hdr = os.path.join(_HERE, "hgca_oracle.h")
    if not force and os.path.exists(_LIB):
        newest = max(os.path.getmtime(_SRC), os.path.getmtime(hdr))
        if os.path.getmtime(_LIB) >= newest:
            return _LIB
    cmd = ["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-fopenmp",
           "-ffp-contract=off", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


class _Shape(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("batch", ctypes.c_int32),
                ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("scale", ctypes.c_double)]


class _Kv(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("seq_lens", ctypes.c_void_p), ("block_table", ctypes.c_void_p),
                ("cap", ctypes.c_int32), ("block_size", ctypes.c_int32),
                ("max_blocks", ctypes.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        for name in ("oracle_scores", "oracle_attend_all", "oracle_attend_indexed",
                     "oracle_attend_union", "oracle_select", "oracle_merge",
                     "oracle_hybrid_step", "oracle_num_threads", "oracle_set_num_threads", "oracle_window_weights",
                     "oracle_maw_update", "oracle_threshold_select", "oracle_select_given"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def set_num_threads(n: int) -> None:
    """Threads the (batch, head) loops use from now on."""
    lib().oracle_set_num_threads(int(n))


@dataclass
class Tier:
    """One KV tier (recent window or older pool) as the oracle sees it."""
    k: np.ndarray                       # contiguous [B,Hkv,cap,d] or paged [n_blocks,Hkv,bs,d]
    v: np.ndarray
    cap: int                            # max logical tokens per sequence
    seq_lens: Optional[np.ndarray] = None      # int32 [B]
    block_table: Optional[np.ndarray] = None   # int32 [B,max_blocks]
    block_size: int = 0

    def lens(self, batch: int) -> np.ndarray:
        if self.seq_lens is None:
            return np.full(batch, self.cap, dtype=np.int32)
        return self.seq_lens


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"oracle takes float32 or uint16 (bf16 bits), got {a.dtype}")


def _shape(q: np.ndarray, tier: Tier, scale: float) -> _Shape:
    assert q.ndim == 3 and q.flags.c_contiguous
    code = _dtype_code(q)
    assert _dtype_code(tier.k) == code and _dtype_code(tier.v) == code
    return _Shape(code, q.shape[0], q.shape[1], tier.k.shape[1], q.shape[2], float(scale))


def _kv(t: Tier, batch: int) -> _Kv:
    assert t.k.flags.c_contiguous and t.v.flags.c_contiguous
    max_blocks = 0
    if t.block_table is not None:
        assert t.block_table.dtype == np.int32 and t.block_table.flags.c_contiguous
        assert t.block_table.shape[0] == batch and t.block_size > 0
        max_blocks = t.block_table.shape[1]
    if t.seq_lens is not None:
        assert t.seq_lens.dtype == np.int32 and t.seq_lens.shape == (batch,)
    return _Kv(_ptr(t.k), _ptr(t.v), _ptr(t.seq_lens), _ptr(t.block_table),
               int(t.cap), int(t.block_size), int(max_blocks))


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


def scores(q, tier: Tier, scale: float) -> np.ndarray:
    sh, kv = _shape(q, tier, scale), _kv(tier, q.shape[0])
    out = np.empty((q.shape[0], q.shape[1], tier.cap), dtype=np.float64)
    _check(lib().oracle_scores(ctypes.byref(sh), _ptr(q), ctypes.byref(kv), _ptr(out)), "scores")
    return out


def attend_all(q, tier: Tier, scale: float):
    sh, kv = _shape(q, tier, scale), _kv(tier, q.shape[0])
    o = np.empty(q.shape, dtype=np.float64)
    lse = np.empty(q.shape[:2], dtype=np.float64)
    _check(lib().oracle_attend_all(ctypes.byref(sh), _ptr(q), ctypes.byref(kv),
                                   _ptr(o), _ptr(lse)), "attend_all")
    return o, lse


def _idx_args(idx, cnt, q):
    assert idx.dtype == np.int32 and cnt.dtype == np.int32
    assert idx.flags.c_contiguous and cnt.flags.c_contiguous
    assert idx.shape[:2] == q.shape[:2] and cnt.shape == q.shape[:2]
    return int(idx.shape[2])


def attend_indexed(q, tier: Tier, idx, cnt, scale: float):
    sh, kv = _shape(q, tier, scale), _kv(tier, q.shape[0])
    k_max = _idx_args(idx, cnt, q)
    o = np.empty(q.shape, dtype=np.float64)
    lse = np.empty(q.shape[:2], dtype=np.float64)
    _check(lib().oracle_attend_indexed(ctypes.byref(sh), _ptr(q), ctypes.byref(kv), _ptr(idx),
                                       _ptr(cnt), k_max, _ptr(o), _ptr(lse)), "attend_indexed")
    return o, lse


def attend_union(q, window: Tier, pool: Tier, idx, cnt, scale: float):
    sh = _shape(q, window, scale)
    assert _dtype_code(pool.k) == sh.dtype
    kw, kp = _kv(window, q.shape[0]), _kv(pool, q.shape[0])
    k_max = 0 if idx is None else _idx_args(idx, cnt, q)
    o = np.empty(q.shape, dtype=np.float64)
    lse = np.empty(q.shape[:2], dtype=np.float64)
    _check(lib().oracle_attend_union(ctypes.byref(sh), _ptr(q), ctypes.byref(kw), ctypes.byref(kp),
                                     _ptr(idx), _ptr(cnt), k_max, _ptr(o), _ptr(lse)), "attend_union")
    return o, lse


def _k_args(k, batch):
    if np.isscalar(k):
        return None, int(k)
    k = np.ascontiguousarray(k, dtype=np.int32)
    assert k.shape == (batch,)
    return k, 0


def select(q, pool: Tier, k, k_max: int, scale: float, round_scores_to_f32: bool = True):
    sh, kv = _shape(q, pool, scale), _kv(pool, q.shape[0])
    k_arr, k_uni = _k_args(k, q.shape[0])
    idx = np.empty(q.shape[:2] + (k_max,), dtype=np.int32)
    cnt = np.empty(q.shape[:2], dtype=np.int32)
    _check(lib().oracle_select(ctypes.byref(sh), _ptr(q), ctypes.byref(kv), _ptr(k_arr), k_uni,
                               int(k_max), int(bool(round_scores_to_f32)), _ptr(idx), _ptr(cnt)),
           "select")
    return idx, cnt


def merge(o_a, lse_a, o_b, lse_b):
    o_a = np.ascontiguousarray(o_a, dtype=np.float64)
    o_b = np.ascontiguousarray(o_b, dtype=np.float64)
    lse_a = np.ascontiguousarray(lse_a, dtype=np.float64)
    lse_b = np.ascontiguousarray(lse_b, dtype=np.float64)
    assert o_a.shape == o_b.shape and lse_a.shape == lse_b.shape == o_a.shape[:-1]
    d = o_a.shape[-1]
    rows = int(np.prod(o_a.shape[:-1], dtype=np.int64))
    o = np.empty_like(o_a)
    lse = np.empty_like(lse_a)
    _check(lib().oracle_merge(ctypes.c_int64(rows), d, _ptr(o_a), _ptr(lse_a), _ptr(o_b), _ptr(lse_b),
                              _ptr(o), _ptr(lse)), "merge")
    return o, lse


def hybrid_step(q, window: Tier, pool: Tier, k, k_max: int, scale: float, idx=None, cnt=None):
    """Dense window, selection (unless idx/cnt are given), sparse part, merge."""
    sh = _shape(q, window, scale)
    kw, kp = _kv(window, q.shape[0]), _kv(pool, q.shape[0])
    k_arr, k_uni = _k_args(k, q.shape[0])
    do_select = idx is None
    if do_select:
        idx = np.empty(q.shape[:2] + (k_max,), dtype=np.int32)
        cnt = np.empty(q.shape[:2], dtype=np.int32)
    else:
        assert _idx_args(idx, cnt, q) == k_max
    o = np.empty(q.shape, dtype=np.float64)
    lse = np.empty(q.shape[:2], dtype=np.float64)
    _check(lib().oracle_hybrid_step(ctypes.byref(sh), _ptr(q), ctypes.byref(kw), ctypes.byref(kp),
                                    _ptr(k_arr), k_uni, int(k_max), int(do_select), _ptr(idx), _ptr(cnt),
                                    _ptr(o), _ptr(lse)), "hybrid_step")
    return o, lse, idx, cnt


def window_weights(q, tier: Tier, scale: float) -> np.ndarray:
    """A_gpu: softmax weights of the query over the window, [B,Hq,cap], zero beyond each length."""
    sh, kv = _shape(q, tier, scale), _kv(tier, q.shape[0])
    a = np.empty((q.shape[0], q.shape[1], tier.cap), dtype=np.float64)
    _check(lib().oracle_window_weights(ctypes.byref(sh), _ptr(q), ctypes.byref(kv), _ptr(a)), "window_weights")
    return a


def _row_lens(lens, shape):
    """Per-sequence lengths [B] -> per-row lengths [B*Hq] (or None)."""
    if lens is None:
        return None
    return np.ascontiguousarray(np.repeat(np.asarray(lens, np.int32), shape[1]))


def maw_update(maw, a, alpha: float, lens=None, n_new: int = 0) -> np.ndarray:
    """maw, a: [B,Hq,cap] float64; returns the updated moving average (a new array)."""
    maw = np.array(maw, dtype=np.float64, order="C")
    a = np.ascontiguousarray(a, dtype=np.float64)
    assert maw.shape == a.shape and maw.ndim == 3
    rl = _row_lens(lens, maw.shape)
    _check(lib().oracle_maw_update(ctypes.c_int64(maw.shape[0] * maw.shape[1]), int(maw.shape[2]), _ptr(rl),
                                   int(n_new), ctypes.c_double(alpha), _ptr(maw), _ptr(a)), "maw_update")
    return maw


def threshold_select(w, beta: float, size, k_max: int, lens=None, normalised: bool = False):
    """w: [B,Hq,cap] float64; size: int or per-sequence int array [B].  Returns idx, cnt (, w_norm)."""
    w = np.ascontiguousarray(w, dtype=np.float64)
    B, Hq, cap = w.shape
    rl = _row_lens(lens, w.shape)
    sizes, size_uni = (None, int(size)) if np.isscalar(size) else (_row_lens(size, w.shape), 0)
    idx = np.empty((B, Hq, k_max), dtype=np.int32)
    cnt = np.empty((B, Hq), dtype=np.int32)
    wn = np.empty((B, Hq, k_max), dtype=np.float64) if normalised else None
    _check(lib().oracle_threshold_select(ctypes.c_int64(B * Hq), int(cap), _ptr(rl), _ptr(sizes), size_uni,
                                         ctypes.c_double(beta), _ptr(w), int(k_max), _ptr(idx), _ptr(cnt),
                                         _ptr(wn)), "threshold_select")
    return (idx, cnt, wn) if normalised else (idx, cnt)


def select_given(scores, k, k_max: int, lens=None):
    """Top-k per (b, h) row of caller-supplied scores [B,Hq,cap]; k: int or per-sequence array [B]."""
    scores = np.ascontiguousarray(scores, dtype=np.float64)
    B, Hq, cap = scores.shape
    rl = _row_lens(lens, scores.shape)
    k_rows, k_uni = (None, int(k)) if np.isscalar(k) else (_row_lens(k, scores.shape), 0)
    idx = np.empty((B, Hq, k_max), dtype=np.int32)
    cnt = np.empty((B, Hq), dtype=np.int32)
    _check(lib().oracle_select_given(ctypes.c_int64(B * Hq), int(cap), _ptr(rl), _ptr(k_rows), k_uni, int(k_max),
                                     _ptr(scores), _ptr(idx), _ptr(cnt)), "select_given")
    return idx, cnt
