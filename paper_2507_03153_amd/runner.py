"""Plumbing around the library calls: upload a generated layer to the GPU, own the output /
workspace buffers, and enqueue one hybrid layer-step.

Order of a step (paper Alg. 2, decode branch): the dense window part and the (select ->) sparse
part are independent; the merge joins them.  Nothing here computes: every step is a libhgca call.

Two ways to finish a step:
  * `fused_tail=False`: dense and sparse each fold their splits into (O, lse), hgca_lse_merge
    combines the two (the four calls, each with its own outputs);
  * `fused_tail=True`: dense and sparse defer their results and hgca_lse_merge_splits folds all
    split partials of both parts in one kernel (two launches fewer per step).
"""
from __future__ import annotations

import ctypes
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

from . import hgca
from .workloads import Layer, TierData


def _to_gpu(a: Optional[np.ndarray], device) -> Optional[torch.Tensor]:
    if a is None:
        return None
    if a.dtype == np.uint16:                                   # bf16 bit patterns
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


def upload_tier(t: TierData, device) -> hgca.Tier:
    return hgca.Tier(_to_gpu(t.k, device), _to_gpu(t.v, device), t.cap, _to_gpu(t.seq_lens, device),
                     _to_gpu(t.block_table, device), t.block_size)


@dataclass
class DeviceLayer:
    q: torch.Tensor
    window: hgca.Tier
    pool: hgca.Tier
    k: object                   # int or int32 GPU tensor [B]
    k_max: int
    shape: hgca.Shape

    @staticmethod
    def upload(layer: Layer, device="cuda:0") -> "DeviceLayer":
        q = _to_gpu(layer.q, device)
        k = layer.k if np.isscalar(layer.k) else _to_gpu(np.ascontiguousarray(layer.k, np.int32), device)
        shape = hgca.make_shape(q, layer.cfg.Hkv, layer.scale)
        return DeviceLayer(q, upload_tier(layer.window, device), upload_tier(layer.pool, device), k,
                           layer.k_max, shape)


class HybridStep:
    """Buffers for one layer-step on `shape`; `run` enqueues dense, select, sparse and merge."""

    def __init__(self, shape: hgca.Shape, max_window: int, max_pool: int, k_max: int, device="cuda:0",
                 out_dtype=torch.float32, two_streams: bool = False, pass_scores: bool = True,
                 fused_tail: bool = False, one_call: bool = False):
        B, Hq, d = shape.batch, shape.n_q_heads, shape.head_dim
        f32 = dict(dtype=torch.float32, device=device)
        self.shape, self.k_max, self.device = shape, k_max, device
        self.pass_scores = pass_scores                              # select hands its scores to the sparse part
        self.fused_tail = fused_tail                                # one fold of all splits instead of three kernels
        self.one_call = one_call                                    # a step = hgca_hybrid_decode_step / _selected
        if one_call and (two_streams or not fused_tail or not pass_scores):
            raise ValueError("one_call implies fused_tail and pass_scores on one stream")
        self.o_w, self.lse_w = torch.empty(B, Hq, d, **f32), torch.empty(B, Hq, **f32)
        self.o_s, self.lse_s = torch.empty(B, Hq, d, **f32), torch.empty(B, Hq, **f32)
        self.o = torch.empty(B, Hq, d, dtype=out_dtype, device=device)
        self.lse = torch.empty(B, Hq, **f32)
        self.idx = torch.full((B, Hq, max(k_max, 1)), -1, dtype=torch.int32, device=device)
        self.cnt = torch.zeros(B, Hq, dtype=torch.int32, device=device)
        self.sel_scores = torch.empty(B, Hq, max(k_max, 1), **f32)   # scores of the kept entries (select -> sparse)
        # the two branches may overlap, so each owns a workspace
        self.ws_dense = hgca.alloc_workspace(shape, max_window, 0, 0, device)
        self.ws_sparse = hgca.alloc_workspace(shape, 0, max_pool, k_max, device)
        self.side = torch.cuda.Stream(device=device) if two_streams else None
        self._fork = torch.cuda.Event() if two_streams else None
        self._join = torch.cuda.Event() if two_streams else None

    def prepare(self, L: DeviceLayer):
        """Marshal the arguments of the calls once; returns run(select=True) for the current stream
        setup.  Keeps Python's per-call cost (struct packing) out of a launch-bound loop."""
        lib, ref, ptr = hgca.lib(), ctypes.byref, hgca._ptr
        sh, win, pool = self.shape, L.window.view(), L.pool.view()
        k_ptr, k_uni = (ptr(L.k), 0) if isinstance(L.k, torch.Tensor) else (None, int(L.k))
        main = torch.cuda.current_stream()
        side = self.side if self.side is not None else main
        s_main, s_side = ctypes.c_void_p(main.cuda_stream), ctypes.c_void_p(side.cuda_stream)
        fused = self.fused_tail
        o_s, l_s = (None, None) if fused else (ptr(self.o_s), ptr(self.lse_s))
        o_w, l_w = (None, None) if fused else (ptr(self.o_w), ptr(self.lse_w))
        a_sel = (ref(sh), ptr(L.q), ref(pool), k_ptr, k_uni, self.k_max, ptr(self.idx), ptr(self.cnt),
                 ptr(self.sel_scores), ptr(self.ws_sparse), self.ws_sparse.numel(), s_side)
        # with a fresh selection its scores feed the sparse part; a reused selection re-reads K
        a_sparse = {given: (ref(sh), ptr(L.q), ref(pool), ptr(self.idx), ptr(self.cnt), self.k_max,
                            ptr(self.sel_scores) if given else None, o_s, l_s,
                            ptr(self.ws_sparse), self.ws_sparse.numel(), s_side) for given in (False, True)}
        a_dense = (ref(sh), ptr(L.q), ref(win), o_w, l_w, ptr(self.ws_dense), self.ws_dense.numel(), s_main)
        a_merge = (ref(sh), ptr(self.o_s), ptr(self.lse_s), ptr(self.o_w), ptr(self.lse_w), ptr(self.o),
                   hgca._dtype_code(self.o), ptr(self.lse), s_main)
        a_splits = (ref(sh), int(L.window.cap), ptr(self.ws_dense), self.ws_dense.numel(), self.k_max,
                    ptr(self.ws_sparse), self.ws_sparse.numel(), ptr(self.o), hgca._dtype_code(self.o),
                    ptr(self.lse), s_main)
        a_step = (ref(sh), ptr(L.q), ref(win), ref(pool), k_ptr, k_uni, self.k_max, ptr(self.idx), ptr(self.cnt),
                  ptr(self.o), hgca._dtype_code(self.o), ptr(self.lse), ptr(self.ws_dense), self.ws_dense.numel(),
                  ptr(self.ws_sparse), self.ws_sparse.numel(), s_main)
        a_selected = (ref(sh), ptr(L.q), ref(win), ref(pool), ptr(self.idx), ptr(self.cnt), self.k_max, None,
                      ptr(self.o), hgca._dtype_code(self.o), ptr(self.lse), ptr(self.ws_dense), self.ws_dense.numel(),
                      ptr(self.ws_sparse), self.ws_sparse.numel(), s_main)
        keep = (sh, win, pool, L)                               # the structs must outlive the closure

        def run(select: bool = True) -> None:
            if self.one_call:
                if select:
                    hgca._check(lib.hgca_hybrid_decode_step(*a_step), "hgca_hybrid_decode_step")
                else:
                    hgca._check(lib.hgca_hybrid_decode_step_selected(*a_selected), "hgca_hybrid_decode_step_selected")
                return
            if self.side is not None:
                self._fork.record(main)
                side.wait_event(self._fork)
            if select:
                hgca._check(lib.hgca_select_salient(*a_sel), "hgca_select_salient")
            hgca._check(lib.hgca_sparse_attn(*a_sparse[select and self.pass_scores]), "hgca_sparse_attn")
            hgca._check(lib.hgca_dense_window_attn(*a_dense), "hgca_dense_window_attn")
            if self.side is not None:
                self._join.record(side)
                main.wait_event(self._join)
            if fused:
                hgca._check(lib.hgca_lse_merge_splits(*a_splits), "hgca_lse_merge_splits")
            else:
                hgca._check(lib.hgca_lse_merge(*a_merge), "hgca_lse_merge")

        run.keep = keep
        return run

    def run(self, L: DeviceLayer, select: bool = True, stream=None) -> None:
        main = torch.cuda.current_stream() if stream is None else stream
        if self.one_call:
            if select:
                hgca.hybrid_decode_step(self.shape, L.q, L.window, L.pool, L.k, self.k_max, self.idx, self.cnt, self.o,
                                        self.lse, self.ws_dense, self.ws_sparse, main)
            else:
                hgca.hybrid_decode_step_selected(self.shape, L.q, L.window, L.pool, self.idx, self.cnt, self.k_max,
                                                 self.o, self.lse, self.ws_dense, self.ws_sparse, main)
            return
        side = main
        if self.side is not None:
            side = self.side
            self._fork.record(main)
            side.wait_event(self._fork)
        given = self.sel_scores if (select and self.pass_scores) else None
        o_s, l_s = (None, None) if self.fused_tail else (self.o_s, self.lse_s)
        o_w, l_w = (None, None) if self.fused_tail else (self.o_w, self.lse_w)
        if select:
            hgca.select_salient(self.shape, L.q, L.pool, L.k, self.k_max, self.idx, self.cnt, self.ws_sparse, side,
                                sel_scores_out=given)
        hgca.sparse_attn(self.shape, L.q, L.pool, self.idx, self.cnt, self.k_max, o_s, l_s, self.ws_sparse, side,
                         sel_scores=given)
        hgca.dense_window_attn(self.shape, L.q, L.window, o_w, l_w, self.ws_dense, main)
        if self.side is not None:
            self._join.record(side)
            main.wait_event(self._join)
        if self.fused_tail:
            hgca.lse_merge_splits(self.shape, L.window.cap, self.ws_dense, self.k_max, self.ws_sparse, self.o,
                                  self.lse, main)
        else:
            hgca.lse_merge(self.shape, self.o_s, self.lse_s, self.o_w, self.lse_w, self.o, self.lse, main)
