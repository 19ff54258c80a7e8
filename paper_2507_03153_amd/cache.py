"""Plumbing for the KV manager calls: owns the device buffers of one layer's cache state (block pool,
block table, window / pool lengths, moving averages, per-head salient lists) and enqueues the calls of
one decode step in the order of the paper's Alg. 2 (attention) and Alg. 1 (management).  Nothing here
computes: every step is a libhgca call."""
from __future__ import annotations

import torch

from . import hgca


class LayerCache:
    """Cache state of one attention layer for a batch of B sequences.

    Sequence b owns the blocks block_table[b, :] (here simply b*max_blocks + j); its pool is the first
    first_win_block[b] of them, its window the following ones."""

    def __init__(self, dtype, B: int, Hq: int, Hkv: int, d: int, block_size: int, win_blocks: int, max_blocks: int,
                 k_max: int, sm_scale: float, device="cuda:0", keep_evicted_maw: bool = False,
                 fused_tail: bool = True, win_cap_blocks: int = 0):
        i32 = dict(dtype=torch.int32, device=device)
        f32 = dict(dtype=torch.float32, device=device)
        self.B, self.Hq, self.Hkv, self.d = B, Hq, Hkv, d
        self.block_size, self.win_blocks, self.max_blocks, self.k_max = block_size, win_blocks, max_blocks, k_max
        self.fused_tail = fused_tail      # one fold of all split partials instead of sparse fold + merge
        # capacity of the window range: l_max for decode steps, l_max - 1 + N for prompts of N tokens
        self.win_cap_blocks = win_cap_blocks or win_blocks
        self.win_cap = self.win_cap_blocks * block_size
        self.pool_cap = max_blocks * block_size
        self.k_blocks = torch.zeros(B * max_blocks, Hkv, block_size, d, dtype=dtype, device=device)
        self.v_blocks = torch.zeros_like(self.k_blocks)
        self.block_table = torch.arange(B * max_blocks, **i32).reshape(B, max_blocks).contiguous()
        self.first_win_block = torch.zeros(B, **i32)
        self.win_lens = torch.zeros(B, **i32)
        self.pool_lens = torch.zeros(B, **i32)
        self.a_maw = torch.zeros(B, Hq, self.win_cap, **f32)
        self.ctx_idx = torch.full((B, Hq, max(k_max, 1)), -1, **i32)
        self.ctx_cnt = torch.zeros(B, Hq, **i32)
        self.a_evicted = torch.zeros(B, Hq, self.pool_cap, **f32) if keep_evicted_maw else None
        self.plan = torch.zeros(B, 4, **i32)
        self.status = torch.zeros(1, **i32)
        q_like = torch.empty(B, Hq, d, dtype=dtype, device=device)
        self.shape = hgca.make_shape(q_like, Hkv, sm_scale)
        p = lambda t: None if t is None else t.data_ptr()
        self.state = hgca.CacheState(p(self.k_blocks), p(self.v_blocks), p(self.block_table), p(self.first_win_block),
                                     p(self.win_lens), p(self.pool_lens), p(self.a_maw), p(self.ctx_idx),
                                     p(self.ctx_cnt), p(self.a_evicted), p(self.plan), p(self.status),
                                     block_size, max_blocks, win_blocks, k_max, self.pool_cap, self.win_cap_blocks)
        self.window = hgca.Tier(self.k_blocks, self.v_blocks, self.win_cap, self.win_lens, self.block_table,
                                block_size, self.first_win_block)
        self.pool = hgca.Tier(self.k_blocks, self.v_blocks, self.pool_cap, self.pool_lens, self.block_table,
                              block_size, None)
        # per-step outputs and scratch
        self.o_w, self.lse_w = torch.empty(B, Hq, d, **f32), torch.empty(B, Hq, **f32)
        self.o_s, self.lse_s = torch.empty(B, Hq, d, **f32), torch.empty(B, Hq, **f32)
        self.o, self.lse = torch.empty(B, Hq, d, **f32), torch.empty(B, Hq, **f32)
        self.a_gpu = torch.zeros(B, Hq, self.win_cap, **f32)
        self.ws_dense = hgca.alloc_workspace(self.shape, self.win_cap, 0, 0, device)
        self.ws_sparse = hgca.alloc_workspace(self.shape, 0, 0, k_max, device)

    def append(self, k_in, v_in, active=None) -> None:
        hgca.kv_append(self.shape, self.state, k_in, v_in, active)

    def attend(self, q, alpha=None, n_new: int = 1) -> None:
        """Alg. 2, decode branch, on a window that already holds the token being decoded.  With `alpha` the
        moving-average update of Alg. 1 rides along with the window's weights."""
        sh = self.shape
        if alpha is None:
            hgca.dense_window_attn_weights(sh, q, self.window, self.o_w, self.lse_w, self.a_gpu, self.ws_dense)
        else:
            hgca.dense_window_attn_maw(sh, q, self.window, self.o_w, self.lse_w, self.a_gpu, self.a_maw, n_new, alpha,
                                       self.ws_dense)
        if self.fused_tail:        # the window's split partials are still in ws_dense: fold them with the sparse ones
            hgca.sparse_attn(sh, q, self.pool, self.ctx_idx, self.ctx_cnt, self.k_max, None, None, self.ws_sparse)
            hgca.lse_merge_splits(sh, self.win_cap, self.ws_dense, self.k_max, self.ws_sparse, self.o, self.lse)
        else:
            hgca.sparse_attn(sh, q, self.pool, self.ctx_idx, self.ctx_cnt, self.k_max, self.o_s, self.lse_s,
                             self.ws_sparse)
            hgca.lse_merge(sh, self.o_s, self.lse_s, self.o_w, self.lse_w, self.o, self.lse)

    def manage(self, alpha: float, beta: float, n_new: int = 1, maw_done: bool = False) -> None:
        """Alg. 1: moving-average update (unless `attend` did it), then eviction and sparsification where a
        window is full."""
        if not maw_done:
            hgca.maw_update(self.shape, self.a_maw, self.a_gpu, self.win_lens, self.win_cap, n_new, alpha)
        hgca.kv_evict(self.shape, self.state, beta)

    def append_buffers(self, n_q: int):
        """Outputs and scratch of append turns of n_q tokens (allocated once per n_q)."""
        if getattr(self, "_append_n", None) != n_q:
            f32 = dict(dtype=torch.float32, device=self.k_blocks.device)
            self._append_n = n_q
            self.a_cpu = torch.zeros(self.B, self.Hq, max(self.pool_cap, 1), **f32)
            self.o_app = torch.empty(self.B, n_q, self.Hq, self.d, **f32)
            self.lse_app = torch.empty(self.B, n_q, self.Hq, **f32)
            self.ws_append = hgca.managed_append_workspace(self.shape, self.state, n_q, self.k_blocks.device)
            self.ws_attn = hgca.append_workspace(self.shape, n_q, max(self.win_cap, self.pool_cap), self.k_blocks.device)
            self.o_aw, self.lse_aw = torch.empty_like(self.o_app), torch.empty_like(self.lse_app)
            self.o_ap, self.lse_ap = torch.empty_like(self.o_app), torch.empty_like(self.lse_app)

    def append_step(self, q, k_in, v_in, alpha: float, beta: float, one_call: bool = True) -> None:
        """One append turn (Alg. 2 append branch, then Alg. 1 with the re-evaluation): q [B,N,Hq,d], k_in / v_in
        [B,N,Hkv,d].  Results in o_app [B,N,Hq,d], lse_app [B,N,Hq], a_gpu, a_cpu."""
        n_q = int(q.shape[1])
        self.append_buffers(n_q)
        sh = self.shape
        if one_call:
            hgca.managed_append_step(sh, self.state, q, k_in, v_in, alpha, beta, self.a_gpu, self.a_cpu, self.o_app,
                                     self.lse_app, self.ws_append)
            return
        hgca.kv_append_tokens(sh, self.state, k_in, v_in)
        hgca.append_attn(sh, q, self.window, True, self.o_aw, self.lse_aw, self.ws_attn)
        hgca.append_attn(sh, q, self.pool, False, self.o_ap, self.lse_ap, self.ws_attn)
        merged = hgca.Shape(sh.dtype, sh.batch * n_q, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.sm_scale)
        hgca.lse_merge(merged, self.o_ap, self.lse_ap, self.o_aw, self.lse_aw, self.o_app, self.lse_app)
        hgca.append_weights(sh, q, self.window, True, self.lse_aw, self.a_gpu)
        hgca.append_weights(sh, q, self.pool, False, self.lse_ap, self.a_cpu)
        hgca.maw_update(sh, self.a_maw, self.a_gpu, self.win_lens, self.win_cap, n_q, alpha)
        hgca.threshold_select(sh, self.a_cpu, self.pool_lens, self.pool_cap, self.pool_lens, beta, self.k_max,
                              self.ctx_idx, self.ctx_cnt)
        hgca.kv_evict(sh, self.state, beta)

    def decode_step(self, q, k_in, v_in, alpha: float, beta: float, fused_maw: bool = True,
                    one_call: bool = False) -> None:
        if one_call:
            hgca.managed_decode_step(self.shape, self.state, q, k_in, v_in, alpha, beta, self.a_gpu, self.o, self.lse,
                                     self.ws_dense, self.ws_sparse)
            return
        self.append(k_in, v_in)
        self.attend(q, alpha if fused_maw else None)
        self.manage(alpha, beta, maw_done=fused_maw)
