"""CPU oracle of group-shared salient lists for grouped-query attention (arXiv 2507.03153,
Sec. 3.3, "CPU-local sparse attention": several adjacent heads are merged into one sparse
attention task, which takes a relaxed per-head sparsification: a merged head may be padded
with entries that do not meet its own criterion).

TEST INFRASTRUCTURE ONLY: plain numpy on top of the C oracle's scores / selection / indexed
attention; shares no code with the HIP library.

With grouped-query attention the heads of a group read the same K/V rows, so the natural merge
unit is the group: ONE list of pool positions per KV head, attended by every head of the group.
Two ways to form it (both are supersets or re-rankings the paper's padding rule allows):
  * union: the union of the group's per-head lists (nothing a head selected is lost);
  * group budget: the k entries with the largest score of ANY head of the group
    (score of an entry for the group = max over the group's heads).
"""
from __future__ import annotations

import numpy as np

import oracle


def group_scores(scores: np.ndarray, n_kv_heads: int) -> np.ndarray:
    """[B, Hq, P] -> [B, Hkv, P]: maximum over the heads of each group (contiguous groups)."""
    B, Hq, P = scores.shape
    return scores.reshape(B, n_kv_heads, Hq // n_kv_heads, P).max(axis=2)


def select_grouped(q, pool: "oracle.Tier", k, k_max: int, scale: float, round_scores_to_f32: bool = True):
    """Per KV head, the k_b entries with the largest group score.  Returns idx [B,Hkv,k_max], cnt [B,Hkv]."""
    s = oracle.scores(q, pool, scale)
    if round_scores_to_f32:
        s = s.astype(np.float32).astype(np.float64)
    lens = pool.lens(q.shape[0])
    s = np.where(np.arange(s.shape[2])[None, None, :] < lens[:, None, None], s, -np.inf)
    return oracle.select_given(group_scores(s, pool.k.shape[1]), k, k_max, lens=lens)


def union_lists(idx: np.ndarray, cnt: np.ndarray, n_kv_heads: int, k_max_out: int):
    """Per KV head, the ascending union of its heads' lists.  idx [B,Hq,k_max], cnt [B,Hq]."""
    B, Hq, _ = idx.shape
    G = Hq // n_kv_heads
    out = np.full((B, n_kv_heads, k_max_out), -1, np.int32)
    out_cnt = np.zeros((B, n_kv_heads), np.int32)
    for b in range(B):
        for kvh in range(n_kv_heads):
            members = set()
            for h in range(kvh * G, (kvh + 1) * G):
                members.update(idx[b, h, :cnt[b, h]].tolist())
            u = sorted(members)
            assert len(u) <= k_max_out
            out[b, kvh, :len(u)] = u
            out_cnt[b, kvh] = len(u)
    return out, out_cnt


def attend_grouped(q, pool: "oracle.Tier", idx_g: np.ndarray, cnt_g: np.ndarray, scale: float):
    """Every head attends to its group's list: the per-head indexed attention on replicated lists."""
    G = q.shape[1] // idx_g.shape[1]
    idx = np.ascontiguousarray(np.repeat(idx_g, G, axis=1))
    cnt = np.ascontiguousarray(np.repeat(cnt_g, G, axis=1))
    return oracle.attend_indexed(q, pool, idx, cnt, scale)
