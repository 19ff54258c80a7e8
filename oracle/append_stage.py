"""CPU oracle of the append stage of hybrid attention (arXiv 2507.03153, Sec. 2.1 and Alg. 2,
append branch; re-evaluation of Sec. 3.2.2 / Alg. 1).

TEST INFRASTRUCTURE ONLY: plain numpy in fp64, loops over sequences, heads and queries.  It
shares no code with the HIP library and is used by the tests only.

An append brings N new tokens at once (Sec. 2.1: S = Q K^T, A = softmax(S), O = A V with
Q in R^{h x N x d} and K, V extended by the N incoming entries).  Alg. 2, append branch:
    KV_gpu' = concat(KV_gpu, KV_in);   O_gpu, lse_g, A_gpu = gpu_attention(Q, KV_gpu')
    O_cpu, lse_c, A_cpu = cpu_attention(Q, KV_cpu)        (the COMPLETE offloaded cache)
    O = merge_state(O_cpu, lse_c, O_gpu, lse_g)
and Alg. 1 then re-evaluates the salient set: ids = A_cpu > beta / A_cpu.size.

Readings taken where the paper is silent:
  * among the N incoming tokens attention is causal: query i (0-based) sees the window's
    older entries and incoming tokens 0..i; every query sees the whole offloaded cache,
    which is older than all of them;
  * A_gpu and A_cpu have one weight per (head, query, entry); the KV manager keeps one value
    per (head, entry), so the N queries' softmax weights are averaged (each query's weights
    sum to 1 over what it sees, hence so does the average); an entry a query does not see has
    weight 0 for that query;
  * each part's weights are normalised within the part (A_gpu over the window, A_cpu over the
    offloaded cache), as each part runs its own softmax and hands back its own lse;
  * scores are scaled by `scale`; query head h reads KV head h // (Hq // Hkv).

Layouts: q [B, N, Hq, d]; a tier is K, V [B, Hkv, cap, d] with lens [B]; in the window tier the
last N valid entries of a sequence are the incoming tokens.
"""
from __future__ import annotations

import numpy as np


def part_attention(q, K, V, lens, scale, causal_tail: bool):
    """Attention of N queries over one tier.  Returns O [B,N,Hq,d], lse [B,N,Hq], A [B,Hq,N,cap]
    (softmax weights, 0 where not visible).  causal_tail: query i sees entries < len - N + i + 1."""
    B, N, Hq, d = q.shape
    Hkv, cap = K.shape[1], K.shape[2]
    G = Hq // Hkv
    O = np.zeros((B, N, Hq, d))
    lse = np.full((B, N, Hq), -np.inf)
    A = np.zeros((B, Hq, N, cap))
    for b in range(B):
        n = int(lens[b])
        for h in range(Hq):
            Kh, Vh = K[b, h // G, :n].astype(np.float64), V[b, h // G, :n].astype(np.float64)
            for i in range(N):
                vis = min(max(n - N + i + 1, 0), n) if causal_tail else n
                if vis == 0:
                    continue
                s = scale * (Kh[:vis] @ q[b, i, h].astype(np.float64))
                m = s.max()
                e = np.exp(s - m)
                z = e.sum()
                A[b, h, i, :vis] = e / z
                O[b, i, h] = (e / z) @ Vh[:vis]
                lse[b, i, h] = m + np.log(z)
    return O, lse, A


def merge_state(o_c, lse_c, o_g, lse_g):
    """Sec. 3.3: z = e^{lse_c} + e^{lse_g}; O = (e^{lse_c} O_cpu + e^{lse_g} O_gpu) / z, element-wise over rows."""
    m = np.maximum(lse_c, lse_g)
    safe = np.where(np.isneginf(m), 0.0, m)
    ec, eg = np.exp(lse_c - safe), np.exp(lse_g - safe)
    z = ec + eg
    o = np.where((z > 0)[..., None], (ec[..., None] * o_c + eg[..., None] * o_g) / np.where(z > 0, z, 1.0)[..., None], 0.0)
    lse = np.where(z > 0, safe + np.log(np.where(z > 0, z, 1.0)), -np.inf)
    return o, lse


def append_step(q, Kw, Vw, w_lens, Kp, Vp, p_lens, scale):
    """The append branch of Alg. 2.  Returns O [B,N,Hq,d], lse [B,N,Hq], A_gpu [B,Hq,W] and A_cpu [B,Hq,P]
    (weights averaged over the N queries)."""
    o_g, lse_g, A_g = part_attention(q, Kw, Vw, w_lens, scale, causal_tail=True)
    o_c, lse_c, A_c = part_attention(q, Kp, Vp, p_lens, scale, causal_tail=False)
    o, lse = merge_state(o_c, lse_c, o_g, lse_g)
    return o, lse, A_g.mean(axis=2), A_c.mean(axis=2)
