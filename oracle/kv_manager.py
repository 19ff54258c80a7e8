"""CPU oracle of the KV manager and the decode branch of hybrid attention over several
steps (arXiv 2507.03153, Alg. 1 "KV manager" and Alg. 2 "Hybrid attention").

TEST INFRASTRUCTURE ONLY: plain numpy in fp64, one sequence and one layer per object,
written from the two algorithms in the paper's order and notation.  It shares no code
with the HIP library and is used by the tests only.

State (names as in Alg. 1):
    KV_gpu   the GPU-resident window, oldest entry first            K_gpu, V_gpu [n, Hkv, d]
    A_maw    moving average of attention weights of the window      [Hq, n]
    KV_cpu   every offloaded entry, in eviction order               K_cpu, V_cpu [m, Hkv, d]
    KV_ctx   per head, the salient offloaded entries; kept here as positions into
             KV_cpu (the paper copies them to per-head contiguous storage, which
             holds the same entries)                                ctx[h] = int array
    A_evict  the moving averages that travelled with the evicted entries (Sec. 3.2.1:
             the MAW is transferred alongside the KV block)         A_cpu_maw [Hq, m]

One decode step (Alg. 2, then Alg. 1):
    KV_gpu' = concat(KV_gpu, KV_in);  O_gpu, lse_g, A_gpu = attention(q, KV_gpu')
    O_cpu[h], lse_c[h] = attention(q[h], KV_ctx[h])
    O = merge_state(O_cpu, lse_c, O_gpu, lse_g)
    A_maw <- (1 - alpha) A_maw + alpha A_gpu      (entries with a history)
    KV_gpu.add(KV_in)                              (its A_maw starts at its first observed weight)
    if l_cur >= l_max:                             l_max = blk_num * blk_size
        l_evict = ceil((l_cur - l_max + 1) / blk_size) * blk_size
        KV_evict, A_evict = KV_gpu[:l_evict], A_maw[:l_evict];  KV_gpu = KV_gpu[l_evict:]
        ids = A_evict > beta / A_gpu.size          (per head; A_gpu.size = l_cur)
        KV_ctx.add(KV_evict[ids]);  KV_cpu.add(KV_evict)

Readings taken where the paper is silent or garbled:
  * the printed eviction length has l_max and l_cur swapped (it would be <= 0 inside
    "if l_cur >= l_max"); it is read as above: the smallest whole number of blocks that
    brings the window below l_max;
  * the printed threshold "beta / = A.size" is read as beta / A.size (Sec. 3.2.2 states it so);
  * a new entry has no moving average yet: it takes its first observed weight;
  * query head h reads KV head h // (Hq // Hkv); scores are scaled by `scale`.
"""
from __future__ import annotations

import numpy as np


def _attention(q_h: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float):
    """Softmax attention of one head's query over keys K [n, d], values V [n, d] (Sec. 2.1).
    Returns O [d], lse, A [n]; an empty set gives O = 0, lse = -inf."""
    if K.shape[0] == 0:
        return np.zeros(V.shape[1]), -np.inf, np.zeros(0)
    s = scale * (K @ q_h)
    m = s.max()
    e = np.exp(s - m)
    z = e.sum()
    return (e / z) @ V, m + np.log(z), e / z


def _merge_state(o_c, lse_c, o_g, lse_g):
    """Sec. 3.3, merging states: z = e^{lse_c} + e^{lse_g}; O = (e^{lse_c} O_cpu + e^{lse_g} O_gpu) / z."""
    m = max(lse_c, lse_g)
    if m == -np.inf:
        return np.zeros_like(o_g), -np.inf
    ec, eg = np.exp(lse_c - m), np.exp(lse_g - m)
    z = ec + eg
    return (ec * o_c + eg * o_g) / z, m + np.log(z)


class KvManager:
    def __init__(self, Hq: int, Hkv: int, d: int, blk_num: int, blk_size: int, alpha: float, beta: float,
                 scale: float):
        self.Hq, self.Hkv, self.d, self.G = Hq, Hkv, d, Hq // Hkv
        self.blk_num, self.blk_size, self.alpha, self.beta, self.scale = blk_num, blk_size, alpha, beta, scale
        self.l_max = blk_num * blk_size
        self.K_gpu = np.zeros((0, Hkv, d))
        self.V_gpu = np.zeros((0, Hkv, d))
        self.A_maw = np.zeros((Hq, 0))
        self.K_cpu = np.zeros((0, Hkv, d))
        self.V_cpu = np.zeros((0, Hkv, d))
        self.ctx = [np.zeros(0, dtype=np.int64) for _ in range(Hq)]
        self.A_cpu_maw = np.zeros((Hq, 0))

    # ---- Alg. 2, decode branch ---------------------------------------------------------------
    def hybrid_attention(self, q: np.ndarray, k_in: np.ndarray, v_in: np.ndarray):
        """q [Hq, d], k_in / v_in [Hkv, d] (the token being decoded).  Returns O [Hq, d], lse [Hq], A_gpu [Hq, n+1]."""
        K = np.concatenate([self.K_gpu, k_in[None].astype(np.float64)])
        V = np.concatenate([self.V_gpu, v_in[None].astype(np.float64)])
        O = np.zeros((self.Hq, self.d))
        lse = np.zeros(self.Hq)
        A_gpu = np.zeros((self.Hq, K.shape[0]))
        for h in range(self.Hq):
            kvh = h // self.G
            qh = q[h].astype(np.float64)
            o_g, lse_g, A_gpu[h] = _attention(qh, K[:, kvh], V[:, kvh], self.scale)
            o_c, lse_c, _ = _attention(qh, self.K_cpu[self.ctx[h], kvh], self.V_cpu[self.ctx[h], kvh], self.scale)
            O[h], lse[h] = _merge_state(o_c, lse_c, o_g, lse_g)
        return O, lse, A_gpu

    # ---- Alg. 1 --------------------------------------------------------------------------------
    def manage(self, k_in: np.ndarray, v_in: np.ndarray, A_gpu: np.ndarray):
        """Returns the number of evicted entries (0 if none)."""
        n_old = self.K_gpu.shape[0]
        l_cur = n_old + 1
        assert A_gpu.shape == (self.Hq, l_cur)
        self.A_maw = np.concatenate([(1.0 - self.alpha) * self.A_maw + self.alpha * A_gpu[:, :n_old],
                                     A_gpu[:, n_old:]], axis=1)
        self.K_gpu = np.concatenate([self.K_gpu, k_in[None].astype(np.float64)])
        self.V_gpu = np.concatenate([self.V_gpu, v_in[None].astype(np.float64)])
        if l_cur < self.l_max:
            return 0
        l_evict = -(-(l_cur - self.l_max + 1) // self.blk_size) * self.blk_size
        K_evict, V_evict, A_evict = self.K_gpu[:l_evict], self.V_gpu[:l_evict], self.A_maw[:, :l_evict]
        self.K_gpu, self.V_gpu, self.A_maw = self.K_gpu[l_evict:], self.V_gpu[l_evict:], self.A_maw[:, l_evict:]
        base = self.K_cpu.shape[0]
        for h in range(self.Hq):
            ids = np.nonzero(A_evict[h] > self.beta / l_cur)[0]
            self.ctx[h] = np.concatenate([self.ctx[h], base + ids])
        self.A_cpu_maw = np.concatenate([self.A_cpu_maw, A_evict], axis=1)
        self.K_cpu = np.concatenate([self.K_cpu, K_evict])
        self.V_cpu = np.concatenate([self.V_cpu, V_evict])
        return l_evict

    def step(self, q, k_in, v_in):
        O, lse, A_gpu = self.hybrid_attention(q, k_in, v_in)
        self.manage(k_in, v_in, A_gpu)
        return O, lse
