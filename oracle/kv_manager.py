"""CPU oracle of the KV manager and of hybrid attention over several steps and turns
(arXiv 2507.03153, Alg. 1 "KV manager" and Alg. 2 "Hybrid attention").

TEST INFRASTRUCTURE ONLY: plain numpy in fp64, one sequence and one layer per object.  It
shares no code with the HIP library and is used by the tests only.

What the object holds (Sec. 3.2.1, 3.2.2):
    window        the recent entries, oldest first                          K_gpu, V_gpu [n, Hkv, d]
    A_maw         per head, the moving average of the attention weight
                  every window entry has received so far                    [Hq, n]
    offloaded     every entry that left the window, in the order it left    K_cpu, V_cpu [m, Hkv, d]
    salient lists per head, which offloaded entries the decode steps attend
                  to, as ascending positions into the offloaded entries
                  (the paper keeps copies of them in per-head contiguous
                  storage: the same set)                                    ctx[h] = int array
    A_cpu_maw     the moving averages the entries had when they left
                  (they travel with the block, Sec. 3.2.1)                  [Hq, m]

A decode step (`step`, Alg. 2 decode branch then Alg. 1) attends densely to the window,
which includes the incoming token, and per head to that head's salient entries, and merges
the two partial results; then the moving averages are updated with the window's weights,
and a window that has reached its limit hands whole blocks of its oldest entries over,
the ones whose average exceeds the threshold joining the salient lists.

An append step (`append`, Alg. 2 append branch then Alg. 1; a new prompt of N tokens)
attends to the window and to ALL offloaded entries, takes the query-averaged weights of
both parts, re-selects the salient lists from the offloaded part's weights
(Sec. 3.2.2 "Re-evaluation"), and then manages the window as a decode step does.

Readings taken where the paper is silent or garbled:
  * the printed eviction length is not positive inside its own condition; it is read as the
    smallest whole number of blocks that brings the window below its limit;
  * the threshold is beta divided by the number of entries the weights were normalised
    over (Sec. 3.2.2 states it so; the listing's fraction is garbled);
  * a new entry has no moving average yet: it takes its first observed weight;
  * query head h reads KV head h // (Hq // Hkv); scores are scaled by `scale`;
  * the N incoming tokens of an append attend causally among themselves and see every
    older entry; one weight per (head, entry) is kept, the mean over the N queries, with
    0 for an entry a query does not see; each part's weights are normalised within the part.
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

    # ---- Alg. 2, append branch -----------------------------------------------------------------
    def append_attention(self, Q: np.ndarray, K_in: np.ndarray, V_in: np.ndarray):
        """Q [N, Hq, d], K_in / V_in [N, Hkv, d] (the incoming prompt, oldest first).  Query i attends to the window's
        older entries, to incoming tokens 0..i, and to every offloaded entry.  Returns O [N, Hq, d], lse [N, Hq], and
        the query-averaged weights of the two parts, A_gpu [Hq, n+N] and A_cpu [Hq, m] (each query's weights are
        normalised within the part; an entry a query does not see counts 0)."""
        N, n, m = Q.shape[0], self.K_gpu.shape[0], self.K_cpu.shape[0]
        K = np.concatenate([self.K_gpu, K_in.astype(np.float64)])
        V = np.concatenate([self.V_gpu, V_in.astype(np.float64)])
        O = np.zeros((N, self.Hq, self.d))
        lse = np.zeros((N, self.Hq))
        A_gpu = np.zeros((self.Hq, n + N))
        A_cpu = np.zeros((self.Hq, m))
        for i in range(N):
            seen = n + i + 1                                        # window entries query i attends to
            for h in range(self.Hq):
                kvh = h // self.G
                qh = Q[i, h].astype(np.float64)
                o_g, lse_g, a_g = _attention(qh, K[:seen, kvh], V[:seen, kvh], self.scale)
                o_c, lse_c, a_c = _attention(qh, self.K_cpu[:, kvh], self.V_cpu[:, kvh], self.scale)
                O[i, h], lse[i, h] = _merge_state(o_c, lse_c, o_g, lse_g)
                A_gpu[h, :seen] += a_g / N
                A_cpu[h] += a_c / N
        return O, lse, A_gpu, A_cpu

    # ---- Alg. 1 for N incoming tokens, with the re-evaluation of the offloaded entries ---------------
    def manage_append(self, K_in: np.ndarray, V_in: np.ndarray, A_gpu: np.ndarray, A_cpu: np.ndarray):
        """Returns the number of evicted entries (0 if none)."""
        N, n_old, m_old = K_in.shape[0], self.K_gpu.shape[0], self.K_cpu.shape[0]
        l_cur = n_old + N
        assert A_gpu.shape == (self.Hq, l_cur) and A_cpu.shape == (self.Hq, m_old)
        # moving averages: entries with a history are blended, the N new ones take their first observed weight
        self.A_maw = np.concatenate([(1.0 - self.alpha) * self.A_maw + self.alpha * A_gpu[:, :n_old],
                                     A_gpu[:, n_old:]], axis=1)
        self.K_gpu = np.concatenate([self.K_gpu, K_in.astype(np.float64)])
        self.V_gpu = np.concatenate([self.V_gpu, V_in.astype(np.float64)])
        # the window hands over the smallest whole number of blocks that brings it below its limit
        l_evict = 0
        if l_cur >= self.l_max:
            l_evict = -(-(l_cur - self.l_max + 1) // self.blk_size) * self.blk_size
        K_evict, V_evict, A_evict = self.K_gpu[:l_evict], self.V_gpu[:l_evict], self.A_maw[:, :l_evict]
        self.K_gpu, self.V_gpu, self.A_maw = self.K_gpu[l_evict:], self.V_gpu[l_evict:], self.A_maw[:, l_evict:]
        # re-evaluation: the salient lists are REPLACED by what the offloaded part's weights select now
        if m_old > 0:
            for h in range(self.Hq):
                self.ctx[h] = np.nonzero(A_cpu[h] > self.beta / m_old)[0].astype(np.int64)
        # sparsification of what has just left the window, as in a decode step
        for h in range(self.Hq):
            ids = np.nonzero(A_evict[h] > self.beta / l_cur)[0]
            self.ctx[h] = np.concatenate([self.ctx[h], m_old + ids])
        self.A_cpu_maw = np.concatenate([self.A_cpu_maw, A_evict], axis=1)
        self.K_cpu = np.concatenate([self.K_cpu, K_evict])
        self.V_cpu = np.concatenate([self.V_cpu, V_evict])
        return l_evict

    def append(self, Q, K_in, V_in):
        O, lse, A_gpu, A_cpu = self.append_attention(Q, K_in, V_in)
        self.manage_append(K_in, V_in, A_gpu, A_cpu)
        return O, lse
