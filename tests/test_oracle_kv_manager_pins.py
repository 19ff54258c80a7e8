"""Pins of the multi-step oracle (KV manager + hybrid attention, paper Alg. 1 and Alg. 2) against
things other than itself (no GPU needed): with beta = 0 every offloaded entry stays salient, so every
step must equal full attention over the whole history (library softmax); with a huge beta nothing
offloaded is attended, so every step equals attention over the window alone; hand-worked moving
averages and eviction decisions on a four-entry window; bookkeeping invariants."""
import numpy as np
import pytest
from scipy.special import logsumexp, softmax

from oracle.kv_manager import KvManager


def tokens(seed, T, Hq, Hkv, d):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((T, Hq, d)), rng.standard_normal((T, Hkv, d)), rng.standard_normal((T, Hkv, d))


def lib_attention(q, K, V, scale, G):
    """softmax(scale q K^T) V and logsumexp per head with library routines; K, V [n, Hkv, d]."""
    Hq = q.shape[0]
    o, lse = np.zeros((Hq, K.shape[2])), np.zeros(Hq)
    for h in range(Hq):
        s = scale * (K[:, h // G] @ q[h])
        o[h], lse[h] = softmax(s) @ V[:, h // G], logsumexp(s)
    return o, lse


@pytest.mark.parametrize("Hq,Hkv,blk_num,blk_size", [(4, 2, 3, 4), (2, 2, 2, 1), (6, 1, 4, 8)])
def test_beta_zero_reproduces_full_attention_over_the_whole_history(Hq, Hkv, blk_num, blk_size):
    T, d, scale = 70, 8, 0.3
    q, k, v = tokens(1, T, Hq, Hkv, d)
    m = KvManager(Hq, Hkv, d, blk_num, blk_size, alpha=0.3, beta=0.0, scale=scale)
    for t in range(T):
        o, lse = m.step(q[t], k[t], v[t])
        o_ref, lse_ref = lib_attention(q[t], k[:t + 1], v[:t + 1], scale, Hq // Hkv)
        np.testing.assert_allclose(o, o_ref, atol=1e-12)
        np.testing.assert_allclose(lse, lse_ref, atol=1e-12)
    assert all(len(c) == m.K_cpu.shape[0] for c in m.ctx) and m.K_cpu.shape[0] > 0


def test_huge_beta_is_attention_over_the_window_alone():
    T, Hq, Hkv, d, blk_num, blk_size, scale = 40, 4, 2, 8, 2, 4, 0.5
    q, k, v = tokens(2, T, Hq, Hkv, d)
    m = KvManager(Hq, Hkv, d, blk_num, blk_size, alpha=0.5, beta=1e9, scale=scale)
    first = 0                                                   # oldest token still in the window
    for t in range(T):
        o, lse = m.step(q[t], k[t], v[t])
        o_ref, lse_ref = lib_attention(q[t], k[first:t + 1], v[first:t + 1], scale, Hq // Hkv)
        np.testing.assert_allclose(o, o_ref, atol=1e-12)
        np.testing.assert_allclose(lse, lse_ref, atol=1e-12)
        if t + 1 - first >= blk_num * blk_size:                 # the window reached l_max: one block leaves
            first += blk_size
    assert all(len(c) == 0 for c in m.ctx)


def test_bookkeeping_invariants():
    T, Hq, Hkv, d, blk_num, blk_size = 100, 4, 2, 4, 3, 8
    q, k, v = tokens(3, T, Hq, Hkv, d)
    m = KvManager(Hq, Hkv, d, blk_num, blk_size, alpha=0.2, beta=1.0, scale=0.5)
    for t in range(T):
        m.step(q[t], k[t], v[t])
        n, c = m.K_gpu.shape[0], m.K_cpu.shape[0]
        assert n + c == t + 1 and c % blk_size == 0             # nothing lost, whole blocks offloaded
        assert n < blk_num * blk_size and (t + 1 < blk_num * blk_size or n >= (blk_num - 1) * blk_size)
        assert m.A_maw.shape == (Hq, n)
        np.testing.assert_array_equal(m.K_cpu, k[:c])           # offloaded in arrival order
        np.testing.assert_array_equal(m.K_gpu, k[c:t + 1])
        for ctx in m.ctx:                                       # positions into KV_cpu, ascending, distinct
            assert np.all(np.diff(ctx) > 0) and (len(ctx) == 0 or (ctx[0] >= 0 and ctx[-1] < c))
    assert 0 < sum(len(ctx) for ctx in m.ctx) < Hq * m.K_cpu.shape[0]     # beta = 1 keeps some, not all


def test_hand_worked_moving_average_and_eviction():
    """q = 0 makes every attention weight 1 / l_cur.  Window of 2 blocks of 2 (l_max = 4), alpha = 1/2.
    MAW by hand:  step 1: e1 = 1
                  step 2: e1 = 1/2 + 1/4 = 3/4,            e2 = 1/2
                  step 3: e1 = 3/8 + 1/6 = 13/24,          e2 = 1/4 + 1/6 = 5/12,   e3 = 1/3
                  step 4: e1 = 13/48 + 1/8 = 19/48,        e2 = 5/24 + 1/8 = 1/3,   e3 = 1/6 + 1/8 = 7/24,  e4 = 1/4
    l_cur = 4 >= l_max: l_evict = ceil(1/2) * 2 = 2; threshold beta / 4 with beta = 1.4 is 0.35:
    e1 = 0.3958 is kept, e2 = 0.3333 is dropped."""
    m = KvManager(1, 1, 1, blk_num=2, blk_size=2, alpha=0.5, beta=1.4, scale=1.0)
    q = np.zeros((1, 1))
    want = [[1.0], [3 / 4, 1 / 2], [13 / 24, 5 / 12, 1 / 3]]
    for t in range(3):
        m.step(q, np.full((1, 1), t + 1.0), np.full((1, 1), 10.0 * (t + 1)))
        np.testing.assert_allclose(m.A_maw[0], want[t], atol=1e-15)
    o, lse = m.step(q, np.full((1, 1), 4.0), np.full((1, 1), 40.0))
    assert o[0, 0] == pytest.approx(25.0) and lse[0] == pytest.approx(np.log(4.0))      # mean of 10..40
    np.testing.assert_allclose(m.A_maw[0], [7 / 24, 1 / 4], atol=1e-15)                 # e3, e4 remain
    assert m.K_cpu[:, 0, 0].tolist() == [1.0, 2.0] and m.ctx[0].tolist() == [0]
    # step 5: window e3 e4 e5, sparse part = e1 only: uniform over 4 entries (e1, e3, e4, e5)
    o, lse = m.step(q, np.full((1, 1), 5.0), np.full((1, 1), 50.0))
    assert o[0, 0] == pytest.approx((10 + 30 + 40 + 50) / 4) and lse[0] == pytest.approx(np.log(4.0))


def test_eviction_length_covers_a_window_that_overshoots():
    """If the window starts beyond l_max (e.g. after a long prompt), enough whole blocks leave at once."""
    m = KvManager(1, 1, 1, blk_num=2, blk_size=2, alpha=0.5, beta=0.0, scale=1.0)
    m.K_gpu = np.arange(7.0).reshape(7, 1, 1)
    m.V_gpu = m.K_gpu.copy()
    m.A_maw = np.full((1, 7), 1 / 7)
    m.step(np.zeros((1, 1)), np.full((1, 1), 7.0), np.full((1, 1), 7.0))
    # l_cur = 8, l_max = 4: ceil(5/2)*2 = 6 leave, 2 stay
    assert m.K_cpu.shape[0] == 6 and m.K_gpu[:, 0, 0].tolist() == [6.0, 7.0]


def test_single_step_parts_agree_with_the_c_oracle(oracle):
    """A_gpu and the threshold decision of one step equal the single-step C oracle's."""
    T, Hq, Hkv, d, blk_num, blk_size, scale = 15, 4, 2, 8, 4, 4, 0.4
    q, k, v = (x.astype(np.float32) for x in tokens(4, T, Hq, Hkv, d))
    m = KvManager(Hq, Hkv, d, blk_num, blk_size, alpha=0.3, beta=1.0, scale=scale)
    for t in range(T):
        K = np.concatenate([m.K_gpu, k[t][None].astype(np.float64)]).astype(np.float32)     # exact: fp32 inputs
        _, _, A_gpu = m.hybrid_attention(q[t], k[t], v[t])
        tier = oracle.Tier(np.ascontiguousarray(K.transpose(1, 0, 2)[None]),
                           np.ascontiguousarray(K.transpose(1, 0, 2)[None]), cap=K.shape[0])
        np.testing.assert_allclose(A_gpu, oracle.window_weights(q[t][None], tier, scale)[0], atol=1e-14)
        maw_before = np.concatenate([(1 - 0.3) * m.A_maw + 0.3 * A_gpu[:, :-1], A_gpu[:, -1:]], axis=1)
        c_before = [c.copy() for c in m.ctx]
        base = m.K_cpu.shape[0]
        ev = m.manage(k[t], v[t], A_gpu)
        if ev:
            idx, cnt = oracle.threshold_select(maw_before[None], 1.0, K.shape[0], ev,
                                               lens=np.array([ev], np.int32))
            for h in range(Hq):
                assert (base + idx[0, h, :cnt[0, h]]).tolist() == m.ctx[h][len(c_before[h]):].tolist()
