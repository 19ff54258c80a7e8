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


# ---------------------------------------------------------------------------------------------------
# Append turns (Alg. 2 append branch, Alg. 1 with N incoming tokens and the re-evaluation of Sec. 3.2.2)

def lib_causal(Q, k, v, t0, scale, G):
    """Query i of a prompt that starts at token t0 attends to tokens 0 .. t0+i: library softmax per query."""
    out = [lib_attention(Q[i], k[:t0 + i + 1], v[:t0 + i + 1], scale, G) for i in range(Q.shape[0])]
    return np.stack([o for o, _ in out]), np.stack([l for _, l in out])


def run_turns(m, q, k, v, turns):
    """turns: list of ('a', N) / ('d', n_steps).  Yields (kind, t0, n, O, lse) per call, tokens taken in order."""
    t = 0
    for kind, n in turns:
        if kind == "a":
            O, lse = m.append(q[t:t + n], k[t:t + n], v[t:t + n])
            yield "a", t, n, O, lse
            t += n
        else:
            for _ in range(n):
                O, lse = m.step(q[t], k[t], v[t])
                yield "d", t, 1, O, lse
                t += 1


TURNS = [("a", 5), ("d", 7), ("a", 13), ("d", 3), ("a", 1), ("d", 9), ("a", 30), ("d", 2)]


@pytest.mark.parametrize("Hq,Hkv,blk_num,blk_size", [(4, 2, 3, 4), (2, 2, 2, 1), (6, 1, 2, 8)])
def test_beta_zero_mixed_turns_reproduce_full_causal_attention(Hq, Hkv, blk_num, blk_size):
    """With beta = 0 nothing offloaded is ever dropped (neither at eviction nor at re-evaluation), so every
    output of every turn equals causal attention over the whole history."""
    T, d, scale = sum(n for _, n in TURNS), 8, 0.3
    q, k, v = tokens(11, T, Hq, Hkv, d)
    m = KvManager(Hq, Hkv, d, blk_num, blk_size, alpha=0.3, beta=0.0, scale=scale)
    for kind, t0, n, O, lse in run_turns(m, q, k, v, TURNS):
        if kind == "a":
            o_ref, l_ref = lib_causal(q[t0:t0 + n], k, v, t0, scale, Hq // Hkv)
        else:
            o_ref, l_ref = lib_attention(q[t0], k[:t0 + 1], v[:t0 + 1], scale, Hq // Hkv)
        np.testing.assert_allclose(O, o_ref, atol=1e-12)
        np.testing.assert_allclose(lse, l_ref, atol=1e-12)
        assert all(len(c) == m.K_cpu.shape[0] for c in m.ctx)
    assert m.K_cpu.shape[0] > 0


def test_huge_beta_append_still_sees_every_offloaded_entry():
    """The append branch attends to ALL offloaded entries whatever the salient lists hold (here a huge beta keeps
    them empty through evictions and re-evaluations alike)."""
    Hq, Hkv, d, blk_num, blk_size, scale = 4, 2, 8, 2, 4, 0.5
    T = sum(n for _, n in TURNS)
    q, k, v = tokens(12, T, Hq, Hkv, d)
    m = KvManager(Hq, Hkv, d, blk_num, blk_size, alpha=0.5, beta=1e9, scale=scale)
    for kind, t0, n, O, lse in run_turns(m, q, k, v, TURNS):
        if kind == "a":
            o_ref, l_ref = lib_causal(q[t0:t0 + n], k, v, t0, scale, Hq // Hkv)
            np.testing.assert_allclose(O, o_ref, atol=1e-12)
            np.testing.assert_allclose(lse, l_ref, atol=1e-12)
        assert all(len(c) == 0 for c in m.ctx)


def test_huge_beta_decode_steps_after_appends_equal_window_attention():
    Hq, Hkv, d, blk_num, blk_size, scale = 2, 1, 4, 2, 4, 0.7
    q, k, v = tokens(13, 60, Hq, Hkv, d)
    m = KvManager(Hq, Hkv, d, blk_num, blk_size, alpha=0.5, beta=1e9, scale=scale)
    t = 0
    for kind, n in [("a", 11), ("d", 6), ("a", 9), ("d", 12)]:
        if kind == "a":
            m.append(q[t:t + n], k[t:t + n], v[t:t + n])
            t += n
            continue
        for _ in range(n):
            first = m.K_cpu.shape[0]                            # the window starts where the offloaded entries end
            O, lse = m.step(q[t], k[t], v[t])
            o_ref, l_ref = lib_attention(q[t], k[first:t + 1], v[first:t + 1], scale, Hq // Hkv)
            np.testing.assert_allclose(O, o_ref, atol=1e-12)
            np.testing.assert_allclose(lse, l_ref, atol=1e-12)
            t += 1


def test_append_of_one_token_manages_the_window_like_a_decode_step():
    """N = 1: the window side of an append (moving averages, insertion, eviction, what leaves) is that of a decode
    step; only the offloaded side differs (complete instead of salient entries, then re-evaluation)."""
    Hq, Hkv, d, blk_num, blk_size, scale = 4, 2, 8, 3, 4, 0.4
    q, k, v = tokens(14, 40, Hq, Hkv, d)
    a = KvManager(Hq, Hkv, d, blk_num, blk_size, alpha=0.3, beta=0.0, scale=scale)
    b = KvManager(Hq, Hkv, d, blk_num, blk_size, alpha=0.3, beta=0.0, scale=scale)
    for t in range(40):
        o_a, l_a = a.append(q[t:t + 1], k[t:t + 1], v[t:t + 1])
        o_b, l_b = b.step(q[t], k[t], v[t])
        np.testing.assert_allclose(o_a[0], o_b, atol=1e-13)     # beta = 0: the lists hold every offloaded entry
        np.testing.assert_allclose(l_a[0], l_b, atol=1e-13)
        np.testing.assert_allclose(a.A_maw, b.A_maw, atol=1e-15)
        np.testing.assert_array_equal(a.K_gpu, b.K_gpu)
        np.testing.assert_array_equal(a.K_cpu, b.K_cpu)
        np.testing.assert_allclose(a.A_cpu_maw, b.A_cpu_maw, atol=1e-15)


def test_bookkeeping_across_turns_and_eviction_of_several_blocks_at_once():
    Hq, Hkv, d, blk_num, blk_size = 4, 2, 4, 3, 8
    T = sum(n for _, n in TURNS)
    q, k, v = tokens(15, T, Hq, Hkv, d)
    m = KvManager(Hq, Hkv, d, blk_num, blk_size, alpha=0.2, beta=1.0, scale=0.5)
    most, c_before = 0, 0
    for kind, t0, n, O, lse in run_turns(m, q, k, v, TURNS):
        n_w, c = m.K_gpu.shape[0], m.K_cpu.shape[0]
        most, c_before = max(most, c - c_before), c
        assert n_w + c == t0 + n and c % blk_size == 0          # nothing lost, whole blocks offloaded
        assert n_w < blk_num * blk_size                          # every call leaves the window below its limit
        assert m.A_maw.shape == (Hq, n_w) and m.A_cpu_maw.shape == (Hq, c)
        np.testing.assert_array_equal(m.K_cpu, k[:c])
        np.testing.assert_array_equal(m.K_gpu, k[c:t0 + n])
        for ctx in m.ctx:
            assert np.all(np.diff(ctx) > 0) and (len(ctx) == 0 or (ctx[0] >= 0 and ctx[-1] < c))
    assert most >= 3 * blk_size                                  # the 30-token prompt pushed out several blocks at once


def test_hand_worked_two_turns_with_reinstatement():
    """One head, d = 1, window of 2 blocks of 2 (l_max = 4), alpha = 1/2, beta = 1.2; values v_i = 10 i.
    Turn 1, prompt of 3 tokens with q = 0 (uniform weights, causal): query 0 sees e1; query 1 e1, e2; query 2
    e1..e3, so the query-averaged weights are (1 + 1/2 + 1/3)/3 = 11/18, (1/2 + 1/3)/3 = 5/18, (1/3)/3 = 1/9,
    which are also the entries' first moving averages.  Decode of e4 (q = 0): every weight 1/4, averages
    e1 = 11/36 + 1/8 = 31/72, e2 = 5/36 + 1/8 = 19/72, e3 = 1/18 + 1/8 = 13/72, e4 = 1/4; l_cur = 4 = l_max: two
    entries leave; threshold 1.2/4 = 0.3: e1 (0.4306) is salient, e2 (0.2639) is not.
    Turn 2, prompt e5, e6 with q = 1 and keys k1 = 0, k2 = ln 3, k3 .. k6 = 0: over the offloaded entries both
    queries weigh e1, e2 as 1/4, 3/4; threshold 1.2/2 = 0.6: e2 is reinstated and e1 dropped (the lists are
    replaced, not extended).  Window weights: query 0 sees e3, e4, e5 (1/3 each), query 1 e3 .. e6 (1/4 each):
    averaged 7/24, 7/24, 7/24, 1/8; moving averages e3 = 13/144 + 7/48 = 17/72, e4 = 1/8 + 7/48 = 13/48, e5 = 7/24,
    e6 = 1/8; l_cur = 4: e3, e4 leave; threshold 0.3: neither is salient.
    Outputs of turn 2 (unnormalised weights e1: 1, e2: 3, window entries: 1 each):
    query 0 = (10 + 60 + 30 + 40 + 50)/7, lse = ln 7; query 1 = (10 + 60 + 30 + 40 + 50 + 60)/8, lse = ln 8.
    Decode of e7 (q = 1, k7 = 0): window e5, e6, e7 and the salient e2: (3*20 + 50 + 60 + 70)/6 = 40, lse = ln 6."""
    m = KvManager(1, 1, 1, blk_num=2, blk_size=2, alpha=0.5, beta=1.2, scale=1.0)
    K = np.array([0.0, np.log(3.0), 0, 0, 0, 0, 0]).reshape(7, 1, 1)
    V = (10.0 * np.arange(1, 8)).reshape(7, 1, 1)
    O, lse = m.append(np.zeros((3, 1, 1)), K[:3], V[:3])
    np.testing.assert_allclose(O[:, 0, 0], [10.0, 15.0, 20.0], atol=1e-13)              # running means of v
    np.testing.assert_allclose(lse[:, 0], np.log([1.0, 2.0, 3.0]), atol=1e-13)
    np.testing.assert_allclose(m.A_maw[0], [11 / 18, 5 / 18, 1 / 9], atol=1e-15)
    m.step(np.zeros((1, 1)), K[3], V[3])
    np.testing.assert_allclose(m.A_cpu_maw[0], [31 / 72, 19 / 72], atol=1e-15)
    np.testing.assert_allclose(m.A_maw[0], [13 / 72, 1 / 4], atol=1e-15)
    assert m.ctx[0].tolist() == [0]
    O, lse = m.append(np.ones((2, 1, 1)), K[4:6], V[4:6])
    np.testing.assert_allclose(O[:, 0, 0], [190 / 7, 250 / 8], atol=1e-12)
    np.testing.assert_allclose(lse[:, 0], np.log([7.0, 8.0]), atol=1e-13)
    assert m.ctx[0].tolist() == [1]                             # e2 reinstated, e1 dropped, e3 and e4 not salient
    np.testing.assert_allclose(m.A_cpu_maw[0], [31 / 72, 19 / 72, 17 / 72, 13 / 48], atol=1e-15)
    np.testing.assert_allclose(m.A_maw[0], [7 / 24, 1 / 8], atol=1e-15)
    assert m.K_cpu[:, 0, 0].tolist() == K[:4, 0, 0].tolist()
    O, lse = m.step(np.ones((1, 1)), K[6], V[6])
    assert O[0, 0] == pytest.approx(40.0) and lse[0] == pytest.approx(np.log(6.0))


def test_append_weights_agree_with_the_stateless_append_oracle():
    """The query-averaged weights and outputs of an append turn equal those of oracle/append_stage.py on the same
    tensors (two independent write-ups of Alg. 2's append branch)."""
    from oracle import append_stage
    Hq, Hkv, d, blk_num, blk_size, scale = 4, 2, 8, 2, 4, 0.4
    q, k, v = tokens(16, 40, Hq, Hkv, d)
    m = KvManager(Hq, Hkv, d, blk_num, blk_size, alpha=0.3, beta=1.0, scale=scale)
    m.append(q[:20], k[:20], v[:20])
    for t in range(20, 25):
        m.step(q[t], k[t], v[t])
    n, c, N = m.K_gpu.shape[0], m.K_cpu.shape[0], 9
    O, lse, A_gpu, A_cpu = m.append_attention(q[25:25 + N], k[25:25 + N], v[25:25 + N])
    win_k = np.concatenate([m.K_gpu, k[25:25 + N]]).transpose(1, 0, 2)[None]
    win_v = np.concatenate([m.V_gpu, v[25:25 + N]]).transpose(1, 0, 2)[None]
    ref = append_stage.append_step(q[25:25 + N][None], win_k, win_v, np.array([n + N]),
                                   m.K_cpu.transpose(1, 0, 2)[None], m.V_cpu.transpose(1, 0, 2)[None], np.array([c]),
                                   scale)
    np.testing.assert_allclose(O, ref[0][0], atol=1e-12)
    np.testing.assert_allclose(lse, ref[1][0], atol=1e-12)
    np.testing.assert_allclose(A_gpu, ref[2][0], atol=1e-14)
    np.testing.assert_allclose(A_cpu, ref[3][0], atol=1e-14)
