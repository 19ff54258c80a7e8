"""Pins of the append-stage oracle (paper Sec. 2.1, Alg. 2 append branch) against things other than
itself: library softmax over an explicitly masked score matrix of the concatenated sequence (the merge
must equal one causal softmax over pool + window), the single-query decode oracle at N = 1, causality,
and normalisation of the averaged weights."""
import numpy as np
import pytest
from scipy.special import logsumexp, softmax

from oracle import append_stage as ap


def make(seed, B, N, Hq, Hkv, d, W, P, w_lens=None, p_lens=None):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, N, Hq, d))
    Kw, Vw = rng.standard_normal((B, Hkv, W, d)), rng.standard_normal((B, Hkv, W, d))
    Kp, Vp = rng.standard_normal((B, Hkv, P, d)), rng.standard_normal((B, Hkv, P, d))
    w_lens = np.full(B, W) if w_lens is None else np.asarray(w_lens)
    p_lens = np.full(B, P) if p_lens is None else np.asarray(p_lens)
    return q, Kw, Vw, w_lens, Kp, Vp, p_lens


@pytest.mark.parametrize("B,N,Hq,Hkv,d,W,P,w_lens,p_lens", [
    (2, 5, 4, 2, 8, 19, 23, None, None),
    (3, 7, 6, 3, 4, 30, 11, (30, 9, 7), (11, 0, 5)),
    (1, 4, 2, 2, 8, 4, 16, None, None),          # the window holds nothing but the incoming tokens
])
def test_merge_equals_one_causal_softmax_over_pool_then_window(B, N, Hq, Hkv, d, W, P, w_lens, p_lens):
    scale = 0.37
    q, Kw, Vw, wl_, Kp, Vp, pl_ = make(1, B, N, Hq, Hkv, d, W, P, w_lens, p_lens)
    o, lse, A_g, A_c = ap.append_step(q, Kw, Vw, wl_, Kp, Vp, pl_, scale)
    G = Hq // Hkv
    for b in range(B):
        nw, npool = int(wl_[b]), int(pl_[b])
        for h in range(Hq):
            K = np.concatenate([Kp[b, h // G, :npool], Kw[b, h // G, :nw]])
            V = np.concatenate([Vp[b, h // G, :npool], Vw[b, h // G, :nw]])
            S = scale * (q[b, :, h] @ K.T)                       # [N, n]
            pos = np.arange(K.shape[0])[None, :]
            last_visible = npool + nw - N + np.arange(N)[:, None]
            S = np.where(pos <= last_visible, S, -np.inf)
            np.testing.assert_allclose(o[b, :, h], softmax(S, axis=1) @ V, atol=1e-12)
            np.testing.assert_allclose(lse[b, :, h], logsumexp(S, axis=1), atol=1e-12)
            # the averaged weights: each part normalised within itself
            Aw = softmax(S[:, npool:], axis=1).mean(0)
            np.testing.assert_allclose(A_g[b, h, :nw], Aw, atol=1e-13)
            if npool:
                np.testing.assert_allclose(A_c[b, h, :npool], softmax(S[:, :npool], axis=1).mean(0), atol=1e-13)
                assert A_c[b, h, :npool].sum() == pytest.approx(1.0, abs=1e-12)
            assert A_g[b, h, :nw].sum() == pytest.approx(1.0, abs=1e-12)
            assert np.all(A_g[b, h, nw:] == 0) and np.all(A_c[b, h, npool:] == 0)


def test_single_query_is_the_decode_step(oracle):
    """N = 1: the append branch is the decode branch with every offloaded entry attended."""
    B, Hq, Hkv, d, W, P = 2, 4, 2, 8, 13, 21
    q, Kw, Vw, wl_, Kp, Vp, pl_ = make(2, B, 1, Hq, Hkv, d, W, P, (13, 6), (21, 17))
    f32 = lambda x: np.ascontiguousarray(x, dtype=np.float32)
    q, Kw, Vw, Kp, Vp = map(f32, (q, Kw, Vw, Kp, Vp))
    o, lse, A_g, _ = ap.append_step(q, Kw, Vw, wl_, Kp, Vp, pl_, 0.5)
    tw = oracle.Tier(Kw, Vw, W, np.asarray(wl_, np.int32))
    tp = oracle.Tier(Kp, Vp, P, np.asarray(pl_, np.int32))
    o_ref, lse_ref = oracle.attend_union(q[:, 0], tw, tp, None, None, 0.5)
    np.testing.assert_allclose(o[:, 0], o_ref, atol=1e-12)
    np.testing.assert_allclose(lse[:, 0], lse_ref, atol=1e-12)
    np.testing.assert_allclose(A_g, oracle.window_weights(q[:, 0], tw, 0.5), atol=1e-13)


def test_causality_later_tokens_do_not_reach_earlier_queries():
    B, N, Hq, Hkv, d, W, P = 1, 6, 2, 1, 4, 20, 9
    q, Kw, Vw, wl_, Kp, Vp, pl_ = make(3, B, N, Hq, Hkv, d, W, P)
    o1, lse1, _, _ = ap.append_step(q, Kw, Vw, wl_, Kp, Vp, pl_, 1.0)
    Kw2, Vw2 = Kw.copy(), Vw.copy()
    Kw2[:, :, W - 2:] += 5.0                                      # the last two incoming tokens change
    Vw2[:, :, W - 2:] -= 3.0
    o2, lse2, _, _ = ap.append_step(q, Kw2, Vw2, wl_, Kp, Vp, pl_, 1.0)
    np.testing.assert_array_equal(o1[:, :N - 2], o2[:, :N - 2])   # queries 0..N-3 never saw them
    np.testing.assert_array_equal(lse1[:, :N - 2], lse2[:, :N - 2])
    assert np.abs(o1[:, N - 2:] - o2[:, N - 2:]).max() > 1e-3


def test_hand_worked_two_queries():
    """d = 1, q = 0 => uniform weights.  Pool of 2, window of 3 whose last 2 entries are incoming.
    Query 0 sees pool(2) + window[0..1]: mean of 4 values; query 1 sees all 5."""
    q = np.zeros((1, 2, 1, 1))
    Kw = np.zeros((1, 1, 3, 1)); Vw = np.array([10.0, 20.0, 30.0]).reshape(1, 1, 3, 1)
    Kp = np.zeros((1, 1, 2, 1)); Vp = np.array([1.0, 2.0]).reshape(1, 1, 2, 1)
    o, lse, A_g, A_c = ap.append_step(q, Kw, Vw, np.array([3]), Kp, Vp, np.array([2]), 1.0)
    assert o[0, 0, 0, 0] == pytest.approx((1 + 2 + 10 + 20) / 4) and lse[0, 0, 0] == pytest.approx(np.log(4))
    assert o[0, 1, 0, 0] == pytest.approx((1 + 2 + 10 + 20 + 30) / 5) and lse[0, 1, 0] == pytest.approx(np.log(5))
    np.testing.assert_allclose(A_g[0, 0], [(1 / 2 + 1 / 3) / 2, (1 / 2 + 1 / 3) / 2, (0 + 1 / 3) / 2], atol=1e-15)
    np.testing.assert_allclose(A_c[0, 0], [0.5, 0.5], atol=1e-15)
