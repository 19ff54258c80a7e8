"""Pins of the oracle's paper-literal sparsifier (no GPU needed): the window's
attention weights A_gpu (paper Alg. 2), their moving average (Alg. 1) and the
per-head threshold rule keep-iff-weight > beta/size (Sec. 3.2.2).

Pinned against library softmax on a numpy contraction, closed forms of the
exponential moving average, hand-worked numbers and a numpy brute force.
"""
import numpy as np
import pytest
from scipy.special import softmax

from paper_2507_03153_amd import workloads as wl


def rand(rng, *shape):
    return rng.standard_normal(shape).astype(np.float32)


def tier(oracle, k, v, **kw):
    return oracle.Tier(np.ascontiguousarray(k), np.ascontiguousarray(v), cap=k.shape[2], **kw)


# ------------------------------------------------------------ window weights

@pytest.mark.parametrize("B,Hq,Hkv,n,d", [(2, 4, 4, 19, 8), (3, 8, 2, 50, 16)])
def test_window_weights_match_library_softmax(oracle, B, Hq, Hkv, n, d):
    rng = np.random.default_rng(5)
    q, K, V = rand(rng, B, Hq, d), rand(rng, B, Hkv, n, d), rand(rng, B, Hkv, n, d)
    G = Hq // Hkv
    a = oracle.window_weights(q, tier(oracle, K, V), 0.31)
    for b in range(B):
        for h in range(Hq):
            s = 0.31 * (K[b, h // G].astype(np.float64) @ q[b, h].astype(np.float64))
            np.testing.assert_allclose(a[b, h], softmax(s), rtol=1e-12, atol=1e-16)
    np.testing.assert_allclose(a.sum(-1), 1.0, atol=1e-13)


def test_window_weights_times_values_is_the_attention_output(oracle):
    rng = np.random.default_rng(6)
    q, K, V = rand(rng, 2, 6, 8), rand(rng, 2, 3, 23, 8), rand(rng, 2, 3, 23, 8)
    lens = np.array([23, 9], np.int32)
    t = tier(oracle, K, V, seq_lens=lens)
    a = oracle.window_weights(q, t, 0.5)
    o, _ = oracle.attend_all(q, t, 0.5)
    Vh = np.repeat(V.astype(np.float64), 2, axis=1)          # [B,Hq,n,d]
    np.testing.assert_allclose(np.einsum("bhn,bhnd->bhd", a, Vh), o, atol=1e-13)
    assert np.all(a[1, :, 9:] == 0.0) and np.all(a[1, :, :9] > 0.0)
    np.testing.assert_allclose(a.sum(-1), 1.0, atol=1e-13)


def test_window_weights_two_keys_closed_form(oracle):
    # scores 0 and ln 3  =>  weights 1/4 and 3/4
    q = np.array([[[1.0, 0.0]]], np.float32)
    K = np.array([[[[0.0, 5.0], [1.0, -2.0]]]], np.float32)
    V = np.zeros_like(K)
    a = oracle.window_weights(q, tier(oracle, K, V), float(np.log(3.0)))
    np.testing.assert_allclose(a[0, 0], [0.25, 0.75], atol=1e-15)


def test_window_weights_bf16_and_empty(oracle):
    rng = np.random.default_rng(7)
    q, K, V = rand(rng, 2, 2, 8), rand(rng, 2, 2, 5, 8), rand(rng, 2, 2, 5, 8)
    qb, Kb, Vb = (wl.f32_to_bf16_bits(x) for x in (q, K, V))
    lens = np.array([0, 5], np.int32)
    a16 = oracle.window_weights(qb, tier(oracle, Kb, Vb, seq_lens=lens), 1.0)
    a32 = oracle.window_weights(wl.bf16_bits_to_f32(qb),
                                tier(oracle, wl.bf16_bits_to_f32(Kb), wl.bf16_bits_to_f32(Vb), seq_lens=lens), 1.0)
    np.testing.assert_array_equal(a16, a32)
    assert np.all(a16[0] == 0.0)


# ------------------------------------------------------------ moving average

def test_maw_hand_worked(oracle):
    maw = np.array([[[0.2, 0.4]]])
    a = np.array([[[0.6, 0.0]]])
    np.testing.assert_allclose(oracle.maw_update(maw, a, 0.25), [[[0.3, 0.3]]], atol=1e-16)
    assert maw[0, 0, 0] == 0.2                                  # input not modified


def test_maw_limits_and_geometric_closed_form(oracle):
    rng = np.random.default_rng(8)
    maw0, a = rng.random((2, 3, 11)), rng.random((2, 3, 11))
    np.testing.assert_array_equal(oracle.maw_update(maw0, a, 0.0), maw0)
    np.testing.assert_allclose(oracle.maw_update(maw0, a, 1.0), a, atol=1e-16)
    alpha, n = 0.3, 9
    m = maw0
    for _ in range(n):
        m = oracle.maw_update(m, a, alpha)
    # constant observation: maw_n = a + (1-alpha)^n (maw_0 - a)
    np.testing.assert_allclose(m, a + (1 - alpha) ** n * (maw0 - a), atol=1e-14)


def test_maw_is_a_convex_combination_and_keeps_row_sums(oracle):
    rng = np.random.default_rng(9)
    maw0 = softmax(rng.standard_normal((2, 2, 16)), axis=-1)
    a = softmax(rng.standard_normal((2, 2, 16)), axis=-1)
    m = oracle.maw_update(maw0, a, 0.4)
    assert np.all(m >= np.minimum(maw0, a) - 1e-16) and np.all(m <= np.maximum(maw0, a) + 1e-16)
    np.testing.assert_allclose(m.sum(-1), 1.0, atol=1e-14)


def test_maw_new_entries_and_lengths(oracle):
    rng = np.random.default_rng(10)
    maw0, a = rng.random((2, 2, 8)), rng.random((2, 2, 8))
    lens = np.array([8, 5], np.int32)
    m = oracle.maw_update(maw0, a, 0.5, lens=lens, n_new=2)
    np.testing.assert_allclose(m[0, :, :6], 0.5 * maw0[0, :, :6] + 0.5 * a[0, :, :6], atol=1e-16)
    np.testing.assert_array_equal(m[0, :, 6:], a[0, :, 6:])     # first observation
    np.testing.assert_allclose(m[1, :, :3], 0.5 * maw0[1, :, :3] + 0.5 * a[1, :, :3], atol=1e-16)
    np.testing.assert_array_equal(m[1, :, 3:5], a[1, :, 3:5])
    np.testing.assert_array_equal(m[1, :, 5:], maw0[1, :, 5:])  # beyond the length: untouched
    # more new entries than the row holds: everything is a first observation
    m = oracle.maw_update(maw0, a, 0.5, lens=lens, n_new=7)
    np.testing.assert_array_equal(m[1, :, :5], a[1, :, :5])


# ------------------------------------------------------------ threshold rule

def test_threshold_hand_worked(oracle):
    # size 4, beta 1: threshold 0.25 -> positions 0 and 2; 0.5/0.8 and 0.3/0.8
    w = np.array([[[0.5, 0.05, 0.3, 0.15]]])
    idx, cnt, wn = oracle.threshold_select(w, 1.0, 4, 4, normalised=True)
    assert cnt[0, 0] == 2 and idx[0, 0].tolist() == [0, 2, -1, -1]
    np.testing.assert_allclose(wn[0, 0], [0.625, 0.375, 0.0, 0.0], atol=1e-16)
    # beta 0.5: threshold 0.125 -> 0, 2, 3
    idx, cnt = oracle.threshold_select(w, 0.5, 4, 4)
    assert cnt[0, 0] == 3 and idx[0, 0].tolist() == [0, 2, 3, -1]


def test_threshold_is_strict_on_uniform_weights(oracle):
    n = 8                                                        # 1/8 is exact in binary
    w = np.full((1, 2, n), 1.0 / n)
    _, cnt = oracle.threshold_select(w, 1.0, n, n)
    assert cnt.tolist() == [[0, 0]]                              # equal to the threshold: dropped
    idx, cnt = oracle.threshold_select(w, 0.99, n, n)
    assert cnt.tolist() == [[n, n]] and idx[0, 0].tolist() == list(range(n))
    # the size the weights were taken over is an argument, not the row length
    _, cnt = oracle.threshold_select(w, 1.0, 2 * n, n)
    assert cnt.tolist() == [[n, n]]


def test_threshold_matches_numpy_brute_force(oracle):
    rng = np.random.default_rng(11)
    B, Hq, cap = 3, 4, 57
    w = softmax(3.0 * rng.standard_normal((B, Hq, cap)), axis=-1)
    lens = np.array([57, 20, 0], np.int32)
    sizes = np.array([57, 64, 5], np.int32)
    idx, cnt, wn = oracle.threshold_select(w, 0.8, sizes, cap, lens=lens, normalised=True)
    for b in range(B):
        for h in range(Hq):
            keep = np.nonzero(w[b, h, :lens[b]] > 0.8 / sizes[b])[0]
            assert cnt[b, h] == len(keep)
            assert idx[b, h, :len(keep)].tolist() == keep.tolist()
            assert np.all(idx[b, h, len(keep):] == -1)
            if len(keep):
                np.testing.assert_allclose(wn[b, h, :len(keep)], w[b, h, keep] / w[b, h, keep].sum(), atol=1e-15)
                assert wn[b, h, :len(keep)].sum() == pytest.approx(1.0, abs=1e-14)
    assert np.all(cnt[2] == 0)


def test_threshold_keeps_the_first_k_max_when_more_pass(oracle):
    w = np.array([[[0.3, 0.0, 0.3, 0.3, 0.1]]])
    idx, cnt, wn = oracle.threshold_select(w, 1.0, 5, 2, normalised=True)
    assert cnt[0, 0] == 2 and idx[0, 0].tolist() == [0, 2]
    np.testing.assert_allclose(wn[0, 0], [0.5, 0.5], atol=1e-16)


def test_peaked_head_keeps_fewer_than_flat_head(oracle):
    """Sec. 3.2.2: the rule adapts per head: sharp distributions keep few entries, flat ones many."""
    rng = np.random.default_rng(12)
    z = rng.standard_normal(256)
    w = np.stack([softmax(8.0 * z), softmax(0.5 * z)])[None]
    _, cnt = oracle.threshold_select(w, 1.0, 256, 256)
    assert 0 < cnt[0, 0] < cnt[0, 1] < 256


# ------------------------------------------------------------ top-k on supplied scores

def test_select_given_matches_stable_argsort_and_the_scoring_select(oracle):
    rng = np.random.default_rng(13)
    B, Hq, cap = 3, 4, 61
    s = np.round(rng.standard_normal((B, Hq, cap)), 1)            # rounded: plenty of exact ties
    lens = np.array([61, 17, 0], np.int32)
    ks = np.array([10, 30, 5], np.int32)
    idx, cnt = oracle.select_given(s, ks, 32, lens=lens)
    for b in range(B):
        kb = min(ks[b], lens[b])
        for h in range(Hq):
            order = np.argsort(-s[b, h, :lens[b]], kind="stable")[:kb]   # stable: lower position first on ties
            assert cnt[b, h] == kb
            assert idx[b, h, :kb].tolist() == sorted(order.tolist())
            assert np.all(idx[b, h, kb:] == -1)
    # fed the oracle's own scores it reproduces the scoring selection
    q, K = rand(rng, 2, 4, 8), rand(rng, 2, 2, 40, 8)
    t = tier(oracle, K, K)
    sc = oracle.scores(q, t, 0.4)
    i1, c1 = oracle.select(q, t, 7, 7, 0.4, round_scores_to_f32=False)
    i2, c2 = oracle.select_given(sc, 7, 7)
    assert np.array_equal(i1, i2) and np.array_equal(c1, c2)


def test_select_given_with_infinite_scores_matches_stable_argsort(oracle):
    """+inf and -inf are ordinary values (masked positions): they rank above / below every finite score, ties among
    them by position; also when the budget reaches into the -inf entries."""
    rng = np.random.default_rng(14)
    B, Hq, cap = 2, 3, 80
    s = rng.standard_normal((B, Hq, cap))
    s[:, :, rng.integers(0, cap, 6)] = np.inf
    s[:, :, rng.integers(0, cap, 30)] = -np.inf
    for k in (1, 5, 40, 70, 79):
        idx, cnt = oracle.select_given(s, k, k)
        for b in range(B):
            for h in range(Hq):
                order = np.argsort(-s[b, h], kind="stable")[:k]
                assert cnt[b, h] == k and idx[b, h].tolist() == sorted(order.tolist())
    hand = np.array([[[-np.inf, 2.0, np.inf, -np.inf, np.inf, 0.5]]])
    assert oracle.select_given(hand, 1, 1)[0][0, 0].tolist() == [2]
    assert oracle.select_given(hand, 3, 3)[0][0, 0].tolist() == [1, 2, 4]
    assert oracle.select_given(hand, 5, 5)[0][0, 0].tolist() == [0, 1, 2, 4, 5]


def test_select_given_hand_worked(oracle):
    s = np.array([[[0.1, 0.7, 0.7, -1.0, 0.3]]])
    idx, cnt = oracle.select_given(s, 2, 3)
    assert idx[0, 0].tolist() == [1, 2, -1] and cnt[0, 0] == 2
    idx, cnt = oracle.select_given(s, 1, 1)
    assert idx[0, 0].tolist() == [1]                              # tie: the lower position is kept
    idx, cnt = oracle.select_given(s, 3, 3)
    assert idx[0, 0].tolist() == [1, 2, 4]
