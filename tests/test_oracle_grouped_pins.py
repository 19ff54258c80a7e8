"""Pins of the group-shared list oracle (paper Sec. 3.3, merged heads) — no GPU needed."""
import numpy as np
import pytest
from scipy.special import logsumexp, softmax

from oracle import grouped


def rand(rng, *s):
    return rng.standard_normal(s).astype(np.float32)


def test_group_scores_hand_worked_and_group_of_one():
    s = np.array([[[1.0, 5.0, 2.0], [4.0, 0.0, 3.0], [7.0, 7.0, 7.0], [-1.0, 8.0, 6.0]]])      # [1, 4, 3]
    np.testing.assert_array_equal(grouped.group_scores(s, 2), [[[4.0, 5.0, 3.0], [7.0, 8.0, 7.0]]])
    np.testing.assert_array_equal(grouped.group_scores(s, 4), s)                                # groups of one head


def test_union_hand_worked():
    idx = np.array([[[0, 3, 9, -1], [3, 4, -1, -1], [1, 2, 3, 4], [-1, -1, -1, -1]]], np.int32)
    cnt = np.array([[3, 2, 4, 0]], np.int32)
    u, c = grouped.union_lists(idx, cnt, 2, 8)
    assert u[0, 0].tolist() == [0, 3, 4, 9, -1, -1, -1, -1] and u[0, 1].tolist() == [1, 2, 3, 4, -1, -1, -1, -1]
    assert c.tolist() == [[4, 4]]
    u1, c1 = grouped.union_lists(idx, cnt, 4, 4)                  # groups of one: the lists themselves
    np.testing.assert_array_equal(u1, idx)
    np.testing.assert_array_equal(c1, cnt)


def test_grouped_budget_matches_argsort_of_the_group_maximum(oracle):
    rng = np.random.default_rng(5)
    B, Hq, Hkv, P, d, k = 2, 8, 2, 90, 8, 11
    q, K = rand(rng, B, Hq, d), rand(rng, B, Hkv, P, d)
    lens = np.array([90, 33], np.int32)
    pool = oracle.Tier(K, K, P, lens)
    idx, cnt = grouped.select_grouped(q, pool, k, k, 0.4, round_scores_to_f32=False)
    for b in range(B):
        for kvh in range(Hkv):
            s = np.stack([0.4 * (K[b, kvh, :lens[b]].astype(np.float64) @ q[b, h].astype(np.float64))
                          for h in range(kvh * 4, kvh * 4 + 4)]).max(axis=0)
            want = sorted(np.argsort(-s, kind="stable")[:k].tolist())
            assert cnt[b, kvh] == k and idx[b, kvh].tolist() == want


def test_attend_grouped_is_library_attention_over_the_shared_rows(oracle):
    rng = np.random.default_rng(6)
    B, Hq, Hkv, P, d = 2, 4, 2, 40, 8
    q, K, V = rand(rng, B, Hq, d), rand(rng, B, Hkv, P, d), rand(rng, B, Hkv, P, d)
    pool = oracle.Tier(K, V, P)
    idx = np.array([[[1, 5, 7, 30, -1], [0, 2, -1, -1, -1]], [[3, -1, -1, -1, -1], [4, 8, 12, 16, 39]]], np.int32)
    cnt = np.array([[4, 2], [1, 5]], np.int32)
    o, lse = grouped.attend_grouped(q, pool, idx, cnt, 0.5)
    for b in range(B):
        for h in range(Hq):
            rows = idx[b, h // 2, :cnt[b, h // 2]]
            s = 0.5 * (K[b, h // 2, rows].astype(np.float64) @ q[b, h].astype(np.float64))
            np.testing.assert_allclose(o[b, h], softmax(s) @ V[b, h // 2, rows].astype(np.float64), atol=1e-13)
            assert lse[b, h] == pytest.approx(logsumexp(s), abs=1e-13)


def test_union_keeps_everything_each_head_selected(oracle):
    rng = np.random.default_rng(7)
    B, Hq, Hkv, P, d, k = 2, 8, 2, 120, 8, 9
    q, K = rand(rng, B, Hq, d), rand(rng, B, Hkv, P, d)
    pool = oracle.Tier(K, K, P)
    idx, cnt = oracle.select(q, pool, k, k, 0.3)
    u, c = grouped.union_lists(idx, cnt, Hkv, 4 * k)
    for b in range(B):
        for h in range(Hq):
            assert set(idx[b, h, :k].tolist()) <= set(u[b, h // 4, :c[b, h // 4]].tolist())
    assert np.all(c >= k) and np.all(c <= 4 * k)
