"""Pins of the CPU oracle against things other than itself (no GPU needed).

Closed forms, hand-derived worked examples (tests/golden), library routines the
oracle does not call (scipy softmax / logsumexp, numpy argsort / matmul),
pure-Python brute force on tiny inputs, and the two invariants the method rests on:
  * merging the partial results of two disjoint sets equals one softmax over
    their union (paper Sec. 3.3, "Merging states");
  * selecting every offloaded entry reproduces full attention (Sec. 2.1, Sec. 3.1).
"""
import math
import os

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

from paper_2507_03153_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tier(oracle, k, v, **kw):
    k = np.ascontiguousarray(k)
    v = np.ascontiguousarray(v)
    return oracle.Tier(k, v, cap=kw.pop("cap", k.shape[2]), **kw)


def as_tier(oracle, t):
    return oracle.Tier(t.k, t.v, t.cap, t.seq_lens, t.block_table, t.block_size)


def rand(rng, *shape):
    return rng.standard_normal(shape).astype(np.float32)


def read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                key, *vals = line.split()
                out[key] = np.array([float(x) for x in vals])
    return out


def lib_attention(q, K, V, scale, G):
    """Independent fp64 formulation with library routines: softmax(scale q K^T) V, logsumexp."""
    B, Hq, d = q.shape
    o = np.zeros((B, Hq, d))
    lse = np.zeros((B, Hq))
    for b in range(B):
        for h in range(Hq):
            s = scale * (K[b, h // G].astype(np.float64) @ q[b, h].astype(np.float64))
            o[b, h] = softmax(s) @ V[b, h // G].astype(np.float64)
            lse[b, h] = logsumexp(s)
    return o, lse


# ---------------------------------------------------------------- closed forms

def test_single_key_returns_its_value_and_score(oracle):
    rng = np.random.default_rng(1)
    q, K, V = rand(rng, 1, 1, 8), rand(rng, 1, 1, 1, 8), rand(rng, 1, 1, 1, 8)
    o, lse = oracle.attend_all(q, tier(oracle, K, V), 0.37)
    expect = 0.37 * float(np.dot(q[0, 0].astype(np.float64), K[0, 0, 0].astype(np.float64)))
    assert lse[0, 0] == pytest.approx(expect, abs=1e-14)
    np.testing.assert_allclose(o[0, 0], V[0, 0, 0].astype(np.float64), atol=1e-15)


def test_identical_keys_average_values(oracle):
    rng = np.random.default_rng(2)
    n, d = 7, 6
    q = rand(rng, 1, 1, d)
    K = np.repeat(rand(rng, 1, 1, 1, d), n, axis=2)
    V = rand(rng, 1, 1, n, d)
    o, lse = oracle.attend_all(q, tier(oracle, K, V), 1.0)
    s = float(np.dot(q[0, 0].astype(np.float64), K[0, 0, 0].astype(np.float64)))
    assert lse[0, 0] == pytest.approx(s + math.log(n), abs=1e-13)
    np.testing.assert_allclose(o[0, 0], V[0, 0].astype(np.float64).mean(0), atol=1e-14)


def test_zero_query_gives_uniform_weights(oracle):
    rng = np.random.default_rng(3)
    n, d = 11, 4
    q = np.zeros((1, 2, d), np.float32)
    K, V = rand(rng, 1, 2, n, d), rand(rng, 1, 2, n, d)
    o, lse = oracle.attend_all(q, tier(oracle, K, V), 0.5)
    np.testing.assert_allclose(lse, math.log(n), atol=1e-14)
    np.testing.assert_allclose(o[0], V[0].astype(np.float64).mean(1), atol=1e-14)


def test_constant_values_pass_through(oracle):
    rng = np.random.default_rng(4)
    q, K = rand(rng, 2, 3, 5), rand(rng, 2, 3, 9, 5)
    V = np.broadcast_to(np.float32([1.5, -2, 0.25, 8, -0.5]), (2, 3, 9, 5)).copy()
    o, _ = oracle.attend_all(q, tier(oracle, K, V), 0.3)
    np.testing.assert_allclose(o, np.broadcast_to(V[0, 0, 0].astype(np.float64), o.shape), atol=1e-13)


def test_two_keys_known_weights(oracle):
    # scores ln 1 and ln 3 => weights 1/4 and 3/4, lse = ln 4
    q = np.float32([[[1.0, 0.0]]])
    K = np.float32([[[[0.0, 5.0], [math.log(3.0), -2.0]]]])
    V = np.float32([[[[8.0, 0.0], [0.0, 4.0]]]])
    o, lse = oracle.attend_all(q, tier(oracle, K, V), 1.0)
    w1 = math.exp(float(np.float32(math.log(3.0))))            # ln 3 as stored in fp32
    assert lse[0, 0] == pytest.approx(math.log(1.0 + w1), abs=1e-14)
    np.testing.assert_allclose(o[0, 0], [8.0 / (1 + w1), 4.0 * w1 / (1 + w1)], atol=1e-14)


def test_gqa_head_to_kv_head_mapping(oracle):
    # Hq = 6 over Hkv = 2: heads 0..2 must read KV head 0, heads 3..5 KV head 1.
    # Within a KV head all keys are equal, so O is the mean of that head's values.
    rng = np.random.default_rng(5)
    q = rand(rng, 1, 6, 4)
    K = np.repeat(rand(rng, 1, 2, 1, 4), 5, axis=2)
    V = rand(rng, 1, 2, 5, 4)
    o, _ = oracle.attend_all(q, tier(oracle, K, V), 1.0)
    for h in range(6):
        np.testing.assert_allclose(o[0, h], V[0, h // 3].astype(np.float64).mean(0), atol=1e-14)


# ------------------------------------------------------- library second opinion

@pytest.mark.parametrize("B,Hq,Hkv,n,d", [(2, 4, 4, 33, 16), (3, 8, 2, 70, 24), (1, 6, 3, 5, 3)])
def test_attend_all_matches_scipy(oracle, B, Hq, Hkv, n, d):
    rng = np.random.default_rng(10 + n)
    q, K, V = rand(rng, B, Hq, d), rand(rng, B, Hkv, n, d), rand(rng, B, Hkv, n, d)
    scale = 1.0 / math.sqrt(d)
    o, lse = oracle.attend_all(q, tier(oracle, K, V), scale)
    eo, el = lib_attention(q, K, V, scale, Hq // Hkv)
    np.testing.assert_allclose(o, eo, atol=1e-13)
    np.testing.assert_allclose(lse, el, atol=1e-13)


def test_scores_match_numpy_contraction(oracle):
    rng = np.random.default_rng(11)
    q, K = rand(rng, 2, 6, 10), rand(rng, 2, 3, 17, 10)
    s = oracle.scores(q, tier(oracle, K, K), 0.7)
    Kq = np.repeat(K.astype(np.float64), 2, axis=1)            # kv head of query head h is h // 2
    expect = 0.7 * np.einsum("bhd,bhtd->bht", q.astype(np.float64), Kq)
    np.testing.assert_allclose(s, expect, atol=1e-13)


def test_brute_force_python_loops(oracle):
    """W=3, P=5, d=4: window attention, indexed attention and union, by explicit loops."""
    rng = np.random.default_rng(12)
    q = rand(rng, 1, 2, 4)
    Kw, Vw = rand(rng, 1, 1, 3, 4), rand(rng, 1, 1, 3, 4)
    Kp, Vp = rand(rng, 1, 1, 5, 4), rand(rng, 1, 1, 5, 4)
    idx = np.array([[[0, 3, 4], [1, 2, -1]]], np.int32)
    cnt = np.array([[3, 2]], np.int32)
    scale = 0.5

    def brute(h, keys_vals):
        ss = []
        for kr, _ in keys_vals:
            ss.append(scale * math.fsum(float(q[0, h, c]) * float(kr[c]) for c in range(4)))
        z = math.fsum(math.exp(s) for s in ss)
        o = [math.fsum(math.exp(s) / z * float(vr[c]) for s, (_, vr) in zip(ss, keys_vals)) for c in range(4)]
        return o, math.log(z)

    tw, tp = tier(oracle, Kw, Vw), tier(oracle, Kp, Vp)
    ow, lw = oracle.attend_all(q, tw, scale)
    os_, ls = oracle.attend_indexed(q, tp, idx, cnt, scale)
    ou, lu = oracle.attend_union(q, tw, tp, idx, cnt, scale)
    for h in range(2):
        win = [(Kw[0, 0, t], Vw[0, 0, t]) for t in range(3)]
        sel = [(Kp[0, 0, t], Vp[0, 0, t]) for t in idx[0, h, :cnt[0, h]]]
        for got_o, got_l, items in ((ow, lw, win), (os_, ls, sel), (ou, lu, win + sel)):
            eo, el = brute(h, items)
            np.testing.assert_allclose(got_o[0, h], eo, atol=1e-14)
            assert got_l[0, h] == pytest.approx(el, abs=1e-14)


# -------------------------------------------------------------- element formats

def test_bf16_bits_are_widened_exactly(oracle):
    # 0x3F80 = 1.0, 0x4000 = 2.0, 0xC040 = -3.0, 0x3E00 = 0.125
    q = np.array([[[0x3F80, 0x0000]]], np.uint16)
    K = np.array([[[[0x4000, 0x7F00]]]], np.uint16)            # second lane huge but q there is 0
    V = np.array([[[[0xC040, 0x3E00]]]], np.uint16)
    o, lse = oracle.attend_all(q, tier(oracle, K, V), 0.25)
    assert lse[0, 0] == 0.5
    np.testing.assert_array_equal(o[0, 0], [-3.0, 0.125])


def test_bf16_matches_f32_of_same_values(oracle):
    rng = np.random.default_rng(13)
    qf, Kf, Vf = rand(rng, 2, 4, 8), rand(rng, 2, 2, 19, 8), rand(rng, 2, 2, 19, 8)
    qb, Kb, Vb = (wl.f32_to_bf16_bits(x) for x in (qf, Kf, Vf))
    o1, l1 = oracle.attend_all(qb, tier(oracle, Kb, Vb), 0.3)
    o2, l2 = oracle.attend_all(*(wl.bf16_bits_to_f32(x) for x in (qb,)), tier(
        oracle, wl.bf16_bits_to_f32(Kb), wl.bf16_bits_to_f32(Vb)), 0.3)
    np.testing.assert_array_equal(o1, o2)
    np.testing.assert_array_equal(l1, l2)


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 3.14159265], np.float32)
    # 1 + 2^-8 is a tie between 0x3F80 and 0x3F81 -> even (0x3F80); 1 + 3*2^-8 ties -> 0x3F82
    np.testing.assert_array_equal(wl.f32_to_bf16_bits(x), [0x3F80, 0x3F80, 0x3F82, 0xBF80, 0x4049])


# ------------------------------------------------------------- ragged and paged

def test_tokens_beyond_seq_len_are_ignored(oracle):
    rng = np.random.default_rng(14)
    q, K, V = rand(rng, 2, 2, 4), rand(rng, 2, 2, 9, 4), rand(rng, 2, 2, 9, 4)
    lens = np.array([4, 9], np.int32)
    Kx, Vx = K.copy(), V.copy()
    Kx[0, :, 4:] = 1e4
    Vx[0, :, 4:] = -1e4
    o, lse = oracle.attend_all(q, tier(oracle, Kx, Vx, seq_lens=lens), 0.5)
    e0 = lib_attention(q[:1], K[:1, :, :4], V[:1, :, :4], 0.5, 1)
    e1 = lib_attention(q[1:], K[1:], V[1:], 0.5, 1)
    np.testing.assert_allclose(o[0], e0[0][0], atol=1e-13)
    np.testing.assert_allclose(o[1], e1[0][0], atol=1e-13)
    np.testing.assert_allclose(lse, np.concatenate([e0[1], e1[1]]), atol=1e-13)


def test_empty_set_is_zero_and_minus_inf(oracle):
    rng = np.random.default_rng(15)
    q, K, V = rand(rng, 2, 2, 4), rand(rng, 2, 2, 3, 4), rand(rng, 2, 2, 3, 4)
    o, lse = oracle.attend_all(q, tier(oracle, K, V, seq_lens=np.array([0, 3], np.int32)), 1.0)
    assert np.all(o[0] == 0) and np.all(np.isneginf(lse[0])) and np.all(np.isfinite(lse[1]))
    idx = np.full((2, 2, 2), -1, np.int32)
    o, lse = oracle.attend_indexed(q, tier(oracle, K, V), idx, np.zeros((2, 2), np.int32), 1.0)
    assert np.all(o == 0) and np.all(np.isneginf(lse))


def test_paged_hand_built_block_table(oracle):
    # 2 physical blocks of 2 tokens; the sequence's logical block 0 lives in physical block 1.
    # Logical token 1 = physical block 1 slot 1.  With one valid... use lens=2 and equal keys.
    K = np.zeros((2, 1, 2, 2), np.float32)
    V = np.zeros((2, 1, 2, 2), np.float32)
    V[1, 0, 0] = [2.0, 4.0]
    V[1, 0, 1] = [6.0, 8.0]
    V[0, 0, :] = 1e6                                           # must not be touched
    t = oracle.Tier(K, V, cap=4, seq_lens=np.array([2], np.int32),
                    block_table=np.array([[1, 0]], np.int32), block_size=2)
    o, lse = oracle.attend_all(np.float32([[[1.0, 1.0]]]), t, 1.0)
    np.testing.assert_allclose(o[0, 0], [4.0, 6.0], atol=1e-15)
    assert lse[0, 0] == pytest.approx(math.log(2.0), abs=1e-15)


def test_paged_equals_contiguous(oracle):
    cfg = wl.scaled(wl.CONFIGS["C5"], B=3, Hq=4, Hkv=2, d=8, W=40, P=100, ragged=(30, 140), block_size=4)
    paged = wl.make_layer(cfg)
    flat = wl.make_layer(wl.scaled(cfg, block_size=0))
    np.testing.assert_array_equal(paged.q, flat.q)
    for name in ("window", "pool"):
        tp, tf = getattr(paged, name), getattr(flat, name)
        assert tp.block_table is not None and tf.block_table is None
        np.testing.assert_array_equal(tp.seq_lens, tf.seq_lens)
        op, lp = oracle.attend_all(paged.q, as_tier(oracle, tp), cfg.scale)
        of, lf = oracle.attend_all(flat.q, as_tier(oracle, tf), cfg.scale)
        np.testing.assert_array_equal(op, of)
        np.testing.assert_array_equal(lp, lf)
    ip, cp = oracle.select(paged.q, as_tier(oracle, paged.pool), paged.k, paged.k_max, cfg.scale)
    if_, cf = oracle.select(flat.q, as_tier(oracle, flat.pool), flat.k, flat.k_max, cfg.scale)
    np.testing.assert_array_equal(ip, if_)
    np.testing.assert_array_equal(cp, cf)


# -------------------------------------------------------------------- selection

def test_select_worked_example(oracle):
    g = read_golden("select_worked_example.txt")
    K = np.stack([g["a"], g["b"]], axis=-1).astype(np.float32)[None]      # [1, 8, 2]
    K = np.stack([K[0], K[0]])[None]                                       # MHA: same keys for both KV heads
    q = np.float32([[[1, 0], [0, 1]]])
    idx, cnt = oracle.select(q, tier(oracle, K, K), int(g["k"][0]), 4, 1.0)
    np.testing.assert_array_equal(cnt, [[3, 3]])
    np.testing.assert_array_equal(idx[0, 0], list(g["head0"].astype(int)) + [-1])
    np.testing.assert_array_equal(idx[0, 1], list(g["head1"].astype(int)) + [-1])


@pytest.mark.parametrize("round32", [False, True])
def test_select_matches_stable_argsort(oracle, round32):
    rng = np.random.default_rng(20)
    B, Hq, Hkv, n, d, k = 2, 6, 2, 200, 8, 37
    q, K = rand(rng, B, Hq, d), rand(rng, B, Hkv, n, d)
    K[:, :, 50:60] = K[:, :, 40:50]                     # exact duplicates => exact ties
    idx, cnt = oracle.select(q, tier(oracle, K, K), k, k, 0.35, round_scores_to_f32=round32)
    for b in range(B):
        for h in range(Hq):
            s = 0.35 * (K[b, h // 3].astype(np.float64) @ q[b, h].astype(np.float64))
            if round32:
                s = s.astype(np.float32).astype(np.float64)
            order = np.argsort(-s, kind="stable")[:k]   # stable: ties keep ascending position
            np.testing.assert_array_equal(idx[b, h], np.sort(order))
    assert np.all(cnt == k)


def test_select_decides_in_fp32_when_asked(oracle):
    # scores 1 + 2^-30 (pos 1) vs 1 (pos 0): distinct in fp64, equal once rounded to fp32.
    q = np.float32([[[1.0, 1.0]]])
    K = np.float32([[[[1.0, 0.0], [1.0, 2.0 ** -30], [0.5, 0.0]]]])
    t = tier(oracle, K, K)
    idx64, _ = oracle.select(q, t, 1, 1, 1.0, round_scores_to_f32=False)
    idx32, _ = oracle.select(q, t, 1, 1, 1.0, round_scores_to_f32=True)
    assert idx64[0, 0, 0] == 1 and idx32[0, 0, 0] == 0


def test_select_budget_edge_cases(oracle):
    rng = np.random.default_rng(21)
    q, K = rand(rng, 3, 2, 4), rand(rng, 3, 2, 10, 4)
    lens = np.array([10, 4, 0], np.int32)
    t = tier(oracle, K, K, seq_lens=lens)
    idx, cnt = oracle.select(q, t, 6, 6, 1.0)                  # k > P_b clamps; P_b = 0 selects nothing
    np.testing.assert_array_equal(cnt, [[6, 6], [4, 4], [0, 0]])
    np.testing.assert_array_equal(idx[1, 0], [0, 1, 2, 3, -1, -1])
    assert np.all(idx[2] == -1)
    idx, cnt = oracle.select(q, t, np.array([0, 2, 5], np.int32), 5, 1.0)   # per-sequence budgets
    np.testing.assert_array_equal(cnt, [[0, 0], [2, 2], [0, 0]])
    for b in range(3):
        for h in range(2):
            row = idx[b, h, :cnt[b, h]]
            assert np.all(np.diff(row) > 0) and np.all(row < lens[b])


def test_planted_keys_are_mostly_selected(oracle):
    L = wl.make_layer(wl.CONFIGS["C1"])
    idx, cnt = oracle.select(L.q, as_tier(oracle, L.pool), L.k, L.k_max, L.scale)
    for h in range(4):
        hit = len(set(L.planted[0][h].tolist()) & set(idx[0, h, :cnt[0, h]].tolist()))
        assert hit >= 12, (h, hit)                             # statistical sanity, 16 planted per head


# ------------------------------------------------------------------------ merge

def test_merge_worked_example(oracle):
    g = read_golden("merge_worked_example.txt")
    q = np.float32([[[1.0, 0.0]]])
    Kw = np.stack([np.log(g["window_exp_scores"]), np.zeros(2)], -1).astype(np.float64)
    Kp = np.stack([np.log(g["pool_exp_scores"]), np.zeros(1)], -1).astype(np.float64)
    # exact-in-fp32 inputs are needed for the oracle; use the rounded keys for the expectation too
    Kw32, Kp32 = Kw.astype(np.float32), Kp.astype(np.float32)
    Vw = g["window_values"].reshape(2, 2).astype(np.float32)
    Vp = g["pool_values"].reshape(1, 2).astype(np.float32)
    og, lg = oracle.attend_all(q, tier(oracle, Kw32[None, None], Vw[None, None]), 1.0)
    oc, lc = oracle.attend_all(q, tier(oracle, Kp32[None, None], Vp[None, None]), 1.0)
    tol = 1e-6                                                 # ln 2, ln 6, ln 8 are rounded to fp32
    assert math.exp(lg[0, 0]) == pytest.approx(g["exp_lse_g"][0], rel=tol)
    assert math.exp(lc[0, 0]) == pytest.approx(g["exp_lse_c"][0], rel=tol)
    np.testing.assert_allclose(og[0, 0], g["o_gpu"], rtol=tol)
    np.testing.assert_allclose(oc[0, 0], g["o_cpu"], rtol=tol)
    # the merge itself, fed the exact printed partials
    o, lse = oracle.merge(g["o_cpu"][None], np.log(g["exp_lse_c"]), g["o_gpu"][None], np.log(g["exp_lse_g"]))
    np.testing.assert_allclose(o[0], g["o"], atol=1e-15)
    assert lse[0] == pytest.approx(math.log(g["exp_lse"][0]), abs=1e-15)


def test_merge_with_empty_side_is_identity_and_both_empty(oracle):
    rng = np.random.default_rng(30)
    o_a, l_a = rng.standard_normal((5, 3)), rng.standard_normal(5)
    zeros, ninf = np.zeros((5, 3)), np.full(5, -np.inf)
    for args in ((o_a, l_a, zeros, ninf), (zeros, ninf, o_a, l_a)):
        o, lse = oracle.merge(*args)
        np.testing.assert_array_equal(o, o_a)
        np.testing.assert_array_equal(lse, l_a)
    o, lse = oracle.merge(zeros, ninf, zeros, ninf)
    assert np.all(o == 0) and np.all(np.isneginf(lse))


def test_merge_printed_formula_commutes_and_survives_large_lse(oracle):
    rng = np.random.default_rng(31)
    o_a, o_b = rng.standard_normal((6, 4)), rng.standard_normal((6, 4))
    l_a, l_b = rng.standard_normal(6) * 3, rng.standard_normal(6) * 3
    o, lse = oracle.merge(o_a, l_a, o_b, l_b)
    z = np.exp(l_a) + np.exp(l_b)                              # the paper's unshifted form
    np.testing.assert_allclose(o, (np.exp(l_a)[:, None] * o_a + np.exp(l_b)[:, None] * o_b) / z[:, None],
                               rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(lse, np.log(z), atol=1e-13)
    o2, lse2 = oracle.merge(o_b, l_b, o_a, l_a)
    np.testing.assert_allclose(o2, o, atol=1e-15)
    np.testing.assert_allclose(lse2, lse, atol=1e-15)
    # shifting both lse by +1000 must not change O (the printed form would overflow)
    o3, lse3 = oracle.merge(o_a, l_a + 1000, o_b, l_b + 1000)
    np.testing.assert_allclose(o3, o, atol=1e-12)
    np.testing.assert_allclose(lse3, lse + 1000, atol=1e-10)


# ------------------------------------------------------- the method's invariants

@pytest.mark.parametrize("name,kw", [
    ("C1", {}),
    ("C2", dict(B=2, Hq=8, Hkv=2, W=96, P=300, k=40)),
    ("C4", dict(B=1, Hq=8, Hkv=1, W=64, P=512, k=96)),
    ("C5", dict(B=4, Hq=4, Hkv=2, d=32, W=48, P=208, ragged=(16, 256), block_size=16)),
])
def test_invariant_merge_equals_softmax_over_union(oracle, name, kw):
    L = wl.make_layer(wl.scaled(wl.CONFIGS[name], **kw))
    tw, tp = as_tier(oracle, L.window), as_tier(oracle, L.pool)
    ow, lw = oracle.attend_all(L.q, tw, L.scale)
    idx, cnt = oracle.select(L.q, tp, L.k, L.k_max, L.scale)
    os_, ls = oracle.attend_indexed(L.q, tp, idx, cnt, L.scale)
    o, lse = oracle.merge(os_, ls, ow, lw)
    ou, lu = oracle.attend_union(L.q, tw, tp, idx, cnt, L.scale)
    np.testing.assert_allclose(o, ou, atol=1e-12)
    np.testing.assert_allclose(lse, lu, atol=1e-12)
    o2, lse2, idx2, cnt2 = oracle.hybrid_step(L.q, tw, tp, L.k, L.k_max, L.scale)
    np.testing.assert_array_equal(idx2, idx)
    np.testing.assert_array_equal(cnt2, cnt)
    np.testing.assert_array_equal(o2, o)
    np.testing.assert_array_equal(lse2, lse)
    o3, _, _, _ = oracle.hybrid_step(L.q, tw, tp, L.k, L.k_max, L.scale, idx=idx, cnt=cnt)
    np.testing.assert_array_equal(o3, o)


@pytest.mark.parametrize("name,kw", [
    ("C1", {}),
    ("C2", dict(B=2, Hq=8, Hkv=2, d=32, W=50, P=130, k=130)),
])
def test_invariant_select_everything_is_full_attention(oracle, name, kw):
    cfg = wl.scaled(wl.CONFIGS[name], **kw)
    cfg = wl.scaled(cfg, k=cfg.P)
    L = wl.make_layer(cfg)
    tw, tp = as_tier(oracle, L.window), as_tier(oracle, L.pool)
    o, lse, idx, cnt = oracle.hybrid_step(L.q, tw, tp, cfg.P, cfg.P, L.scale)
    assert np.all(cnt == cfg.P) and np.all(idx == np.arange(cfg.P, dtype=np.int32))
    # brute-force full attention over all W + P tokens with library routines
    K = np.concatenate([wl.to_f32(L.window.k), wl.to_f32(L.pool.k)], axis=2)
    V = np.concatenate([wl.to_f32(L.window.v), wl.to_f32(L.pool.v)], axis=2)
    eo, el = lib_attention(wl.to_f32(L.q), K, V, L.scale, cfg.G)
    np.testing.assert_allclose(o, eo, atol=1e-12)
    np.testing.assert_allclose(lse, el, atol=1e-12)
    ou, lu = oracle.attend_union(L.q, tw, tp, None, None, L.scale)
    np.testing.assert_allclose(ou, eo, atol=1e-12)
    np.testing.assert_allclose(lu, el, atol=1e-12)


def test_any_partition_of_the_window_merges_to_the_same_result(oracle):
    rng = np.random.default_rng(40)
    q, K, V = rand(rng, 2, 4, 16), rand(rng, 2, 2, 61, 16), rand(rng, 2, 2, 61, 16)
    whole_o, whole_l = oracle.attend_all(q, tier(oracle, K, V), 0.25)
    cuts = [0, 7, 8, 40, 61]
    acc_o, acc_l = np.zeros(q.shape), np.full(q.shape[:2], -np.inf)
    for a, b in reversed(list(zip(cuts[:-1], cuts[1:]))):      # merge in reverse order on purpose
        po, pl = oracle.attend_all(q, tier(oracle, K[:, :, a:b], V[:, :, a:b]), 0.25)
        acc_o, acc_l = oracle.merge(acc_o, acc_l, po, pl)
    np.testing.assert_allclose(acc_o, whole_o, atol=1e-13)
    np.testing.assert_allclose(acc_l, whole_l, atol=1e-13)


def test_batch_and_head_permutation_only_permutes_outputs(oracle):
    rng = np.random.default_rng(41)
    q, K, V = rand(rng, 3, 4, 8), rand(rng, 3, 4, 21, 8), rand(rng, 3, 4, 21, 8)
    pb, ph = np.array([2, 0, 1]), np.array([3, 1, 0, 2])
    o, lse = oracle.attend_all(q, tier(oracle, K, V), 0.4)
    o2, lse2 = oracle.attend_all(np.ascontiguousarray(q[pb][:, ph]),
                                 tier(oracle, K[pb][:, ph], V[pb][:, ph]), 0.4)
    np.testing.assert_array_equal(o2, o[pb][:, ph])
    np.testing.assert_array_equal(lse2, lse[pb][:, ph])
    idx, _ = oracle.select(q, tier(oracle, K, K), 5, 5, 0.4)
    idx2, _ = oracle.select(np.ascontiguousarray(q[pb][:, ph]), tier(oracle, K[pb][:, ph], K[pb][:, ph]), 5, 5, 0.4)
    np.testing.assert_array_equal(idx2, idx[pb][:, ph])


def test_indexed_attention_matches_library_on_gathered_rows(oracle):
    rng = np.random.default_rng(42)
    B, Hq, Hkv, n, d, k = 2, 4, 2, 50, 8, 9
    q, K, V = rand(rng, B, Hq, d), rand(rng, B, Hkv, n, d), rand(rng, B, Hkv, n, d)
    idx = np.stack([[np.sort(rng.choice(n, k, replace=False)) for _ in range(Hq)] for _ in range(B)]).astype(np.int32)
    cnt = np.array([[k, k - 3, 1, k], [2, k, k, 0]], np.int32)
    o, lse = oracle.attend_indexed(q, tier(oracle, K, V), idx, cnt, 0.3)
    for b in range(B):
        for h in range(Hq):
            rows = idx[b, h, :cnt[b, h]]
            if rows.size == 0:
                assert np.all(o[b, h] == 0) and np.isneginf(lse[b, h])
                continue
            s = 0.3 * (K[b, h // 2, rows].astype(np.float64) @ q[b, h].astype(np.float64))
            np.testing.assert_allclose(o[b, h], softmax(s) @ V[b, h // 2, rows].astype(np.float64), atol=1e-13)
            assert lse[b, h] == pytest.approx(logsumexp(s), abs=1e-13)
