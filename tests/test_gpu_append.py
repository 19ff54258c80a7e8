"""Parity of the append stage (N queries per sequence; paper Sec. 2.1 and Alg. 2, append branch) with the
numpy fp64 oracle, through the C ABI: causal attention over the window, attention over the complete older
pool, their merge, the query-averaged weights of each part, and the re-evaluation threshold on A_cpu.

Bars (bf16 inputs; scores accumulate exact products in fp32; the probabilities enter the second
contraction as a high and a low bf16 part): lse within 2e-5, O within 2e-4 (the stated bar is 2e-2),
averaged weights within 2e-5 and summing to 1 within 1e-4.  With HGCA_APPEND_ONE_PART_P (weights rounded
once to bf16) lse is the same bit for bit and O is held to 1e-2 (2^-9 max|v|)."""
import sys

import numpy as np
import pytest

from oracle import append_stage as ap
from paper_2507_03153_amd import workloads as wl

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2507_03153_amd import hgca, runner
    hgca.lib()
    return torch, hgca, runner


def make_inputs(seed, B, N, Hq, Hkv, d, W, P, w_lens, p_lens, lean=0.6):
    rng = np.random.default_rng(seed)
    bits = lambda *s: wl.f32_to_bf16_bits(rng.standard_normal(s).astype(np.float32))
    q, Kw, Vw, Kp, Vp = bits(B, N, Hq, d), bits(B, Hkv, W, d), bits(B, Hkv, W, d), bits(B, Hkv, max(P, 1), d), \
        bits(B, Hkv, max(P, 1), d)
    # a few pool keys lean towards the first query of each head's group so that some weights stand out
    qf = wl.bf16_bits_to_f32(q)
    for b in range(B):
        for kvh in range(Hkv):
            for j in range(0, P, 37):
                kf = wl.bf16_bits_to_f32(Kp[b, kvh, j]) + lean * qf[b, 0, kvh * (Hq // Hkv)]
                Kp[b, kvh, j] = wl.f32_to_bf16_bits(kf.astype(np.float32))
    w_lens = np.full(B, W, np.int32) if w_lens is None else np.asarray(w_lens, np.int32)
    p_lens = np.full(B, P, np.int32) if p_lens is None else np.asarray(p_lens, np.int32)
    return q, Kw, Vw, w_lens, Kp, Vp, p_lens


def to_paged(runner, hgca, torch, K, V, lens, cap, block, seed, dev):
    """The same logical tier in shuffled 16-token blocks, addressed through a table row that starts at a
    per-sequence offset (first_block)."""
    B, Hkv, _, d = K.shape
    nb = (cap + block - 1) // block
    rng = np.random.default_rng(seed)
    first = rng.integers(0, 3, B).astype(np.int32)
    table = np.full((B, nb + 3), 0, np.int32)
    perm = rng.permutation(B * nb).astype(np.int32)
    kb = np.zeros((B * nb, Hkv, block, d), K.dtype)
    vb = np.zeros_like(kb)
    for b in range(B):
        for j in range(nb):
            blk = perm[b * nb + j]
            table[b, first[b] + j] = blk
            n = min(block, cap - j * block)
            kb[blk, :, :n] = K[b, :, j * block:j * block + n]
            vb[blk, :, :n] = V[b, :, j * block:j * block + n]
    g = lambda a: runner._to_gpu(a, dev)
    return hgca.Tier(g(kb), g(vb), cap, g(lens), g(table), block, g(first))


def run_case(gpu, seed, B, N, Hq, Hkv, d, W, P, w_lens=None, p_lens=None, paged=False, lean=0.6):
    torch, hgca, runner = gpu
    dev = "cuda:0"
    say(f"\n[case] append N={N} B={B} Hq={Hq} Hkv={Hkv} d={d} W={W} P={P} w_lens={w_lens} p_lens={p_lens} paged={paged}")
    q, Kw, Vw, wl_, Kp, Vp, pl_ = make_inputs(seed, B, N, Hq, Hkv, d, W, P, w_lens, p_lens, lean)
    scale = 1.0 / np.sqrt(d)
    f = lambda x: wl.bf16_bits_to_f32(x).astype(np.float64)
    o_g, l_g, A_g = ap.part_attention(f(q), f(Kw), f(Vw), wl_, scale, True)
    o_c, l_c, A_c = ap.part_attention(f(q), f(Kp), f(Vp), pl_, scale, False)
    o_ref, l_ref = ap.merge_state(o_c, l_c, o_g, l_g)

    g = lambda a: runner._to_gpu(a, dev)
    qd = g(q)
    if paged:
        win = to_paged(runner, hgca, torch, Kw, Vw, wl_, W, 16, seed + 1, dev)
        pool = to_paged(runner, hgca, torch, Kp, Vp, pl_, max(P, 1), 16, seed + 2, dev)
        pool.cap = P
    else:
        win = hgca.Tier(g(Kw), g(Vw), W, g(wl_))
        pool = hgca.Tier(g(Kp), g(Vp), P, g(pl_))
    shape = hgca.Shape(hgca.BF16, B, Hq, Hkv, d, scale)
    f32 = dict(dtype=torch.float32, device=dev)
    ws = hgca.append_workspace(shape, N, max(W, P), dev)
    ow, lw = torch.full((B, N, Hq, d), float("nan"), **f32), torch.full((B, N, Hq), float("nan"), **f32)
    op, lp = torch.full_like(ow, float("nan")), torch.full_like(lw, float("nan"))
    hgca.append_attn(shape, qd, win, True, ow, lw, ws)
    hgca.append_attn(shape, qd, pool, False, op, lp, ws)
    o, lse = torch.empty_like(ow), torch.empty_like(lw)
    merged_shape = hgca.Shape(hgca.BF16, B * N, Hq, Hkv, d, scale)
    hgca.lse_merge(merged_shape, op, lp, ow, lw, o, lse)
    a_gpu = torch.full((B, Hq, W), float("nan"), **f32)
    a_cpu = torch.full((B, Hq, max(P, 1)), float("nan"), **f32)
    hgca.append_weights(shape, qd, win, True, lw, a_gpu)
    hgca.append_weights(shape, qd, pool, False, lp, a_cpu)
    torch.cuda.synchronize()

    def check(name, o_t, l_t, o_r, l_r):
        o_t, l_t = o_t.double().cpu().numpy(), l_t.double().cpu().numpy()
        empty = np.isneginf(l_r)
        assert np.array_equal(np.isneginf(l_t), empty), f"{name}: empty sets differ"
        assert np.all(np.isfinite(o_t)) and np.all(o_t[empty] == 0)
        err_l = np.max(np.abs(l_t[~empty] - l_r[~empty]), initial=0.0)
        err_o = np.max(np.abs(o_t - o_r), initial=0.0)
        say(f"    {name}: max|dO|={err_o:.2e} max|dlse|={err_l:.2e}")
        assert err_l <= 2e-5 and err_o <= 2e-4, f"{name}: dO={err_o} dlse={err_l}"
    check("window (causal)", ow, lw, o_g, l_g)
    check("pool", op, lp, o_c, l_c)
    check("merged", o, lse, o_ref, l_ref)

    # both tiers in one call (one launch for the splits of both, one fold): the merged result and each tier's lse
    ws2 = hgca.append_tiers_workspace(shape, N, W, P, dev)
    o2, lse2 = torch.full_like(ow, float("nan")), torch.full_like(lw, float("nan"))
    lw2, lp2 = torch.full_like(lw, float("nan")), torch.full_like(lw, float("nan"))
    hgca.append_attn_tiers(shape, qd, win, pool, o2, lse2, ws2, lse_window_out=lw2, lse_pool_out=lp2)
    o3, lse3 = torch.full_like(ow, float("nan")), torch.full_like(lw, float("nan"))
    hgca.append_attn_tiers(shape, qd, win, pool, o3, lse3, ws2)                  # without the per-tier outputs
    torch.cuda.synchronize()
    check("two tiers, one call", o2, lse2, o_ref, l_ref)
    assert torch.equal(o3, o2) and torch.equal(lse3, lse2)
    for name, got, want in (("window lse", lw2, l_g), ("pool lse", lp2, l_c)):
        got = got.double().cpu().numpy()
        assert np.array_equal(np.isneginf(got), np.isneginf(want)), name
        fin = ~np.isneginf(want)
        assert np.max(np.abs(got[fin] - want[fin]), initial=0.0) <= 2e-5, name

    # the same with the weights rounded once to bf16 for the second product: lse is untouched (bit for bit); every
    # weight is off by at most 2^-9 of itself and the weights sum to 1, so |dO| <= 2^-9 max|v| (about 9e-3 for
    # N(0,1) values; reached when a query sees only a few tokens)
    ow1, lw1 = torch.full_like(ow, float("nan")), torch.full_like(lw, float("nan"))
    op1, lp1 = torch.full_like(ow, float("nan")), torch.full_like(lw, float("nan"))
    hgca.append_attn(shape, qd, win, True, ow1, lw1, ws, one_part_p=True)
    hgca.append_attn(shape, qd, pool, False, op1, lp1, ws, one_part_p=True)
    torch.cuda.synchronize()
    assert torch.equal(lw1, lw) and torch.equal(lp1, lp)
    for name, got, want in (("window", ow1, o_g), ("pool", op1, o_c)):
        err = float(np.max(np.abs(got.double().cpu().numpy() - want), initial=0.0))
        say(f"    {name}, one-part P: max|dO|={err:.2e}")
        assert np.all(np.isfinite(got.cpu().numpy())) and err <= 1e-2

    # the weights of both tiers in one launch, normalised by the per-tier lse of the two-tier attention call
    a_gpu2 = torch.full((B, Hq, W), float("nan"), **f32)
    a_cpu2 = torch.full((B, Hq, max(P, 1)), float("nan"), **f32)
    hgca.append_weights_tiers(shape, qd, win, pool, lw2, lp2, a_gpu2, a_cpu2)
    torch.cuda.synchronize()
    for name, a_t, A, lens, cap in (("A_gpu", a_gpu, A_g, wl_, W), ("A_cpu", a_cpu, A_c, pl_, P),
                                    ("A_gpu, two tiers", a_gpu2, A_g, wl_, W), ("A_cpu, two tiers", a_cpu2, A_c, pl_, P)):
        a_t = a_t.double().cpu().numpy()[:, :, :cap]
        a_r = A.mean(axis=2)
        err = np.max(np.abs(a_t - a_r), initial=0.0)
        say(f"    {name}: max|dA|={err:.2e}")
        assert err <= 2e-5
        for b in range(B):
            assert np.all(a_t[b, :, lens[b]:] == 0.0)
            if lens[b] and (name.startswith("A_cpu") or lens[b] >= N):
                assert np.max(np.abs(a_t[b, :, :lens[b]].sum(-1) - 1.0)) <= 1e-4
    return shape, a_cpu, A_c.mean(axis=2), pl_


@pytest.mark.parametrize("kw", [
    dict(B=2, N=5, Hq=8, Hkv=2, d=128, W=100, P=333),                       # one partly filled row tile
    dict(B=2, N=32, Hq=8, Hkv=2, d=128, W=700, P=1500),                      # 128 rows: every wave two tiles
    dict(B=1, N=40, Hq=8, Hkv=2, d=128, W=300, P=900),                       # 160 rows: two query blocks
    dict(B=3, N=7, Hq=4, Hkv=4, d=128, W=130, P=257),                        # MHA
    dict(B=1, N=16, Hq=16, Hkv=2, d=128, W=96, P=640),                       # GQA 8
    dict(B=2, N=9, Hq=4, Hkv=2, d=64, W=333, P=1111),                        # head_dim 64
    dict(B=1, N=1, Hq=8, Hkv=2, d=128, W=64, P=200),                         # a single query: the decode step
], ids=["n5", "n32", "n40_two_blocks", "mha", "gqa8", "d64", "n1"])
def test_append_shapes(gpu, kw):
    run_case(gpu, 31, **kw)


@pytest.mark.parametrize("lean", [8.0, -8.0], ids=["scores_plus_90", "scores_minus_90"])
def test_append_extreme_scores(gpu, lean):
    """Every 37th pool key leans towards (away from) a query by 8 |q|: scaled scores of about +-90 for that query's
    head.  The running maximum is kept on raw scores and the scale folded into the exponent; nothing may overflow,
    and the merge of a pool part that outweighs the window by e^80 must stay finite and equal to the oracle's."""
    run_case(gpu, 37, B=2, N=8, Hq=8, Hkv=2, d=128, W=200, P=1500, lean=lean)


def test_append_ragged_and_degenerate_lengths(gpu):
    # a window that holds only the incoming tokens, an empty pool, a window shorter than the chunk tail
    run_case(gpu, 32, B=4, N=6, Hq=8, Hkv=2, d=128, W=200, P=500, w_lens=(200, 6, 37, 150), p_lens=(500, 0, 1, 33))
    run_case(gpu, 33, B=2, N=12, Hq=8, Hkv=2, d=128, W=64, P=0, w_lens=(64, 12))


def test_append_paged_tiers_with_first_block_offsets(gpu):
    run_case(gpu, 34, B=3, N=10, Hq=8, Hkv=2, d=128, W=208, P=1000, w_lens=(208, 100, 10), p_lens=(1000, 17, 640),
             paged=True)


def test_append_long_pool_many_splits_and_row_table_refills(gpu):
    run_case(gpu, 35, B=1, N=32, Hq=8, Hkv=2, d=128, W=256, P=9000)


@pytest.mark.timeout(600)
@pytest.mark.timeout(600)
def test_append_full_size_c2_every_unit(gpu):
    """The shape and launch configuration bench.py times for the append stage (B=8, N=32, 32 query heads on 8 KV
    heads, window 4096, pool 28672); the oracle computes every one of the 256 (sequence, head) units: all N queries
    of the unit, both parts, the merge and the two query-averaged weight rows."""
    torch, hgca, runner = gpu
    dev = "cuda:0"
    c2 = wl.CONFIGS["C2"]
    B, N, Hq, Hkv, d, W, P = c2.B, 32, c2.Hq, c2.Hkv, c2.d, c2.W, c2.P
    G = Hq // Hkv
    say(f"\n[case] append full size N={N} B={B} Hq={Hq} Hkv={Hkv} d={d} W={W} P={P}")
    q, Kw, Vw, wl_, Kp, Vp, pl_ = make_inputs(41, B, N, Hq, Hkv, d, W, P, None, None)
    wl_[1], pl_[1] = W - 1000, P - 5001                         # one sequence with ragged tails in both tiers
    scale = 1.0 / np.sqrt(d)
    g = lambda a: runner._to_gpu(a, dev)
    qd = g(q)
    win, pool = hgca.Tier(g(Kw), g(Vw), W, g(wl_)), hgca.Tier(g(Kp), g(Vp), P, g(pl_))
    shape = hgca.Shape(hgca.BF16, B, Hq, Hkv, d, scale)
    f32 = dict(dtype=torch.float32, device=dev)
    ws = hgca.append_workspace(shape, N, max(W, P), dev)
    ow, lw = torch.full((B, N, Hq, d), float("nan"), **f32), torch.full((B, N, Hq), float("nan"), **f32)
    op, lp = torch.full_like(ow, float("nan")), torch.full_like(lw, float("nan"))
    hgca.append_attn(shape, qd, win, True, ow, lw, ws)
    hgca.append_attn(shape, qd, pool, False, op, lp, ws)
    o, lse = torch.empty_like(ow), torch.empty_like(lw)
    hgca.lse_merge(hgca.Shape(hgca.BF16, B * N, Hq, Hkv, d, scale), op, lp, ow, lw, o, lse)
    a_gpu, a_cpu = torch.full((B, Hq, W), float("nan"), **f32), torch.full((B, Hq, P), float("nan"), **f32)
    hgca.append_weights(shape, qd, win, True, lw, a_gpu)
    hgca.append_weights(shape, qd, pool, False, lp, a_cpu)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(o).all()) and bool(torch.isfinite(lse).all())
    assert bool(torch.isfinite(a_gpu).all()) and bool(torch.isfinite(a_cpu).all())
    # a second run gives the same bits (a stage read before its loads had landed would show here or in the sums below)
    ow2, lw2, op2, lp2 = (torch.full_like(x, float("nan")) for x in (ow, lw, op, lp))
    hgca.append_attn(shape, qd, win, True, ow2, lw2, ws)
    hgca.append_attn(shape, qd, pool, False, op2, lp2, ws)
    torch.cuda.synchronize()
    assert torch.equal(ow2, ow) and torch.equal(lw2, lw) and torch.equal(op2, op) and torch.equal(lp2, lp)
    # both tiers in one call, as bench.py times it: the merged result and the per-tier lse agree with the calls above
    ws_t = hgca.append_tiers_workspace(shape, N, W, P, dev)
    o_t, lse_t = torch.full_like(ow, float("nan")), torch.full_like(lw, float("nan"))
    lw_t, lp_t = torch.full_like(lw, float("nan")), torch.full_like(lw, float("nan"))
    hgca.append_attn_tiers(shape, qd, win, pool, o_t, lse_t, ws_t, lse_window_out=lw_t, lse_pool_out=lp_t)
    torch.cuda.synchronize()
    # (other split sizes, hence another order of the fp32 sums: both are held to the oracle below, each to its bar)
    assert float((o_t - o).abs().max()) <= 4e-4 and float((lse_t - lse).abs().max()) <= 4e-5
    assert float((lw_t - lw).abs().max()) <= 4e-5 and float((lp_t - lp).abs().max()) <= 4e-5
    # every averaged weight row sums to 1 over what is visible (holds at any size)
    assert float((a_gpu.sum(-1) - 1).abs().max()) <= 1e-4 and float((a_cpu.sum(-1) - 1).abs().max()) <= 1e-4

    # every (sequence, head) unit against the oracle: all N queries of the unit, both parts, the merge, and the two
    # query-averaged weight rows (a few of them printed)
    f = lambda x: wl.bf16_bits_to_f32(x).astype(np.float64)
    got = {name: t.double().cpu().numpy() for name, t in (("O_gpu", ow), ("lse_g", lw), ("O_cpu", op), ("lse_c", lp),
                                                          ("O", o), ("lse", lse), ("A_gpu", a_gpu), ("A_cpu", a_cpu),
                                                          ("O_tiers", o_t), ("lse_tiers", lse_t), ("lse_g_tiers", lw_t),
                                                          ("lse_c_tiers", lp_t))}

    def unit_group(b, kvh):
        """The G heads that share KV head kvh of sequence b: worst error per quantity."""
        kw, vw, kp, vp = (f(x[b:b + 1, kvh:kvh + 1]) for x in (Kw, Vw, Kp, Vp))
        worst = {}
        for h in range(kvh * G, (kvh + 1) * G):
            qs = f(q[b:b + 1, :, h:h + 1])
            o_g, l_g, A_g = ap.part_attention(qs, kw, vw, wl_[b:b + 1], scale, True)
            o_c, l_c, A_c = ap.part_attention(qs, kp, vp, pl_[b:b + 1], scale, False)
            o_r, l_r = ap.merge_state(o_c, l_c, o_g, l_g)
            want = {"O_gpu": o_g[0, :, 0], "lse_g": l_g[0, :, 0], "O_cpu": o_c[0, :, 0], "lse_c": l_c[0, :, 0],
                    "O": o_r[0, :, 0], "lse": l_r[0, :, 0], "A_gpu": A_g[0, 0].mean(axis=0), "A_cpu": A_c[0, 0].mean(axis=0),
                    "O_tiers": o_r[0, :, 0], "lse_tiers": l_r[0, :, 0], "lse_g_tiers": l_g[0, :, 0], "lse_c_tiers": l_c[0, :, 0]}
            for name, ref in want.items():
                mine = got[name][b, h] if name.startswith("A_") else got[name][b, :, h]
                worst[name] = max(worst.get(name, 0.0), float(np.max(np.abs(mine - ref))))
            assert np.all(got["A_gpu"][b, h, wl_[b]:] == 0) and np.all(got["A_cpu"][b, h, pl_[b]:] == 0)
        return b, kvh, worst

    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(8) as pool_:
        results = list(pool_.map(lambda bk: unit_group(*bk), [(b, kvh) for b in range(B) for kvh in range(Hkv)]))
    assert len(results) * G == B * Hq                           # all 256 units
    for b, kvh, errs in results:
        if kvh in (0, Hkv - 1):
            say(f"    (b={b}, heads {kvh * G}..{kvh * G + G - 1}): " + " ".join(f"{k}={v:.1e}" for k, v in errs.items()))
        assert max(errs["O_gpu"], errs["O_cpu"], errs["O"], errs["O_tiers"]) <= 2e-4, (b, kvh, errs)
        assert max(errs["lse_g"], errs["lse_c"], errs["lse"], errs["A_gpu"], errs["A_cpu"], errs["lse_tiers"],
                   errs["lse_g_tiers"], errs["lse_c_tiers"]) <= 2e-5, (b, kvh, errs)


def run_case_f32(gpu, seed, B, N, Hq, Hkv, d, W, P, w_lens=None, p_lens=None, paged=False):
    """fp32 inputs: the bar is 1e-5 on O and lse of both parts and of the merge, and on the averaged weights."""
    torch, hgca, runner = gpu
    dev = "cuda:0"
    say(f"\n[case] append fp32 N={N} B={B} Hq={Hq} Hkv={Hkv} d={d} W={W} P={P} w_lens={w_lens} p_lens={p_lens} paged={paged}")
    qb, Kwb, Vwb, wl_, Kpb, Vpb, pl_ = make_inputs(seed, B, N, Hq, Hkv, d, W, P, w_lens, p_lens)
    rng = np.random.default_rng(seed + 100)
    # fp32 values with a full mantissa: the bf16 draw plus a small fp32 perturbation
    full = lambda bits: (wl.bf16_bits_to_f32(bits) + 1e-3 * rng.standard_normal(bits.shape)).astype(np.float32)
    q, Kw, Vw, Kp, Vp = (full(x) for x in (qb, Kwb, Vwb, Kpb, Vpb))
    scale = 1.0 / np.sqrt(d)
    f = lambda x: x.astype(np.float64)
    o_g, l_g, A_g = ap.part_attention(f(q), f(Kw), f(Vw), wl_, scale, True)
    o_c, l_c, A_c = ap.part_attention(f(q), f(Kp), f(Vp), pl_, scale, False)
    o_ref, l_ref = ap.merge_state(o_c, l_c, o_g, l_g)
    g = lambda a: runner._to_gpu(a, dev)
    qd = g(q)
    if paged:
        win = to_paged(runner, hgca, torch, Kw, Vw, wl_, W, 16, seed + 1, dev)
        pool = to_paged(runner, hgca, torch, Kp, Vp, pl_, max(P, 1), 16, seed + 2, dev)
        pool.cap = P
    else:
        win = hgca.Tier(g(Kw), g(Vw), W, g(wl_))
        pool = hgca.Tier(g(Kp), g(Vp), P, g(pl_))
    shape = hgca.Shape(hgca.F32, B, Hq, Hkv, d, scale)
    f32 = dict(dtype=torch.float32, device=dev)
    ws = hgca.append_workspace(shape, N, max(W, P), dev)
    ow, lw = torch.full((B, N, Hq, d), float("nan"), **f32), torch.full((B, N, Hq), float("nan"), **f32)
    op, lp = torch.full_like(ow, float("nan")), torch.full_like(lw, float("nan"))
    hgca.append_attn(shape, qd, win, True, ow, lw, ws)
    hgca.append_attn(shape, qd, pool, False, op, lp, ws)
    o, lse = torch.empty_like(ow), torch.empty_like(lw)
    hgca.lse_merge(hgca.Shape(hgca.F32, B * N, Hq, Hkv, d, scale), op, lp, ow, lw, o, lse)
    a_gpu = torch.full((B, Hq, W), float("nan"), **f32)
    a_cpu = torch.full((B, Hq, max(P, 1)), float("nan"), **f32)
    hgca.append_weights(shape, qd, win, True, lw, a_gpu)
    hgca.append_weights(shape, qd, pool, False, lp, a_cpu)
    torch.cuda.synchronize()
    for name, o_t, l_t, o_r, l_r in (("window (causal)", ow, lw, o_g, l_g), ("pool", op, lp, o_c, l_c),
                                     ("merged", o, lse, o_ref, l_ref)):
        o_t, l_t = o_t.double().cpu().numpy(), l_t.double().cpu().numpy()
        empty = np.isneginf(l_r)
        assert np.array_equal(np.isneginf(l_t), empty), f"{name}: empty sets differ"
        assert np.all(np.isfinite(o_t)) and np.all(o_t[empty] == 0)
        err_l = np.max(np.abs(l_t[~empty] - l_r[~empty]), initial=0.0)
        err_o = np.max(np.abs(o_t - o_r), initial=0.0)
        say(f"    {name}: max|dO|={err_o:.2e} max|dlse|={err_l:.2e} (bar 1e-5)")
        assert err_l <= 1e-5 and err_o <= 1e-5, f"{name}: dO={err_o} dlse={err_l}"
    for name, a_t, A, lens, cap in (("A_gpu", a_gpu, A_g, wl_, W), ("A_cpu", a_cpu, A_c, pl_, P)):
        a_t = a_t.double().cpu().numpy()[:, :, :cap]
        err = np.max(np.abs(a_t - A.mean(axis=2)), initial=0.0)
        say(f"    {name}: max|dA|={err:.2e}")
        assert err <= 1e-5
        for b in range(B):
            assert np.all(a_t[b, :, lens[b]:] == 0.0)
            if lens[b] and (name.startswith("A_cpu") or lens[b] >= N):
                assert np.max(np.abs(a_t[b, :, :lens[b]].sum(-1) - 1.0)) <= 1e-5


def test_append_fp32_tiny_config_shape(gpu):
    """The fp32 configuration's shape (B=1, 4 MHA heads of 64, window 256, pool 2048) with a prompt of 32 tokens."""
    run_case_f32(gpu, 51, B=1, N=32, Hq=4, Hkv=4, d=64, W=256, P=2048)


@pytest.mark.parametrize("kw", [
    dict(B=2, N=5, Hq=8, Hkv=2, d=128, W=100, P=333),
    dict(B=3, N=17, Hq=8, Hkv=1, d=64, W=300, P=700, w_lens=(300, 17, 5), p_lens=(700, 0, 64)),     # a prompt longer than the window
    dict(B=2, N=9, Hq=4, Hkv=2, d=128, W=160, P=600, w_lens=(160, 33), p_lens=(555, 600), paged=True),
    dict(B=1, N=3, Hq=2, Hkv=2, d=64, W=64, P=0),
], ids=["gqa4", "gqa8_ragged", "paged", "no_pool"])
def test_append_fp32_shapes(gpu, kw):
    run_case_f32(gpu, 52, **kw)


def test_reevaluation_threshold_on_a_cpu(gpu, oracle):
    """Alg. 1, append: ids = A_cpu > beta / A_cpu.size; both sides threshold their own A_cpu, entries within
    rounding of the threshold may differ."""
    torch, hgca, runner = gpu
    shape, a_cpu, a_ref, p_lens = run_case(gpu, 36, B=2, N=16, Hq=8, Hkv=2, d=128, W=128, P=2000, p_lens=(2000, 1234))
    P = a_ref.shape[2]
    idx = torch.empty(2, 8, P, dtype=torch.int32, device="cuda:0")
    cnt = torch.empty(2, 8, dtype=torch.int32, device="cuda:0")
    lens_d = torch.from_numpy(p_lens).to("cuda:0")
    hgca.threshold_select(shape, a_cpu, lens_d, P, lens_d, 1.0, P, idx, cnt)
    torch.cuda.synchronize()
    idx_ref, cnt_ref = oracle.threshold_select(a_ref, 1.0, p_lens, P, lens=p_lens)
    idx, cnt = idx.cpu().numpy(), cnt.cpu().numpy()
    differing = 0
    for b in range(2):
        thr = 1.0 / p_lens[b]
        for h in range(8):
            got, want = set(idx[b, h, :cnt[b, h]].tolist()), set(idx_ref[b, h, :cnt_ref[b, h]].tolist())
            for j in got ^ want:
                assert abs(a_ref[b, h, j] - thr) <= 1e-4 * thr
                differing += 1
    say(f"    kept per head {cnt_ref.min()}..{cnt_ref.max()} of {p_lens.tolist()}; decided differently inside the "
        f"rounding band: {differing}")
    assert 0 < cnt_ref.min() and cnt_ref.max() < p_lens.min()
