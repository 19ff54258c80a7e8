"""Multi-step parity of the KV manager and the paper-literal decode step (paper Alg. 1 and Alg. 2)
with the numpy fp64 oracle: both sides run the whole loop on their own from the same seeded tokens.

Bars: O and lse of every step within 2e-4 (bf16 inputs, fp32 accumulation; the stated bar is 2e-2);
moving averages within 2e-5; per-head salient lists identical except for entries whose moving average
lies within 1e-5 (relative) of the threshold, where the two sides' rounding may decide differently
(after such a difference the outputs are held to the stated 2e-2 only); window / pool contents,
lengths and block boundaries exact."""
import sys

import numpy as np
import pytest

from oracle.kv_manager import KvManager
from paper_2507_03153_amd import workloads as wl

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2507_03153_amd import cache, hgca, runner
    hgca.lib()
    return torch, hgca, runner, cache


def make_tokens(seed, T, B, Hq, Hkv, d, boost=3.0):
    """Seeded q, k, v per step as bf16 bit patterns.  Every 7th token's key leans towards a fixed
    direction u of its KV head and every query leans the same way, so those tokens collect weight."""
    rng = np.random.default_rng(seed)
    u = rng.standard_normal((B, Hkv, d))
    u /= np.linalg.norm(u, axis=-1, keepdims=True)
    q = rng.standard_normal((T, B, Hq, d)) + 2.5 * np.repeat(u, Hq // Hkv, axis=1)[None] * np.sqrt(d) / 4
    k = rng.standard_normal((T, B, Hkv, d))
    k[3::7] += boost * u[None] * np.sqrt(d) / 4
    v = rng.standard_normal((T, B, Hkv, d))
    return tuple(wl.f32_to_bf16_bits(x.astype(np.float32)) for x in (q, k, v))


def run_loop(gpu, B, Hq, Hkv, d, block_size, win_blocks, max_blocks, k_max, prefill, steps, alpha, beta, seed,
             expect_list_full=False, fused_tail=True, fused_maw=True, one_call=False, boost=3.0):
    torch, hgca, runner, cache = gpu
    dev = "cuda:0"
    T = max(prefill) + steps
    say(f"\n[case] decode loop B={B} Hq={Hq} Hkv={Hkv} d={d} block={block_size} l_max={win_blocks * block_size} "
        f"prefill={prefill} steps={steps} alpha={alpha} beta={beta} k_max={k_max} one_call={one_call}")
    qb, kb, vb = make_tokens(seed, T, B, Hq, Hkv, d, boost)
    qf, kf, vf = (wl.bf16_bits_to_f32(x).astype(np.float64) for x in (qb, kb, vb))
    scale = 1.0 / np.sqrt(d)
    C = cache.LayerCache(torch.bfloat16, B, Hq, Hkv, d, block_size, win_blocks, max_blocks, k_max, scale, dev,
                         keep_evicted_maw=True, fused_tail=fused_tail)
    mgr = [KvManager(Hq, Hkv, d, win_blocks, block_size, alpha, beta, scale) for _ in range(B)]

    # prefill: sequence b starts with prefill[b] < l_max window entries whose moving average is 1/prefill[b]
    for t in range(max(prefill)):
        active = np.array([t < p for p in prefill], np.int32)
        C.append(runner._to_gpu(kb[t], dev), runner._to_gpu(vb[t], dev), torch.from_numpy(active).to(dev))
    maw0 = np.zeros((B, Hq, C.win_cap), np.float32)
    for b, p in enumerate(prefill):
        assert p < win_blocks * block_size
        maw0[b, :, :p] = 1.0 / max(p, 1)
        mgr[b].K_gpu, mgr[b].V_gpu = kf[:p, b].copy(), vf[:p, b].copy()
        mgr[b].A_maw = maw0[b, :, :p].astype(np.float64)
    C.a_maw.copy_(torch.from_numpy(maw0))
    torch.cuda.synchronize()
    assert C.win_lens.cpu().tolist() == list(prefill)

    differing, worst_o, worst_l, evictions = 0, 0.0, 0.0, 0
    for s in range(steps):
        t = max(prefill) + s
        C.decode_step(runner._to_gpu(qb[t], dev), runner._to_gpu(kb[t], dev), runner._to_gpu(vb[t], dev), alpha, beta,
                      fused_maw=fused_maw, one_call=one_call)
        torch.cuda.synchronize()
        o_g, l_g = C.o.double().cpu().numpy(), C.lse.double().cpu().numpy()
        cnt_g, idx_g = C.ctx_cnt.cpu().numpy(), C.ctx_idx.cpu().numpy()
        for b in range(B):
            o_ref, l_ref, A_gpu = mgr[b].hybrid_attention(qf[t, b], kf[t, b], vf[t, b])
            l_cur = mgr[b].K_gpu.shape[0] + 1
            tol = 2e-4 if differing == 0 else 2e-2
            err_o, err_l = np.max(np.abs(o_g[b] - o_ref)), np.max(np.abs(l_g[b] - l_ref))
            assert err_o <= tol and err_l <= tol, f"step {s} seq {b}: dO={err_o} dlse={err_l}"
            worst_o, worst_l = max(worst_o, err_o), max(worst_l, err_l)
            maw_at_evict = None
            if l_cur >= mgr[b].l_max:                           # what the threshold will look at
                maw_at_evict = np.concatenate([(1 - alpha) * mgr[b].A_maw + alpha * A_gpu[:, :-1], A_gpu[:, -1:]], 1)
            ev = mgr[b].manage(kf[t, b], vf[t, b], A_gpu)
            evictions += ev > 0
            for h in range(Hq):
                if expect_list_full:                            # the library's list keeps the first k_max it is given
                    mgr[b].ctx[h] = mgr[b].ctx[h][:k_max]
                got = set(idx_g[b, h, :cnt_g[b, h]].tolist())
                want = set(mgr[b].ctx[h].tolist())
                if got != want:
                    base = mgr[b].K_cpu.shape[0] - ev
                    for j in got ^ want:                        # only this step's evicted entries, within rounding
                        assert ev and j >= base, f"step {s} seq {b} head {h}: list differs at old entry {j}"
                        thr = beta / l_cur
                        assert abs(maw_at_evict[h, j - base] - thr) <= 1e-5 * thr
                        differing += 1
                row = idx_g[b, h, :cnt_g[b, h]]
                assert np.all(np.diff(row) > 0) and np.all(idx_g[b, h, cnt_g[b, h]:k_max] == -1)
    # final state
    win_lens, pool_lens, first = (x.cpu().numpy() for x in (C.win_lens, C.pool_lens, C.first_win_block))
    maw_g, aev_g = C.a_maw.double().cpu().numpy(), C.a_evicted.double().cpu().numpy()
    kblk, vblk, table = C.k_blocks.cpu().view(torch.int16).numpy().view(np.uint16), \
        C.v_blocks.cpu().view(torch.int16).numpy().view(np.uint16), C.block_table.cpu().numpy()
    for b in range(B):
        n, m = mgr[b].K_gpu.shape[0], mgr[b].K_cpu.shape[0]
        assert win_lens[b] == n and pool_lens[b] == m and first[b] * block_size == m
        assert np.max(np.abs(maw_g[b, :, :n] - mgr[b].A_maw), initial=0.0) <= 2e-5
        assert np.all(maw_g[b, :, n:] == 0.0)
        assert np.max(np.abs(aev_g[b, :, :m] - mgr[b].A_cpu_maw), initial=0.0) <= 2e-5
        total = prefill[b] + steps                               # every token of the sequence, in arrival order
        toks = [tt for tt in range(T) if tt < prefill[b] or tt >= max(prefill)]
        assert len(toks) == total == n + m
        for pos, tt in enumerate(toks):
            blk, slot = table[b, pos // block_size], pos % block_size
            assert np.array_equal(kblk[blk, :, slot], kb[tt, b]) and np.array_equal(vblk[blk, :, slot], vb[tt, b])
    status = int(C.status.cpu()[0])
    say(f"    {evictions} evictions; max|dO|={worst_o:.2e} max|dlse|={worst_l:.2e}; list entries decided differently "
        f"inside the rounding band: {differing}; kept per head: {cnt_g.min()}..{cnt_g.max()} of {pool_lens.max()}; "
        f"status={status}")
    return C, mgr, status


def test_decode_loop_ragged_windows_gqa4(gpu):
    C, mgr, status = run_loop(gpu, B=3, Hq=8, Hkv=2, d=128, block_size=16, win_blocks=4, max_blocks=24, k_max=384,
                              prefill=(0, 37, 63), steps=260, alpha=0.3, beta=1.0, seed=11)
    assert status == 0
    kept = C.ctx_cnt.cpu().numpy()
    pool = C.pool_lens.cpu().numpy()
    assert kept.min() > 0 and np.all(kept.max(axis=1) < pool)    # beta = 1 keeps some entries, not all


def test_decode_loop_in_one_call_per_step(gpu):
    """The same loop through hgca_managed_decode_step: one library call per decode step."""
    C, mgr, status = run_loop(gpu, B=3, Hq=8, Hkv=2, d=128, block_size=16, win_blocks=4, max_blocks=24, k_max=384,
                              prefill=(0, 37, 63), steps=260, alpha=0.3, beta=1.0, seed=11, one_call=True)
    assert status == 0
    _, _, status = run_loop(gpu, B=2, Hq=4, Hkv=4, d=64, block_size=32, win_blocks=3, max_blocks=8, k_max=256,
                            prefill=(5, 90), steps=150, alpha=0.5, beta=0.7, seed=12, one_call=True)
    assert status == 0


def test_decode_loop_in_one_call_other_group_sizes(gpu):
    """Groups of 2 (two launches per step: the token joins inside the window's split launch) and of 8 (insert, window
    splits and gather as launches of their own, the tail as one): the same loop, the same checks."""
    _, _, status = run_loop(gpu, B=2, Hq=4, Hkv=2, d=64, block_size=32, win_blocks=3, max_blocks=9, k_max=256,
                            prefill=(7, 70), steps=130, alpha=0.4, beta=0.8, seed=21, one_call=True)
    assert status == 0
    _, _, status = run_loop(gpu, B=2, Hq=8, Hkv=1, d=128, block_size=16, win_blocks=3, max_blocks=14, k_max=256,
                            prefill=(0, 33), steps=140, alpha=0.3, beta=1.0, seed=22, one_call=True)
    assert status == 0


def test_decode_loop_with_sharply_peaked_attention(gpu):
    """Every 7th key leans ten times as far towards the queries' direction: scaled scores of about 70 against
    N(0,1) for the rest, so the window weights are ~1/n_boosted on a few entries and underflow to zero on the others;
    the moving averages, the thresholds and the merge must cope (one call per step and separate calls)."""
    for one_call in (False, True):
        _, _, status = run_loop(gpu, B=2, Hq=8, Hkv=2, d=128, block_size=16, win_blocks=3, max_blocks=16, k_max=256,
                                prefill=(0, 40), steps=150, alpha=0.3, beta=1.0, seed=15, one_call=one_call, boost=30.0)
        assert status == 0


def test_decode_loop_mha_head_dim_64_blocks_of_32(gpu):
    _, _, status = run_loop(gpu, B=2, Hq=4, Hkv=4, d=64, block_size=32, win_blocks=3, max_blocks=8, k_max=256,
                            prefill=(5, 90), steps=150, alpha=0.5, beta=0.7, seed=12, fused_tail=False,
                            fused_maw=False)
    assert status == 0


@pytest.mark.timeout(600)
def test_decode_loop_at_the_benchmark_window_size(gpu):
    """B=8, 32 query heads on 8 KV heads, l_max = 4096 in 16-token blocks (the window of the benchmark shape), so
    that every kernel of the managed step runs in the launch configuration bench.py times; two evictions."""
    C, _, status = run_loop(gpu, B=8, Hq=32, Hkv=8, d=128, block_size=16, win_blocks=256, max_blocks=264, k_max=64,
                            prefill=(4090, 4090, 4000, 4095, 4090, 3, 4090, 4089), steps=24, alpha=0.3, beta=1.0,
                            seed=14)
    assert status == 0
    assert int(C.pool_lens.max()) == 32
    C, _, status = run_loop(gpu, B=8, Hq=32, Hkv=8, d=128, block_size=16, win_blocks=256, max_blocks=264, k_max=64,
                            prefill=(4090, 4090, 4000, 4095, 4090, 3, 4090, 4089), steps=24, alpha=0.3, beta=1.0,
                            seed=14, one_call=True)
    assert status == 0


def test_beta_zero_keeps_everything_and_matches_full_attention(gpu):
    """With beta = 0 every evicted entry stays salient, so each step is full attention over the history
    (the oracle is pinned to exactly that with library softmax)."""
    C, mgr, status = run_loop(gpu, B=2, Hq=8, Hkv=1, d=128, block_size=16, win_blocks=2, max_blocks=12, k_max=192,
                              prefill=(0, 20), steps=120, alpha=0.2, beta=0.0, seed=13)
    assert status == 0
    assert np.array_equal(C.ctx_cnt.cpu().numpy(), np.repeat(C.pool_lens.cpu().numpy()[:, None], 8, axis=1))


def test_status_bits_for_full_list_full_window_and_full_context(gpu):
    torch, hgca, runner, cache = gpu
    # a salient list shorter than what passes: the first k_max stay, the bit is raised, nothing else breaks
    C, mgr, status = run_loop(gpu, B=2, Hq=4, Hkv=2, d=128, block_size=16, win_blocks=2, max_blocks=10, k_max=8,
                              prefill=(0, 9), steps=100, alpha=0.3, beta=0.0, seed=14, expect_list_full=True)
    assert status == hgca.CACHE_LIST_FULL
    assert np.all(C.ctx_cnt.cpu().numpy() == 8)
    assert np.array_equal(C.ctx_idx.cpu().numpy()[:, :, :8], np.broadcast_to(np.arange(8, dtype=np.int32), (2, 4, 8)))
    # appending without ever evicting fills the window: the token is dropped and the bit is raised
    say("\n[case] append on a full window / beyond the table row")
    C = cache.LayerCache(torch.bfloat16, 1, 4, 2, 128, 16, 2, 4, 16, 0.1)
    tok = torch.ones(1, 2, 128, dtype=torch.bfloat16, device="cuda:0")
    for _ in range(33):
        C.append(tok, tok)
    torch.cuda.synchronize()
    assert int(C.win_lens.cpu()[0]) == 32 and int(C.status.cpu()[0]) == hgca.CACHE_WINDOW_FULL
    # evicting each time the window fills walks to the end of the 4-block table row: then the context is full
    # (the one-call step inserts the token inside its first launch and stores the length in its last: same outcome)
    q = torch.ones(1, 4, 128, dtype=torch.bfloat16, device="cuda:0")
    state = {}
    for one_call in (False, True):
        C = cache.LayerCache(torch.bfloat16, 1, 4, 2, 128, 16, 2, 4, 64, 0.1)
        for _ in range(70):
            C.decode_step(q, tok, tok, 0.5, 1.0, one_call=one_call)
        torch.cuda.synchronize()
        assert int(C.status.cpu()[0]) & hgca.CACHE_CONTEXT_FULL
        assert int(C.pool_lens.cpu()[0]) + int(C.win_lens.cpu()[0]) == 64     # nothing written beyond the row
        state[one_call] = (int(C.status.cpu()[0]), C.win_lens.cpu().tolist(), C.pool_lens.cpu().tolist(),
                           C.first_win_block.cpu().tolist(), C.ctx_cnt.cpu().tolist(), C.lse.cpu().numpy().copy())
    assert state[False][:5] == state[True][:5]
    np.testing.assert_allclose(state[True][5], state[False][5], atol=2e-5, rtol=0)


@pytest.mark.parametrize("one_call", [False, True], ids=["separate_calls", "one_call"])
def test_graph_replay_of_the_decode_step_equals_eager(gpu, one_call):
    """The decode step takes every decision on the device, so one captured launch sequence serves every step.
    Each replay is checked against an eager twin fed the same tokens, with eager work and synchronisation
    between the replays, across two evictions."""
    torch, hgca, runner, cache = gpu
    B, Hq, Hkv, d, bs, wb = 2, 8, 2, 128, 16, 2
    say("\n[case] HIP graph replay of the decode step vs eager")
    qb, kb, vb = make_tokens(21, 60, B, Hq, Hkv, d)
    dev = "cuda:0"
    mk = lambda: cache.LayerCache(torch.bfloat16, B, Hq, Hkv, d, bs, wb, 8, 96, 1.0 / np.sqrt(d), dev)
    E, G = mk(), mk()
    q, k, v = (runner._to_gpu(x[0], dev).clone() for x in (qb, kb, vb))        # static inputs of the graph
    side = torch.cuda.Stream(device=dev)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                                # capture on a non-default stream
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            G.decode_step(q, k, v, 0.3, 1.0, one_call=one_call)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    assert int(G.win_lens.cpu()[0]) == 0                         # capturing executes nothing
    for t in range(60):
        q.copy_(runner._to_gpu(qb[t], dev)); k.copy_(runner._to_gpu(kb[t], dev)); v.copy_(runner._to_gpu(vb[t], dev))
        graph.replay()
        E.decode_step(q, k, v, 0.3, 1.0, one_call=one_call)
        torch.cuda.synchronize()
        for name in ("o", "lse", "a_maw", "ctx_idx", "ctx_cnt", "win_lens", "pool_lens", "first_win_block"):
            assert torch.equal(getattr(E, name), getattr(G, name)), f"step {t}: {name} differs"
    assert int(G.pool_lens.cpu()[0]) == 32 and int(G.status.cpu()[0]) == 0


def test_full_list_is_flagged_even_when_it_was_exactly_full_before(gpu):
    """The salient list fills exactly to k_max without overflow at one eviction; the next eviction finds salient
    entries it cannot list and must say so."""
    torch, hgca, runner, cache = gpu
    say("\n[case] list exactly full, then one more salient entry")
    C = cache.LayerCache(torch.bfloat16, 1, 2, 1, 128, 16, 1, 4, 16, 0.1)       # window of one block, list of 16
    tok = torch.ones(1, 1, 128, dtype=torch.bfloat16, device="cuda:0")
    q = torch.ones(1, 2, 128, dtype=torch.bfloat16, device="cuda:0")
    for _ in range(16):                                           # first eviction: 16 entries, all salient at beta = 0
        C.decode_step(q, tok, tok, 0.5, 0.0)
    torch.cuda.synchronize()
    assert C.ctx_cnt.cpu().tolist() == [[16, 16]] and int(C.status.cpu()[0]) == 0
    for _ in range(16):                                           # second eviction: nothing fits any more
        C.decode_step(q, tok, tok, 0.5, 0.0)
    torch.cuda.synchronize()
    assert C.ctx_cnt.cpu().tolist() == [[16, 16]] and int(C.status.cpu()[0]) == hgca.CACHE_LIST_FULL
    assert int(C.pool_lens.cpu()[0]) == 32
