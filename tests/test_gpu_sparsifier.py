"""Parity of the paper-literal sparsifier (window attention weights A_gpu, their moving average,
the beta/size threshold rule; paper Alg. 1, Alg. 2, Sec. 3.2.2) with the fp64 CPU oracle, through
the C ABI.

Bars:
  * attention weights: 2e-6 absolute for fp32 inputs, 2e-5 for bf16 inputs (weights are <= 1; the
    path accumulates exact bf16 products in fp32), rows sum to 1 within 1e-5;
  * moving average: 1e-6 absolute (one fp32 multiply-add per entry);
  * threshold rule on the SAME fp32 weights: bit-exact positions and counts (both sides compare the
    exactly widened weight with beta/size in fp64); re-normalised weights 1e-6;
  * the chained decode loop (weights -> moving average -> threshold): positions exact outside a band
    of 1e-5 relative to the threshold, where the two sides' rounding may differ.
"""
import sys

import numpy as np
import pytest
from scipy.special import softmax

from paper_2507_03153_amd import workloads as wl

pytestmark = pytest.mark.gpu

W_TOL = {"f32": 2e-6, "bf16": 2e-5}


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


def otier(oracle, t):
    return oracle.Tier(t.k, t.v, t.cap, t.seq_lens, t.block_table, t.block_size)


def window_weights_case(gpu, oracle, cfg):
    torch, hgca, runner = gpu
    say(f"\n[case] window weights {cfg.name} dtype={cfg.dtype} B={cfg.B} Hq={cfg.Hq} Hkv={cfg.Hkv} d={cfg.d} "
        f"W={cfg.W} ragged={cfg.ragged} block={cfg.block_size}")
    L = wl.make_layer(cfg)
    D = runner.DeviceLayer.upload(L)
    f32 = dict(dtype=torch.float32, device="cuda:0")
    ws = hgca.alloc_workspace(D.shape, cfg.W, 0, 0, "cuda:0")
    o, lse = torch.empty(cfg.B, cfg.Hq, cfg.d, **f32), torch.empty(cfg.B, cfg.Hq, **f32)
    o2, lse2 = torch.empty_like(o), torch.empty_like(lse)
    a = torch.full((cfg.B, cfg.Hq, max(cfg.W, 1)), float("nan"), **f32)
    hgca.dense_window_attn_weights(D.shape, D.q, D.window, o, lse, a, ws)
    hgca.dense_window_attn(D.shape, D.q, D.window, o2, lse2, ws)
    torch.cuda.synchronize()
    assert torch.equal(o, o2) and torch.equal(lse, lse2)       # the extra output changes nothing else
    a = a.double().cpu().numpy()[:, :, :cfg.W]
    a_ref = oracle.window_weights(L.q, otier(oracle, L.window), L.scale)
    err = np.max(np.abs(a - a_ref)) if a.size else 0.0
    say(f"    max|dA|={err:.3e} (tol {W_TOL[cfg.dtype]:g})")
    assert err <= W_TOL[cfg.dtype]
    lens = L.window.lens(cfg.B)
    for b in range(cfg.B):
        assert np.all(a[b, :, lens[b]:] == 0.0)                # zero beyond the length, NaN prefill gone
        if lens[b]:
            assert np.max(np.abs(a[b, :, :lens[b]].sum(-1) - 1.0)) <= 1e-5
    return a_ref


@pytest.mark.parametrize("kw", [
    dict(B=2, Hq=8, Hkv=2, W=700, P=64, k=8),
    dict(B=3, Hq=4, Hkv=4, W=130, P=64, k=8),
    dict(B=1, Hq=16, Hkv=2, W=1100, P=64, k=8),
    dict(B=2, Hq=4, Hkv=2, d=64, W=333, P=64, k=8),
    dict(B=2, Hq=8, Hkv=2, W=1, P=64, k=8),
    dict(B=2, Hq=8, Hkv=2, W=0, P=64, k=8),
], ids=["gqa4", "mha", "gqa8", "gqa2_d64", "W1", "W0"])
def test_window_weights_bf16(gpu, oracle, kw):
    window_weights_case(gpu, oracle, wl.scaled(wl.CONFIGS["C2"], **kw))


def test_window_weights_fp32(gpu, oracle):
    window_weights_case(gpu, oracle, wl.CONFIGS["C1"])
    window_weights_case(gpu, oracle, wl.scaled(wl.CONFIGS["C1"], B=2, Hq=8, Hkv=2, d=128, W=300, P=64, k=8))


def test_window_weights_ragged_paged_with_empty_sequences(gpu, oracle):
    window_weights_case(gpu, oracle, wl.scaled(wl.CONFIGS["C5"], B=6, Hq=8, Hkv=2, W=256, P=1792, ragged=(100, 2048)))
    window_weights_case(gpu, oracle, wl.scaled(wl.CONFIGS["C5"], B=6, Hq=8, Hkv=2, W=256, P=1792, ragged=(200, 2048),
                                               block_size=0))


def test_window_weights_full_size_c2(gpu, oracle):
    window_weights_case(gpu, oracle, wl.scaled(wl.CONFIGS["C2"], P=64, k=8))


# ------------------------------------------------------------------------ moving average

@pytest.mark.parametrize("B,Hq,cap,n_new,alpha", [
    (2, 8, 700, 1, 0.25), (3, 4, 1024, 0, 0.5), (2, 2, 5, 9, 0.1), (1, 4, 4097, 3, 1.0), (2, 4, 64, 1, 0.0),
    (8, 32, 4096, 1, 0.3),
])
def test_maw_update_matches_oracle(gpu, oracle, B, Hq, cap, n_new, alpha):
    torch, hgca, _ = gpu
    say(f"\n[case] maw_update B={B} Hq={Hq} cap={cap} n_new={n_new} alpha={alpha}")
    rng = np.random.default_rng(100 + cap)
    maw0 = softmax(rng.standard_normal((B, Hq, cap)), axis=-1).astype(np.float32)
    a = softmax(2.0 * rng.standard_normal((B, Hq, cap)), axis=-1).astype(np.float32)
    lens = rng.integers(0, cap + 1, B).astype(np.int32)
    lens[0] = cap
    sh = hgca.Shape(hgca.BF16, B, Hq, Hq, 128, 1.0)
    for use_lens in (True, False):
        m = torch.from_numpy(maw0).cuda()
        hgca.maw_update(sh, m, torch.from_numpy(a).cuda(), torch.from_numpy(lens).cuda() if use_lens else None,
                        cap, n_new, alpha)
        torch.cuda.synchronize()
        m = m.cpu().numpy()
        ref = oracle.maw_update(maw0, a, alpha, lens=lens if use_lens else None, n_new=n_new)
        assert np.max(np.abs(m - ref)) <= 1e-6
        if use_lens:
            for b in range(B):                                 # beyond the length: bit-identical to the input
                assert np.array_equal(m[b, :, lens[b]:], maw0[b, :, lens[b]:])
                first_new = max(lens[b] - n_new, 0)            # first observations are copied, not blended
                assert np.array_equal(m[b, :, first_new:lens[b]], a[b, :, first_new:lens[b]])


# ------------------------------------------------------------------------ threshold rule

def threshold_case(gpu, oracle, w, beta, size, k_max, lens=None):
    torch, hgca, _ = gpu
    B, Hq, cap = w.shape
    sh = hgca.Shape(hgca.BF16, B, Hq, Hq, 128, 1.0)
    dev = "cuda:0"
    idx = torch.full((B, Hq, max(k_max, 1)), -7, dtype=torch.int32, device=dev)
    cnt = torch.full((B, Hq), -7, dtype=torch.int32, device=dev)
    wn = torch.full((B, Hq, max(k_max, 1)), float("nan"), dtype=torch.float32, device=dev)
    size_arg = size if np.isscalar(size) else torch.from_numpy(np.asarray(size, np.int32)).to(dev)
    lens_arg = None if lens is None else torch.from_numpy(lens).to(dev)
    w_dev = torch.from_numpy(w).to(dev) if w.size else torch.empty(B, Hq, 1, dtype=torch.float32, device=dev)
    hgca.threshold_select(sh, w_dev, lens_arg, cap, size_arg, beta, k_max, idx, cnt, wn)
    idx2 = torch.full_like(idx, -7)
    cnt2 = torch.full_like(cnt, -7)
    hgca.threshold_select(sh, w_dev, lens_arg, cap, size_arg, beta, k_max, idx2, cnt2, None)
    torch.cuda.synchronize()
    idx_ref, cnt_ref, wn_ref = oracle.threshold_select(w, beta, size, k_max, lens=lens, normalised=True)
    idx, cnt, wn = idx.cpu().numpy()[:, :, :k_max], cnt.cpu().numpy(), wn.cpu().numpy()[:, :, :k_max]
    assert np.array_equal(cnt, cnt_ref)
    assert np.array_equal(idx, idx_ref)
    assert np.array_equal(idx2.cpu().numpy()[:, :, :k_max], idx_ref) and np.array_equal(cnt2.cpu().numpy(), cnt_ref)
    assert np.max(np.abs(wn - wn_ref), initial=0.0) <= 1e-6
    return cnt_ref


@pytest.mark.parametrize("B,Hq,cap,beta,sharp", [
    (2, 8, 700, 1.0, 3.0), (3, 4, 1023, 0.5, 1.0), (1, 4, 5000, 1.0, 6.0), (2, 2, 1, 0.5, 1.0), (2, 4, 257, 0.0, 1.0),
    (8, 32, 4096, 1.0, 4.0),
])
def test_threshold_select_is_exact_on_the_same_weights(gpu, oracle, B, Hq, cap, beta, sharp):
    say(f"\n[case] threshold_select B={B} Hq={Hq} cap={cap} beta={beta}")
    rng = np.random.default_rng(200 + cap)
    w = softmax(sharp * rng.standard_normal((B, Hq, cap)), axis=-1).astype(np.float32)
    cnt = threshold_case(gpu, oracle, w, beta, cap, cap)
    say(f"    kept per head: min {cnt.min()} mean {cnt.mean():.1f} max {cnt.max()} of {cap}")
    # ragged rows, per-sequence sizes, and a budget smaller than what passes
    lens = rng.integers(0, cap + 1, B).astype(np.int32)
    lens[-1] = 0
    sizes = np.maximum(lens, 1).astype(np.int32)
    threshold_case(gpu, oracle, w, beta, sizes, cap, lens=lens)
    threshold_case(gpu, oracle, w, beta * 0.5, cap, max(int(cnt.max()) // 2, 1))
    threshold_case(gpu, oracle, w, beta, cap, 0)


def test_threshold_is_strict_and_handles_all_or_nothing(gpu, oracle):
    say("\n[case] threshold_select: weights equal to the threshold, all kept, none kept")
    w = np.full((2, 4, 2048), 1.0 / 2048, np.float32)          # 2^-11 is exact: equal to beta/size at beta = 1
    assert threshold_case(gpu, oracle, w, 1.0, 2048, 2048).max() == 0
    assert threshold_case(gpu, oracle, w, 0.999, 2048, 2048).min() == 2048
    assert threshold_case(gpu, oracle, w, 1.0, 4096, 2048).min() == 2048   # size is an argument, not the row length
    w[:, :, 1000] = np.float32(1.0 / 2048) + np.float32(2.0 ** -34)        # one ulp above the threshold
    cnt = threshold_case(gpu, oracle, w, 1.0, 2048, 2048)
    assert cnt.min() == 1 and cnt.max() == 1


# ------------------------------------------------------------------------ the chain, over decode steps

def test_decode_steps_maw_then_threshold_then_sparse_attention(gpu, oracle):
    """Alg. 1 over a few decode steps: every step the window grows by one token, A_gpu updates the moving
    average, and at the end the oldest l_evict entries are filtered by MAW > beta / window size; the
    kept entries are then attended sparsely (Alg. 2, cpu_attention).  Both sides run the whole chain
    on their own from the same seeded inputs."""
    torch, hgca, runner = gpu
    cfg = wl.scaled(wl.CONFIGS["C2"], B=2, Hq=8, Hkv=2, W=1200, P=64, k=8)
    steps, alpha, beta, l_evict = 5, 0.3, 1.0, 512
    say(f"\n[case] decode loop: {steps} steps, alpha={alpha}, beta={beta}, evict {l_evict} of {cfg.W}")
    L = wl.make_layer(cfg)
    tw = otier(oracle, L.window)
    D = runner.DeviceLayer.upload(L)
    dev = "cuda:0"
    f32 = dict(dtype=torch.float32, device=dev)
    ws = hgca.alloc_workspace(D.shape, cfg.W, 0, l_evict, dev)
    o, lse = torch.empty(cfg.B, cfg.Hq, cfg.d, **f32), torch.empty(cfg.B, cfg.Hq, **f32)
    a_gpu = torch.empty(cfg.B, cfg.Hq, cfg.W, **f32)
    maw = torch.zeros(cfg.B, cfg.Hq, cfg.W, **f32)
    maw_ref = np.zeros((cfg.B, cfg.Hq, cfg.W))
    base = np.array([cfg.W - steps, cfg.W - steps - 300], np.int32)   # window lengths before the first step
    for t in range(steps):
        lens = (base + t + 1).astype(np.int32)
        q_t = wl.make_layer(cfg, layer=t + 1).q                 # a fresh seeded query per step
        n_new = int(lens.max()) if t == 0 else 1               # first step: every entry is a first observation
        D.window.seq_lens = torch.from_numpy(lens).to(dev)
        hgca.dense_window_attn_weights(D.shape, runner._to_gpu(q_t, dev), D.window, o, lse, a_gpu, ws)
        hgca.maw_update(D.shape, maw, a_gpu, D.window.seq_lens, cfg.W, n_new, alpha)
        tw.seq_lens = lens
        a_ref = oracle.window_weights(q_t, tw, L.scale)
        maw_ref = oracle.maw_update(maw_ref, a_ref, alpha, lens=lens, n_new=n_new)
    torch.cuda.synchronize()
    err = np.max(np.abs(maw.double().cpu().numpy() - maw_ref))
    say(f"    max|dMAW| after {steps} steps = {err:.3e}")
    assert err <= W_TOL["bf16"]

    evict = np.full(cfg.B, l_evict, np.int32)
    idx = torch.empty(cfg.B, cfg.Hq, l_evict, dtype=torch.int32, device=dev)
    cnt = torch.empty(cfg.B, cfg.Hq, dtype=torch.int32, device=dev)
    hgca.threshold_select(D.shape, maw, torch.from_numpy(evict).to(dev), cfg.W, D.window.seq_lens, beta, l_evict,
                          idx, cnt)
    torch.cuda.synchronize()
    idx_ref, cnt_ref = oracle.threshold_select(maw_ref, beta, lens, l_evict, lens=evict)
    idx_g, cnt_g = idx.cpu().numpy(), cnt.cpu().numpy()
    say(f"    kept per head: min {cnt_ref.min()} mean {cnt_ref.mean():.1f} max {cnt_ref.max()} of {l_evict}")
    assert 0 < cnt_ref.min() and cnt_ref.max() < l_evict
    differing = 0
    for b in range(cfg.B):
        thr = beta / lens[b]
        for h in range(cfg.Hq):
            got = set(idx_g[b, h, :cnt_g[b, h]].tolist())
            want = set(idx_ref[b, h, :cnt_ref[b, h]].tolist())
            assert np.all(np.diff(idx_g[b, h, :cnt_g[b, h]]) > 0) and np.all(idx_g[b, h, cnt_g[b, h]:] == -1)
            for j in got ^ want:                               # only entries within rounding of the threshold
                assert abs(maw_ref[b, h, j] - thr) <= 1e-5 * thr
                differing += 1
    say(f"    entries decided differently inside the rounding band: {differing}")

    # the salient entries of the evicted block, attended sparsely with the last query
    o_s, lse_s = torch.empty_like(o), torch.empty_like(lse)
    hgca.sparse_attn(D.shape, runner._to_gpu(q_t, dev), D.window, idx, cnt, l_evict, o_s, lse_s, ws)
    torch.cuda.synchronize()
    if differing == 0:
        o_ref, l_ref = oracle.attend_indexed(q_t, tw, idx_ref, cnt_ref, L.scale)
        assert np.max(np.abs(o_s.double().cpu().numpy() - o_ref)) <= 2e-4
        assert np.max(np.abs(lse_s.double().cpu().numpy() - l_ref)) <= 2e-4


# ------------------------------------------------------------------------ top-k on supplied scores

@pytest.mark.parametrize("B,Hq,cap,k,kind", [
    (2, 8, 700, 100, "normal"), (2, 4, 4097, 512, "maw"), (1, 4, 33000, 1200, "maw"), (3, 2, 64, 64, "coarse"),
    (8, 32, 4096, 409, "maw"),
    # more rows than compute units (512-thread workgroups): rows held as fp32, rows held as bytes with plenty of ties
    (10, 32, 4096, 409, "maw"), (10, 32, 9000, 900, "coarse"), (9, 32, 20001, 6667, "normal"),
    # rows too long for LDS as fp32 (sampled pre-filter, then the exact selection among what it retains): the usual
    # case, a budget of one, a peaked row, ties everywhere (the filter gives up: crowded bin), scores that grow
    # along the row (the last waves' lists overflow: the filter gives up), a budget too large for the filter
    (2, 8, 122880, 4096, "normal"), (1, 4, 70001, 1, "normal"), (1, 4, 140000, 3000, "maw"),
    (1, 2, 100000, 1500, "coarse"), (1, 4, 90000, 2500, "trend"), (1, 2, 80000, 30000, "normal"),
    (1, 4, 100000, 2000, "tie"),                # a handful of equal scores exactly where the budget cuts
    # more rows than compute units AND rows held as bytes: the 512-thread workgroups try the pre-filter too (sample of
    # 2 048 scores): the usual case, a tie at the cut, a trend (the filter gives up), a budget beyond its reach
    (9, 32, 14336, 1024, "normal"), (9, 32, 12000, 700, "tie"), (9, 32, 14000, 800, "trend"), (9, 32, 9000, 2000, "normal"),
    (9, 32, 8300, 1, "maw"),
    # infinite scores (a caller's masked positions): a few of either sign; so many -inf that the budget reaches into
    # them (ties among them are cut by position); on every path: registers, LDS, bytes, pre-filter, from memory
    (2, 8, 700, 100, "inf"), (2, 4, 28672, 2048, "inf"), (1, 4, 33000, 1200, "inf"), (1, 4, 100000, 2000, "inf"),
    (2, 4, 200000, 25000, "inf"), (9, 32, 9000, 900, "inf"),
    (2, 8, 700, 500, "masked"), (2, 4, 28672, 20000, "masked"), (1, 4, 40000, 30000, "masked"),
    (1, 2, 150000, 100000, "masked"), (9, 32, 9000, 6000, "masked"),
])
def test_select_topk_on_supplied_scores_is_exact(gpu, oracle, B, Hq, cap, k, kind):
    torch, hgca, _ = gpu
    say(f"\n[case] select_topk B={B} Hq={Hq} cap={cap} k={k} scores={kind}")
    rng = np.random.default_rng(300 + cap)
    z = rng.standard_normal((B, Hq, cap))
    if kind == "maw":                                           # weights of a peaked softmax: many tiny values, exact zeros
        s = softmax(12.0 * z, axis=-1).astype(np.float32)
        s[s < 1e-12] = 0.0
    elif kind == "inf":
        s = z.astype(np.float32)
        s[:, :, rng.integers(0, cap, 5)] = np.inf
        s[:, :, rng.integers(0, cap, 5)] = -np.inf
    elif kind == "masked":                                      # half of the positions are -inf
        s = np.where(rng.random((B, Hq, cap)) < 0.5, -np.inf, z).astype(np.float32)
    elif kind == "tie":
        s = z.astype(np.float32)
        for b in range(B):
            for h in range(Hq):
                order = np.argsort(-s[b, h], kind="stable")
                s[b, h, order[k + 40:k + 46]] = s[b, h, order[k - 1]]   # six more entries with the k-th largest score
    elif kind == "trend":
        s = (z + np.linspace(0.0, 12.0, cap)).astype(np.float32)
    elif kind == "coarse":
        s = np.round(z, 1).astype(np.float32)                   # plenty of exact ties
    else:
        s = z.astype(np.float32)
    lens = rng.integers(0, cap + 1, B).astype(np.int32)
    lens[0] = cap
    sh = hgca.Shape(hgca.BF16, B, Hq, Hq, 128, 1.0)
    dev = "cuda:0"
    s_dev = torch.from_numpy(s).to(dev)
    for use_lens in (False, True):
        idx = torch.full((B, Hq, k), -7, dtype=torch.int32, device=dev)
        cnt = torch.full((B, Hq), -7, dtype=torch.int32, device=dev)
        sel = torch.full((B, Hq, k), float("nan"), dtype=torch.float32, device=dev)
        hgca.select_topk(sh, s_dev, torch.from_numpy(lens).to(dev) if use_lens else None, cap, k, k, idx, cnt, sel)
        torch.cuda.synchronize()
        idx_ref, cnt_ref = oracle.select_given(s, k, k, lens=lens if use_lens else None)
        idx, cnt, sel = idx.cpu().numpy(), cnt.cpu().numpy(), sel.cpu().numpy()
        assert np.array_equal(cnt, cnt_ref)
        assert np.array_equal(idx, idx_ref)
        kept = np.arange(k)[None, None, :] < cnt[:, :, None]
        want = np.take_along_axis(s, np.where(kept, idx, 0).astype(np.int64), axis=2)
        assert np.array_equal(sel[kept], want[kept])            # the kept entries' own scores, bit for bit


def test_seeded_sweep_of_supplied_scores(gpu, oracle):
    """Forty seeded draws of (rows, row length, budget, score distribution, lengths) through hgca_select_topk: few
    long rows and many short ones, ties, trends along the row, peaked and bimodal rows, a constant first half,
    infinities; positions, counts and kept scores bit for bit against the oracle."""
    torch, hgca, _ = gpu
    dev = "cuda:0"
    rng = np.random.default_rng(4711)
    for it in range(40):
        if it % 2 == 0:                                         # few long rows: the 1024-thread workgroups
            B, Hq = int(rng.integers(1, 3)), int(rng.choice([1, 2, 4]))
            cap = int(rng.choice([34000, 66000, 70001, 100000, 131072, 140000]))
        else:                                                   # more rows than compute units: the 512-thread ones
            B, Hq = int(rng.integers(9, 12)), 32
            cap = int(rng.choice([4100, 8192, 8300, 9001, 12000, 14336, 20000]))
        k = int(rng.choice([1, 7, 64, 300, 1024, 2048, 4096, cap // 20, cap // 8, cap // 3]))
        k = max(1, min(k, cap - 1))
        kind = str(rng.choice(["normal", "coarse", "trend", "peaked", "bimodal", "sawtooth", "tie", "const_head", "inf"]))
        z = rng.standard_normal((B, Hq, cap))
        if kind == "coarse":
            s = np.round(z, int(rng.integers(0, 3)))
        elif kind == "trend":
            s = z + np.linspace(0, float(rng.choice([-12, 3, 12])), cap)
        elif kind == "peaked":
            s = np.exp(6 * z)
            s[s < 1e-6] = 0
        elif kind == "bimodal":
            s = z + 8.0 * (rng.random((B, Hq, cap)) < 0.03)
        elif kind == "sawtooth":
            s = z + 4.0 * ((np.arange(cap) // 256) % 7 == 0)
        elif kind == "tie":
            s = z.copy()
            for b in range(B):
                for h in range(Hq):
                    order = np.argsort(-s[b, h], kind="stable")
                    s[b, h, order[k:k + int(rng.integers(1, 40))]] = s[b, h, order[k - 1]]
        elif kind == "const_head":
            s = z.copy()
            s[:, :, :cap // 2] = 0.25
        elif kind == "inf":
            s = z.copy()
            s[:, :, rng.integers(0, cap, 5)] = np.inf
            s[:, :, rng.integers(0, cap, 5)] = -np.inf
        else:
            s = z
        s = s.astype(np.float32)
        lens = rng.integers(0, cap + 1, B).astype(np.int32)
        lens[0] = cap
        use_lens = bool(rng.random() < 0.5)
        say(f"\n[case] sweep {it}: B={B} Hq={Hq} cap={cap} k={k} scores={kind} lens={use_lens}")
        sh = hgca.Shape(hgca.BF16, B, Hq, Hq, 128, 1.0)
        idx = torch.full((B, Hq, k), -7, dtype=torch.int32, device=dev)
        cnt = torch.full((B, Hq), -7, dtype=torch.int32, device=dev)
        sel = torch.full((B, Hq, k), float("nan"), dtype=torch.float32, device=dev)
        hgca.select_topk(sh, torch.from_numpy(s).to(dev), torch.from_numpy(lens).to(dev) if use_lens else None, cap, k, k,
                         idx, cnt, sel)
        torch.cuda.synchronize()
        idx_ref, cnt_ref = oracle.select_given(s, k, k, lens=lens if use_lens else None)
        idx_g, cnt_g, sel_g = idx.cpu().numpy(), cnt.cpu().numpy(), sel.cpu().numpy()
        assert np.array_equal(cnt_g, cnt_ref) and np.array_equal(idx_g, idx_ref)
        kept = np.arange(k)[None, None, :] < cnt_g[:, :, None]
        want = np.take_along_axis(s, np.where(kept, idx_g, 0).astype(np.int64), axis=2)
        assert np.array_equal(sel_g[kept], want[kept])


def test_dense_with_moving_average_equals_the_two_calls(gpu, oracle):
    torch, hgca, runner = gpu
    cfg = wl.scaled(wl.CONFIGS["C5"], B=4, Hq=8, Hkv=2, W=256, P=1792, ragged=(100, 2048))
    say("\n[case] dense_window_attn_maw vs dense_window_attn_weights + maw_update")
    L = wl.make_layer(cfg)
    D = runner.DeviceLayer.upload(L)
    f32 = dict(dtype=torch.float32, device="cuda:0")
    ws = hgca.alloc_workspace(D.shape, cfg.W, 0, 0, "cuda:0")
    g = torch.Generator(device="cpu").manual_seed(3)
    maw0 = torch.rand(cfg.B, cfg.Hq, cfg.W, generator=g).cuda()
    outs = []
    for fused in (False, True):
        o, lse = torch.empty(cfg.B, cfg.Hq, cfg.d, **f32), torch.empty(cfg.B, cfg.Hq, **f32)
        a, maw = torch.empty(cfg.B, cfg.Hq, cfg.W, **f32), maw0.clone()
        if fused:
            hgca.dense_window_attn_maw(D.shape, D.q, D.window, o, lse, a, maw, 2, 0.3, ws)
        else:
            hgca.dense_window_attn_weights(D.shape, D.q, D.window, o, lse, a, ws)
            hgca.maw_update(D.shape, maw, a, D.window.seq_lens, cfg.W, 2, 0.3)
        torch.cuda.synchronize()
        outs.append((o, lse, a, maw))
    for x, y in zip(*outs):
        assert torch.equal(x, y)
    a_ref = oracle.window_weights(L.q, otier(oracle, L.window), L.scale)
    ref = oracle.maw_update(maw0.double().cpu().numpy(), a_ref, 0.3, lens=L.window.seq_lens, n_new=2)
    assert np.max(np.abs(outs[1][3].double().cpu().numpy() - ref)) <= W_TOL["bf16"]
