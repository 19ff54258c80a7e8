"""KV_ctx of the KV manager (paper Alg. 1, KV_ctx.add(KV_evict[ids]); Sec. 3.2.2): the copy of listed pool
entries into per-head contiguous storage is byte work and is held to bit equality with a numpy gather of the same
inputs; attention over the compacted storage (every head a sequence of its own for the dense kernel) is held to
the bars of the sparse part: 2e-4 for bf16 inputs (stated bar 2e-2), 1e-5 for fp32."""
import sys

import numpy as np
import pytest

from paper_2507_03153_amd import workloads as wl
from test_gpu_append import to_paged
from test_gpu_parity import TIGHT, TOL, assert_partial, otier

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


def bits_of(t):
    """A device tensor's bytes as a numpy integer array (bf16 -> uint16, fp32 -> uint32)."""
    import torch
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.view(torch.int32).cpu().numpy().view(np.uint32)


@pytest.mark.parametrize("dtype,B,Hq,Hkv,d,P,k_max,ctx_cap,paged", [
    ("bf16", 3, 8, 2, 128, 1000, 300, 400, False),
    ("bf16", 2, 4, 4, 64, 515, 129, 129, False),
    ("f32", 2, 8, 2, 128, 333, 64, 100, False),
    ("f32", 1, 2, 1, 64, 100, 100, 50, False),
    ("bf16", 3, 8, 2, 128, 1008, 200, 260, True),
], ids=["bf16_gqa4", "bf16_mha_d64", "f32_gqa4", "f32_list_longer_than_ctx", "bf16_paged"])
def test_ctx_compact_is_a_bitwise_gather(gpu, dtype, B, Hq, Hkv, d, P, k_max, ctx_cap, paged):
    torch, hgca, runner = gpu
    dev = "cuda:0"
    say(f"\n[case] ctx_compact {dtype} B={B} Hq={Hq} Hkv={Hkv} d={d} P={P} k_max={k_max} ctx_cap={ctx_cap} paged={paged}")
    rng = np.random.default_rng(2507 + P)
    G = Hq // Hkv
    if dtype == "bf16":
        K, V = (rng.integers(0, 1 << 16, (B, Hkv, P, d)).astype(np.uint16) for _ in range(2))   # any bit pattern
        sentinel, code = np.uint16(0xABCD), hgca.BF16
    else:
        K, V = (rng.standard_normal((B, Hkv, P, d)).astype(np.float32) for _ in range(2))
        sentinel, code = np.float32(-123.5), hgca.F32
    p_lens = rng.integers(P // 2, P + 1, B).astype(np.int32)
    p_lens[0] = P
    cnt = rng.integers(0, k_max + 1, (B, Hq)).astype(np.int32)
    cnt[0, 0], cnt[-1, -1] = k_max, 0
    cnt = np.minimum(cnt, p_lens[:, None])
    idx = np.full((B, Hq, k_max), -1, np.int32)
    for b in range(B):
        for h in range(Hq):
            idx[b, h, :cnt[b, h]] = np.sort(rng.choice(p_lens[b], cnt[b, h], replace=False))
    first = rng.integers(0, ctx_cap // 3 + 1, (B, Hq)).astype(np.int32)
    first[0, 0] = 0
    first[0, 1] = ctx_cap                                       # a head whose storage is already full

    g = lambda a: runner._to_gpu(a, dev)
    pool = to_paged(runner, hgca, torch, K, V, p_lens, P, 16, 77, dev) if paged else hgca.Tier(g(K), g(V), P, g(p_lens))
    shape = hgca.Shape(code, B, Hq, Hkv, d, 1.0)
    k_ctx = g(np.full((B, Hq, ctx_cap, d), sentinel, K.dtype))
    v_ctx = g(np.full((B, Hq, ctx_cap, d), sentinel, K.dtype))
    cnt_out = torch.full((B, Hq), -7, dtype=torch.int32, device=dev)
    hgca.ctx_compact(shape, pool, g(idx), g(cnt), k_max, k_ctx, v_ctx, ctx_cap, first_row=g(first), cnt_out=cnt_out)
    torch.cuda.synchronize()

    want_k = np.full((B, Hq, ctx_cap, d), sentinel, K.dtype)
    want_v = want_k.copy()
    want_cnt = np.minimum(first + cnt, ctx_cap)
    for b in range(B):
        for h in range(Hq):
            n = want_cnt[b, h] - first[b, h]
            want_k[b, h, first[b, h]:first[b, h] + n] = K[b, h // G, idx[b, h, :n]]
            want_v[b, h, first[b, h]:first[b, h] + n] = V[b, h // G, idx[b, h, :n]]
    as_bits = lambda a: a.view(np.uint32) if a.dtype == np.float32 else a
    assert np.array_equal(bits_of(k_ctx), as_bits(want_k))
    assert np.array_equal(bits_of(v_ctx), as_bits(want_v))
    assert np.array_equal(cnt_out.cpu().numpy(), want_cnt)
    say(f"    rows copied per head {int((want_cnt - first).min())}..{int((want_cnt - first).max())}, "
        f"cut at ctx_cap in {int(np.sum(first + cnt > ctx_cap))} heads")


@pytest.mark.parametrize("name,kw", [
    ("C2", dict(B=2, Hq=8, Hkv=2, W=300, P=3001, k=300)),
    ("C2", dict(B=1, Hq=16, Hkv=2, W=128, P=5000, k=640)),
    ("C1", dict(B=2, Hq=8, Hkv=2, d=128, W=100, P=1200, k=77)),
    ("C5", dict(B=6, Hq=8, Hkv=2, W=256, P=1792, ragged=(100, 2048))),
], ids=["bf16_gqa4", "bf16_gqa8", "f32", "bf16_ragged_paged"])
def test_attention_over_kv_ctx_matches_the_oracle(gpu, oracle, name, kw):
    """Select with the oracle, compact in two instalments (as two evictions would), attend over KV_ctx as a
    stream, merge with the window part: equal to the oracle's sparse part and hybrid result."""
    torch, hgca, runner = gpu
    cfg = wl.scaled(wl.CONFIGS[name], **kw)
    say(f"\n[case] attention over KV_ctx {cfg.name} dtype={cfg.dtype} B={cfg.B} Hq={cfg.Hq} Hkv={cfg.Hkv} d={cfg.d} "
        f"W={cfg.W} P={cfg.P} k={cfg.k} ragged={cfg.ragged}")
    L = wl.make_layer(cfg)
    tw, tp = otier(oracle, L.window), otier(oracle, L.pool)
    D = runner.DeviceLayer.upload(L)
    dev = D.q.device
    B, Hq, d, k_max = cfg.B, cfg.Hq, cfg.d, L.k_max
    idx_ref, cnt_ref = oracle.select(L.q, tp, L.k, k_max, L.scale)
    o_ref, l_ref = oracle.attend_indexed(L.q, tp, idx_ref, cnt_ref, L.scale)

    # first instalment: the first half of every list; second: the rest, behind it
    half = cnt_ref // 2
    idx2 = np.full_like(idx_ref, -1)
    for b in range(B):
        for h in range(Hq):
            idx2[b, h, :cnt_ref[b, h] - half[b, h]] = idx_ref[b, h, half[b, h]:cnt_ref[b, h]]
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    k_ctx = torch.zeros(B, Hq, k_max, d, dtype=D.q.dtype, device=dev)
    v_ctx = torch.zeros_like(k_ctx)
    n1 = torch.zeros(B, Hq, dtype=torch.int32, device=dev)
    n2 = torch.zeros_like(n1)
    hgca.ctx_compact(D.shape, D.pool, to_dev(idx_ref), to_dev(half.astype(np.int32)), k_max, k_ctx, v_ctx, k_max,
                     cnt_out=n1)
    hgca.ctx_compact(D.shape, D.pool, to_dev(idx2), to_dev((cnt_ref - half).astype(np.int32)), k_max, k_ctx, v_ctx,
                     k_max, first_row=n1, cnt_out=n2)
    torch.cuda.synchronize()
    assert np.array_equal(n2.cpu().numpy(), cnt_ref)

    # every (sequence, head) is a sequence of its own with one head
    per_head = hgca.Shape(D.shape.dtype, B * Hq, 1, 1, d, D.shape.sm_scale)
    ctx = hgca.Tier(k_ctx.view(B * Hq, 1, k_max, d), v_ctx.view(B * Hq, 1, k_max, d), k_max, n2.view(-1))
    o_s = torch.full((B, Hq, d), float("nan"), dtype=torch.float32, device=dev)
    l_s = torch.full((B, Hq), float("nan"), dtype=torch.float32, device=dev)
    ws = hgca.alloc_workspace(per_head, k_max, 0, 0, dev)
    hgca.dense_window_attn(per_head, D.q.view(B * Hq, 1, d), ctx, o_s.view(B * Hq, 1, d), l_s.view(B * Hq, 1), ws)
    torch.cuda.synchronize()
    tight = min(TOL[cfg.dtype], TIGHT[cfg.dtype])
    assert_partial("attention over KV_ctx", o_s, l_s, o_ref, l_ref, tight)

    step = runner.HybridStep(D.shape, cfg.W, cfg.P, k_max)
    hgca.dense_window_attn(D.shape, D.q, D.window, step.o_w, step.lse_w, step.ws_dense)
    hgca.lse_merge(D.shape, o_s, l_s, step.o_w, step.lse_w, step.o, step.lse)
    torch.cuda.synchronize()
    o_w, l_w = oracle.attend_all(L.q, tw, L.scale)
    o_h, l_h = oracle.merge(o_ref, l_ref, o_w, l_w)
    assert_partial("hybrid over KV_ctx", step.o, step.lse, o_h, l_h, tight)
