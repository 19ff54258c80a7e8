"""Parity of the group-shared salient lists for GQA (paper Sec. 3.3, merged heads) with the oracle, through
the C ABI: group-budget selection (tie band as for the per-head selection), union of per-head lists (exact),
sparse attention on shared lists (2e-4 for bf16 inputs, 1e-5 for fp32; stated bars 2e-2 / 1e-5)."""
import sys

import numpy as np
import pytest

from oracle import grouped
from paper_2507_03153_amd import workloads as wl
from test_gpu_parity import BAND, TIGHT, TOL, assert_partial, assert_selection, otier

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


def run_case(gpu, oracle, cfg):
    torch, hgca, runner = gpu
    say(f"\n[case] grouped {cfg.name} dtype={cfg.dtype} B={cfg.B} Hq={cfg.Hq} Hkv={cfg.Hkv} d={cfg.d} W={cfg.W} P={cfg.P} "
        f"k={cfg.k} ragged={cfg.ragged} block={cfg.block_size}")
    L = wl.make_layer(cfg)
    tw, tp = otier(oracle, L.window), otier(oracle, L.pool)
    D = runner.DeviceLayer.upload(L)
    dev = D.q.device
    step = runner.HybridStep(D.shape, cfg.W, cfg.P, L.k_max)
    B, Hq, Hkv, G = cfg.B, cfg.Hq, cfg.Hkv, cfg.Hq // cfg.Hkv
    p_lens = L.pool.lens(B)
    k_b = np.full(B, L.k, np.int64) if np.isscalar(L.k) else np.asarray(L.k, np.int64)
    tight = min(TOL[cfg.dtype], TIGHT[cfg.dtype])

    say("  select_salient_grouped")
    idx_g = torch.full((B, Hkv, max(L.k_max, 1)), -7, dtype=torch.int32, device=dev)
    cnt_g = torch.full((B, Hkv), -7, dtype=torch.int32, device=dev)
    hgca.select_salient_grouped(D.shape, D.q, D.pool, D.k, L.k_max, idx_g, cnt_g, step.ws_sparse)
    torch.cuda.synchronize()
    gs = grouped.group_scores(oracle.scores(L.q, tp, L.scale), Hkv)
    n_band = assert_selection("grouped select", idx_g.cpu().numpy()[:, :, :L.k_max], cnt_g.cpu().numpy(), gs, p_lens,
                              k_b, BAND[cfg.dtype])
    idx_ref, cnt_ref = grouped.select_grouped(L.q, tp, L.k, L.k_max, L.scale)
    assert np.array_equal(cnt_g.cpu().numpy(), cnt_ref)
    same = float(np.mean(np.all(idx_g.cpu().numpy()[:, :, :L.k_max] == idx_ref, axis=-1))) if idx_ref.size else 1.0
    say(f"    rows identical to the oracle's: {same:.4f}; rows with a tie inside the band: {n_band}")

    say("  sparse_attn_grouped on the oracle's lists")
    idx_d = torch.from_numpy(np.ascontiguousarray(idx_ref)).to(dev) if L.k_max else idx_g
    cnt_d = torch.from_numpy(cnt_ref).to(dev)
    hgca.sparse_attn_grouped(D.shape, D.q, D.pool, idx_d, cnt_d, L.k_max, step.o_s, step.lse_s, step.ws_sparse)
    torch.cuda.synchronize()
    o_ref, l_ref = grouped.attend_grouped(L.q, tp, idx_ref, cnt_ref, L.scale)
    assert_partial("grouped sparse", step.o_s, step.lse_s, o_ref, l_ref, tight)

    say("  union_lists of the oracle's per-head lists, then attention on the union")
    idx_h, cnt_h = oracle.select(L.q, tp, L.k, L.k_max, L.scale)
    ku = G * L.k_max
    u_idx = torch.full((B, Hkv, max(ku, 1)), -7, dtype=torch.int32, device=dev)
    u_cnt = torch.full((B, Hkv), -7, dtype=torch.int32, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    idx_hd = torch.from_numpy(np.ascontiguousarray(idx_h)).to(dev) if L.k_max else idx_g
    hgca.union_lists(D.shape, idx_hd, torch.from_numpy(cnt_h).to(dev), L.k_max, max(cfg.P, 1), u_idx, u_cnt, ku, status)
    torch.cuda.synchronize()
    u_ref, uc_ref = grouped.union_lists(idx_h, cnt_h, Hkv, ku)
    assert np.array_equal(u_cnt.cpu().numpy(), uc_ref) and np.array_equal(u_idx.cpu().numpy()[:, :, :ku], u_ref)
    assert int(status.cpu()[0]) == 0
    ws_u = hgca.alloc_workspace(D.shape, 0, 0, ku, dev)
    hgca.sparse_attn_grouped(D.shape, D.q, D.pool, u_idx, u_cnt, ku, step.o_s, step.lse_s, ws_u)
    torch.cuda.synchronize()
    o_u, l_u = grouped.attend_grouped(L.q, tp, u_ref, uc_ref, L.scale)
    assert_partial("sparse on the union", step.o_s, step.lse_s, o_u, l_u, tight)
    say(f"    union sizes {uc_ref.min()}..{uc_ref.max()} for per-head lists of {cnt_h.min()}..{cnt_h.max()}")

    say("  whole step with the group budget: dense, grouped select, grouped sparse (deferred), one fold")
    hgca.dense_window_attn(D.shape, D.q, D.window, None, None, step.ws_dense)
    hgca.select_salient_grouped(D.shape, D.q, D.pool, D.k, L.k_max, idx_g, cnt_g, step.ws_sparse)
    hgca.sparse_attn_grouped(D.shape, D.q, D.pool, idx_g, cnt_g, L.k_max, None, None, step.ws_sparse)
    hgca.lse_merge_splits(D.shape, cfg.W, step.ws_dense, L.k_max, step.ws_sparse, step.o, step.lse)
    torch.cuda.synchronize()
    o_w, l_w = oracle.attend_all(L.q, tw, L.scale)
    o_h, l_h = oracle.merge(o_ref, l_ref, o_w, l_w)
    assert_partial("grouped hybrid", step.o, step.lse, o_h, l_h, TOL[cfg.dtype] if n_band else tight)


@pytest.mark.parametrize("kw", [
    dict(B=2, Hq=8, Hkv=2, W=300, P=3001, k=300),
    dict(B=1, Hq=16, Hkv=2, W=128, P=5000, k=640),
    dict(B=2, Hq=4, Hkv=2, d=64, W=100, P=2222, k=100),
    dict(B=3, Hq=4, Hkv=4, W=64, P=1500, k=257),                 # groups of one head: the per-head case
    dict(B=2, Hq=8, Hkv=2, W=64, P=512, k=0),
    dict(B=2, Hq=8, Hkv=2, W=64, P=0, k=16),
    dict(B=36, Hq=16, Hkv=8, d=64, W=40, P=1500, k=150),         # 288 lists: the selection's small workgroups
    dict(B=33, Hq=16, Hkv=8, d=64, W=40, P=6000, k=700),         # the same with rows held as bytes
], ids=["gqa4", "gqa8", "gqa2_d64", "mha", "k0", "P0", "many_lists", "many_lists_byte_cache"])
def test_grouped_bf16(gpu, oracle, kw):
    run_case(gpu, oracle, wl.scaled(wl.CONFIGS["C2"], **kw))


@pytest.mark.timeout(600)
def test_grouped_full_size_c2(gpu, oracle):
    """The shape bench.py times the grouped calls on."""
    run_case(gpu, oracle, wl.CONFIGS["C2"])


def test_grouped_fp32(gpu, oracle):
    run_case(gpu, oracle, wl.scaled(wl.CONFIGS["C1"], B=2, Hq=8, Hkv=2, d=128, W=100, P=1200, k=77))


def test_grouped_ragged_paged(gpu, oracle):
    run_case(gpu, oracle, wl.scaled(wl.CONFIGS["C5"], B=6, Hq=8, Hkv=2, W=256, P=1792, ragged=(100, 2048)))


def test_union_longer_than_its_row_is_cut_and_flagged(gpu, oracle):
    torch, hgca, _ = gpu
    dev = "cuda:0"
    say("\n[case] union longer than k_max_out")
    sh = hgca.Shape(hgca.BF16, 1, 4, 1, 128, 1.0)
    idx = torch.tensor([[[0, 10, 20], [1, 11, 21], [2, 12, 22], [3, 13, 23]]], dtype=torch.int32, device=dev)
    cnt = torch.full((1, 4), 3, dtype=torch.int32, device=dev)
    out = torch.full((1, 1, 5), -7, dtype=torch.int32, device=dev)
    out_cnt = torch.zeros(1, 1, dtype=torch.int32, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    hgca.union_lists(sh, idx, cnt, 3, 64, out, out_cnt, 5, status)
    torch.cuda.synchronize()
    assert out.cpu().tolist() == [[[0, 1, 2, 3, 10]]] and int(out_cnt.cpu()[0, 0]) == 5 and int(status.cpu()[0]) == 1
