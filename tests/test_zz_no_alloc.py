"""The allocation-free dense window attention (hgca_dense_window_attn_static) against the entry point it is a
variant of (hgca_dense_window_attn) and against the fp64 oracle, through the C ABI.

The two entry points run the same kernels with the same split sizes, so their outputs are compared bit for bit;
the oracle comparison holds the usual bars (1e-5 fp32 inputs, 2e-2 and the tighter 2e-4 for bf16 inputs).  The
library's device array keeps whatever the previous call left in it, so the calls come in pairs, the second on
a smaller input, with nothing cleared in between.
"""
import sys

import numpy as np
import pytest

from paper_2507_03153_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-4}


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


def check_pair(gpu, oracle, cfg, poison=False):
    torch, hgca, runner = gpu
    say(f"\n[static] {cfg.name} dtype={cfg.dtype} B={cfg.B} Hq={cfg.Hq} Hkv={cfg.Hkv} d={cfg.d} W={cfg.W} "
        f"ragged={cfg.ragged} block={cfg.block_size}")
    L = wl.make_layer(cfg)
    D = runner.DeviceLayer.upload(L)
    f32 = dict(dtype=torch.float32, device=D.q.device)
    o_s = torch.full((cfg.B, cfg.Hq, cfg.d), float("nan"), **f32)
    l_s = torch.full((cfg.B, cfg.Hq), float("nan"), **f32)
    o_w, l_w = torch.empty_like(o_s), torch.empty_like(l_s)
    ws = hgca.alloc_workspace(D.shape, cfg.W, 0, 0, D.q.device)
    assert ws.numel() <= hgca.STATIC_SCRATCH_BYTES
    before = torch.cuda.memory_allocated()
    hgca.dense_window_attn_static(D.shape, D.q, D.window, o_s, l_s)
    assert torch.cuda.memory_allocated() == before             # nothing taken from torch's allocator either
    hgca.dense_window_attn(D.shape, D.q, D.window, o_w, l_w, ws)
    torch.cuda.synchronize()
    assert torch.equal(o_s, o_w) and torch.equal(l_s, l_w), "static and workspace variants differ"
    t = L.window
    o_ref, l_ref = oracle.attend_all(L.q, oracle.Tier(t.k, t.v, t.cap, t.seq_lens, t.block_table, t.block_size), L.scale)
    o, lse = o_s.double().cpu().numpy(), l_s.double().cpu().numpy()
    empty = np.isneginf(l_ref)
    assert np.array_equal(np.isneginf(lse), empty)
    err_o = float(np.max(np.abs(o - o_ref)))
    err_l = float(np.max(np.abs(lse[~empty] - l_ref[~empty]))) if (~empty).any() else 0.0
    say(f"    max|dO|={err_o:.3e} max|dlse|={err_l:.3e} (tol {TOL[cfg.dtype]:g})")
    assert err_o <= TOL[cfg.dtype] and err_l <= TOL[cfg.dtype]


def test_two_calls_in_a_row_second_smaller_bf16(gpu, oracle):
    big = wl.scaled(wl.CONFIGS["C2"], B=4, Hq=16, Hkv=4, W=1500, P=64, k=8)
    small = wl.scaled(wl.CONFIGS["C2"], B=2, Hq=8, Hkv=2, W=300, P=64, k=8)
    check_pair(gpu, oracle, big)
    check_pair(gpu, oracle, small)


def test_two_calls_in_a_row_second_smaller_fp32_ragged_paged(gpu, oracle):
    big = wl.scaled(wl.CONFIGS["C5"], dtype="f32", B=5, Hq=8, Hkv=4, d=64, W=700, P=2000 - 700, ragged=(100, 2000))
    small = wl.scaled(wl.CONFIGS["C5"], B=3, Hq=8, Hkv=1, W=160, P=500 - 160, ragged=(1, 500))
    check_pair(gpu, oracle, big)
    check_pair(gpu, oracle, small)


def test_c2_window_fits_and_matches(gpu, oracle):
    """The benchmarked shape's window part (B=8, Hq=32, W=4096) fits the array; a smaller call follows it."""
    check_pair(gpu, oracle, wl.scaled(wl.CONFIGS["C2"], P=64, k=8))
    check_pair(gpu, oracle, wl.scaled(wl.CONFIGS["C2"], B=1, Hq=4, Hkv=1, W=64, P=64, k=8))


def test_sizes_beyond_the_array_are_refused(gpu):
    torch, hgca, _ = gpu
    sh = hgca.Shape(hgca.BF16, 64, 64, 8, 128, 0.1)             # 4096 rows x 64 splits of 128 floats: 128 MiB of partials
    assert hgca.workspace_bytes(sh, 4096, 0, 0) > hgca.STATIC_SCRATCH_BYTES
    q = torch.zeros(64, 64, 128, dtype=torch.bfloat16, device="cuda:0")
    kv = torch.zeros(16, dtype=torch.bfloat16, device="cuda:0")  # never read: the call is refused on the host
    o, lse = torch.zeros(64, 64, 128, device="cuda:0"), torch.zeros(64, 64, device="cuda:0")
    with pytest.raises(hgca.HgcaError) as e:
        hgca.dense_window_attn_static(sh, q, hgca.Tier(kv, kv, 4096), o, lse)
    assert e.value.status == hgca.ERR_WORKSPACE
