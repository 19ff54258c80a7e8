"""Host-only checks of the C ABI: the library loads, exports what include/hgca.h declares,
sizes its workspace sensibly and rejects bad arguments before touching the device.
No call here reaches a kernel launch."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def hg():
    from paper_2507_03153_amd import build, hgca
    build.build(force=False)
    hgca.lib()
    return hgca


def test_every_declared_symbol_is_exported(hg):
    with open(os.path.join(ROOT, "include", "hgca.h")) as f:
        header = re.sub(r"/\*.*?\*/", "", f.read(), flags=re.S)
    declared = set(re.findall(r"\b(hgca_\w+)\s*\(", header))
    assert declared == set(hg.EXPORTS)
    L = ctypes.CDLL(os.path.join(ROOT, "paper_2507_03153_amd", "libhgca.so"))
    for name in declared:
        assert getattr(L, name) is not None


def test_batch_and_head_count_limits(hg):
    assert hg.workspace_bytes(hg.Shape(hg.BF16, 65535, 8, 2, 128, 1.0), 16, 16, 4) > 0
    assert hg.workspace_bytes(hg.Shape(hg.BF16, 65536, 8, 2, 128, 1.0), 16, 16, 4) == 0
    sh = hg.Shape(hg.BF16, 65536, 8, 2, 128, 1.0)
    assert hg.lib().hgca_maw_update(ctypes.byref(sh), FAKE, FAKE, None, 64, 1, 0.5, None) == hg.ERR_UNSUPPORTED


def test_status_strings(hg):
    texts = {hg.status_string(s) for s in (0, -1, -2, -3, -4)}
    assert len(texts) == 5 and hg.status_string(-99) == "unknown status"


def test_workspace_bytes(hg):
    sh = hg.Shape(hg.BF16, 8, 32, 8, 128, 0.088)
    small = hg.workspace_bytes(sh, 4096, 0, 0)
    full = hg.workspace_bytes(sh, 4096, 28672, 2048)
    assert 0 < small < full
    assert full >= 8 * 32 * 28672 * 4                        # room for one fp32 score per pool token and head
    assert hg.workspace_bytes(sh, 0, 0, 0) > 0
    assert hg.workspace_bytes(hg.Shape(hg.BF16, 8, 32, 5, 128, 1.0), 16, 16, 4) == 0
    assert hg.workspace_bytes(sh, -1, 0, 0) == 0


FAKE = ctypes.c_void_p(0x10000)       # non-null, 16-byte aligned, never dereferenced on these paths
ODD = ctypes.c_void_p(0x10004)


def _view(hg, cap=64, k=FAKE, v=FAKE, table=None, bs=0, mb=0):
    return hg.KvView(k, v, None, table, cap, bs, mb, None)


def _dense(hg, sh, view, q=FAKE, o=FAKE, lse=FAKE, ws=FAKE, ws_bytes=1 << 40):
    return hg.lib().hgca_dense_window_attn(ctypes.byref(sh), q, ctypes.byref(view), o, lse, ws, ws_bytes, None)


def test_dense_rejects_bad_arguments(hg):
    good = hg.Shape(hg.F32, 1, 4, 4, 64, 0.125)
    v = _view(hg)
    assert _dense(hg, hg.Shape(hg.F32, 1, 4, 3, 64, 0.125), v) == hg.ERR_INVALID_ARG     # Hq % Hkv
    assert _dense(hg, hg.Shape(hg.F32, 1, 4, 4, 80, 0.125), v) == hg.ERR_UNSUPPORTED     # head_dim
    assert _dense(hg, hg.Shape(7, 1, 4, 4, 64, 0.125), v) == hg.ERR_UNSUPPORTED          # dtype
    assert _dense(hg, hg.Shape(hg.F32, 1, 48, 4, 64, 0.125), v) == hg.ERR_UNSUPPORTED    # group of 12
    assert _dense(hg, hg.Shape(hg.F32, -1, 4, 4, 64, 0.125), v) == hg.ERR_INVALID_ARG
    assert _dense(hg, hg.Shape(hg.F32, 1, 4, 4, 64, float("nan")), v) == hg.ERR_INVALID_ARG
    assert _dense(hg, good, v, q=None) == hg.ERR_INVALID_ARG
    assert _dense(hg, good, v, q=ODD) == hg.ERR_INVALID_ARG
    assert _dense(hg, good, v, o=None) == hg.ERR_INVALID_ARG
    assert _dense(hg, good, v, lse=None) == hg.ERR_INVALID_ARG
    assert _dense(hg, good, _view(hg, k=None)) == hg.ERR_INVALID_ARG
    assert _dense(hg, good, _view(hg, v=None)) == hg.ERR_INVALID_ARG
    assert _dense(hg, good, _view(hg, k=ODD)) == hg.ERR_INVALID_ARG
    assert _dense(hg, good, _view(hg, cap=-3)) == hg.ERR_INVALID_ARG
    assert _dense(hg, good, _view(hg, table=FAKE, bs=24, mb=8)) == hg.ERR_UNSUPPORTED    # block size % 16
    assert _dense(hg, good, _view(hg, table=FAKE, bs=16, mb=3)) == hg.ERR_INVALID_ARG    # table too short
    assert _dense(hg, good, _view(hg, table=FAKE, bs=0, mb=4)) == hg.ERR_INVALID_ARG
    assert _dense(hg, good, v, ws=None) == hg.ERR_WORKSPACE
    assert _dense(hg, good, v, ws_bytes=16) == hg.ERR_WORKSPACE
    need = hg.workspace_bytes(good, 64, 0, 0)
    assert _dense(hg, good, v, ws_bytes=need - 1) == hg.ERR_WORKSPACE
    assert hg.lib().hgca_dense_window_attn(None, FAKE, ctypes.byref(v), FAKE, FAKE, FAKE, 1 << 40, None) \
        == hg.ERR_INVALID_ARG
    assert hg.lib().hgca_dense_window_attn(ctypes.byref(good), FAKE, None, FAKE, FAKE, FAKE, 1 << 40, None) \
        == hg.ERR_INVALID_ARG


def test_static_dense_rejects_bad_arguments_and_sizes_beyond_its_array(hg):
    """The allocation-free variant validates like hgca_dense_window_attn, wants both outputs, and refuses a shape
    whose split partials exceed the library's device array before anything touches the device."""
    def call(sh, view, q=FAKE, o=FAKE, lse=FAKE):
        return hg.lib().hgca_dense_window_attn_static(ctypes.byref(sh), q, ctypes.byref(view), o, lse, None)
    good = hg.Shape(hg.F32, 1, 4, 4, 64, 0.125)
    v = _view(hg)
    assert call(hg.Shape(hg.F32, 1, 4, 3, 64, 0.125), v) == hg.ERR_INVALID_ARG
    assert call(hg.Shape(hg.F32, 1, 4, 4, 80, 0.125), v) == hg.ERR_UNSUPPORTED
    assert call(good, v, o=None) == hg.ERR_INVALID_ARG           # no deferred result here
    assert call(good, v, lse=None) == hg.ERR_INVALID_ARG
    assert call(good, v, o=None, lse=None) == hg.ERR_INVALID_ARG
    assert call(good, _view(hg, k=None)) == hg.ERR_INVALID_ARG
    assert call(good, _view(hg, table=FAKE, bs=24, mb=8)) == hg.ERR_UNSUPPORTED
    big = hg.Shape(hg.BF16, 64, 64, 8, 128, 0.1)
    assert hg.workspace_bytes(big, 4096, 0, 0) > hg.STATIC_SCRATCH_BYTES
    assert call(big, _view(hg, cap=4096)) == hg.ERR_WORKSPACE
    c2 = hg.Shape(hg.BF16, 8, 32, 8, 128, 0.088)                 # the benchmarked shape's window fits
    assert hg.workspace_bytes(c2, 4096, 0, 0) <= hg.STATIC_SCRATCH_BYTES
    assert call(hg.Shape(hg.BF16, 0, 32, 8, 128, 0.088), v) == hg.OK   # batch 0: a no-op


def test_select_and_sparse_reject_bad_arguments(hg):
    sh = hg.Shape(hg.BF16, 2, 8, 2, 128, 0.088)
    v = _view(hg, cap=256)
    L = hg.lib()

    def select(k_ptr=None, k_uni=8, k_max=8, idx=FAKE, cnt=FAKE, ws=FAKE, ws_bytes=1 << 40, view=v, q=FAKE):
        return L.hgca_select_salient(ctypes.byref(sh), q, ctypes.byref(view), k_ptr, k_uni, k_max, idx, cnt, None,
                                     ws, ws_bytes, None)

    assert select(k_uni=9) == hg.ERR_INVALID_ARG              # k > k_max
    assert select(k_uni=-1) == hg.ERR_INVALID_ARG
    assert select(k_max=-1) == hg.ERR_INVALID_ARG
    assert select(idx=None) == hg.ERR_INVALID_ARG
    assert select(cnt=None) == hg.ERR_INVALID_ARG
    assert select(q=None) == hg.ERR_INVALID_ARG
    assert select(ws_bytes=1024) == hg.ERR_WORKSPACE
    assert select(view=_view(hg, cap=256, k=None, v=None)) == hg.ERR_INVALID_ARG
    need = hg.workspace_bytes(sh, 0, 256, 0)                  # the selection alone keeps no kept-entry scores
    assert select(ws_bytes=need - 1) == hg.ERR_WORKSPACE

    def sparse(idx=FAKE, cnt=FAKE, k_max=8, o=FAKE, lse=FAKE, ws=FAKE, ws_bytes=1 << 40, view=v):
        return L.hgca_sparse_attn(ctypes.byref(sh), FAKE, ctypes.byref(view), idx, cnt, k_max, None, o, lse, ws,
                                  ws_bytes, None)

    assert sparse(idx=None) == hg.ERR_INVALID_ARG
    assert sparse(cnt=None) == hg.ERR_INVALID_ARG
    assert sparse(k_max=-2) == hg.ERR_INVALID_ARG
    assert sparse(o=ODD) == hg.ERR_INVALID_ARG
    assert sparse(view=_view(hg, cap=256, v=None)) == hg.ERR_INVALID_ARG      # sparse attention reads V
    assert sparse(ws=None) == hg.ERR_WORKSPACE


def test_merge_rejects_bad_arguments(hg):
    sh = hg.Shape(hg.F32, 2, 4, 4, 128, 1.0)
    L = hg.lib()

    def merge(o_a=FAKE, l_a=FAKE, o_b=ctypes.c_void_p(0x20000), l_b=FAKE, out=ctypes.c_void_p(0x30000),
              dt=hg.F32, shape=sh):
        return L.hgca_lse_merge(ctypes.byref(shape), o_a, l_a, o_b, l_b, out, dt, None, None)

    assert merge(o_a=None) == hg.ERR_INVALID_ARG
    assert merge(l_b=None) == hg.ERR_INVALID_ARG
    assert merge(out=None) == hg.ERR_INVALID_ARG
    assert merge(dt=5) == hg.ERR_UNSUPPORTED
    assert merge(out=FAKE, dt=hg.BF16) == hg.ERR_INVALID_ARG                  # bf16 result over an fp32 input
    assert merge(shape=hg.Shape(hg.F32, 2, 4, 4, 96, 1.0)) == hg.ERR_UNSUPPORTED


def test_binding_refuses_cpu_tensors(hg):
    import torch
    q = torch.zeros(1, 4, 64)
    with pytest.raises(ValueError):
        hg.make_shape(q, 4, 0.125)


def test_sparsifier_entry_points_reject_bad_arguments(hg):
    L = hg.lib()
    sh = hg.Shape(hg.BF16, 2, 8, 2, 128, 0.088)
    view = _view(hg)
    byref = ctypes.byref
    # the weights cannot be produced without the window's own result
    assert L.hgca_dense_window_attn_weights(byref(sh), FAKE, byref(view), None, None, FAKE, FAKE, 1 << 40, None) \
        == hg.ERR_INVALID_ARG
    assert L.hgca_dense_window_attn_weights(byref(sh), FAKE, byref(view), FAKE, FAKE, None, FAKE, 1 << 40, None) \
        == hg.ERR_INVALID_ARG
    assert L.hgca_dense_window_attn_weights(byref(sh), FAKE, byref(view), FAKE, FAKE, FAKE, FAKE, 16, None) \
        == hg.ERR_WORKSPACE
    # moving average: alpha in [0, 1], sizes non-negative, pointers present
    for alpha in (-0.1, 1.5, float("nan")):
        assert L.hgca_maw_update(byref(sh), FAKE, FAKE, None, 64, 1, alpha, None) == hg.ERR_INVALID_ARG
    assert L.hgca_maw_update(byref(sh), FAKE, FAKE, None, -1, 1, 0.5, None) == hg.ERR_INVALID_ARG
    assert L.hgca_maw_update(byref(sh), FAKE, FAKE, None, 64, -1, 0.5, None) == hg.ERR_INVALID_ARG
    assert L.hgca_maw_update(byref(sh), None, FAKE, None, 64, 1, 0.5, None) == hg.ERR_INVALID_ARG
    assert L.hgca_maw_update(byref(sh), FAKE, None, None, 64, 1, 0.5, None) == hg.ERR_INVALID_ARG
    assert L.hgca_maw_update(byref(sh), None, None, None, 0, 1, 0.5, None) == hg.OK       # nothing to do
    # threshold rule
    def thr(w=FAKE, cap=64, sizes=None, size=64, beta=1.0, k_max=64, idx=FAKE, cnt=FAKE):
        return L.hgca_threshold_select(byref(sh), w, None, cap, sizes, size, beta, k_max, idx, cnt, None, None)
    assert thr(size=0) == hg.ERR_INVALID_ARG
    assert thr(beta=-1.0) == hg.ERR_INVALID_ARG
    assert thr(beta=float("nan")) == hg.ERR_INVALID_ARG
    assert thr(k_max=-1) == hg.ERR_INVALID_ARG
    assert thr(cap=-1) == hg.ERR_INVALID_ARG
    assert thr(w=None) == hg.ERR_INVALID_ARG
    assert thr(idx=None) == hg.ERR_INVALID_ARG
    assert thr(cnt=None) == hg.ERR_INVALID_ARG
    empty = hg.Shape(hg.BF16, 0, 8, 2, 128, 0.088)
    assert L.hgca_threshold_select(byref(empty), None, None, 64, None, 64, 1.0, 64, None, None, None, None) == hg.OK


def test_select_topk_rejects_bad_arguments(hg):
    L = hg.lib()
    sh = hg.Shape(hg.BF16, 2, 8, 2, 128, 0.088)

    def topk(scores=FAKE, cap=64, k=8, k_max=8, idx=FAKE, cnt=FAKE):
        return L.hgca_select_topk(ctypes.byref(sh), scores, None, cap, None, k, k_max, idx, cnt, None, None)
    assert topk(scores=None) == hg.ERR_INVALID_ARG
    assert topk(scores=ODD) == hg.ERR_INVALID_ARG
    assert topk(cap=-1) == hg.ERR_INVALID_ARG
    assert topk(k=-1) == hg.ERR_INVALID_ARG
    assert topk(k=9) == hg.ERR_INVALID_ARG                     # budget beyond the row length of idx_out
    assert topk(idx=None) == hg.ERR_INVALID_ARG
    assert topk(cnt=None) == hg.ERR_INVALID_ARG


def test_kv_manager_entry_points_reject_bad_arguments(hg):
    L = hg.lib()
    sh = hg.Shape(hg.BF16, 2, 8, 2, 128, 0.088)
    p = 0x10000

    def state(**kw):
        f = dict(k_blocks=p, v_blocks=p, block_table=p, first_win_block=p, win_lens=p, pool_lens=p, a_maw=p,
                 ctx_idx=p, ctx_cnt=p, a_evicted=None, plan=p, status=p,
                 block_size=16, max_blocks=8, win_blocks=4, k_max=64, pool_cap=128, win_cap_blocks=0)
        f.update(kw)
        return hg.CacheState(**f)

    def append(st, k=FAKE, v=FAKE):
        return L.hgca_kv_append(ctypes.byref(sh), ctypes.byref(st), k, v, None, None)

    def append_n(st, n, k=FAKE, v=FAKE):
        return L.hgca_kv_append_tokens(ctypes.byref(sh), ctypes.byref(st), k, v, n, None, None)

    def turn(st, q=FAKE, k=FAKE, v=FAKE, n_q=8, alpha=0.3, beta=1.0, flags=0, a_gpu=FAKE, a_cpu=FAKE, o=FAKE, lse=FAKE,
             ws=FAKE, ws_bytes=1 << 40):
        return L.hgca_managed_append_step(ctypes.byref(sh), ctypes.byref(st), q, k, v, n_q, alpha, beta, flags, a_gpu,
                                          a_cpu, o, lse, ws, ws_bytes, None)
    assert append_n(state(), -1) == hg.ERR_INVALID_ARG
    assert append_n(state(), 0, k=None) == hg.OK                 # nothing to insert
    assert append_n(state(), 5, k=None) == hg.ERR_INVALID_ARG
    assert append_n(state(win_cap_blocks=3), 5) == hg.ERR_INVALID_ARG        # capacity below l_max
    assert append_n(state(win_cap_blocks=9), 5) == hg.ERR_INVALID_ARG        # capacity beyond the table row
    need = L.hgca_managed_append_workspace_bytes(ctypes.byref(sh), ctypes.byref(state(win_cap_blocks=6)), 8)
    assert need > 0
    assert L.hgca_managed_append_workspace_bytes(ctypes.byref(sh), ctypes.byref(state()), -1) == 0
    assert L.hgca_managed_append_workspace_bytes(ctypes.byref(sh), ctypes.byref(state(block_size=0)), 8) == 0
    st6 = state(win_cap_blocks=6)
    assert turn(st6, q=None) == hg.ERR_INVALID_ARG
    assert turn(st6, k=ODD) == hg.ERR_INVALID_ARG
    assert turn(st6, a_gpu=None) == hg.ERR_INVALID_ARG
    assert turn(st6, a_cpu=None) == hg.ERR_INVALID_ARG
    assert turn(st6, o=None) == hg.ERR_INVALID_ARG
    assert turn(st6, lse=None) == hg.ERR_INVALID_ARG
    assert turn(st6, alpha=1.5) == hg.ERR_INVALID_ARG
    assert turn(st6, beta=-1.0) == hg.ERR_INVALID_ARG
    assert turn(st6, flags=64) == hg.ERR_INVALID_ARG
    assert turn(st6, n_q=-1) == hg.ERR_INVALID_ARG
    assert turn(st6, ws=None) == hg.ERR_WORKSPACE
    assert turn(st6, ws_bytes=need - 1) == hg.ERR_WORKSPACE
    assert turn(state(block_size=24)) == hg.ERR_UNSUPPORTED
    f32 = hg.Shape(hg.F32, 2, 8, 2, 128, 0.088)
    assert L.hgca_managed_append_step(ctypes.byref(f32), ctypes.byref(st6), FAKE, FAKE, FAKE, 8, 0.3, 1.0, 0, FAKE, FAKE,
                                      FAKE, FAKE, FAKE, 64, None) == hg.ERR_WORKSPACE          # fp32 is served too
    assert turn(st6, n_q=0, q=None) == hg.OK                     # an empty prompt: nothing to do

    def evict(st, beta=1.0):
        return L.hgca_kv_evict(ctypes.byref(sh), ctypes.byref(st), beta, None)
    for bad in (dict(block_size=0), dict(win_blocks=0), dict(win_blocks=9), dict(max_blocks=0), dict(k_max=-1),
                dict(pool_cap=-1), dict(k_blocks=None), dict(v_blocks=0x10004), dict(block_table=None),
                dict(win_lens=None), dict(a_maw=None), dict(ctx_idx=None), dict(plan=None), dict(status=None)):
        assert append(state(**bad)) == hg.ERR_INVALID_ARG, bad
        assert evict(state(**bad)) == hg.ERR_INVALID_ARG, bad
    assert append(state(block_size=24)) == hg.ERR_UNSUPPORTED
    assert append(state(), k=None) == hg.ERR_INVALID_ARG
    assert append(state(), v=ODD) == hg.ERR_INVALID_ARG
    assert evict(state(), beta=-0.5) == hg.ERR_INVALID_ARG
    assert evict(state(), beta=float("nan")) == hg.ERR_INVALID_ARG
    assert L.hgca_kv_append(ctypes.byref(sh), None, FAKE, FAKE, None, None) == hg.ERR_INVALID_ARG
    empty = hg.Shape(hg.BF16, 0, 8, 2, 128, 0.088)
    assert L.hgca_kv_evict(ctypes.byref(empty), ctypes.byref(state(k_blocks=None)), 1.0, None) == hg.OK


def test_append_entry_points_reject_bad_arguments(hg):
    L = hg.lib()
    sh = hg.Shape(hg.BF16, 2, 8, 2, 128, 0.088)
    view = _view(hg)
    byref = ctypes.byref
    assert hg.lib().hgca_append_workspace_bytes(byref(sh), 32, 4096) > 0
    assert hg.lib().hgca_append_workspace_bytes(byref(sh), -1, 4096) == 0
    assert hg.lib().hgca_append_workspace_bytes(byref(hg.Shape(hg.BF16, 2, 8, 3, 128, 1.0)), 4, 64) == 0

    def attn(shape=sh, q=FAKE, n_q=4, o=FAKE, lse=FAKE, ws=FAKE, ws_bytes=1 << 40, flags=1):
        return L.hgca_append_attn(byref(shape), q, n_q, byref(view), flags, o, lse, ws, ws_bytes, None)
    assert attn(q=None) == hg.ERR_INVALID_ARG
    assert attn(shape=hg.Shape(hg.BF16, 2, 8, 2, 128, 0.0)) == hg.ERR_INVALID_ARG      # scale must be > 0 here
    assert attn(shape=hg.Shape(hg.BF16, 2, 8, 2, 128, -0.1)) == hg.ERR_INVALID_ARG
    assert attn(shape=hg.Shape(hg.BF16, 2, 8, 2, 128, float("inf"))) == hg.ERR_INVALID_ARG
    assert attn(flags=4) == hg.ERR_INVALID_ARG                  # an unknown flag bit
    assert attn(flags=-1) == hg.ERR_INVALID_ARG
    assert attn(q=ODD) == hg.ERR_INVALID_ARG
    assert attn(n_q=-1) == hg.ERR_INVALID_ARG
    assert attn(n_q=5000) == hg.ERR_INVALID_ARG
    assert attn(o=None) == hg.ERR_INVALID_ARG
    assert attn(lse=None) == hg.ERR_INVALID_ARG
    assert attn(ws=None) == hg.ERR_WORKSPACE
    assert attn(ws_bytes=64) == hg.ERR_WORKSPACE
    assert attn(shape=hg.Shape(hg.F32, 2, 8, 2, 128, 0.088), ws_bytes=64) == hg.ERR_WORKSPACE   # fp32 is served too
    assert attn(shape=hg.Shape(hg.F32, 4096, 8, 2, 128, 0.088), n_q=32) == hg.ERR_UNSUPPORTED     # B * n_q > 65 535
    assert attn(n_q=0) == hg.OK                                                          # nothing to do
    # (KV head, block of 128 query rows) pairs are one grid dimension: 2048 heads x 32 blocks do not fit 65 535
    assert attn(shape=hg.Shape(hg.BF16, 1, 2048, 2048, 128, 0.088), n_q=4096) == hg.ERR_UNSUPPORTED
    assert attn(shape=hg.Shape(hg.BF16, 1, 2047, 2047, 128, 0.088), n_q=4096, ws_bytes=64) == hg.ERR_WORKSPACE

    # both tiers in one call
    assert L.hgca_append_tiers_workspace_bytes(byref(sh), 32, 4096, 28672) > 0
    assert L.hgca_append_tiers_workspace_bytes(byref(sh), 32, -1, 64) == 0
    assert L.hgca_append_tiers_workspace_bytes(byref(sh), -1, 64, 64) == 0

    def tiers(shape=sh, q=FAKE, n_q=4, o=FAKE, lse=FAKE, ws=FAKE, ws_bytes=1 << 40, flags=1):
        return L.hgca_append_attn_tiers(byref(shape), q, n_q, byref(view), byref(view), flags, o, lse, None, None, ws,
                                        ws_bytes, None)
    assert tiers(q=None) == hg.ERR_INVALID_ARG
    assert tiers(flags=4) == hg.ERR_INVALID_ARG
    assert tiers(n_q=5000) == hg.ERR_INVALID_ARG
    assert tiers(o=None) == hg.ERR_INVALID_ARG
    assert tiers(lse=None) == hg.ERR_INVALID_ARG
    assert tiers(ws=None) == hg.ERR_WORKSPACE
    assert tiers(ws_bytes=64) == hg.ERR_WORKSPACE
    assert tiers(shape=hg.Shape(hg.F32, 2, 8, 2, 128, 0.088)) == hg.ERR_UNSUPPORTED     # per-tier calls serve fp32
    assert tiers(shape=hg.Shape(hg.BF16, 1, 2048, 2048, 128, 0.088), n_q=4096) == hg.ERR_UNSUPPORTED
    assert tiers(n_q=0) == hg.OK

    def weights2(shape=sh, q=FAKE, n_q=4, lw=FAKE, lp=FAKE, ag=FAKE, ac=FAKE):
        return L.hgca_append_weights_tiers(byref(shape), q, n_q, byref(view), byref(view), 1, lw, lp, ag, ac, None)
    assert weights2(q=None) == hg.ERR_INVALID_ARG
    assert weights2(n_q=0) == hg.ERR_INVALID_ARG
    assert weights2(lw=None) == hg.ERR_INVALID_ARG
    assert weights2(ac=None) == hg.ERR_INVALID_ARG
    assert weights2(shape=hg.Shape(hg.F32, 2, 8, 2, 128, 0.088)) == hg.ERR_UNSUPPORTED

    def weights(q=FAKE, n_q=4, lse=FAKE, a=FAKE):
        return L.hgca_append_weights(byref(sh), q, n_q, byref(view), 0, lse, a, None)
    assert weights(q=None) == hg.ERR_INVALID_ARG
    assert weights(n_q=0) == hg.ERR_INVALID_ARG
    assert weights(lse=None) == hg.ERR_INVALID_ARG
    assert weights(a=None) == hg.ERR_INVALID_ARG


def test_grouped_entry_points_reject_bad_arguments(hg):
    L = hg.lib()
    sh = hg.Shape(hg.BF16, 2, 8, 2, 128, 0.088)
    view = _view(hg)
    byref = ctypes.byref

    def sel(q=FAKE, k=8, k_max=8, idx=FAKE, cnt=FAKE, ws=FAKE, ws_bytes=1 << 40):
        return L.hgca_select_salient_grouped(byref(sh), q, byref(view), None, k, k_max, idx, cnt, ws, ws_bytes, None)
    assert sel(q=None) == hg.ERR_INVALID_ARG
    assert sel(k=9) == hg.ERR_INVALID_ARG
    assert sel(idx=None) == hg.ERR_INVALID_ARG
    assert sel(cnt=None) == hg.ERR_INVALID_ARG
    assert sel(ws_bytes=16) == hg.ERR_WORKSPACE

    def uni(idx=FAKE, cnt=FAKE, k_max=8, n_pos=64, out=FAKE, out_cnt=FAKE, k_out=32):
        return L.hgca_union_lists(byref(sh), idx, cnt, k_max, n_pos, out, out_cnt, k_out, None, None)
    assert uni(idx=None) == hg.ERR_INVALID_ARG
    assert uni(cnt=None) == hg.ERR_INVALID_ARG
    assert uni(out=None) == hg.ERR_INVALID_ARG
    assert uni(n_pos=-1) == hg.ERR_INVALID_ARG
    # one bit per position must fit the 64 KiB of LDS a launch gets without asking for more: refused on the host
    assert uni(n_pos=523776 + 1) == hg.ERR_UNSUPPORTED
    assert uni(n_pos=1 << 19) == hg.ERR_UNSUPPORTED
    assert uni(k_max=-1) == hg.ERR_INVALID_ARG

    def att(q=FAKE, idx=FAKE, cnt=FAKE, k_max=8, o=FAKE, lse=FAKE, ws=FAKE, ws_bytes=1 << 40):
        return L.hgca_sparse_attn_grouped(byref(sh), q, byref(view), idx, cnt, k_max, o, lse, ws, ws_bytes, None)
    assert att(q=ODD) == hg.ERR_INVALID_ARG
    assert att(idx=None) == hg.ERR_INVALID_ARG
    assert att(cnt=None) == hg.ERR_INVALID_ARG
    assert att(o=None) == hg.ERR_INVALID_ARG                   # one output without the other
    assert att(ws=None) == hg.ERR_WORKSPACE


def test_hybrid_decode_step_rejects_bad_arguments(hg):
    sh = hg.Shape(hg.BF16, 2, 8, 2, 128, 0.088)
    win, pool = _view(hg, cap=64), _view(hg, cap=256)
    WS2 = ctypes.c_void_p(0x40000)

    def step(shape=sh, q=FAKE, w=win, p=pool, k_uni=8, k_max=8, idx=FAKE, cnt=FAKE, o=FAKE, o_dtype=0, wd=FAKE,
             wd_bytes=1 << 40, wsp=WS2, wsp_bytes=1 << 40):
        return hg.lib().hgca_hybrid_decode_step(ctypes.byref(shape), q, ctypes.byref(w), ctypes.byref(p), None, k_uni,
                                                k_max, idx, cnt, o, o_dtype, None, wd, wd_bytes, wsp, wsp_bytes, None)

    assert step(shape=hg.Shape(hg.BF16, 2, 8, 3, 128, 0.088)) == hg.ERR_INVALID_ARG
    assert step(q=None) == hg.ERR_INVALID_ARG
    assert step(o=None) == hg.ERR_INVALID_ARG
    assert step(o_dtype=5) == hg.ERR_UNSUPPORTED
    assert step(idx=None) == hg.ERR_INVALID_ARG
    assert step(cnt=None) == hg.ERR_INVALID_ARG
    assert step(k_uni=9) == hg.ERR_INVALID_ARG                 # k > k_max
    assert step(k_max=-1) == hg.ERR_INVALID_ARG
    assert step(w=_view(hg, cap=64, k=None)) == hg.ERR_INVALID_ARG
    assert step(p=_view(hg, cap=256, v=None)) == hg.ERR_INVALID_ARG
    assert step(wd=None) == hg.ERR_WORKSPACE
    assert step(wsp=None) == hg.ERR_WORKSPACE
    assert step(wsp=FAKE) == hg.ERR_WORKSPACE                  # one buffer for both parts
    assert step(wd_bytes=hg.workspace_bytes(sh, 64, 0, 0) - 1) == hg.ERR_WORKSPACE
    assert step(wsp_bytes=hg.workspace_bytes(sh, 0, 256, 8) - 1) == hg.ERR_WORKSPACE
    assert step(shape=hg.Shape(hg.BF16, 0, 8, 2, 128, 0.088), q=None, o=None) == hg.OK   # empty batch: nothing to do


def test_hybrid_decode_step_selected_rejects_bad_arguments(hg):
    sh = hg.Shape(hg.BF16, 2, 8, 2, 128, 0.088)
    win, pool = _view(hg, cap=256), _view(hg, cap=1024)
    big = 1 << 40

    def call(shape=sh, q=FAKE, w=win, p=pool, idx=FAKE, cnt=FAKE, k_max=64, sel=None, o=FAKE, o_dtype=hg.F32, lse=FAKE,
             wd=FAKE, wd_bytes=big, ws=ctypes.c_void_p(0x20000), ws_bytes=big):
        return hg.lib().hgca_hybrid_decode_step_selected(ctypes.byref(shape), q, ctypes.byref(w), ctypes.byref(p), idx,
                                                         cnt, k_max, sel, o, o_dtype, lse, wd, wd_bytes, ws, ws_bytes,
                                                         None)
    assert call(shape=hg.Shape(hg.BF16, 2, 8, 3, 128, 0.088)) == hg.ERR_INVALID_ARG
    assert call(shape=hg.Shape(hg.BF16, 2, 8, 2, 96, 0.088)) == hg.ERR_UNSUPPORTED
    assert call(o_dtype=5) == hg.ERR_UNSUPPORTED
    assert call(q=None) == hg.ERR_INVALID_ARG
    assert call(q=ODD) == hg.ERR_INVALID_ARG
    assert call(o=None) == hg.ERR_INVALID_ARG
    assert call(cnt=None) == hg.ERR_INVALID_ARG
    assert call(idx=None) == hg.ERR_INVALID_ARG
    assert call(k_max=-1) == hg.ERR_INVALID_ARG
    assert call(w=_view(hg, cap=256, v=None)) == hg.ERR_INVALID_ARG
    assert call(p=_view(hg, cap=1024, v=None)) == hg.ERR_INVALID_ARG        # the sparse part reads V
    assert call(wd=None) == hg.ERR_WORKSPACE
    assert call(ws=None) == hg.ERR_WORKSPACE
    assert call(wd_bytes=hg.workspace_bytes(sh, 256, 0, 0) - 1) == hg.ERR_WORKSPACE
    assert call(ws_bytes=hg.workspace_bytes(sh, 0, 0, 64) - 1) == hg.ERR_WORKSPACE
    assert call(ws=FAKE) == hg.ERR_WORKSPACE                               # the two workspaces must differ
    assert call(shape=hg.Shape(hg.BF16, 0, 8, 2, 128, 0.088), q=None, o=None) == hg.OK     # batch 0: a no-op


def test_ctx_compact_rejects_bad_arguments(hg):
    sh = hg.Shape(hg.BF16, 2, 8, 2, 128, 0.088)
    pool = _view(hg, cap=256)
    K2, V2, C2 = ctypes.c_void_p(0x20000), ctypes.c_void_p(0x30000), ctypes.c_void_p(0x40000)

    def compact(shape=sh, p=pool, idx=FAKE, cnt=FAKE, k_max=8, first=None, k=K2, v=V2, cap=16, cnt_out=C2):
        return hg.lib().hgca_ctx_compact(ctypes.byref(shape), ctypes.byref(p), idx, cnt, k_max, first, k, v, cap,
                                         cnt_out, None)

    assert compact(shape=hg.Shape(hg.BF16, 2, 8, 3, 128, 0.088)) == hg.ERR_INVALID_ARG
    assert compact(idx=None) == hg.ERR_INVALID_ARG
    assert compact(cnt=None) == hg.ERR_INVALID_ARG
    assert compact(k_max=-1) == hg.ERR_INVALID_ARG
    assert compact(cap=-1) == hg.ERR_INVALID_ARG
    assert compact(k=None) == hg.ERR_INVALID_ARG
    assert compact(v=K2) == hg.ERR_INVALID_ARG                  # K and V storage must differ
    assert compact(k=ODD) == hg.ERR_INVALID_ARG
    assert compact(first=C2) == hg.ERR_INVALID_ARG              # cnt_out is written while other workgroups read first_row
    assert compact(cnt=C2) == hg.ERR_INVALID_ARG
    assert compact(p=_view(hg, cap=256, k=None)) == hg.ERR_INVALID_ARG
    assert compact(shape=hg.Shape(hg.BF16, 0, 8, 2, 128, 0.088), idx=None, cnt=None) == hg.OK


def test_header_is_valid_c99():
    """include/hgca.h is a C header: a C99 compiler accepts it on its own."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = '#include "hgca.h"\nint main(void) { return sizeof(hgca_shape) + sizeof(hgca_kv_view) + sizeof(hgca_cache_state) > 0 ? 0 : 1; }\n'
    run = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", "-x", "c",
                          "-I" + os.path.join(root, "include"), "-"], input=src, capture_output=True, text=True)
    assert run.returncode == 0, run.stderr


def test_managed_decode_step_rejects_bad_arguments(hg):
    sh = hg.Shape(hg.BF16, 2, 8, 2, 128, 0.088)
    WS2, A = ctypes.c_void_p(0x40000), ctypes.c_void_p(0x50000)

    def state(**kw):
        f = dict(k_blocks=0x10000, v_blocks=0x20000, block_table=0x30000, first_win_block=0x30100, win_lens=0x30200,
                 pool_lens=0x30300, a_maw=0x30400, ctx_idx=0x30500, ctx_cnt=0x30600, a_evicted=None, plan=0x30700,
                 status=0x30800, block_size=16, max_blocks=8, win_blocks=2, k_max=32, pool_cap=128)
        f.update(kw)
        return hg.CacheState(**f)

    def step(st=None, shape=sh, q=FAKE, k=FAKE, v=FAKE, alpha=0.3, beta=1.0, a=A, o=FAKE, o_dtype=0, wd=FAKE,
             wd_bytes=1 << 40, wsp=WS2, wsp_bytes=1 << 40):
        st = st or state()
        return hg.lib().hgca_managed_decode_step(ctypes.byref(shape), ctypes.byref(st), q, k, v, alpha, beta, a, o,
                                                 o_dtype, None, wd, wd_bytes, wsp, wsp_bytes, None)

    assert step(st=state(block_size=24)) == hg.ERR_UNSUPPORTED
    assert step(st=state(win_lens=None)) == hg.ERR_INVALID_ARG
    assert step(q=None) == hg.ERR_INVALID_ARG
    assert step(k=None) == hg.ERR_INVALID_ARG
    assert step(v=ODD) == hg.ERR_INVALID_ARG
    assert step(a=None) == hg.ERR_INVALID_ARG
    assert step(o=None) == hg.ERR_INVALID_ARG
    assert step(o_dtype=9) == hg.ERR_UNSUPPORTED
    assert step(alpha=1.5) == hg.ERR_INVALID_ARG
    assert step(beta=-1.0) == hg.ERR_INVALID_ARG
    assert step(wd=None) == hg.ERR_WORKSPACE
    assert step(wsp=FAKE) == hg.ERR_WORKSPACE                  # one buffer for both parts
    assert step(wd_bytes=hg.workspace_bytes(sh, 32, 0, 0) - 1) == hg.ERR_WORKSPACE
    assert step(wsp_bytes=hg.workspace_bytes(sh, 0, 0, 32) - 1) == hg.ERR_WORKSPACE
    assert step(shape=hg.Shape(hg.BF16, 0, 8, 2, 128, 0.088), q=None, o=None, a=None) == hg.OK
