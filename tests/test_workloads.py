"""Host-only checks of the seeded input generator (shapes, determinism, byte model)."""
import numpy as np

from paper_2507_03153_amd import workloads as wl


def test_generation_is_deterministic_and_layers_differ():
    cfg = wl.scaled(wl.CONFIGS["C2"], B=2, Hq=8, Hkv=2, W=64, P=256, k=32)
    a, b, c = wl.make_layer(cfg), wl.make_layer(cfg), wl.make_layer(cfg, layer=1)
    for x, y in ((a.q, b.q), (a.window.k, b.window.k), (a.pool.v, b.pool.v)):
        np.testing.assert_array_equal(x, y)
    assert a.q.dtype == np.uint16 and a.window.k.shape == (2, 2, 64, 128)
    assert not np.array_equal(a.pool.k, c.pool.k)


def test_planted_keys_align_with_their_query_head():
    cfg = wl.scaled(wl.CONFIGS["C2"], B=1, Hq=8, Hkv=2, W=16, P=2000, k=32)
    L = wl.make_layer(cfg)
    q, kp = wl.to_f32(L.q), wl.to_f32(L.pool.k)
    for kvh in range(2):
        pos = L.planted[0][kvh]
        assert pos.size == 20 and np.all(np.diff(pos) > 0)
        for i, p in enumerate(pos):
            h = cfg.G * kvh + i % cfg.G
            s = cfg.scale * float(q[0, h] @ kp[0, kvh, p])
            assert s > 0.0, (kvh, i, s)                     # ~ N(0,1) + 2.5
    runs = wl.make_layer(wl.scaled(wl.CONFIGS["C4"], B=1, Hq=8, Hkv=1, W=16, P=6400, k=64))
    pos = runs.planted[0][0]
    assert pos.size == 64 and np.all(pos.reshape(-1, 32)[:, 0] % 32 == 0)
    assert np.all(np.diff(pos.reshape(-1, 32), axis=1) == 1)


def test_ragged_paged_layout_is_consistent():
    cfg = wl.scaled(wl.CONFIGS["C5"], B=5, Hq=4, Hkv=2, d=16, W=32, P=96, ragged=(16, 128))
    L = wl.make_layer(cfg)
    w, p, k = wl.seq_lengths(cfg)
    np.testing.assert_array_equal(L.window.seq_lens, w)
    np.testing.assert_array_equal(L.pool.seq_lens, p)
    assert np.all(w == np.minimum(32, w + p)) and np.all(k == np.floor(0.1 * p))
    used = np.concatenate([L.pool.block_table[b, :(p[b] + 15) // 16] for b in range(5)])
    assert used.size == np.unique(used).size == L.pool.k.shape[0] or p.sum() == 0
    assert L.k_max == int(k.max())


def test_algorithmic_bytes_of_the_full_configs():
    # window K+V per KV head + pool K per KV head + index lists + k gathered K+V rows per query head
    expect = {"C1": (524288, 2098176, 132096), "C2": (134217728, 471859200, 270532608),
              "C3": (1342177280, 4702863360, 676331520), "C4": (134217728, 1010827264, 541065216)}
    for name, (s1, s2, s3) in expect.items():
        cfg = wl.CONFIGS[name]
        b = wl.step_bytes(cfg, *wl.seq_lengths(cfg))
        assert (b["dense"], b["select"], b["sparse"]) == (s1, s2, s3)
        assert b["full"] == s1 + s2 + s3 and b["steady"] == s1 + s3
