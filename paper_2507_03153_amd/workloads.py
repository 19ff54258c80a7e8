"""Seeded synthetic inputs for the hybrid decode-attention step.

This module only *draws inputs*: it holds none of the method's arithmetic and is
the one piece shared by the HIP path's tests/benchmark and the CPU oracle's
tests.  Arrays are numpy; bf16 tensors are uint16 bit patterns (rounded once,
round-to-nearest-even, from the fp32 draw) so that both sides consume the very
same bits.

The shapes stand in for the workloads of the paper's evaluation (decoder heads of
dimension 128, a bounded recent window in fast memory, a long offloaded context
in which a few entries per head carry most of the attention mass -- Sec. 2.3
observations O-1..O-3 and Sec. 4).  "Planted" keys model those salient entries:
k_j = n_j + c * q_hat, n_j ~ N(0, I), q_hat the unit vector of the query of one
head of the group, so their scaled score is about N(0,1) + c.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Optional

import numpy as np

BASE_SEED = 250703153


@dataclass(frozen=True)
class Config:
    name: str
    index: int              # enters the seed
    dtype: str              # "f32" | "bf16"
    B: int
    Hq: int
    Hkv: int
    d: int
    W: int                  # recent-window capacity (tokens per sequence)
    P: int                  # older-pool capacity
    k: int                  # per-head selection budget (uniform configs)
    plant_frac: float = 0.01   # fraction of pool keys planted per KV head
    plant_count: int = 0       # if > 0: exact number per KV head instead
    plant_scale: float = 2.5
    plant_run: int = 1         # planted keys come in contiguous runs of this length
    ragged: Optional[tuple] = None   # (min_len, max_len) => per-sequence lengths
    k_frac: float = 0.0        # ragged: k_b = floor(k_frac * P_b)
    block_size: int = 0        # > 0 => both tiers paged with this block size

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.d))

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2


CONFIGS = {
    "C1": Config("C1", 1, "f32", B=1, Hq=4, Hkv=4, d=64, W=256, P=2048, k=64,
                 plant_count=16, plant_scale=3.0),
    "C2": Config("C2", 2, "bf16", B=8, Hq=32, Hkv=8, d=128, W=4096, P=28672, k=2048),
    "C3": Config("C3", 3, "bf16", B=32, Hq=40, Hkv=40, d=128, W=2048, P=14336, k=1024),
    "C4": Config("C4", 4, "bf16", B=4, Hq=64, Hkv=8, d=128, W=8192, P=122880, k=4096,
                 plant_run=32),
    "C5": Config("C5", 5, "bf16", B=64, Hq=32, Hkv=8, d=128, W=2048, P=16384 - 2048, k=0,
                 ragged=(2048, 16384), k_frac=0.10, block_size=16),
}


def scaled(cfg: Config, **kw) -> Config:
    """A smaller/modified variant of a config (same recipe, same seed index)."""
    return replace(cfg, **kw)


@dataclass
class TierData:
    k: np.ndarray                 # contiguous [B,Hkv,cap,d]; paged [n_blocks,Hkv,bs,d]
    v: np.ndarray
    cap: int
    seq_lens: Optional[np.ndarray] = None      # int32 [B]
    block_table: Optional[np.ndarray] = None   # int32 [B,max_blocks]
    block_size: int = 0

    def lens(self, batch: int) -> np.ndarray:
        return np.full(batch, self.cap, np.int32) if self.seq_lens is None else self.seq_lens


@dataclass
class Layer:
    cfg: Config
    q: np.ndarray                 # [B,Hq,d]
    window: TierData
    pool: TierData
    k: object                     # int, or int32 [B] for ragged configs
    k_max: int
    scale: float
    planted: list                 # planted[b][kvh] = sorted int32 positions in the pool

    def kv_bytes(self) -> int:
        return sum(a.nbytes for a in (self.window.k, self.window.v, self.pool.k, self.pool.v))


# ---- bf16 bit patterns --------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_f32(a: np.ndarray) -> np.ndarray:
    return a if a.dtype == np.float32 else bf16_bits_to_f32(a)


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.float32) if dtype == "f32" else f32_to_bf16_bits(x)


# ---- generation ------------------------------------------------------------------

def _rng(cfg: Config, layer: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(
        np.random.SeedSequence([BASE_SEED, cfg.index, layer, stream])))


def seq_lengths(cfg: Config, layer: int = 0):
    """(window_len[B], pool_len[B], k[B] or int).  Ragged lengths come from their own stream."""
    if cfg.ragged is None:
        return (np.full(cfg.B, cfg.W, np.int32), np.full(cfg.B, cfg.P, np.int32), int(cfg.k))
    lo, hi = cfg.ragged
    total = _rng(cfg, layer, 1 << 20).integers(lo, hi + 1, size=cfg.B).astype(np.int64)
    w = np.minimum(cfg.W, total)
    p = total - w
    k = np.floor(cfg.k_frac * p).astype(np.int64)
    return w.astype(np.int32), p.astype(np.int32), k.astype(np.int32)


def _plant_positions(rng, cfg: Config, p_len: int) -> np.ndarray:
    n = cfg.plant_count if cfg.plant_count > 0 else int(round(cfg.plant_frac * p_len))
    n = min(n, p_len)
    if n <= 0:
        return np.zeros(0, np.int32)
    run = max(1, cfg.plant_run)
    if run == 1:
        pos = rng.choice(p_len, size=n, replace=False)
    else:
        n_runs = max(1, n // run)
        slots = p_len // run
        n_runs = min(n_runs, slots)
        if n_runs == 0:
            return np.zeros(0, np.int32)
        starts = rng.choice(slots, size=n_runs, replace=False) * run
        pos = (starts[:, None] + np.arange(run)[None, :]).reshape(-1)
    return np.sort(pos).astype(np.int32)


def _one_sequence(cfg: Config, layer: int, b: int, w_len: int, p_len: int):
    """Draw order per sequence: q, K_window, V_window, K_pool, V_pool, plant positions per KV head."""
    rng = _rng(cfg, layer, b)
    f = np.float32
    q = rng.standard_normal((cfg.Hq, cfg.d), dtype=f)
    kw = rng.standard_normal((cfg.Hkv, w_len, cfg.d), dtype=f)
    vw = rng.standard_normal((cfg.Hkv, w_len, cfg.d), dtype=f)
    kp = rng.standard_normal((cfg.Hkv, p_len, cfg.d), dtype=f)
    vp = rng.standard_normal((cfg.Hkv, p_len, cfg.d), dtype=f)
    q_hat = q / np.linalg.norm(q, axis=-1, keepdims=True)
    planted = []
    for kvh in range(cfg.Hkv):
        pos = _plant_positions(rng, cfg, p_len)
        if pos.size:
            heads = cfg.G * kvh + (np.arange(pos.size) % cfg.G)
            kp[kvh, pos, :] += f(cfg.plant_scale) * q_hat[heads, :]
        planted.append(pos)
    return (_store(q, cfg.dtype), _store(kw, cfg.dtype), _store(vw, cfg.dtype),
            _store(kp, cfg.dtype), _store(vp, cfg.dtype), planted)


def _n_workers() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def make_layer(cfg: Config, layer: int = 0) -> Layer:
    """All inputs of one layer-step for `cfg`; `layer` selects an independent draw."""
    w_lens, p_lens, k = seq_lengths(cfg, layer)
    np_dt = np.float32 if cfg.dtype == "f32" else np.uint16
    with ThreadPoolExecutor(_n_workers()) as ex:
        seqs = list(ex.map(lambda b: _one_sequence(cfg, layer, b, int(w_lens[b]), int(p_lens[b])),
                           range(cfg.B)))
    q = np.stack([s[0] for s in seqs]) if cfg.B else np.zeros((0, cfg.Hq, cfg.d), np_dt)
    planted = [s[5] for s in seqs]
    ragged = cfg.ragged is not None

    if cfg.block_size > 0:
        window = _paged_tier(cfg, layer, 0, [s[1] for s in seqs], [s[2] for s in seqs], w_lens, cfg.W, np_dt)
        pool = _paged_tier(cfg, layer, 1, [s[3] for s in seqs], [s[4] for s in seqs], p_lens, cfg.P, np_dt)
    else:
        window = _contig_tier(cfg, [s[1] for s in seqs], [s[2] for s in seqs], w_lens, cfg.W, np_dt, ragged)
        pool = _contig_tier(cfg, [s[3] for s in seqs], [s[4] for s in seqs], p_lens, cfg.P, np_dt, ragged)

    k_max = int(np.max(k)) if not np.isscalar(k) else int(min(k, cfg.P))
    if not np.isscalar(k) and cfg.B == 0:
        k_max = 0
    return Layer(cfg, q, window, pool, k, max(k_max, 0), cfg.scale, planted)


def _contig_tier(cfg, ks, vs, lens, cap, np_dt, ragged) -> TierData:
    K = np.zeros((cfg.B, cfg.Hkv, cap, cfg.d), np_dt)
    V = np.zeros((cfg.B, cfg.Hkv, cap, cfg.d), np_dt)
    for b in range(cfg.B):
        K[b, :, :lens[b]] = ks[b]
        V[b, :, :lens[b]] = vs[b]
    return TierData(K, V, cap, seq_lens=lens.copy() if ragged else None)


def _paged_tier(cfg, layer, which, ks, vs, lens, cap, np_dt) -> TierData:
    """Scatter each sequence's tokens into fixed-size blocks placed by a seeded permutation."""
    bs = cfg.block_size
    n_blk = [(int(n) + bs - 1) // bs for n in lens]
    total = int(sum(n_blk))
    max_blocks = max(1, (cap + bs - 1) // bs)
    perm = _rng(cfg, layer, (1 << 21) + which).permutation(max(total, 1)).astype(np.int32)
    K = np.zeros((max(total, 1), cfg.Hkv, bs, cfg.d), np_dt)
    V = np.zeros((max(total, 1), cfg.Hkv, bs, cfg.d), np_dt)
    table = np.zeros((cfg.B, max_blocks), np.int32)
    at = 0
    for b in range(cfg.B):
        ids = perm[at:at + n_blk[b]]
        at += n_blk[b]
        table[b, :n_blk[b]] = ids
        n = int(lens[b])
        if n == 0:
            continue
        pad = n_blk[b] * bs - n
        for src, dst in ((ks[b], K), (vs[b], V)):
            x = src if pad == 0 else np.concatenate(
                [src, np.zeros((cfg.Hkv, pad, cfg.d), np_dt)], axis=1)
            # [Hkv, n_blk*bs, d] -> [n_blk, Hkv, bs, d]
            dst[ids] = x.reshape(cfg.Hkv, n_blk[b], bs, cfg.d).transpose(1, 0, 2, 3)
    return TierData(K, V, cap, seq_lens=lens.copy(), block_table=table, block_size=bs)


# ---- algorithmic HBM bytes of one layer-step ---------------------------------------

def step_bytes(cfg: Config, w_lens, p_lens, k) -> dict:
    """Bytes the method must move: window K+V once per KV head, pool K once per KV head for
    scoring (+ index list written), k gathered K+V rows per query head (+ index list read)."""
    e, d = cfg.elem_bytes, cfg.d
    w_lens = np.asarray(w_lens, np.int64)
    p_lens = np.asarray(p_lens, np.int64)
    kb = np.minimum(np.full(cfg.B, k, np.int64) if np.isscalar(k) else np.asarray(k, np.int64), p_lens)
    s1 = int(2 * w_lens.sum() * cfg.Hkv * d * e)
    s2 = int(p_lens.sum() * cfg.Hkv * d * e + 4 * cfg.Hq * kb.sum())
    s3 = int(2 * cfg.Hq * kb.sum() * d * e + 4 * cfg.Hq * kb.sum())
    return {"dense": s1, "select": s2, "sparse": s3, "full": s1 + s2 + s3, "steady": s1 + s3}
