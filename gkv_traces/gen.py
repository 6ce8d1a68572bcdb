"""Counter-based synthetic decode traces.

Every (stream, layer, sequence, block of 64 steps) has its own Philox key, so
the values for one (layer, sequence) pair can be drawn without materialising
the rest of the batch, and the same values come out whatever chunking the
caller uses.  Values are rounded to the configuration's storage dtype here,
once, so every consumer widens the very same bits.

Recipes
-------
gauss_sink   Q, K, V ~ N(0,1); the key at position 0 is scaled x8 (an
             attention sink).
recurring    K ~ N(0,1) with 4 outlier channels per (layer, KV head) scaled
             x10; V ~ N(0,1); a fixed unit vector u per (layer, KV head);
             1% of positions get k += a*u; Q ~ N(0,1) and, during "recall
             bursts" (32 steps starting at t = 100 mod 320), q += a*u for
             every head of the group, a = sqrt(8*sqrt(d)).  With s=128, w=16
             the observation window meets a burst only at every 5th
             compression, so boosted keys are needed again long after a
             local score has stopped seeing them.
heavy_tail   K entries Student-t(nu=3); Q, V ~ N(0,1); per-sequence keys.
"""
from __future__ import annotations

import numpy as np

from .configs import WorkloadConfig

BLOCK = 64                      # steps per RNG block
_KIND_Q, _KIND_K, _KIND_V, _KIND_STATIC = 0, 1, 2, 3
BURST_PERIOD, BURST_START, BURST_LEN = 320, 100, 32
BOOST_RATE = 0.01
N_OUTLIER, OUTLIER_SCALE = 4, 10.0
SINK_SCALE = 8.0


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float32 (exact)."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16, returned as float32."""
    return from_bf16_bits(to_bf16_bits(x))


def _rng(seed: int, kind: int, layer: int, seq: int, block: int) -> np.random.Generator:
    assert 0 <= layer < (1 << 10) and 0 <= seq < (1 << 20) and 0 <= block < (1 << 31)
    stream = (kind << 61) | (layer << 51) | (seq << 31) | block
    return np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF, stream]))


class Trace:
    """Synthetic decode trace for one workload configuration."""

    def __init__(self, cfg: WorkloadConfig):
        self.cfg = cfg
        d = cfg.head_dim
        self.boost = float(np.sqrt(8.0 * np.sqrt(d)))
        self._static = {}

    # ---- per-layer constants of the "recurring" recipe --------------------
    def static(self, layer: int):
        """(u [h_kv, d] unit vectors, outlier channel ids [h_kv, 4]) of a layer."""
        if layer not in self._static:
            cfg = self.cfg
            g = _rng(cfg.seed, _KIND_STATIC, layer, 0, 0)
            u = g.standard_normal((cfg.n_kv_heads, cfg.head_dim))
            u /= np.linalg.norm(u, axis=-1, keepdims=True)
            ch = np.stack([g.permutation(cfg.head_dim)[:N_OUTLIER]
                           for _ in range(cfg.n_kv_heads)])
            self._static[layer] = (u.astype(np.float32), ch)
        return self._static[layer]

    # ---- one block of 64 steps for one (layer, sequence) ------------------
    def _block(self, layer: int, seq: int, block: int, need_q: bool = True):
        """need_q=False skips drawing the queries (q comes back as None); every stream has its own
        generator, so k and v are the same values either way."""
        cfg = self.cfg
        hq, hkv, d, grp = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.group
        t = np.arange(block * BLOCK, (block + 1) * BLOCK)
        gq = _rng(cfg.seed, _KIND_Q, layer, seq, block)
        gk = _rng(cfg.seed, _KIND_K, layer, seq, block)
        gv = _rng(cfg.seed, _KIND_V, layer, seq, block)
        q = gq.standard_normal((BLOCK, hq, d), dtype=np.float32) if need_q else None
        v = gv.standard_normal((BLOCK, hkv, d), dtype=np.float32)
        if cfg.recipe == "heavy_tail":
            k = gk.standard_t(3.0, size=(BLOCK, hkv, d)).astype(np.float32)
        else:
            k = gk.standard_normal((BLOCK, hkv, d), dtype=np.float32)
        if cfg.recipe == "gauss_sink":
            if block == 0:
                k[0] *= SINK_SCALE
        elif cfg.recipe == "recurring":
            u, ch = self.static(layer)
            for j in range(hkv):
                k[:, j, ch[j]] *= OUTLIER_SCALE
            boosted = gk.random(BLOCK) < BOOST_RATE
            k[boosted] += self.boost * u[None, :, :]
            burst = ((t - BURST_START) % BURST_PERIOD) < BURST_LEN
            if need_q:
                uq = np.repeat(u, grp, axis=0)          # [h_q, d]: head i -> group i // grp
                q[burst] += self.boost * uq[None, :, :]
        elif cfg.recipe != "heavy_tail":
            raise ValueError(cfg.recipe)
        if cfg.dtype == "bf16":
            q, k, v = (bf16_round(q) if need_q else None), bf16_round(k), bf16_round(v)
        return q, k, v

    def unit_steps(self, layer: int, seq: int, t0: int, n: int, need_q: bool = True):
        """q [n,h_q,d], k [n,h_kv,d], v [n,h_kv,d] (float32, dtype-rounded) for steps t0..t0+n-1
        (q is None with need_q=False)."""
        out_q, out_k, out_v = [], [], []
        blk0, blk1 = t0 // BLOCK, (t0 + n - 1) // BLOCK
        for blk in range(blk0, blk1 + 1):
            q, k, v = self._block(layer, seq, blk, need_q)
            lo = max(t0, blk * BLOCK) - blk * BLOCK
            hi = min(t0 + n, (blk + 1) * BLOCK) - blk * BLOCK
            if need_q:
                out_q.append(q[lo:hi])
            out_k.append(k[lo:hi]); out_v.append(v[lo:hi])
        return (np.concatenate(out_q) if need_q else None, np.concatenate(out_k), np.concatenate(out_v))

    def batch_steps(self, t0: int, n: int, layers=None, seqs=None, workers: int = 1, need_q: bool = True):
        """q [n,L,B,h_q,d], k/v [n,L,B,h_kv,d] (float32, dtype-rounded) for the whole batch.
        `workers` > 1 draws the (layer, sequence) pairs on a thread pool (same values);
        need_q=False returns q = None (a prompt needs keys and values only)."""
        cfg = self.cfg
        layers = range(cfg.n_layers) if layers is None else layers
        seqs = range(cfg.batch) if seqs is None else seqs
        L, B = len(layers), len(seqs)
        q = np.empty((n, L, B, cfg.n_q_heads, cfg.head_dim), np.float32) if need_q else None
        k = np.empty((n, L, B, cfg.n_kv_heads, cfg.head_dim), np.float32)
        v = np.empty_like(k)
        for layer in layers:
            self.static(layer)

        def fill(args):
            li, layer, bi, seq = args
            qq, k[:, li, bi], v[:, li, bi] = self.unit_steps(layer, seq, t0, n, need_q)
            if need_q:
                q[:, li, bi] = qq

        jobs = [(li, layer, bi, seq) for li, layer in enumerate(layers) for bi, seq in enumerate(seqs)]
        if workers > 1:
            from concurrent.futures import ThreadPoolExecutor
            with ThreadPoolExecutor(workers) as ex:
                list(ex.map(fill, jobs))
        else:
            for j in jobs:
                fill(j)
        return q, k, v
