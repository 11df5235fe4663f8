"""Seeded synthetic inputs for the slow/fast decode-attention path.

This module only *generates inputs*: bf16 bit patterns for q / K / V, context
lengths and the slow/fast schedule of each workload.  It holds none of the
method's arithmetic (no logits, no softmax, no selection), so that both the CPU
oracle's tests and the HIP path's tests can draw identical bits from it without
sharing any computation.

bf16 values travel as ``numpy.uint16`` bit patterns (the upper half of the
IEEE-754 binary32 encoding, rounded to nearest-even).

Workloads stand in for the KV caches of the paper's Qwen3 serving runs
(Sec. 5 "Efficiency Analysis") whose weights and prompts are not available:
K/V ~ N(0,1) with planted high-norm "support" key rows, which give the
attention map the concentrated, slowly moving support the paper's Fig. 1
describes.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

HEAD_DIM = 128
N_SINK = 4

# tensor ids for the counter-based generator (seed, tensor id) -> stream
_TID_K, _TID_V, _TID_Q, _TID_SUPPORT, _TID_LEN, _TID_SCHED, _TID_DRIFT = 1, 2, 3, 4, 5, 6, 7


def rng_for(seed: int, tensor_id: int, sub: int = 0) -> np.random.Generator:
    """Philox stream addressed by (seed, tensor id, sub-stream)."""
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(tensor_id * 1_000_003 + sub)]))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(rng: np.random.Generator, shape, row_scale: Optional[np.ndarray] = None) -> np.ndarray:
    """N(0,1) samples, optionally scaled per row (second-to-last axis) before rounding.  Large 2-D requests are
    drawn a block of rows at a time (the generator's stream, hence every bit, is the same as in one draw; the
    temporaries then stay cache-sized, which is what lets several threads fill slices side by side)."""
    if len(shape) == 2 and shape[0] * shape[1] > (1 << 20):
        out = np.empty(shape, dtype=np.uint16)
        step = max(1, (1 << 18) // shape[1])
        for r0 in range(0, shape[0], step):
            r1 = min(shape[0], r0 + step)
            out[r0:r1] = normal_bf16(rng, (r1 - r0, shape[1]), None if row_scale is None else row_scale[r0:r1])
        return out
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if row_scale is not None:
        x *= row_scale[..., None].astype(np.float32)
    return f32_to_bf16_bits(x)


@dataclass
class Workload:
    """One synthetic decode workload (shapes + tensors + schedule)."""

    name: str
    B: int
    Hq: int
    Hkv: int
    L0: np.ndarray            # int32 [B] context length at step 0 (rows already in the cache)
    steps: int
    budget: int
    recent: int
    n_sink: int = N_SINK
    d: int = HEAD_DIM
    seed: int = 0
    L_alloc: int = 0          # rows allocated per (sequence, KV head)
    K: Optional[np.ndarray] = None   # uint16 [B, Hkv, L_alloc, d]
    V: Optional[np.ndarray] = None
    slow: Optional[np.ndarray] = None  # bool [steps, B]: is step t a slow step for sequence b
    support: Optional[np.ndarray] = None  # int64 [B, Hkv, n_support] planted row positions (may be empty)
    meta: Dict = field(default_factory=dict)

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    def q(self, step: int) -> np.ndarray:
        """Fresh query for decode step ``step``: uint16 [B, Hq, d]."""
        return normal_bf16(rng_for(self.seed, _TID_Q, step), (self.B, self.Hq, self.d))

    def ctx_len(self, step: int) -> np.ndarray:
        return (self.L0 + step).astype(np.int32)

    def recent_start(self, step: int) -> np.ndarray:
        L = self.ctx_len(step)
        return np.maximum(self.n_sink, L - self.recent).astype(np.int32)

    def kv_bytes_slow(self, step: int) -> int:
        return int(self.ctx_len(step).astype(np.int64).sum()) * self.Hkv * self.d * 2 * 2

    def kv_bytes_fast(self, step: int, n_sel: Optional[np.ndarray] = None) -> int:
        L = self.ctx_len(step).astype(np.int64)
        rs = self.recent_start(step).astype(np.int64)
        nj = np.maximum(0, L - self.recent - self.n_sink)
        ns = np.minimum(self.budget, nj) if n_sel is None else n_sel
        rows = np.minimum(self.n_sink, L) + ns + (L - rs)
        return int(rows.sum()) * self.Hkv * self.d * 2 * 2


def _alloc_kv(w: Workload, row_scale: Optional[np.ndarray]) -> None:
    """Every (b, h) slice comes from its own Philox stream, so the slices can be filled by a few threads at once
    (numpy's generators release the interpreter lock) and the bits do not depend on how many."""
    from concurrent.futures import ThreadPoolExecutor

    shape = (w.B, w.Hkv, w.L_alloc, w.d)
    w.K = np.empty(shape, dtype=np.uint16)
    w.V = np.empty(shape, dtype=np.uint16)

    def fill(sub: int) -> None:
        b, h = divmod(sub, w.Hkv)
        rs = None if row_scale is None else row_scale[b, h]
        w.K[b, h] = normal_bf16(rng_for(w.seed, _TID_K, sub), (w.L_alloc, w.d), rs)
        w.V[b, h] = normal_bf16(rng_for(w.seed, _TID_V, sub), (w.L_alloc, w.d))

    n = w.B * w.Hkv
    if n * w.L_alloc * w.d < (1 << 22):
        for sub in range(n):
            fill(sub)
    else:
        with ThreadPoolExecutor(max_workers=8) as ex:
            list(ex.map(fill, range(n)))


def _fixed_schedule(steps: int, B: int, every: int) -> np.ndarray:
    s = np.zeros((steps, B), dtype=bool)
    s[::every, :] = True
    return s


def _uniform_support(w: Workload, n_support: int, lo: int, hi: np.ndarray) -> np.ndarray:
    """n_support distinct positions per (b, h), uniform in [lo, hi[b])."""
    out = np.empty((w.B, w.Hkv, n_support), dtype=np.int64)
    for b in range(w.B):
        for h in range(w.Hkv):
            r = rng_for(w.seed, _TID_SUPPORT, b * w.Hkv + h)
            out[b, h] = np.sort(r.choice(np.arange(lo, int(hi[b])), size=n_support, replace=False))
    return out


def make_tiny(L0: int = 4096, steps: int = 16, seed: int = 0, B: int = 1, Hq: int = 8, Hkv: int = 2,
              budget: int = 256, recent: int = 64, slow_every: int = 8, n_support: int = 32) -> Workload:
    """Config 1: one small stream; 32 support rows (x4) per KV head and a x4 sink row at position 0."""
    w = Workload("tiny", B, Hq, Hkv, np.full(B, L0, np.int32), steps, budget, recent, seed=seed)
    w.L_alloc = L0 + steps
    hi = w.L0 - recent
    w.support = _uniform_support(w, n_support, w.n_sink, hi)
    scale = np.ones((B, Hkv, w.L_alloc), dtype=np.float32)
    for b in range(B):
        for h in range(Hkv):
            scale[b, h, w.support[b, h]] = 4.0
    scale[:, :, 0] = 4.0
    _alloc_kv(w, scale)
    w.slow = _fixed_schedule(steps, B, slow_every)
    return w


def make_llama8b(L0: int = 32768, steps: int = 64, seed: int = 0, B: int = 4, Hq: int = 32, Hkv: int = 8,
                 budget: int = 2048, recent: int = 128, slow_every: int = 16, support_frac: float = 0.01) -> Workload:
    """Config 2: Llama-3-8B-shaped layer; 1% support rows (x4).  ``drift`` re-draws 10% of them."""
    w = Workload("llama8b", B, Hq, Hkv, np.full(B, L0, np.int32), steps, budget, recent, seed=seed)
    w.L_alloc = L0 + steps
    n_support = max(1, int(round(support_frac * L0)))
    hi = w.L0 - recent
    w.support = _uniform_support(w, n_support, w.n_sink, hi)
    scale = np.ones((B, Hkv, w.L_alloc), dtype=np.float32)
    for b in range(B):
        for h in range(Hkv):
            scale[b, h, w.support[b, h]] = 4.0
    _alloc_kv(w, scale)
    w.slow = _fixed_schedule(steps, B, slow_every)
    return w


def drift_support(w: Workload, epoch: int, frac: float = 0.10):
    """Re-draw ``frac`` of each (b, h)'s support positions (old rows back to x1, new rows x4).

    Mutates ``w.K`` / ``w.support`` in place and returns a list of
    (b, h, positions int64[n], rows uint16[n, d]) patches for a device copy of K.
    The unscaled row values are regenerated from the same stream as at allocation.
    """
    patches = []
    for b in range(w.B):
        for h in range(w.Hkv):
            sub = b * w.Hkv + h
            base = rng_for(w.seed, _TID_K, sub).standard_normal(size=(w.L_alloc, w.d), dtype=np.float32)
            r = rng_for(w.seed, _TID_DRIFT, epoch * 65536 + sub)
            sup = w.support[b, h]
            n_move = max(1, int(round(frac * len(sup))))
            leave = r.choice(len(sup), size=n_move, replace=False)
            free = np.setdiff1d(np.arange(w.n_sink, int(w.L0[b]) - w.recent), sup)
            enter = r.choice(free, size=n_move, replace=False)
            old_pos = sup[leave]
            new_sup = sup.copy()
            new_sup[leave] = enter
            w.support[b, h] = np.sort(new_sup)
            pos = np.concatenate([old_pos, enter])
            rows = np.concatenate([base[old_pos], base[enter] * np.float32(4.0)])
            bits = f32_to_bf16_bits(rows)
            w.K[b, h, pos] = bits
            patches.append((b, h, pos, bits))
    return patches


def make_long(L0: int = 131072, steps: int = 128, seed: int = 0, B: int = 1, Hq: int = 32, Hkv: int = 8,
              budget: int = 4096, recent: int = 256, slow_every: int = 32, n_clusters: int = 64,
              cluster_rows: int = 32) -> Workload:
    """Config 3: one long stream; clustered support (Gaussian-bump row scales)."""
    w = Workload("long", B, Hq, Hkv, np.full(B, L0, np.int32), steps, budget, recent, seed=seed)
    w.L_alloc = L0 + steps
    sigma = cluster_rows / 6.0
    scale = np.ones((B, Hkv, w.L_alloc), dtype=np.float32)
    centres = np.empty((B, Hkv, n_clusters), dtype=np.int64)
    half = cluster_rows // 2
    for b in range(B):
        for h in range(Hkv):
            r = rng_for(seed, _TID_SUPPORT, b * Hkv + h)
            lo, hi = w.n_sink + half, int(w.L0[b]) - recent - half
            c = np.sort(r.integers(lo, max(lo + 1, hi), size=n_clusters))
            centres[b, h] = c
            for ci in c:
                i = np.arange(ci - half, ci + half)
                bump = 1.0 + 3.0 * np.exp(-((i - ci) ** 2) / (2.0 * sigma * sigma))
                scale[b, h, i] = np.maximum(scale[b, h, i], bump.astype(np.float32))
    w.support = centres
    _alloc_kv(w, scale)
    w.slow = _fixed_schedule(steps, B, slow_every)
    return w


def make_cot(L0: int = 8192, steps: int = 2048, seed: int = 0, B: int = 8, Hq: int = 40, Hkv: int = 8,
             budget: int = 1024, recent: int = 128, slow_every: int = 24) -> Workload:
    """Config 4: long-CoT growth window starting at context ``L0``; plain N(0,1) K/V."""
    w = Workload("cot", B, Hq, Hkv, np.full(B, L0, np.int32), steps, budget, recent, seed=seed)
    w.L_alloc = L0 + steps
    w.support = np.empty((B, Hkv, 0), dtype=np.int64)
    _alloc_kv(w, None)
    w.slow = _fixed_schedule(steps, B, slow_every)
    return w


def make_serving(steps: int = 256, seed: int = 0, B: int = 32, Hq: int = 64, Hkv: int = 8, budget: int = 2048,
                 recent: int = 128, len_lo: int = 16384, len_hi: int = 65536, mean_gap: float = 20.0,
                 support_frac: float = 0.005, alloc: bool = True) -> Workload:
    """Config 5: ragged high-batch mix; per-sequence slow steps at geometric gaps (first step slow).
    alloc=False leaves K / V unset (lengths, support positions and schedule only), for callers that
    fill the cache on the device."""
    r = rng_for(seed, _TID_LEN)
    L0 = r.integers(len_lo, len_hi + 1, size=B).astype(np.int32)
    w = Workload("serving", B, Hq, Hkv, L0, steps, budget, recent, seed=seed)
    w.L_alloc = int(L0.max()) + steps
    n_support = max(1, int(round(support_frac * float(L0.min()))))
    w.support = _uniform_support(w, n_support, w.n_sink, (L0 - recent))
    if alloc:
        scale = np.ones((B, Hkv, w.L_alloc), dtype=np.float32)
        for b in range(B):
            for h in range(Hkv):
                scale[b, h, w.support[b, h]] = 4.0
        _alloc_kv(w, scale)
    rs = rng_for(seed, _TID_SCHED)
    slow = np.zeros((steps, B), dtype=bool)
    for b in range(B):
        t = 0
        while t < steps:
            slow[t, b] = True
            t += int(rs.geometric(1.0 / mean_gap))
    w.slow = slow
    return w


def make_retention_sweep(retention: float, L: int = 16384, B: int = 16, Hq: int = 32, Hkv: int = 8,
                         seed: int = 0, recent: int = 128) -> Workload:
    """Shape of the paper's kernel-speedup table (KV length 16K, batch 16, bf16): budget set by retention."""
    rows = int(round(retention * L))
    budget = max(0, min(L - recent - N_SINK, rows - recent - N_SINK))
    w = Workload("retention", B, Hq, Hkv, np.full(B, L, np.int32), 1, budget, recent, seed=seed)
    w.L_alloc = L
    w.support = np.empty((B, Hkv, 0), dtype=np.int64)
    _alloc_kv(w, None)
    w.slow = np.ones((1, B), dtype=bool)
    return w


def roll_rows(x: np.ndarray, shift: int, L: int) -> np.ndarray:
    """A distinct 'virtual layer' from a base K or V: rows [0, L) rolled by ``shift`` (tail rows kept)."""
    y = x.copy()
    y[:, :, :L] = np.roll(x[:, :, :L], shift, axis=2)
    return y


def random_sel(seed: int, B: int, Hkv: int, budget: int, n_sel: np.ndarray, lo: int, hi: np.ndarray) -> np.ndarray:
    """Arbitrary valid index sets (ascending, unique, in [lo, hi[b])) padded with -1: int32 [B, Hkv, budget]."""
    out = np.full((B, Hkv, max(budget, 1)), -1, dtype=np.int32)
    for b in range(B):
        for h in range(Hkv):
            n = int(n_sel[b, h])
            if n > 0:
                r = rng_for(seed, _TID_SUPPORT, 7_000_000 + b * Hkv + h)
                out[b, h, :n] = np.sort(r.choice(np.arange(lo, int(hi[b])), size=n, replace=False)).astype(np.int32)
    return out


def checksum(a: np.ndarray) -> int:
    """Order-sensitive 64-bit checksum of a tensor's bytes (to prove two sides hold the same bits)."""
    v = np.ascontiguousarray(a).view(np.uint8)
    pad = (-v.size) % 8
    if pad:
        v = np.concatenate([v.ravel(), np.zeros(pad, np.uint8)])
    u = v.ravel().view(np.uint64)
    idx = (np.arange(u.size, dtype=np.uint64) * np.uint64(0x9E3779B97F4A7C15)) | np.uint64(1)
    with np.errstate(over="ignore"):
        return int(np.bitwise_xor.reduce(u * idx))
