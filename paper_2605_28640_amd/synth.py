"""Seeded synthetic workloads (needle-structured), shared by tests and bench.

This module draws random inputs only.  It holds none of the method's arithmetic
(no recurrence, no scoring, no attention): those live in the HIP library and,
separately, in the test oracle.

Every (tensor, batch, head) unit has its own Philox stream, so one unit of a large
workload can be regenerated alone (the full-size parity tests do that).
Floating arrays are float32 holding values exactly representable in the workload's
storage dtype (bf16 values have a zero low half).
"""
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from functools import lru_cache
import os

import numpy as np

BASE_SEED = 20260528

# tensor ids of the Philox key
_T_K, _T_V, _T_G, _T_QDIR, _T_NEEDLE, _T_POS, _T_DEC, _T_QPRE, _T_QWIN = range(9)


@dataclass(frozen=True)
class Workload:
    name: str
    config_id: int
    B: int
    Hq: int
    Hkv: int
    D: int
    T: int
    dtype: str  # storage dtype of q, k, v and the cache: "f32" or "bf16"
    P: int = 16  # Quest page size
    n_needles: int = 8
    needle_mode: str = "per_head"  # per_head | per_seq_uniform | random_depth
    steps: int = 0  # decode steps appended after the prefill
    budgets: tuple = ()  # Quest budgets (fractions of the prefill page count)
    block: int = 0  # MoBA block size
    topk_blocks: int = 0
    W: int = 0  # SnapKV observation window
    keep_frac: float = 0.0
    pool: int = 0

    @property
    def G(self):
        return self.Hq // self.Hkv

    def scaled(self, **kw):
        return replace(self, **kw)


# The five configurations this build is measured and checked on.
C1 = Workload("C1-tiny-f32", 1, B=1, Hq=2, Hkv=2, D=64, T=2048, dtype="f32", n_needles=4,
              steps=16, budgets=(1 / 8,))
C2 = Workload("C2-gqa-32k", 2, B=1, Hq=32, Hkv=8, D=128, T=32768, dtype="bf16", n_needles=8,
              steps=256, budgets=(1 / 4, 1 / 8, 1 / 16))
C3 = Workload("C3-olmo2-7b-64k", 3, B=4, Hq=32, Hkv=32, D=128, T=65536, dtype="bf16",
              n_needles=16, needle_mode="per_seq_uniform", steps=512, budgets=(1 / 16, 1 / 4))
C4 = Workload("C4-moba-prefill-32k", 4, B=1, Hq=32, Hkv=32, D=128, T=32768, dtype="bf16",
              n_needles=16, needle_mode="per_seq_uniform", block=512, topk_blocks=3)
C5 = Workload("C5-snapkv-128k", 5, B=1, Hq=32, Hkv=8, D=128, T=131072, dtype="bf16",
              n_needles=8, needle_mode="random_depth", steps=256, W=32, keep_frac=1 / 8, pool=7)
CONFIGS = {w.config_id: w for w in (C1, C2, C3, C4, C5)}


def _rng(seed, config_id, tensor_id, unit):
    key = [np.uint64(seed), np.uint64((config_id << 48) | (tensor_id << 40) | unit)]
    return np.random.Generator(np.random.Philox(key=key))


def to_bf16_grid(x):
    """Round float32 values to the nearest bfloat16 (ties to even); still float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def _store(w, x):
    return to_bf16_grid(x) if w.dtype == "bf16" else np.ascontiguousarray(x, dtype=np.float32)


def _gate(rng, shape):
    z = rng.standard_normal(shape, dtype=np.float32)
    x = np.float32(4.2) + np.float32(0.5) * z
    return (np.float32(1.0) / (np.float32(1.0) + np.exp(-x))).astype(np.float32)


@lru_cache(maxsize=None)
def _q_dir(config_id, D, unit, seed):
    d = _rng(seed, config_id, _T_QDIR, unit).standard_normal(D)
    return (d * np.sqrt(D) / np.linalg.norm(d)).astype(np.float32)


def q_dir(w, b, kvh, seed=BASE_SEED):
    """Retrieval direction of one KV head: N(0, I) rescaled to norm sqrt(D)."""
    return _q_dir(w.config_id, w.D, b * w.Hkv + kvh, seed)


def needle_positions(w, b, kvh, seed=BASE_SEED):
    n = w.n_needles
    if n == 0:
        return np.zeros(0, dtype=np.int64)
    if w.needle_mode == "per_seq_uniform":  # same positions for every head of a sequence
        return ((np.arange(n) + 0.5) * w.T / n).astype(np.int64)
    if w.needle_mode == "random_depth":
        r = _rng(seed, w.config_id, _T_POS, b)
        return np.sort((r.uniform(0.1, 0.9, n) * w.T).astype(np.int64))
    r = _rng(seed, w.config_id, _T_POS, b * w.Hkv + kvh)
    return np.sort(r.choice(w.T, size=n, replace=False)).astype(np.int64)


def prefill_unit(w, b, kvh, seed=BASE_SEED):
    """Inputs of the recurrence for one (batch, KV head): k, v, g of shape [T, D]."""
    u = b * w.Hkv + kvh
    k = _rng(seed, w.config_id, _T_K, u).standard_normal((w.T, w.D), dtype=np.float32)
    v = _rng(seed, w.config_id, _T_V, u).standard_normal((w.T, w.D), dtype=np.float32)
    g = _gate(_rng(seed, w.config_id, _T_G, u), (w.T, w.D))
    pos = needle_positions(w, b, kvh, seed)
    if len(pos):
        noise = _rng(seed, w.config_id, _T_NEEDLE, u).standard_normal((len(pos), w.D))
        k[pos] = (3.0 * q_dir(w, b, kvh, seed)[None, :] + 0.3 * noise).astype(np.float32)
    return _store(w, k), _store(w, v), g


def _units(w, fn, units=None, threads=None):
    units = [(b, h) for b in range(w.B) for h in range(w.Hkv)] if units is None else units
    threads = threads or min(16, os.cpu_count() or 1)
    if threads > 1 and len(units) > 1:
        with ThreadPoolExecutor(threads) as ex:
            return units, list(ex.map(lambda bh: fn(*bh), units))
    return units, [fn(*bh) for bh in units]


def prefill(w, seed=BASE_SEED):
    """k, v, g of shape [B, Hkv, T, D]."""
    k = np.empty((w.B, w.Hkv, w.T, w.D), dtype=np.float32)
    v = np.empty_like(k)
    g = np.empty_like(k)
    units, res = _units(w, lambda b, h: prefill_unit(w, b, h, seed))
    for (b, h), (ku, vu, gu) in zip(units, res):
        k[b, h], v[b, h], g[b, h] = ku, vu, gu
    return k, v, g


def decode_step(w, step, seed=BASE_SEED):
    """Inputs of decode step `step`: k_t, v_t, g_t [B, Hkv, 1, D] and q_t [B, Hq, D]."""
    r = _rng(seed, w.config_id, _T_DEC, step)
    k = r.standard_normal((w.B, w.Hkv, 1, w.D), dtype=np.float32)
    v = r.standard_normal((w.B, w.Hkv, 1, w.D), dtype=np.float32)
    g = _gate(r, (w.B, w.Hkv, 1, w.D))
    q = np.empty((w.B, w.Hq, w.D), dtype=np.float32)
    noise = r.standard_normal((w.B, w.Hq, w.D), dtype=np.float32)
    for b in range(w.B):
        for h in range(w.Hq):
            q[b, h] = q_dir(w, b, h // w.G, seed) + np.float32(0.25) * noise[b, h]
    return _store(w, k), _store(w, v), g, _store(w, q)


def prefill_queries_unit(w, b, h, seed=BASE_SEED, every=64):
    """Prefill queries of one query head, [T, D]: background N(0, I); every `every`-th
    row looks for the needles (q_dir + 0.25 N(0, I))."""
    r = _rng(seed, w.config_id, _T_QPRE, b * w.Hq + h)
    q = r.standard_normal((w.T, w.D), dtype=np.float32)
    rows = np.arange(every - 1, w.T, every)
    q[rows] = q_dir(w, b, h // w.G, seed)[None, :] + np.float32(0.25) * q[rows]
    return _store(w, q)


def prefill_queries(w, seed=BASE_SEED):
    q = np.empty((w.B, w.Hq, w.T, w.D), dtype=np.float32)
    for b in range(w.B):
        for h in range(w.Hq):
            q[b, h] = prefill_queries_unit(w, b, h, seed)
    return q


def window_queries(w, seed=BASE_SEED):
    """Observation-window queries [B, Hq, W, D]: q_dir + 0.25 N(0, I)."""
    q = np.empty((w.B, w.Hq, w.W, w.D), dtype=np.float32)
    for b in range(w.B):
        for h in range(w.Hq):
            r = _rng(seed, w.config_id, _T_QWIN, b * w.Hq + h)
            q[b, h] = q_dir(w, b, h // w.G, seed)[None, :] + np.float32(0.25) * \
                r.standard_normal((w.W, w.D), dtype=np.float32)
    return _store(w, q)
