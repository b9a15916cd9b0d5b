"""Seeded synthetic inputs for the AhaKV eviction path.

This module only draws numbers and shapes them like the paper's workloads
(decoder attention Q/K/V per layer and head, an attention sink at token 0, a
small fraction of heavy-hitter keys, optional per-channel scales and rotary
position embedding).  It contains none of the method's arithmetic, so both
the GPU path and the float64 CPU checker may be fed from it.  Real model
activations and the paper's evaluation sets are not available offline; these
inputs stand in for them and take only their shapes and structure.

Every (layer, batch, KV head) slice has its own counter-based stream, so any
subset of heads can be generated alone and equals the same slice of the full
tensor.

Values are returned as float32 numpy arrays already rounded to the storage
dtype of the workload (bf16 workloads hold bf16-representable values), so the
same bits reach every consumer.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Sequence

import numpy as np

BASE_SEED = 20250603


@dataclass(frozen=True)
class Workload:
    name: str
    cfg_id: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seq_len: int
    window: int          # observation window r
    budget: int          # total cache budget B
    recent: int          # recent budget B_r
    dtype: str           # "f32" | "bf16"
    channel_scale: bool = False
    rope: bool = False
    hh_frac: float = 0.01
    hh_even: bool = False
    sink_mult: float = 4.0
    q_bias: float = 2.0
    beta: float = 1.0
    layers: int = 1
    decode_steps: int = 0

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


# The five benchmark shapes.
C1 = Workload("c1_tiny_f32", 1, 1, 2, 2, 64, 512, 32, 128, 32, "f32", hh_frac=0.02)
C2 = Workload("c2_llama2_7b_layer", 2, 1, 32, 32, 128, 4096, 64, 512, 64, "bf16",
              channel_scale=True)
C3 = Workload("c3_gqa_32k", 3, 1, 32, 8, 128, 32768, 64, 2048, 64, "bf16",
              rope=True, hh_even=True)
C3_B1024 = replace(C3, name="c3_gqa_32k_b1024", budget=1024)
C4 = Workload("c4_batched_decode", 4, 8, 32, 32, 128, 4096, 64, 1024, 64, "bf16",
              channel_scale=True, decode_steps=256)
C5 = Workload("c5_full_depth", 5, 4, 32, 32, 128, 16384, 64, 3276, 64, "bf16",
              layers=32)

CONFIGS = {w.name: w for w in (C1, C2, C3, C3_B1024, C4, C5)}


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bf16 (ties to even); result stays float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
         & np.uint32(0xFFFF0000))
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already bf16-representable."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16)


def store_round(x: np.ndarray, dtype: str) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    return round_bf16(x) if dtype == "bf16" else x


def _rng(w: Workload, layer: int, *key: int) -> np.random.Generator:
    seed = BASE_SEED + 1000 * w.cfg_id + layer
    return np.random.Generator(np.random.PCG64([seed, *key]))


def _rope(x: np.ndarray, base: float = 10000.0) -> np.ndarray:
    """Rotate-half rotary embedding over the last two axes [n, d] (float64)."""
    n, d = x.shape[-2], x.shape[-1]
    half = d // 2
    inv = base ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    ang = np.arange(n, dtype=np.float64)[:, None] * inv[None, :]
    cos, sin = np.cos(ang), np.sin(ang)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * cos - x2 * sin, x2 * cos + x1 * sin], axis=-1)


def layer_knobs(w: Workload, layer: int):
    """(sink multiplier, heavy-hitter fraction) of a layer."""
    if w.layers > 1:
        t = layer / float(w.layers - 1)
        return 2.0 + 4.0 * t, 0.005 + 0.025 * t
    return w.sink_mult, w.hh_frac


def heavy_hitter_positions(w: Workload, layer: int, b: int, hk: int) -> np.ndarray:
    n, r = w.seq_len, w.window
    _, frac = layer_knobs(w, layer)
    m = int(np.ceil(frac * n))
    span = n - r - 1  # positions 1 .. n-r-1
    m = max(0, min(m, span))
    if m == 0:
        return np.zeros(0, dtype=np.int64)
    if w.hh_even:
        pos = np.floor((np.arange(m) + 0.5) * (n - r) / m).astype(np.int64)
        return np.clip(pos, 1, n - r - 1)
    rng = _rng(w, layer, b, hk, 7)
    return np.sort(1 + rng.choice(span, size=m, replace=False)).astype(np.int64)


def make_head(w: Workload, layer: int, b: int, hk: int):
    """One KV head's inputs: Q [G, n, d], K [n, d], V [n, d] (float32, rounded)."""
    G, n, d = w.group, w.seq_len, w.head_dim
    rng = _rng(w, layer, b, hk, 0)
    Q = rng.standard_normal((G, n, d), dtype=np.float32).astype(np.float64)
    K = rng.standard_normal((n, d), dtype=np.float32).astype(np.float64)
    V = rng.standard_normal((n, d), dtype=np.float32).astype(np.float64)
    if w.channel_scale:
        Q *= rng.uniform(0.5, 2.0, size=(G, 1, d))
        K *= rng.uniform(0.5, 2.0, size=(1, d))
        V *= rng.uniform(0.5, 2.0, size=(1, d))
    if w.rope:
        Q = _rope(Q)
        K = _rope(K)
    u = rng.standard_normal((G, d))
    u /= np.linalg.norm(u, axis=-1, keepdims=True)
    Q += w.q_bias * u[:, None, :]
    sink, _ = layer_knobs(w, layer)
    K[0] *= sink
    hh = heavy_hitter_positions(w, layer, b, hk)
    if hh.size:
        qbar = Q[:, n - w.window:, :].mean(axis=(0, 1))
        qbar /= np.linalg.norm(qbar)
        K[hh] += w.beta * np.sqrt(d) * qbar
    return (store_round(Q, w.dtype), store_round(K, w.dtype), store_round(V, w.dtype))


def make_prefill(w: Workload, layer: int = 0,
                 batches: Optional[Sequence[int]] = None,
                 kv_heads: Optional[Sequence[int]] = None,
                 threads: int = 8):
    """Q [b, Hq', n, d], K, V [b, Hkv', n, d] for the chosen batches / KV heads.

    With subsets, the result equals the same slices of the full tensors (the
    query heads of a KV head travel with it).
    """
    from concurrent.futures import ThreadPoolExecutor

    bs = list(range(w.batch)) if batches is None else list(batches)
    hs = list(range(w.n_kv_heads)) if kv_heads is None else list(kv_heads)
    G, n, d = w.group, w.seq_len, w.head_dim
    Q = np.empty((len(bs), len(hs) * G, n, d), dtype=np.float32)
    K = np.empty((len(bs), len(hs), n, d), dtype=np.float32)
    V = np.empty((len(bs), len(hs), n, d), dtype=np.float32)

    def work(t):
        bi, hi = t
        q, k, v = make_head(w, layer, bs[bi], hs[hi])
        Q[bi, hi * G:(hi + 1) * G] = q
        K[bi, hi] = k
        V[bi, hi] = v

    jobs = [(bi, hi) for bi in range(len(bs)) for hi in range(len(hs))]
    if threads > 1 and len(jobs) > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, jobs))
    else:
        for t in jobs:
            work(t)
    return Q, K, V


def make_decode_inputs(w: Workload, step: int):
    """Fresh Gaussian q [b, Hq, d], k, v [b, Hkv, d] of one generation step."""
    rng = _rng(w, 0, 1_000_000 + step)
    q = rng.standard_normal((w.batch, w.n_q_heads, w.head_dim), dtype=np.float32)
    k = rng.standard_normal((w.batch, w.n_kv_heads, w.head_dim), dtype=np.float32)
    v = rng.standard_normal((w.batch, w.n_kv_heads, w.head_dim), dtype=np.float32)
    return store_round(q, w.dtype), store_round(k, w.dtype), store_round(v, w.dtype)


def scaled(w: Workload, **kw) -> Workload:
    """A reshaped copy (tests use smaller or ragged variants of a shape)."""
    return replace(w, **kw)
