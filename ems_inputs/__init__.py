"""Seeded synthetic Q/K/V for the EMS prefill-compression path.

This module serves both the CPU oracle's tests and the HIP library's tests / benchmark.
It holds data generation and number-format conversion only -- none of the method's
arithmetic -- and imports neither side.

Recipe (stands in for real LLM activations, which need model weights and datasets):
  * Q, K, V ~ N(0,1) i.i.d., rounded to bf16 (round-to-nearest-even).
  * one unit direction u per (batch, kv-head), shared by the q-heads of the group;
    every query gets +1*u;
  * "heavy hitter" keys at seeded random positions get +3*u;
  * optional attention-sink key at position 0 gets +4*u;
  * optional "needle": 16 contiguous keys at a seeded start get +3*u.
  V is left untouched.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 20241208


@dataclass(frozen=True)
class Workload:
    name: str
    index: int              # 1-based config number
    batch: int
    q_heads: int
    kv_heads: int
    head_dim: int
    seq_len: int
    window: int
    budget: int
    merge_ratio: float = 0.5
    tau: float = 0.6
    pool_kernel: int = 7
    heavy: float = 0.0      # >= 1: count per head ; < 1: fraction of seq_len
    sink: bool = False
    needle: int = 0         # length of the contiguous needle span (0 = none)
    layers: int = 1


WORKLOADS = {
    "tiny": Workload("tiny", 1, 1, 4, 4, 64, 1024, 32, 64, heavy=8),
    "llama2_7b_4k": Workload("llama2_7b_4k", 2, 1, 32, 32, 128, 4096, 32, 256,
                             heavy=0.01, sink=True),
    "mistral_7b_16k": Workload("mistral_7b_16k", 3, 1, 32, 8, 128, 16384, 32, 256,
                               heavy=0.005, sink=True),
    "llama3_8b_32k": Workload("llama3_8b_32k", 4, 4, 32, 8, 128, 32768, 64, 128,
                              heavy=0.005, sink=True, needle=16),
    "extreme_128k": Workload("extreme_128k", 5, 1, 32, 8, 128, 131072, 64, 2048,
                             heavy=0.002, sink=True, needle=16, layers=32),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even); returns the 16-bit patterns as uint16."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32)
            << np.uint32(16)).view(np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 values rounded to the nearest bf16-representable float32."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x))


@dataclass
class Inputs:
    workload: Workload
    layer: int
    q: np.ndarray           # uint16 bf16 bits [B,Hq,N,D]
    k: np.ndarray           # uint16 bf16 bits [B,Hkv,N,D]
    v: np.ndarray           # uint16 bf16 bits [B,Hkv,N,D]
    heavy_pos: list = field(default_factory=list)   # [B][Hkv] -> int array
    needle_start: list = field(default_factory=list)

    def f32(self, name: str) -> np.ndarray:
        return bf16_bits_to_f32(getattr(self, name))


def _n_heavy(w: Workload) -> int:
    if w.heavy <= 0:
        return 0
    return int(w.heavy) if w.heavy >= 1 else max(1, int(round(w.heavy * w.seq_len)))


def generate(w: Workload, layer: int = 0, seed: int | None = None,
             batch_slice: slice | None = None) -> Inputs:
    """Generate one layer's inputs.  `batch_slice` restricts which batch entries are
    produced (each entry has its own stream, so slices match the full tensor)."""
    seed = BASE_SEED if seed is None else seed
    G = w.q_heads // w.kv_heads
    N, D = w.seq_len, w.head_dim
    batches = range(w.batch)[batch_slice] if batch_slice is not None else range(w.batch)
    nb = len(batches)
    q = np.empty((nb, w.q_heads, N, D), np.uint16)
    k = np.empty((nb, w.kv_heads, N, D), np.uint16)
    v = np.empty((nb, w.kv_heads, N, D), np.uint16)
    heavy_pos, needle_start = [], []
    n_heavy = _n_heavy(w)
    for bi, b in enumerate(batches):
        hp_b, ns_b = [], []
        for kvh in range(w.kv_heads):
            rng = np.random.Generator(np.random.PCG64([seed, w.index, layer, b, kvh]))
            u = rng.standard_normal(D)
            u = (u / np.sqrt((u * u).sum())).astype(np.float32)
            kk = rng.standard_normal((N, D), dtype=np.float32)
            vv = rng.standard_normal((N, D), dtype=np.float32)
            pos = np.sort(rng.choice(np.arange(1, N), size=n_heavy, replace=False)) \
                if n_heavy else np.zeros(0, np.int64)
            kk[pos] += 3.0 * u
            if w.sink:
                kk[0] += 4.0 * u
            start = -1
            if w.needle:
                start = int(rng.integers(w.window, N - w.window - w.needle))
                kk[start:start + w.needle] += 3.0 * u
            k[bi, kvh] = f32_to_bf16_bits(kk)
            v[bi, kvh] = f32_to_bf16_bits(vv)
            for g in range(G):
                qq = rng.standard_normal((N, D), dtype=np.float32)
                qq += u
                q[bi, kvh * G + g] = f32_to_bf16_bits(qq)
            hp_b.append(pos)
            ns_b.append(start)
        heavy_pos.append(hp_b)
        needle_start.append(ns_b)
    return Inputs(w, layer, q, k, v, heavy_pos, needle_start)


def small(batch, q_heads, kv_heads, head_dim, seq_len, seed=0, heavy=4, sink=True,
          scale=1.0) -> Inputs:
    """Free-form small case for tests (same recipe, arbitrary shape)."""
    w = Workload(f"small_{batch}x{q_heads}x{kv_heads}x{seq_len}x{head_dim}", 0, batch,
                 q_heads, kv_heads, head_dim, seq_len, 1, 1,
                 heavy=min(heavy, max(seq_len - 1, 0)), sink=sink)
    inp = generate(w, seed=BASE_SEED + 1000 + seed)
    if scale != 1.0:
        for name in ("q", "k", "v"):
            setattr(inp, name, f32_to_bf16_bits(inp.f32(name) * np.float32(scale)))
    return inp
