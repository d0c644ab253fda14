"""Seeded synthetic workloads for the DynamicKV prefill-compression path.

This module only *draws inputs*: window queries, keys, values and the planted
"heavy" key positions that stand in for the salient tokens of the paper's
long-context workloads (LongBench-length and needle-style prompts, Section 5).
It contains none of the method's arithmetic (no softmax, pooling, selection or
budget maths) and imports neither the CPU oracle nor the HIP library, so both
may consume its arrays.

Shapes follow the model table of the paper's appendix (Llama-3-8B,
Mistral-7B, Qwen2-7B: layers / query heads / KV heads / head size); values are
synthetic: Q, K, V ~ N(0, 1) from a counter-based Philox stream keyed by
(seed, layer, tensor), rounded to the storage type so that every consumer sees
the same bit patterns.

Layout of one layer (all float32 numpy arrays holding storage-representable
values):
    q_win [n_seqs, Hq, w, d]      the last w query rows of every sequence
    k, v  [Hkv, T, d]             head-major, sequences packed along T
    cu_seqlens [n_seqs + 1] int32 packed-sequence offsets, T = cu_seqlens[-1]
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Tuple

import numpy as np

_TENSOR_Q, _TENSOR_K, _TENSOR_V, _TENSOR_PLANT, _TENSOR_LEN = range(5)


@dataclass(frozen=True)
class Workload:
    """One synthetic configuration (symbols as in Algorithm 1 of the paper).

    L layers, Hq query heads, Hkv KV heads, head size d, window ws = w, pooling
    kernel P, mean per-layer budget wt - ws = mean_budget, per-layer maximum
    B^l = layer_max, update interval m = interval.
    """
    name: str
    L: int
    Hq: int
    Hkv: int
    d: int
    seqlens: Tuple[int, ...]
    dtype: str                 # "f32" or "bf16" (storage type of Q, K, V)
    w: int
    P: int
    mean_budget: int
    layer_max: int
    interval: int
    seed: int
    plant: str = "loguniform"  # "int", "loguniform", "cluster8", "front8"
    plant_lo: int = 16
    plant_hi: int = 512
    gain: float = 3.0
    plant_normalize: bool = False   # rescale the mean query to norm sqrt(d) before applying gain

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def n_seqs(self) -> int:
        return len(self.seqlens)

    @property
    def total_tokens(self) -> int:
        return int(sum(self.seqlens))

    @property
    def cu_seqlens(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.seqlens)]).astype(np.int32)

    @property
    def global_budget(self) -> int:
        return self.mean_budget * self.L

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


def _rng(seed: int, layer: int, tensor: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(seed << 20) ^ (layer << 4) ^ tensor, 0x9E3779B9]))


def _ragged_lengths(seed: int, n: int, lo: int, hi: int) -> Tuple[int, ...]:
    return tuple(int(x) for x in _rng(seed, 0, _TENSOR_LEN).integers(lo, hi + 1, size=n))


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); returns float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of bf16-representable float32 values."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16)


def standard_configs() -> Dict[str, Workload]:
    """The five benchmark configurations (index = order of definition)."""
    cfgs = [
        Workload("tiny", L=4, Hq=4, Hkv=2, d=64, seqlens=(1024,), dtype="f32", w=16, P=7,
                 mean_budget=128, layer_max=256, interval=2, seed=1000, plant="int", plant_lo=8, plant_hi=64),
        Workload("llama3_8b_8k", L=32, Hq=32, Hkv=8, d=128, seqlens=(8192,), dtype="bf16", w=32, P=7,
                 mean_budget=128, layer_max=512, interval=4, seed=1001, plant="loguniform"),
        Workload("mistral_7b_32k", L=32, Hq=32, Hkv=8, d=128, seqlens=(32768,), dtype="bf16", w=32, P=7,
                 mean_budget=512, layer_max=2048, interval=4, seed=1002, plant="cluster8"),
        Workload("qwen2_7b_32k_extreme", L=28, Hq=28, Hkv=4, d=128, seqlens=(32768,), dtype="bf16", w=32, P=7,
                 mean_budget=64, layer_max=256, interval=4, seed=1003, plant="front8"),
        Workload("ragged_batch8", L=32, Hq=32, Hkv=8, d=128, seqlens=_ragged_lengths(1004, 8, 4096, 16384),
                 dtype="bf16", w=32, P=7, mean_budget=256, layer_max=1024, interval=4, seed=1004,
                 plant="loguniform"),
    ]
    return {c.name: c for c in cfgs}


def extended_configs() -> Dict[str, Workload]:
    """Beyond the five benchmark configurations: config 3's shape at four and at sixteen times the context."""
    base = standard_configs()["mistral_7b_32k"]
    return {"mistral_7b_128k": base.with_(name="mistral_7b_128k", seqlens=(131072,), seed=1005),
            "mistral_7b_512k": base.with_(name="mistral_7b_512k", seqlens=(524288,), seed=1006)}


def all_configs() -> Dict[str, Workload]:
    cfgs = standard_configs()
    cfgs.update(extended_configs())
    return cfgs


def planted_count(cfg: Workload, layer: int) -> int:
    """Number of planted heavy-key positions of one layer (same for every sequence)."""
    r = _rng(cfg.seed, layer, _TENSOR_PLANT)
    if cfg.plant == "int":
        return int(r.integers(cfg.plant_lo, cfg.plant_hi + 1))
    lo, hi = cfg.plant_lo, cfg.plant_hi
    if cfg.plant == "front8" and layer >= 8:
        return int(r.integers(0, 17))
    return int(round(float(np.exp(r.uniform(np.log(lo), np.log(hi))))))


def planted_positions(cfg: Workload, layer: int, seq: int) -> np.ndarray:
    """Sorted sequence-local prefix positions whose key rows are overwritten."""
    S = cfg.seqlens[seq]
    prefix = S - cfg.w
    c = min(planted_count(cfg, layer), max(prefix, 0))
    if c <= 0:
        return np.zeros(0, dtype=np.int64)
    r = _rng(cfg.seed + 7919 * (seq + 1), layer, _TENSOR_PLANT)
    if cfg.plant == "cluster8":
        width = 8
        n_clusters = max(1, c // width)
        slots = max(prefix // width, 1)
        starts = r.choice(slots, size=min(n_clusters, slots), replace=False) * width
        pos = (starts[:, None] + np.arange(width)[None, :]).reshape(-1)
        pos = pos[pos < prefix]
    else:
        pos = r.choice(prefix, size=c, replace=False)
    return np.sort(pos.astype(np.int64))


def make_layer(cfg: Workload, layer: int, with_v: bool = True) -> Dict[str, np.ndarray]:
    """Draw one layer's q_win, k, v (float32 arrays of storage-representable values)."""
    T = cfg.total_tokens
    q = _rng(cfg.seed, layer, _TENSOR_Q).standard_normal((cfg.n_seqs, cfg.Hq, cfg.w, cfg.d), dtype=np.float32)
    k = _rng(cfg.seed, layer, _TENSOR_K).standard_normal((cfg.Hkv, T, cfg.d), dtype=np.float32)
    if cfg.dtype == "bf16":
        q = round_to_bf16(q)
        k = round_to_bf16(k)
    cu = cfg.cu_seqlens
    for s in range(cfg.n_seqs):
        pos = planted_positions(cfg, layer, s)
        if pos.size == 0:
            continue
        # heavy key of KV head h = gain x mean of that head's G*w window query rows
        mean_q = q[s].reshape(cfg.Hkv, cfg.G * cfg.w, cfg.d).mean(axis=1, dtype=np.float32)
        if cfg.plant_normalize:
            norm = np.sqrt((mean_q.astype(np.float64) ** 2).sum(axis=1, keepdims=True))
            mean_q = (mean_q * (np.sqrt(cfg.d) / np.maximum(norm, 1e-30))).astype(np.float32)
        heavy = (np.float32(cfg.gain) * mean_q).astype(np.float32)
        if cfg.dtype == "bf16":
            heavy = round_to_bf16(heavy)
        k[:, cu[s] + pos, :] = heavy[:, None, :]
    out = {"q_win": q, "k": k, "cu_seqlens": cu}
    if with_v:
        v = _rng(cfg.seed, layer, _TENSOR_V).standard_normal((cfg.Hkv, T, cfg.d), dtype=np.float32)
        out["v"] = round_to_bf16(v) if cfg.dtype == "bf16" else v
    return out
