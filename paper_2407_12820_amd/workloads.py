"""Seeded synthetic decode workloads shaped like long-context Llama-3 attention layers.

This module only draws random tensors and formats them.  It holds none of the
method's arithmetic (no clustering, no scoring, no selection, no attention): both
the CPU oracle's tests and the GPU path take their inputs from here, and the K-Means
initial sample positions (the only random numbers the method itself draws) are
produced here as well and handed to whichever side builds the PQ structures.

Shapes follow the paper's notation (Table "Notations"): batch B, query heads Hq,
key/value heads Hkv, head dimension D, N cached tokens, M PQ partitions with
C = 2**b centroids each.  Selection sizes follow Section 4.1 (a fixed ratio of the
sequence) plus the always-kept initial and local windows of Section 3.1.

All values are drawn in fp32 from a counter-based generator (Philox) keyed by
(seed, tensor tag, unit index), so any unit can be regenerated independently.
bf16 tensors are the fp32 draw rounded to nearest-even and are returned as uint16
bit patterns, so both sides consume identical bits.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np

_TAG_Q, _TAG_K, _TAG_V, _TAG_PLANT, _TAG_OUTLIER, _TAG_INIT = 1, 2, 3, 4, 5, 6


@dataclass(frozen=True)
class Workload:
    """One decode-step problem: a single attention layer with its PQ geometry."""

    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_tokens: int
    pq_m: int
    pq_centroids: int
    topk: int
    n_init: int
    n_local: int
    dtype: str  # "f32" or "bf16": storage type of q, K and V
    kmeans_iters: int
    recipe: str  # "plain" | "planted_q" | "planted_mean_q" | "outlier_channels"
    plant_count: int = 0  # number of planted tokens per KV head (planted recipes)
    plant_gain: float = 0.0  # planted key = gain * query + N(0,1)
    outlier_channels: int = 0
    outlier_gain: float = 1.0
    topk_ratio_den: int = 0  # K = N // den when rescaled; 0 keeps K fixed

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def sub_dim(self) -> int:
        return self.head_dim // self.pq_m

    @property
    def n_selected(self) -> int:
        return self.n_init + self.topk + self.n_local

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def scaled(self, **changes) -> "Workload":
        """A smaller (or otherwise altered) variant that keeps the recipe.

        When n_tokens changes and the workload's K is a ratio of N, K follows.
        planted counts that are a ratio of N follow as well.
        """
        new = dataclasses.replace(self, **changes)
        if "n_tokens" in changes and "topk" not in changes and self.topk_ratio_den:
            new = dataclasses.replace(new, topk=new.n_tokens // self.topk_ratio_den)
        if ("n_tokens" in changes and "plant_count" not in changes
                and self.recipe == "planted_mean_q"):
            new = dataclasses.replace(new, plant_count=max(1, round(new.n_tokens * 0.01)))
        if "name" not in changes:
            new = dataclasses.replace(new, name=self.name + "_scaled")
        return new

    def algorithmic_bytes(self) -> int:
        """Bytes one decode step must move: codes + selected K/V rows + q + look-up table."""
        units = self.batch * self.n_kv_heads
        codes = units * self.n_tokens * self.pq_m
        kv = units * self.n_selected * self.head_dim * 2 * self.elem_bytes
        q = self.batch * self.n_q_heads * self.head_dim * self.elem_bytes
        lut = units * self.pq_m * self.pq_centroids * 4
        return codes + kv + q + lut


def _mk(name, B, Hq, Hkv, N, M, C, den, dtype, iters, recipe, **kw) -> Workload:
    return Workload(name=name, batch=B, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=128,
                    n_tokens=N, pq_m=M, pq_centroids=C, topk=N // den if den else kw.pop("topk"),
                    n_init=4, n_local=64, dtype=dtype, kmeans_iters=iters, recipe=recipe,
                    topk_ratio_den=den, **kw)


# The five benchmark configurations.  K-Means iteration counts other than the first
# are this build's choice (the paper caps iterations adaptively, Section 3.3).
CONFIGS: Dict[str, Workload] = {
    "tiny_f32": _mk("tiny_f32", 1, 1, 1, 4096, 2, 64, 0, "f32", 25, "planted_q",
                    topk=512, plant_count=40, plant_gain=3.0),
    "llama8b_32k": _mk("llama8b_32k", 1, 32, 8, 32768, 2, 64, 5, "bf16", 10,
                       "outlier_channels", outlier_channels=4, outlier_gain=8.0),
    "llama8b_128k": _mk("llama8b_128k", 1, 32, 8, 131072, 2, 64, 10, "bf16", 8,
                        "planted_mean_q", plant_count=1311, plant_gain=2.0),
    "batch8_32k": _mk("batch8_32k", 8, 32, 8, 32768, 4, 256, 5, "bf16", 4, "plain"),
    "llama70b_128k": _mk("llama70b_128k", 4, 64, 8, 131072, 4, 256, 10, "bf16", 3,
                         "outlier_channels", outlier_channels=4, outlier_gain=8.0),
}
CONFIG_ORDER = ["tiny_f32", "llama8b_32k", "llama8b_128k", "batch8_32k", "llama70b_128k"]


# --------------------------------------------------------------------------- bf16
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_f32(x: np.ndarray, dtype: str) -> np.ndarray:
    """The fp32 value of a stored tensor, whatever its storage type."""
    return x.astype(np.float32, copy=False) if dtype == "f32" else bf16_bits_to_f32(x)


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.float32) if dtype == "f32" else f32_to_bf16_bits(x)


def _rng(seed: int, tag: int, unit: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(tag * (1 << 32) + unit)]))


# ---------------------------------------------------------------------- generation
def generate(w: Workload, seed: int = 0, threads: int = 8) -> Dict[str, np.ndarray]:
    """Draw q [B,Hq,D], k and v [B,Hkv,N,D] for a workload.

    Returns storage arrays (float32, or uint16 bf16 bits) plus the bookkeeping
    needed to describe the draw: planted token positions and outlier channels.
    """
    B, Hq, Hkv, D, N = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_tokens
    G = w.group
    sdt = np.float32 if w.dtype == "f32" else np.uint16
    q32 = _rng(seed, _TAG_Q).standard_normal((B, Hq, D), dtype=np.float32)
    q = _store(q32, w.dtype)
    qv = to_f32(q, w.dtype)  # the values both sides will actually see
    k = np.empty((B, Hkv, N, D), dtype=sdt)
    v = np.empty((B, Hkv, N, D), dtype=sdt)
    planted = np.zeros((B, Hkv, max(w.plant_count, 1)), dtype=np.int64)
    outliers = np.zeros((B, Hkv, max(w.outlier_channels, 1)), dtype=np.int64)
    lo, hi = w.n_init, N - w.n_local  # planted tokens sit among the middle tokens

    def unit(u: int) -> None:
        b, g = divmod(u, Hkv)
        x = _rng(seed, _TAG_K, u).standard_normal((N, D), dtype=np.float32)
        if w.recipe in ("planted_q", "planted_mean_q") and w.plant_count and hi > lo:
            cnt = min(w.plant_count, hi - lo)
            pos = lo + _rng(seed, _TAG_PLANT, u).choice(hi - lo, size=cnt, replace=False)
            pos.sort()
            planted[b, g, :cnt] = pos
            target = qv[b, g * G:(g + 1) * G].mean(axis=0, dtype=np.float32)
            x[pos] += np.float32(w.plant_gain) * target
        if w.recipe == "outlier_channels" and w.outlier_channels:
            ch = _rng(seed, _TAG_OUTLIER, u).choice(D, size=w.outlier_channels, replace=False)
            ch.sort()
            outliers[b, g, :] = ch
            x[:, ch] *= np.float32(w.outlier_gain)
        k[b, g] = _store(x, w.dtype)
        del x
        y = _rng(seed, _TAG_V, u).standard_normal((N, D), dtype=np.float32)
        v[b, g] = _store(y, w.dtype)

    units = B * Hkv
    if threads > 1 and units > 1:
        with ThreadPoolExecutor(max_workers=min(threads, units)) as pool:
            list(pool.map(unit, range(units)))
    else:
        for u in range(units):
            unit(u)
    return {"q": q, "k": k, "v": v, "planted": planted, "outlier_channels": outliers}


def kmeans_init_indices(w: Workload, seed: int = 0) -> np.ndarray:
    """Token positions whose sub-vectors seed the K-Means centroids.

    Shape [B,Hkv,M,C] int32, distinct within each (b, head, partition) whenever
    N >= C.  These are the random numbers the PQ construction draws; they are an
    input to whichever implementation runs the clustering.
    """
    B, Hkv, M, C, N = w.batch, w.n_kv_heads, w.pq_m, w.pq_centroids, w.n_tokens
    out = np.empty((B, Hkv, M, C), dtype=np.int32)
    for u in range(B * Hkv):
        b, g = divmod(u, Hkv)
        r = _rng(seed, _TAG_INIT, u)
        for j in range(M):
            out[b, g, j] = r.choice(N, size=C, replace=N < C).astype(np.int32)
    return out


def softmax_scale(w: Workload) -> float:
    """The usual 1/sqrt(d_h) factor applied to query-key products before softmax."""
    return float(1.0 / np.sqrt(np.float64(w.head_dim)))


def get(name: str, **changes) -> Workload:
    w = CONFIGS[name]
    return w.scaled(**changes) if changes else w
