"""Shared helpers of the GPU parity tests: problem construction (inputs from the
seeded generator, PQ structures from the oracle's K-Means) and the comparison rules.

Comparison rules (per unit = (sequence, KV head)):
  * index sets: the GPU's attended set must equal the oracle's.  If they differ, every
    token in the symmetric difference must have an fp32 score within 1e-4 relative of
    the oracle's K-th score (such near-ties are counted and reported, anything else
    fails).  Both sides rank the same fp32 scores, so the expected count is zero.
  * attention: max |gpu - ref| / max|ref| per head <= 2e-3 for bf16 inputs, 1e-5 for
    fp32 inputs, the reference being the oracle's double-precision attention over the
    GPU's own index list (so that a legal tie swap cannot hide or cause an error).
"""
from __future__ import annotations

import dataclasses
from typing import Dict, Optional, Sequence

import numpy as np

import oracle
from paper_2407_12820_amd import workloads as wl

ATTN_TOL = {"bf16": 2e-3, "f32": 1e-5}
NEAR_TIE_REL = 1e-4


@dataclasses.dataclass
class Problem:
    w: wl.Workload
    q: np.ndarray
    k: np.ndarray
    v: np.ndarray
    centroids: np.ndarray
    codes: np.ndarray
    checked_units: Sequence[int]  # units whose PQ structures come from the oracle's K-Means


_CACHE: Dict[tuple, Problem] = {}


def build_problem(w: wl.Workload, seed: int = 0, checked_units: Optional[Sequence[int]] = None) -> Problem:
    """Inputs for one workload.  With checked_units given, only those units get K-Means
    PQ structures; the others get centroids drawn from their keys and random codes, which
    are valid inputs too (scores, selection and attention need no clustering), so a test
    can still compare every unit with the oracle by passing `units` to the checks."""
    key = (w, seed, None if checked_units is None else tuple(checked_units))
    if key in _CACHE:
        return _CACHE[key]
    d = wl.generate(w, seed)
    init = wl.kmeans_init_indices(w, seed)
    B, Hkv, N, D, M, C = w.batch, w.n_kv_heads, w.n_tokens, w.head_dim, w.pq_m, w.pq_centroids
    if checked_units is None:
        cent, codes, _ = oracle.pq_build(d["k"], w.dtype, M, C, w.kmeans_iters, init)
        units = list(range(B * Hkv))
    else:
        units = list(checked_units)
        rng = np.random.default_rng(seed + 12345)
        cent = np.empty((B, Hkv, M, C, D // M), np.float32)
        codes = rng.integers(0, C, size=(B, Hkv, N, M), dtype=np.uint8)
        kf = None
        for u in range(B * Hkv):
            b, g = divmod(u, Hkv)
            if u in units:
                c1, cd1, _ = oracle.pq_build(d["k"][b:b + 1, g:g + 1], w.dtype, M, C, w.kmeans_iters, init[b:b + 1, g:g + 1])
                cent[b, g], codes[b, g] = c1[0, 0], cd1[0, 0]
            else:
                rows = wl.to_f32(d["k"][b, g][init[b, g].reshape(-1)], w.dtype).reshape(M, C, D)
                for j in range(M):
                    cent[b, g, j] = rows[j][:, j * (D // M):(j + 1) * (D // M)]
    p = Problem(w, d["q"], d["k"], d["v"], cent, codes, units)
    if N * B * Hkv <= (1 << 21):
        _CACHE[key] = p
    return p


def unit_slice(p: Problem, u: int):
    """The [1,1,...] sub-problem of unit u (and its G query heads)."""
    w = p.w
    b, g = divmod(u, w.n_kv_heads)
    G = w.group
    return (p.q[b:b + 1, g * G:(g + 1) * G], p.centroids[b:b + 1, g:g + 1], p.codes[b:b + 1, g:g + 1],
            p.k[b:b + 1, g:g + 1], p.v[b:b + 1, g:g + 1])


def check_indices(p: Problem, idx_gpu: np.ndarray, units: Optional[Sequence[int]] = None) -> int:
    """Returns the number of near-tie substitutions (expected 0); raises on any real mismatch."""
    w = p.w
    I, K, L, N = w.n_init, w.topk, w.n_local, w.n_tokens
    assert idx_gpu.shape == (w.batch, w.n_kv_heads, I + K + L) and idx_gpu.dtype == np.int32
    near = 0
    for u in (p.checked_units if units is None else units):
        b, g = divmod(u, w.n_kv_heads)
        q1, c1, cd1, _, _ = unit_slice(p, u)
        s32, _ = oracle.scores(q1, w.dtype, c1, cd1)
        want = oracle.select(s32, K, I, L)[0, 0]
        got = idx_gpu[b, g]
        assert got[:I].tolist() == list(range(I)), f"unit {u}: initial window"
        assert got[I + K:].tolist() == list(range(N - L, N)), f"unit {u}: local window"
        top = got[I:I + K]
        assert len(set(top.tolist())) == K, f"unit {u}: duplicate retrieved tokens"
        assert K == 0 or (top.min() >= I and top.max() < N - L), f"unit {u}: retrieved token outside the middle range"
        diff = set(top.tolist()) ^ set(want[I:I + K].tolist())
        if diff:
            tau = float(s32[0, 0, want[I + K - 1]])
            bad = [t for t in diff if abs(float(s32[0, 0, t]) - tau) > NEAR_TIE_REL * abs(tau)]
            assert not bad, f"unit {u}: {len(bad)} tokens differ outside the near-tie band, e.g. {bad[:5]}"
            near += len(diff)
    return near


def check_structure(p: Problem, idx_gpu: np.ndarray, out_gpu: np.ndarray) -> None:
    """Invariants that hold for every unit whatever the PQ structures are."""
    w = p.w
    I, K, L, N = w.n_init, w.topk, w.n_local, w.n_tokens
    assert np.all(np.isfinite(out_gpu))
    assert np.all(idx_gpu[:, :, :I] == np.arange(I)) and np.all(idx_gpu[:, :, I + K:] == np.arange(N - L, N))
    top = np.sort(idx_gpu[:, :, I:I + K], axis=-1)
    if K:
        assert top.min() >= I and top.max() < N - L
        assert np.all(np.diff(top, axis=-1) > 0), "duplicate retrieved tokens"


def attn_error(p: Problem, idx_gpu: np.ndarray, out_gpu: np.ndarray, units: Optional[Sequence[int]] = None,
               scale: Optional[float] = None) -> float:
    """Max over checked heads of max|gpu - ref| / max|ref|."""
    w = p.w
    scale = wl.softmax_scale(w) if scale is None else scale
    G = w.group
    worst = 0.0
    for u in (p.checked_units if units is None else units):
        b, g = divmod(u, w.n_kv_heads)
        q1, _, _, k1, v1 = unit_slice(p, u)
        ref = oracle.attention(q1, k1, v1, w.dtype, idx_gpu[b:b + 1, g:g + 1], scale)[0]
        got = out_gpu[b, g * G:(g + 1) * G].astype(np.float64)
        err = np.abs(got - ref).max(axis=1) / np.maximum(np.abs(ref).max(axis=1), 1e-30)
        worst = max(worst, float(err.max()))
    return worst
