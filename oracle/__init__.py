"""ctypes loader for the C oracle (oracle/pqc_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  It never imports the GPU package and the GPU
package never imports it.  Arrays are numpy, host memory; bf16 tensors are uint16
bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

_LIB = None


def lib() -> C.CDLL:
    global _LIB
    if _LIB is None:
        # PQC_ORACLE_LIB: another build of pqc_oracle.c to load instead (the mutation tests plant mistakes
        # in copies of the source and check that the pins notice)
        path = os.environ.get("PQC_ORACLE_LIB") or _build.LIB
        if not os.path.exists(path):
            _build.build()
        _LIB = C.CDLL(path)
        for name in ("pqo_kmeans", "pqo_pq_build", "pqo_nearest_codes", "pqo_scores",
                     "pqo_exact_scores", "pqo_select", "pqo_attention", "pqo_decode",
                     "pqo_block_counts", "pqo_block_topk", "pqo_threads"):
            getattr(_LIB, name).restype = C.c_int
    return _LIB


def _dt(dtype: str) -> int:
    return {"f32": 0, "bf16": 1}[dtype]


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(rc: int, what: str) -> None:
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def _stored(a: np.ndarray, dtype: str) -> np.ndarray:
    want = np.float32 if dtype == "f32" else np.uint16
    assert a.dtype == want, (a.dtype, want)
    return np.ascontiguousarray(a)


def threads() -> int:
    return int(lib().pqo_threads())


def kmeans(x: np.ndarray, n_centroids: int, iters: int, init_idx: np.ndarray):
    """Lloyd K-Means on x [n, dm] f32 -> (centroids [c, dm] f32, codes [n] u8, inertia [iters+1])."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    n, dm = x.shape
    init_idx = np.ascontiguousarray(init_idx, dtype=np.int32)
    assert init_idx.shape == (n_centroids,)
    cent = np.empty((n_centroids, dm), np.float32)
    codes = np.empty(n, np.uint8)
    inertia = np.empty(iters + 1, np.float64)
    _chk(lib().pqo_kmeans(_p(x), C.c_int64(n), dm, n_centroids, iters, _p(init_idx), _p(cent),
                          _p(codes), _p(inertia)), "kmeans")
    return cent, codes, inertia


def pq_build(keys: np.ndarray, dtype: str, pq_m: int, n_centroids: int, iters: int,
             init_idx: np.ndarray):
    """keys [B,Hkv,N,D] -> (centroids [B,Hkv,M,C,Dm] f32, codes [B,Hkv,N,M] u8, inertia [B,Hkv,M,iters+1])."""
    keys = _stored(keys, dtype)
    B, Hkv, N, D = keys.shape
    init_idx = np.ascontiguousarray(init_idx, dtype=np.int32)
    assert init_idx.shape == (B, Hkv, pq_m, n_centroids)
    cent = np.empty((B, Hkv, pq_m, n_centroids, D // pq_m), np.float32)
    codes = np.empty((B, Hkv, N, pq_m), np.uint8)
    inertia = np.empty((B, Hkv, pq_m, iters + 1), np.float64)
    _chk(lib().pqo_pq_build(_p(keys), _dt(dtype), B, Hkv, C.c_int64(N), D, pq_m, n_centroids, iters,
                            _p(init_idx), _p(cent), _p(codes), _p(inertia)), "pq_build")
    return cent, codes, inertia


def nearest_codes(key: np.ndarray, dtype: str, centroids: np.ndarray) -> np.ndarray:
    """key [B,Hkv,D], centroids [B,Hkv,M,C,Dm] -> code [B,Hkv,M] u8."""
    key = _stored(key, dtype)
    centroids = np.ascontiguousarray(centroids, dtype=np.float32)
    B, Hkv, M, Cn, Dm = centroids.shape
    assert key.shape == (B, Hkv, M * Dm)
    out = np.empty((B, Hkv, M), np.uint8)
    _chk(lib().pqo_nearest_codes(_p(key), _dt(dtype), _p(centroids), B, Hkv, M * Dm, M, Cn, _p(out)),
         "nearest_codes")
    return out


def scores(q: np.ndarray, dtype: str, centroids: np.ndarray, codes: np.ndarray):
    """-> (score32 [B,Hkv,N] f32 in the reference fp32 order, score64 [B,Hkv,N] f64)."""
    q = _stored(q, dtype)
    centroids = np.ascontiguousarray(centroids, dtype=np.float32)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    B, Hq, D = q.shape
    _, Hkv, M, Cn, Dm = centroids.shape
    N = codes.shape[2]
    assert codes.shape == (B, Hkv, N, M) and M * Dm == D
    s32 = np.empty((B, Hkv, N), np.float32)
    s64 = np.empty((B, Hkv, N), np.float64)
    _chk(lib().pqo_scores(_p(q), _dt(dtype), _p(centroids), _p(codes), B, Hq, Hkv, C.c_int64(N), D, M,
                          Cn, _p(s32), _p(s64)), "scores")
    return s32, s64


def exact_scores(q: np.ndarray, k: np.ndarray, dtype: str) -> np.ndarray:
    q = _stored(q, dtype)
    k = _stored(k, dtype)
    B, Hq, D = q.shape
    _, Hkv, N, _ = k.shape
    out = np.empty((B, Hkv, N), np.float64)
    _chk(lib().pqo_exact_scores(_p(q), _p(k), _dt(dtype), B, Hq, Hkv, C.c_int64(N), D, _p(out)),
         "exact_scores")
    return out


def select(score32: np.ndarray, topk: int, n_init: int, n_local: int) -> np.ndarray:
    """score32 [B,Hkv,N] -> idx [B,Hkv,I+K+L] int32 (initial asc, retrieved best first, local asc)."""
    score32 = np.ascontiguousarray(score32, dtype=np.float32)
    B, Hkv, N = score32.shape
    out = np.empty((B, Hkv, n_init + topk + n_local), np.int32)
    _chk(lib().pqo_select(_p(score32), B, Hkv, C.c_int64(N), C.c_int64(topk), C.c_int64(n_init),
                          C.c_int64(n_local), _p(out)), "select")
    return out


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, dtype: str, idx: np.ndarray,
              scale: float) -> np.ndarray:
    """Softmax attention of every query head over the listed tokens of its KV head -> [B,Hq,D] f64."""
    q, k, v = _stored(q, dtype), _stored(k, dtype), _stored(v, dtype)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    B, Hq, D = q.shape
    _, Hkv, N, _ = k.shape
    assert v.shape == k.shape and idx.shape[:2] == (B, Hkv)
    out = np.empty((B, Hq, D), np.float64)
    _chk(lib().pqo_attention(_p(q), _p(k), _p(v), _dt(dtype), B, Hq, Hkv, C.c_int64(N), D, _p(idx),
                             C.c_int64(idx.shape[2]), C.c_double(scale), _p(out)), "attention")
    return out


def decode(q, centroids, codes, k, v, dtype: str, topk: int, n_init: int, n_local: int, scale: float):
    """Scores -> selection -> attention in one call -> (idx [B,Hkv,I+K+L], out [B,Hq,D] f64, score32)."""
    q, k, v = _stored(q, dtype), _stored(k, dtype), _stored(v, dtype)
    centroids = np.ascontiguousarray(centroids, dtype=np.float32)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    B, Hq, D = q.shape
    _, Hkv, N, _ = k.shape
    M, Cn = centroids.shape[2], centroids.shape[3]
    s32 = np.empty((B, Hkv, N), np.float32)
    idx = np.empty((B, Hkv, n_init + topk + n_local), np.int32)
    out = np.empty((B, Hq, D), np.float64)
    _chk(lib().pqo_decode(_p(q), _p(centroids), _p(codes), _p(k), _p(v), _dt(dtype), B, Hq, Hkv,
                          C.c_int64(N), D, M, Cn, C.c_int64(topk), C.c_int64(n_init), C.c_int64(n_local),
                          C.c_double(scale), _p(s32), _p(idx), _p(out)), "decode")
    return idx, out, s32


def block_counts(idx: np.ndarray, n_tokens: int, block: int) -> np.ndarray:
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    B, Hkv, n_idx = idx.shape
    nb = (n_tokens + block - 1) // block
    out = np.empty((B, Hkv, nb), np.int32)
    _chk(lib().pqo_block_counts(_p(idx), B, Hkv, C.c_int64(n_tokens), C.c_int64(n_idx), block, _p(out)),
         "block_counts")
    return out


def block_topk(counts: np.ndarray, k_cache: int) -> np.ndarray:
    """The k_cache blocks with the most selected tokens, best first (ties: lower block index)."""
    counts = np.ascontiguousarray(counts, dtype=np.int32)
    B, Hkv, nb = counts.shape
    out = np.empty((B, Hkv, k_cache), np.int32)
    _chk(lib().pqo_block_topk(_p(counts), B, Hkv, C.c_int64(nb), C.c_int64(k_cache), _p(out)), "block_topk")
    return out


def block_cache_update(slot_block: np.ndarray, slot_stamp: np.ndarray, slot_uses: np.ndarray, counts: np.ndarray,
                       blocks: np.ndarray, step: int, policy: str):
    """One refresh of the block-level cache of Section 3.4, for every unit, written out sequentially.

    State per unit: n_slots slots, each empty (block -1) or holding a block with the step of its last use
    (`stamp`) and the number of steps in which it was requested (`uses`).  `counts` [B,Hkv,nb] are this
    step's retrieved tokens per block, `blocks` [B,Hkv,k_cache] the blocks the step requests (the k_cache
    blocks holding the most retrieved tokens), in the order they are to be served; entries that are not
    block numbers (outside [0, nb)) are skipped.

    The retrieved tokens are first looked up in the cache as it stands: hit_tokens = retrieved tokens that
    lie in resident blocks, hit_blocks = requested blocks that are resident.  Then the cache is refreshed:
    a requested resident block is marked used (stamp = step, uses + 1); a requested absent block takes the
    lowest-numbered empty slot, or else replaces the victim of the policy among the slots not requested in
    this step -- "lru": the oldest stamp, "lfu": the fewest uses, then the oldest stamp; remaining ties go
    to the lowest slot -- and starts with stamp = step, uses = 1; when every slot holds a block requested
    in this step the remaining requests are dropped.

    Returns (slot_block, slot_stamp, slot_uses, stats [B,Hkv,4] = hit_tokens, hit_blocks, inserted, evicted).
    """
    assert policy in ("lru", "lfu")
    sb, ss, su = (np.array(a, dtype=np.int32, copy=True) for a in (slot_block, slot_stamp, slot_uses))
    B, Hkv, n_slots = sb.shape
    stats = np.zeros((B, Hkv, 4), np.int32)
    for b in range(B):
        for g in range(Hkv):
            blk, stamp, uses = sb[b, g], ss[b, g], su[b, g]
            nb = counts.shape[-1]
            wanted = [int(v) for v in blocks[b, g] if 0 <= int(v) < nb]  # anything else is not a block: skipped
            resident = {int(x): s for s, x in enumerate(blk) if x >= 0}
            stats[b, g, 0] = sum(int(counts[b, g, x]) for x in resident)
            stats[b, g, 1] = sum(1 for x in wanted if x in resident)
            requested_slots = set()
            for x in wanted:
                if x in resident:
                    s = resident[x]
                    stamp[s] = step
                    uses[s] += 1
                    requested_slots.add(s)
            for x in wanted:
                if x in resident:
                    continue
                empty = [s for s in range(n_slots) if blk[s] < 0]
                if empty:
                    s = empty[0]
                else:
                    free = [s for s in range(n_slots) if s not in requested_slots]
                    if not free:
                        break
                    if policy == "lru":
                        s = min(free, key=lambda t: (int(stamp[t]), t))
                    else:
                        s = min(free, key=lambda t: (int(uses[t]), int(stamp[t]), t))
                    del resident[int(blk[s])]
                    stats[b, g, 3] += 1
                blk[s], stamp[s], uses[s] = x, step, 1
                resident[x] = s
                requested_slots.add(s)
                stats[b, g, 2] += 1
    return sb, ss, su, stats
