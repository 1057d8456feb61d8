"""ctypes binding over the C ABI of libpqcache (include/pqcache.h).

Argument marshalling only: every step of the decode path runs in the HIP kernels of
the shared library.  PyTorch supplies device memory and the current stream.  There
is no fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import dataclasses
import os
from typing import Optional, Tuple

import torch

from .workloads import Workload

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpqcache.so")

PQC_F32, PQC_BF16 = 0, 1
STATUS = {0: "PQC_OK", -1: "PQC_EINVAL", -2: "PQC_EUNSUPPORTED", -3: "PQC_EWORKSPACE", -4: "PQC_EHIP", -5: "PQC_ESCRATCH"}


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("batch", "n_q_heads", "n_kv_heads", "head_dim", "n_tokens", "pq_m",
                                         "pq_centroids", "topk", "n_init", "n_local", "kv_dtype")] + [
                                             ("softmax_scale", C.c_float), ("n_capacity", C.c_int32)]


_lib = None


def load() -> C.CDLL:
    """Load libpqcache.so, compiling it first if it has not been built; raises if that fails (there is no other path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        # nothing built yet: compile the library now (hipcc cross-compiles gfx950 without a GPU)
        from . import build as _build

        if os.path.abspath(LIB_PATH) == os.path.abspath(_build.LIB):
            _build.build()
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing and could not be built with `python -m paper_2407_12820_amd.build` "
                           "(the decode path has no CPU or PyTorch fallback)")
    lib = C.CDLL(LIB_PATH)
    vp, cp = C.c_void_p, C.POINTER(Config)
    lib.pqc_version.restype = C.c_int
    lib.pqc_strerror.restype = C.c_char_p
    lib.pqc_strerror.argtypes = [C.c_int]
    lib.pqc_workspace_bytes.restype = C.c_size_t
    lib.pqc_workspace_bytes.argtypes = [cp]
    lib.pqc_create.restype = C.c_int
    lib.pqc_create.argtypes = [C.POINTER(vp), cp, vp, C.c_size_t]
    lib.pqc_set_length.restype = C.c_int
    lib.pqc_set_length.argtypes = [vp, C.c_int32, C.c_int32]
    lib.pqc_destroy.restype = None
    lib.pqc_destroy.argtypes = [vp]
    lib.pqc_last_hip_error.restype = C.c_int
    lib.pqc_last_hip_error.argtypes = [vp]
    lib.pqc_decode.restype = C.c_int
    lib.pqc_decode.argtypes = [vp] * 9
    lib.pqc_static_scratch_bytes.restype = C.c_size_t
    lib.pqc_static_scratch_bytes.argtypes = []
    lib.pqc_decode_static.restype = C.c_int
    lib.pqc_decode_static.argtypes = [cp] + [vp] * 8
    lib.pqc_decode_append.restype = C.c_int
    lib.pqc_decode_append.argtypes = [vp] * 7 + [C.c_int32] + [vp] * 3
    lib.pqc_decode_indexed_append.restype = C.c_int
    lib.pqc_decode_indexed_append.argtypes = [vp] * 8 + [C.c_int32] + [vp] * 3
    lib.pqc_decode_phase.restype = C.c_int
    lib.pqc_decode_phase.argtypes = [vp, C.c_int] + [vp] * 8
    lib.pqc_lut.restype = C.c_int
    lib.pqc_lut.argtypes = [vp] * 5
    lib.pqc_scan.restype = C.c_int
    lib.pqc_scan.argtypes = [vp] * 5
    lib.pqc_topk.restype = C.c_int
    lib.pqc_topk.argtypes = [vp] * 4
    lib.pqc_gather_attn.restype = C.c_int
    lib.pqc_gather_attn.argtypes = [vp] * 7
    lib.pqc_pq_build_workspace_bytes.restype = C.c_size_t
    lib.pqc_pq_build_workspace_bytes.argtypes = [cp]
    lib.pqc_pq_build.restype = C.c_int
    lib.pqc_pq_build.argtypes = [cp, vp, vp, C.c_int32, vp, vp, vp, C.c_size_t, vp]
    lib.pqc_pq_assign.restype = C.c_int
    lib.pqc_pq_assign.argtypes = [cp, vp, vp, vp, vp]
    lib.pqc_pq_encode_token.restype = C.c_int
    lib.pqc_pq_encode_token.argtypes = [cp, vp, vp, vp, C.c_int32, vp]
    lib.pqc_decode_indexed.restype = C.c_int
    lib.pqc_decode_indexed.argtypes = [vp] * 10
    lib.pqc_pair_counts.restype = C.c_int
    lib.pqc_pair_counts.argtypes = [cp, vp, vp, vp]
    lib.pqc_pair_counts_add.restype = C.c_int
    lib.pqc_pair_counts_add.argtypes = [cp, vp, C.c_int32, vp, vp]
    lib.pqc_block_cache_update.restype = C.c_int
    lib.pqc_block_cache_update.argtypes = [cp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp, vp, C.c_int32, vp, vp, vp, vp, vp]
    lib.pqc_block_stats.restype = C.c_int
    lib.pqc_block_stats.argtypes = [cp, vp, C.c_int64, C.c_int32, C.c_int32, vp, vp, vp]
    _lib = lib
    return lib


def make_config(w: Workload, softmax_scale: float = 0.0, capacity: int = 0) -> Config:
    """capacity: tokens the K/V, key and code tensors have room for per head (0: exactly n_tokens)."""
    return Config(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_tokens, w.pq_m, w.pq_centroids, w.topk,
                  w.n_init, w.n_local, PQC_F32 if w.dtype == "f32" else PQC_BF16, softmax_scale, capacity)


class PQCacheError(RuntimeError):
    def __init__(self, status: int, what: str, hip: int = 0):
        self.status = status
        msg = load().pqc_strerror(status).decode()
        super().__init__(f"{what}: {STATUS.get(status, status)} ({msg})" + (f", hipError {hip}" if hip else ""))


class PQCache:
    """One decode context: a configuration plus its device workspace."""

    def __init__(self, w: Workload, device: str = "cuda:0", softmax_scale: float = 0.0, capacity: int = 0):
        self.lib = load()
        self.w = w
        self.capacity = capacity or w.n_tokens
        self.device = torch.device(device)
        self.cfg = make_config(w, softmax_scale, capacity)
        nbytes = self.lib.pqc_workspace_bytes(C.byref(self.cfg))
        if nbytes == 0:
            # let pqc_create say why
            h = C.c_void_p()
            raise PQCacheError(self.lib.pqc_create(C.byref(h), C.byref(self.cfg), None, 0), "pqc_create")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.handle = C.c_void_p()
        rc = self.lib.pqc_create(C.byref(self.handle), C.byref(self.cfg), self.workspace.data_ptr(), nbytes)
        if rc != 0:
            raise PQCacheError(rc, "pqc_create")
        self.kv_torch = torch.float32 if w.dtype == "f32" else torch.bfloat16

    def set_length(self, n_tokens: int, topk: int) -> None:
        """The cache now holds n_tokens tokens (<= capacity) and topk of the middle ones are retrieved."""
        self._check(self.lib.pqc_set_length(self.handle, n_tokens, topk), "pqc_set_length")
        self.w = dataclasses.replace(self.w, n_tokens=n_tokens, topk=topk)
        self.cfg.n_tokens, self.cfg.topk = n_tokens, topk

    def close(self) -> None:
        if getattr(self, "handle", None) is not None and self.handle.value:
            self.lib.pqc_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- marshalling helpers
    def _ptr(self, t: torch.Tensor, dtype, shape) -> int:
        if t.device != self.device or not t.is_contiguous():
            raise ValueError("tensor must be contiguous and on the context's device")
        if t.dtype != dtype or tuple(t.shape) != tuple(shape):
            raise ValueError(f"expected {dtype} {tuple(shape)}, got {t.dtype} {tuple(t.shape)}")
        return t.data_ptr()

    def _stream(self, stream) -> int:
        s = stream if stream is not None else torch.cuda.current_stream(self.device)
        return s.cuda_stream

    def _check(self, rc: int, what: str) -> None:
        if rc != 0:
            raise PQCacheError(rc, what, self.lib.pqc_last_hip_error(self.handle))

    # -- shapes
    @property
    def shapes(self):
        w = self.w
        return {
            "q": (w.batch, w.n_q_heads, w.head_dim),
            "centroids": (w.batch, w.n_kv_heads, w.pq_m, w.pq_centroids, w.sub_dim),
            "codes": (w.batch, w.n_kv_heads, self.capacity, w.pq_m),
            "kv": (w.batch, w.n_kv_heads, self.capacity, w.head_dim),
            "idx": (w.batch, w.n_kv_heads, w.n_selected),
            "out": (w.batch, w.n_q_heads, w.head_dim),
            "table": (w.batch, w.n_kv_heads, w.pq_m, w.pq_centroids),
            "scores": (w.batch, w.n_kv_heads, w.n_tokens),
        }

    def empty_outputs(self) -> Tuple[torch.Tensor, torch.Tensor]:
        sh = self.shapes
        return (torch.empty(sh["idx"], dtype=torch.int32, device=self.device),
                torch.empty(sh["out"], dtype=torch.float32, device=self.device))

    # -- entry points (same names as the C ABI)
    def decode(self, q, centroids, codes, k_cache, v_cache, out_idx=None, out_attn=None, stream=None):
        sh = self.shapes
        if out_idx is None or out_attn is None:
            out_idx, out_attn = self.empty_outputs()
        rc = self.lib.pqc_decode(self.handle, self._ptr(q, self.kv_torch, sh["q"]),
                                 self._ptr(centroids, torch.float32, sh["centroids"]),
                                 self._ptr(codes, torch.uint8, sh["codes"]),
                                 self._ptr(k_cache, self.kv_torch, sh["kv"]), self._ptr(v_cache, self.kv_torch, sh["kv"]),
                                 self._ptr(out_idx, torch.int32, sh["idx"]), self._ptr(out_attn, torch.float32, sh["out"]),
                                 self._stream(stream))
        self._check(rc, "pqc_decode")
        return out_idx, out_attn

    def decode_append(self, q, centroids, codes, k_cache, v_cache, new_key, position: int, out_idx=None, out_attn=None,
                      stream=None):
        """pqc_decode plus the code of the token at `position` (its key: new_key [B,Hkv,D]), in the same launches."""
        sh = self.shapes
        if out_idx is None or out_attn is None:
            out_idx, out_attn = self.empty_outputs()
        w = self.w
        rc = self.lib.pqc_decode_append(self.handle, self._ptr(q, self.kv_torch, sh["q"]),
                                        self._ptr(centroids, torch.float32, sh["centroids"]),
                                        self._ptr(codes, torch.uint8, sh["codes"]),
                                        self._ptr(k_cache, self.kv_torch, sh["kv"]), self._ptr(v_cache, self.kv_torch, sh["kv"]),
                                        self._ptr(new_key, self.kv_torch, (w.batch, w.n_kv_heads, w.head_dim)), position,
                                        self._ptr(out_idx, torch.int32, sh["idx"]), self._ptr(out_attn, torch.float32, sh["out"]),
                                        self._stream(stream))
        self._check(rc, "pqc_decode_append")
        return out_idx, out_attn

    def decode_indexed_append(self, q, centroids, codes, pair_counts, k_cache, v_cache, new_key, position: int, out_idx=None,
                              out_attn=None, stream=None):
        """pqc_decode_indexed plus the code (and the counted code pair) of the token at `position`."""
        if out_idx is None or out_attn is None:
            out_idx, out_attn = self.empty_outputs()
        qp, cp, cdp, kp, vp_, oi, oa = self.marshal_decode_args(q, centroids, codes, k_cache, v_cache, out_idx, out_attn)
        w = self.w
        rc = self.lib.pqc_decode_indexed_append(self.handle, qp, cp, cdp, self._pair_ptr(pair_counts), kp, vp_,
                                                self._ptr(new_key, self.kv_torch, (w.batch, w.n_kv_heads, w.head_dim)), position,
                                                oi, oa, self._stream(stream))
        self._check(rc, "pqc_decode_indexed_append")
        return out_idx, out_attn

    def marshal_decode_args(self, q, centroids, codes, k_cache, v_cache, out_idx, out_attn):
        """Checks the seven tensors of a decode call once and returns their device addresses, for
        callers that repeat the same call and want the per-call Python cost out of the way."""
        sh = self.shapes
        return (self._ptr(q, self.kv_torch, sh["q"]), self._ptr(centroids, torch.float32, sh["centroids"]),
                self._ptr(codes, torch.uint8, sh["codes"]), self._ptr(k_cache, self.kv_torch, sh["kv"]),
                self._ptr(v_cache, self.kv_torch, sh["kv"]), self._ptr(out_idx, torch.int32, sh["idx"]),
                self._ptr(out_attn, torch.float32, sh["out"]))

    def decode_marshalled(self, args, stream_handle: int) -> None:
        self._check(self.lib.pqc_decode(self.handle, *args, stream_handle), "pqc_decode")

    def decode_indexed(self, q, centroids, codes, pair_counts, k_cache, v_cache, out_idx=None, out_attn=None, stream=None):
        """pqc_decode_indexed: the same step with the threshold taken from code-pair counts (two partitions)."""
        if out_idx is None or out_attn is None:
            out_idx, out_attn = self.empty_outputs()
        a = self.marshal_decode_args(q, centroids, codes, k_cache, v_cache, out_idx, out_attn)
        self.decode_indexed_marshalled(a, self._pair_ptr(pair_counts), self._stream(stream))
        return out_idx, out_attn

    def _pair_ptr(self, pair_counts) -> int:
        w = self.w
        return self._ptr(pair_counts, torch.int32, (w.batch, w.n_kv_heads, w.pq_centroids * w.pq_centroids))

    def decode_indexed_marshalled(self, args, pair_ptr: int, stream_handle: int) -> None:
        q, cent, codes, k, v, oi, oa = args
        self._check(self.lib.pqc_decode_indexed(self.handle, q, cent, codes, pair_ptr, k, v, oi, oa, stream_handle),
                    "pqc_decode_indexed")

    def decode_phase_marshalled(self, phase: int, args, stream_handle: int) -> None:
        """One kernel of pqc_decode (0 histogram, 1 select + attention, 2 finalize); see the header."""
        self._check(self.lib.pqc_decode_phase(self.handle, phase, *args, stream_handle), "pqc_decode_phase")

    def decode_phase(self, phase, q, centroids, codes, k_cache, v_cache, out_idx, out_attn, stream=None):
        self.decode_phase_marshalled(int(phase), self.marshal_decode_args(q, centroids, codes, k_cache, v_cache, out_idx, out_attn),
                                     self._stream(stream))

    def lut(self, q, centroids, table=None, stream=None):
        sh = self.shapes
        if table is None:
            table = torch.empty(sh["table"], dtype=torch.float32, device=self.device)
        rc = self.lib.pqc_lut(self.handle, self._ptr(q, self.kv_torch, sh["q"]),
                              self._ptr(centroids, torch.float32, sh["centroids"]),
                              self._ptr(table, torch.float32, sh["table"]), self._stream(stream))
        self._check(rc, "pqc_lut")
        return table

    def scan(self, table, codes, scores=None, stream=None):
        sh = self.shapes
        if scores is None:
            scores = torch.empty(sh["scores"], dtype=torch.float32, device=self.device)
        rc = self.lib.pqc_scan(self.handle, self._ptr(table, torch.float32, sh["table"]),
                               self._ptr(codes, torch.uint8, sh["codes"]),
                               self._ptr(scores, torch.float32, sh["scores"]), self._stream(stream))
        self._check(rc, "pqc_scan")
        return scores

    def topk(self, scores, out_idx=None, stream=None):
        sh = self.shapes
        if out_idx is None:
            out_idx = torch.empty(sh["idx"], dtype=torch.int32, device=self.device)
        rc = self.lib.pqc_topk(self.handle, self._ptr(scores, torch.float32, sh["scores"]),
                               self._ptr(out_idx, torch.int32, sh["idx"]), self._stream(stream))
        self._check(rc, "pqc_topk")
        return out_idx

    def gather_attn(self, q, k_cache, v_cache, idx, out_attn=None, stream=None):
        sh = self.shapes
        if out_attn is None:
            out_attn = torch.empty(sh["out"], dtype=torch.float32, device=self.device)
        rc = self.lib.pqc_gather_attn(self.handle, self._ptr(q, self.kv_torch, sh["q"]),
                                      self._ptr(k_cache, self.kv_torch, sh["kv"]), self._ptr(v_cache, self.kv_torch, sh["kv"]),
                                      self._ptr(idx, torch.int32, sh["idx"]), self._ptr(out_attn, torch.float32, sh["out"]),
                                      self._stream(stream))
        self._check(rc, "pqc_gather_attn")
        return out_attn


def _kv_dtype(w: Workload):
    return torch.float32 if w.dtype == "f32" else torch.bfloat16


def _need(t: torch.Tensor, dtype, shape, what: str) -> int:
    if not t.is_cuda or not t.is_contiguous() or t.dtype != dtype or tuple(t.shape) != tuple(shape):
        raise ValueError(f"{what}: expected contiguous device {dtype} {tuple(shape)}, got {t.dtype} {tuple(t.shape)}")
    return t.data_ptr()


def decode_static(w: Workload, q, centroids, codes, k_cache, v_cache, out_idx, out_attn, stream=None, capacity: int = 0,
                  softmax_scale: float = 0.0) -> None:
    """pqc_decode_static: the decode step on the library's own static scratch memory (no context, no workspace)."""
    lib = load()
    cfg = make_config(w, softmax_scale, capacity)
    ntok = capacity or w.n_tokens
    kvt = _kv_dtype(w)
    st = (stream if stream is not None else torch.cuda.current_stream(q.device)).cuda_stream
    rc = lib.pqc_decode_static(
        C.byref(cfg), _need(q, kvt, (w.batch, w.n_q_heads, w.head_dim), "q"),
        _need(centroids, torch.float32, (w.batch, w.n_kv_heads, w.pq_m, w.pq_centroids, w.sub_dim), "centroids"),
        _need(codes, torch.uint8, (w.batch, w.n_kv_heads, ntok, w.pq_m), "codes"),
        _need(k_cache, kvt, (w.batch, w.n_kv_heads, ntok, w.head_dim), "k_cache"),
        _need(v_cache, kvt, (w.batch, w.n_kv_heads, ntok, w.head_dim), "v_cache"),
        _need(out_idx, torch.int32, (w.batch, w.n_kv_heads, w.n_selected), "out_idx"),
        _need(out_attn, torch.float32, (w.batch, w.n_q_heads, w.head_dim), "out_attn"), st)
    if rc != 0:
        raise PQCacheError(rc, "pqc_decode_static")


def pq_build(w: Workload, keys: torch.Tensor, init_idx: torch.Tensor, iters: Optional[int] = None, stream=None,
             capacity: int = 0):
    """K-Means PQ construction on the GPU -> (centroids [B,Hkv,M,C,Dm] f32, codes [B,Hkv,N,M] u8).

    capacity (here and below): token room of `keys` and `codes` per head when it exceeds w.n_tokens."""
    lib = load()
    cfg = make_config(w, capacity=capacity)
    ntok = capacity or w.n_tokens
    dev = keys.device
    iters = w.kmeans_iters if iters is None else iters
    nbytes = lib.pqc_pq_build_workspace_bytes(C.byref(cfg))
    if nbytes == 0:
        raise PQCacheError(-1, "pqc_pq_build_workspace_bytes")
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    cent = torch.empty((w.batch, w.n_kv_heads, w.pq_m, w.pq_centroids, w.sub_dim), dtype=torch.float32, device=dev)
    codes = torch.zeros((w.batch, w.n_kv_heads, ntok, w.pq_m), dtype=torch.uint8, device=dev)
    st = (stream if stream is not None else torch.cuda.current_stream(dev)).cuda_stream
    rc = lib.pqc_pq_build(C.byref(cfg), _need(keys, _kv_dtype(w), (w.batch, w.n_kv_heads, ntok, w.head_dim), "keys"),
                          _need(init_idx, torch.int32, (w.batch, w.n_kv_heads, w.pq_m, w.pq_centroids), "init_idx"),
                          iters, cent.data_ptr(), codes.data_ptr(), ws.data_ptr(), nbytes, st)
    if rc != 0:
        raise PQCacheError(rc, "pqc_pq_build")
    return cent, codes


def pq_assign(w: Workload, keys: torch.Tensor, centroids: torch.Tensor, stream=None, capacity: int = 0) -> torch.Tensor:
    lib = load()
    cfg = make_config(w, capacity=capacity)
    ntok = capacity or w.n_tokens
    dev = keys.device
    codes = torch.zeros((w.batch, w.n_kv_heads, ntok, w.pq_m), dtype=torch.uint8, device=dev)
    st = (stream if stream is not None else torch.cuda.current_stream(dev)).cuda_stream
    rc = lib.pqc_pq_assign(C.byref(cfg), _need(keys, _kv_dtype(w), (w.batch, w.n_kv_heads, ntok, w.head_dim), "keys"),
                           _need(centroids, torch.float32, (w.batch, w.n_kv_heads, w.pq_m, w.pq_centroids, w.sub_dim), "centroids"),
                           codes.data_ptr(), st)
    if rc != 0:
        raise PQCacheError(rc, "pqc_pq_assign")
    return codes


def pq_encode_token(w: Workload, key: torch.Tensor, centroids: torch.Tensor, codes: torch.Tensor, position: int,
                    stream=None, capacity: int = 0) -> None:
    """Write the nearest-centroid codes of one new key per (sequence, KV head) at `position` of `codes`."""
    lib = load()
    cfg = make_config(w, capacity=capacity)
    st = (stream if stream is not None else torch.cuda.current_stream(key.device)).cuda_stream
    rc = lib.pqc_pq_encode_token(C.byref(cfg), _need(key, _kv_dtype(w), (w.batch, w.n_kv_heads, w.head_dim), "key"),
                                 _need(centroids, torch.float32, (w.batch, w.n_kv_heads, w.pq_m, w.pq_centroids, w.sub_dim), "centroids"),
                                 _need(codes, torch.uint8, (w.batch, w.n_kv_heads, capacity or w.n_tokens, w.pq_m), "codes"),
                                 position, st)
    if rc != 0:
        raise PQCacheError(rc, "pqc_pq_encode_token")


def pair_counts(w: Workload, codes: torch.Tensor, stream=None, capacity: int = 0) -> torch.Tensor:
    """Tokens per pair of codes, [B][Hkv][C*C] (uint32 values in an int32 tensor); two partitions only."""
    lib = load()
    cfg = make_config(w, capacity=capacity)
    _need(codes, torch.uint8, (w.batch, w.n_kv_heads, capacity or w.n_tokens, w.pq_m), "codes")
    out = torch.empty((w.batch, w.n_kv_heads, w.pq_centroids * w.pq_centroids), dtype=torch.int32, device=codes.device)
    st = (stream if stream is not None else torch.cuda.current_stream(codes.device)).cuda_stream
    rc = lib.pqc_pair_counts(C.byref(cfg), codes.data_ptr(), out.data_ptr(), st)
    if rc != 0:
        raise PQCacheError(rc, "pqc_pair_counts")
    return out


def pair_counts_add(w: Workload, codes: torch.Tensor, position: int, counts: torch.Tensor, stream=None,
                    capacity: int = 0) -> None:
    lib = load()
    cfg = make_config(w, capacity=capacity)
    st = (stream if stream is not None else torch.cuda.current_stream(codes.device)).cuda_stream
    rc = lib.pqc_pair_counts_add(C.byref(cfg), codes.data_ptr(), position, counts.data_ptr(), st)
    if rc != 0:
        raise PQCacheError(rc, "pqc_pair_counts_add")


def block_stats(w: Workload, idx: torch.Tensor, block_tokens: int, k_cache: int, stream=None):
    """Listed tokens per block and the k_cache fullest blocks -> (counts [B][Hkv][nb], blocks [B][Hkv][k_cache])."""
    lib = load()
    cfg = make_config(w)
    if idx.dtype != torch.int32 or idx.dim() != 3 or tuple(idx.shape[:2]) != (w.batch, w.n_kv_heads) or not idx.is_contiguous():
        raise ValueError("idx must be a contiguous int32 tensor [B][Hkv][n_idx]")
    nb = (w.n_tokens + block_tokens - 1) // block_tokens
    counts = torch.empty((w.batch, w.n_kv_heads, nb), dtype=torch.int32, device=idx.device)
    blocks = torch.empty((w.batch, w.n_kv_heads, k_cache), dtype=torch.int32, device=idx.device)
    st = (stream if stream is not None else torch.cuda.current_stream(idx.device)).cuda_stream
    rc = lib.pqc_block_stats(C.byref(cfg), idx.data_ptr(), idx.shape[2], block_tokens, k_cache, counts.data_ptr(),
                             blocks.data_ptr() if k_cache > 0 else None, st)
    if rc != 0:
        raise PQCacheError(rc, "pqc_block_stats")
    return counts, blocks


def to_device(a, dtype: str, device="cuda:0") -> torch.Tensor:
    """Upload a numpy array produced by `workloads` (bf16 arrives as uint16 bit patterns)."""
    import numpy as np

    if a.dtype == np.uint16 and dtype == "bf16":
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


def block_cache_update(w: Workload, block_tokens: int, policy: str, step: int, counts: torch.Tensor, blocks: torch.Tensor,
                       slot_block: torch.Tensor, slot_stamp: torch.Tensor, slot_uses: torch.Tensor, stream=None) -> torch.Tensor:
    """One look-up and refresh of the block cache state (updated in place) -> stats [B,Hkv,4] int32."""
    lib = load()
    cfg = make_config(w)
    nb = (w.n_tokens + block_tokens - 1) // block_tokens
    n_slots, k_cache = slot_block.shape[-1], blocks.shape[-1]
    _need(counts, torch.int32, (w.batch, w.n_kv_heads, nb), "counts")
    _need(blocks, torch.int32, (w.batch, w.n_kv_heads, k_cache), "blocks")
    for t, name in ((slot_block, "slot_block"), (slot_stamp, "slot_stamp"), (slot_uses, "slot_uses")):
        _need(t, torch.int32, (w.batch, w.n_kv_heads, n_slots), name)
    stats = torch.empty((w.batch, w.n_kv_heads, 4), dtype=torch.int32, device=counts.device)
    st = (stream if stream is not None else torch.cuda.current_stream(counts.device)).cuda_stream
    rc = lib.pqc_block_cache_update(C.byref(cfg), block_tokens, n_slots, {"lru": 0, "lfu": 1}[policy], step, counts.data_ptr(),
                                    blocks.data_ptr() if k_cache else None, k_cache, slot_block.data_ptr(),
                                    slot_stamp.data_ptr(), slot_uses.data_ptr(), stats.data_ptr(), st)
    if rc != 0:
        raise PQCacheError(rc, "pqc_block_cache_update")
    return stats
