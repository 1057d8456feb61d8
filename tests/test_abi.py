"""Host-only checks of the C ABI: the library loads without a GPU, exports every symbol the
header declares, and its host logic (configuration checks, workspace sizing) behaves."""
import ctypes as C
import dataclasses
import os
import re

import numpy as np
import pytest

from paper_2407_12820_amd import binding, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            text = open(os.path.join(ROOT, "include", fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(pqc_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = binding.load()
    names = _declared()
    assert {"pqc_decode", "pqc_lut", "pqc_scan", "pqc_topk", "pqc_gather_attn", "pqc_create", "pqc_destroy",
            "pqc_workspace_bytes", "pqc_strerror", "pqc_version", "pqc_last_hip_error"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_version_and_messages():
    lib = binding.load()
    assert lib.pqc_version() >= 100
    assert lib.pqc_strerror(0) == b"ok"
    assert len({lib.pqc_strerror(s) for s in (0, -1, -2, -3, -4, -99)}) == 6


def test_workspace_bytes_for_the_benchmark_shapes():
    lib = binding.load()
    for name in wl.CONFIG_ORDER:
        w = wl.CONFIGS[name]
        n = lib.pqc_workspace_bytes(C.byref(binding.make_config(w)))
        assert n > 0 and n % 256 == 0
        # a few words per cached token at most (staging of selected ids / candidates)
        assert n < 64 * w.batch * w.n_kv_heads * w.n_tokens + (1 << 22)


@pytest.mark.parametrize("change,status", [
    (dict(batch=0), -1), (dict(n_tokens=0), -1), (dict(n_kv_heads=3), -1), (dict(pq_m=3), -1),
    (dict(topk=4096), -1), (dict(topk=0, n_init=0, n_local=0), -1), (dict(dtype_code=7), -1),
    (dict(head_dim=64), -2), (dict(pq_centroids=257), -2), (dict(n_q_heads=16, n_kv_heads=1), -2),
    (dict(pq_m=16), -2), (dict(n_tokens=(1 << 22) + 1), -2),
])
def test_rejected_configurations(change, status):
    lib = binding.load()
    cfg = binding.make_config(wl.CONFIGS["tiny_f32"])
    for k, v in change.items():
        setattr(cfg, "kv_dtype" if k == "dtype_code" else k, v)
    assert lib.pqc_workspace_bytes(C.byref(cfg)) == 0
    h = C.c_void_p(123)
    assert lib.pqc_create(C.byref(h), C.byref(cfg), C.c_void_p(256), 1 << 30) == status
    assert not h.value


def test_create_checks_workspace_and_null_arguments():
    lib = binding.load()
    cfg = binding.make_config(wl.CONFIGS["tiny_f32"])
    need = lib.pqc_workspace_bytes(C.byref(cfg))
    h = C.c_void_p()
    assert lib.pqc_create(C.byref(h), C.byref(cfg), None, need) == -3
    assert lib.pqc_create(C.byref(h), C.byref(cfg), C.c_void_p(4096), need - 1) == -3
    assert lib.pqc_create(C.byref(h), C.byref(cfg), C.c_void_p(4096 + 16), need) == -3
    assert lib.pqc_create(None, C.byref(cfg), C.c_void_p(4096), need) == -1
    assert lib.pqc_create(C.byref(h), None, C.c_void_p(4096), need) == -1
    # a well-formed create is host-only: no device call happens until an entry point is used
    assert lib.pqc_create(C.byref(h), C.byref(cfg), C.c_void_p(4096), need) == 0 and h.value
    assert lib.pqc_decode(h, None, None, None, None, None, None, None, None) == -1
    assert lib.pqc_decode(None, *([C.c_void_p(16)] * 7), None) == -1
    assert lib.pqc_topk(h, C.c_void_p(8), C.c_void_p(16), None) == -1  # misaligned pointer
    assert lib.pqc_last_hip_error(h) == 0
    lib.pqc_destroy(h)
    lib.pqc_destroy(None)


def test_argument_checks_of_the_newer_entry_points():
    # all of these are refused on the host, before any device call
    lib = binding.load()
    tiny = wl.CONFIGS["tiny_f32"]            # M = 2, C = 64, N = 4096
    cfg = binding.make_config(tiny)
    p = C.c_void_p(4096)
    # block statistics: block size 1..2047, 0 <= k_cache <= number of blocks, blocks needed when k_cache > 0
    assert lib.pqc_block_stats(C.byref(cfg), p, 10, 0, 1, p, p, None) == -1
    assert lib.pqc_block_stats(C.byref(cfg), p, 10, 2048, 1, p, p, None) == -1
    assert lib.pqc_block_stats(C.byref(cfg), p, 10, 128, 33, p, p, None) == -1
    assert lib.pqc_block_stats(C.byref(cfg), p, 10, 128, 4, p, None, None) == -1
    assert lib.pqc_block_stats(C.byref(cfg), None, 10, 128, 4, p, p, None) == -1
    assert lib.pqc_block_stats(C.byref(cfg), p, -1, 128, 4, p, p, None) == -1
    # code-pair counts exist for two partitions of at most 64 centroids
    four = binding.make_config(wl.CONFIGS["batch8_32k"])
    assert lib.pqc_pair_counts(C.byref(four), p, p, None) == -2
    assert lib.pqc_pair_counts_add(C.byref(four), p, 0, p, None) == -2
    assert lib.pqc_pair_counts(C.byref(cfg), None, p, None) == -1
    assert lib.pqc_pair_counts_add(C.byref(cfg), p, 4096, p, None) == -1
    # decode phases 0..2 only; indexed decode needs its pair counts and a supported shape
    need = lib.pqc_workspace_bytes(C.byref(cfg))
    h = C.c_void_p()
    assert lib.pqc_create(C.byref(h), C.byref(cfg), C.c_void_p(4096), need) == 0
    assert lib.pqc_decode_phase(h, 3, *([p] * 7), None) == -1
    assert lib.pqc_decode_phase(h, -1, *([p] * 7), None) == -1
    assert lib.pqc_decode_indexed(h, p, p, p, None, p, p, p, p, None) == -1
    lib.pqc_destroy(h)
    need4 = lib.pqc_workspace_bytes(C.byref(four))
    assert lib.pqc_create(C.byref(h), C.byref(four), C.c_void_p(4096), need4) == 0
    assert lib.pqc_decode_indexed(h, *([p] * 9), None) == -2
    lib.pqc_destroy(h)


def test_workspace_for_a_capacity_covers_every_length():
    # a context that follows a growing cache keeps its workspace: the size reported for a capacity must
    # be at least the exact size of every shorter dense shape (lengths chosen around the grid's switch points)
    lib = binding.load()
    for base in ("llama8b_128k", "batch8_32k", "tiny_f32"):
        w = wl.get(base)
        cap = w.n_tokens
        small = dataclasses.replace(w, n_tokens=max(200, w.n_init + w.n_local + 8), topk=8)
        bound = lib.pqc_workspace_bytes(C.byref(binding.make_config(small, capacity=cap)))
        assert bound > 0
        lengths = sorted({cap, cap - 1, cap // 2, cap // 2 + 1, cap // 3, 4097, 4096, 2049, 1025, 513, 512, 511, 200} |
                         {int(x) for x in np.random.default_rng(5).integers(200, cap, 60)})
        for n in (x for x in lengths if x <= cap):
            for k in (0, (n - w.n_init - w.n_local) // 10, n - w.n_init - w.n_local):
                dense = dataclasses.replace(w, n_tokens=n, topk=k)
                need = lib.pqc_workspace_bytes(C.byref(binding.make_config(dense)))
                assert 0 < need <= bound, (base, n, k, need, bound)
                # the same length inside the capacity is planned the same way
                need_cap = lib.pqc_workspace_bytes(C.byref(binding.make_config(dense, capacity=cap)))
                assert need_cap == (need if n == cap else bound)


def test_set_length_checks():
    lib = binding.load()
    w = wl.get("llama8b_32k")
    cap = 40000
    cfg = binding.make_config(w, capacity=cap)
    need = lib.pqc_workspace_bytes(C.byref(cfg))
    h = C.c_void_p()
    assert lib.pqc_create(C.byref(h), C.byref(cfg), C.c_void_p(4096), need) == 0
    assert lib.pqc_set_length(None, 1000, 10) == -1
    assert lib.pqc_set_length(h, cap, 4000) == 0
    assert lib.pqc_set_length(h, cap + 1, 4000) == -1          # beyond the capacity
    assert lib.pqc_set_length(h, 1000, 1000) == -1             # I + K + L > N
    assert lib.pqc_set_length(h, 68, 0) == 0                   # windows only
    assert lib.pqc_set_length(h, 0, 0) == -1
    lib.pqc_destroy(h)
    # a workspace sized for the short dense shape cannot take a longer one
    short = dataclasses.replace(w, n_tokens=2000, topk=100)
    cfg2 = binding.make_config(short, capacity=cap)
    exact = lib.pqc_workspace_bytes(C.byref(binding.make_config(short)))
    assert lib.pqc_create(C.byref(h), C.byref(cfg2), C.c_void_p(4096), exact) == 0
    assert lib.pqc_set_length(h, cap, 4000) == -3
    assert lib.pqc_set_length(h, 1900, 100) == 0
    lib.pqc_destroy(h)
    # capacity below the length, or negative
    assert lib.pqc_workspace_bytes(C.byref(binding.make_config(w, capacity=w.n_tokens - 1))) == 0
    assert lib.pqc_workspace_bytes(C.byref(binding.make_config(w, capacity=-5))) == 0


def test_block_cache_update_argument_checks():
    lib = binding.load()
    cfg = binding.make_config(wl.get("llama8b_32k"))
    p = C.c_void_p(4096)
    ok = dict(block_tokens=128, n_slots=32, policy=0, step=1, counts=p, blocks=p, k_cache=32, sb=p, ss=p, su=p, stats=p)

    def call(**kw):
        a = dict(ok, **kw)
        return lib.pqc_block_cache_update(C.byref(cfg), a["block_tokens"], a["n_slots"], a["policy"], a["step"], a["counts"],
                                          a["blocks"], a["k_cache"], a["sb"], a["ss"], a["su"], a["stats"], None)

    for bad in (dict(block_tokens=0), dict(n_slots=0), dict(n_slots=1025), dict(policy=2), dict(policy=-1), dict(k_cache=-1),
                dict(k_cache=1025), dict(counts=None), dict(blocks=None), dict(sb=None), dict(ss=None), dict(su=None),
                dict(stats=None)):
        assert call(**bad) == -1, bad
    assert lib.pqc_block_cache_update(None, 128, 32, 0, 1, p, p, 32, p, p, p, p, None) == -1


def test_missing_library_is_an_error_not_a_fallback(monkeypatch):
    # no CPU or PyTorch stand-in exists: a library that is not there (and is not the one the
    # package knows how to build) must raise
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", os.path.join(ROOT, "paper_2407_12820_amd", "no_such_library.so"))
    with pytest.raises(RuntimeError, match="no CPU or PyTorch fallback"):
        binding.load()
