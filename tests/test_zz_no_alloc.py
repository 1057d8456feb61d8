"""GPU test of pqc_decode_static, the decode step for callers that cannot allocate: it runs on a scratch
array inside the library instead of a caller's workspace and must give exactly what pqc_decode gives
(same kernels), call after call on the one shared array, whatever the previous call left there."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2407_12820_amd import workloads as wl

from parity_utils import ATTN_TOL, attn_error, build_problem, check_indices

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def pqc():
    from paper_2407_12820_amd import binding
    binding.load()
    return binding


def _inputs(pqc, p):
    w = p.w
    return (pqc.to_device(p.q, w.dtype, DEV), torch.from_numpy(p.centroids).to(DEV), torch.from_numpy(p.codes).to(DEV),
            pqc.to_device(p.k, w.dtype, DEV), pqc.to_device(p.v, w.dtype, DEV))


def _both(pqc, p):
    """(idx, out) of pqc_decode on a context with its own workspace, and of pqc_decode_static."""
    w = p.w
    dev = _inputs(pqc, p)
    ctx = pqc.PQCache(w, DEV)
    idx_a, out_a = ctx.decode(*dev)
    idx_b, out_b = ctx.empty_outputs()
    idx_b.fill_(-7)
    out_b.fill_(float("nan"))
    pqc.decode_static(w, *dev, idx_b, out_b)
    torch.cuda.synchronize()
    return (idx_a.cpu().numpy(), out_a.cpu().numpy()), (idx_b.cpu().numpy(), out_b.cpu().numpy())


def test_static_scratch_decode_equals_decode_on_two_calls_in_a_row(pqc):
    big = wl.get("llama70b_128k", batch=1, n_tokens=30011)   # M=4, C=256, G=8: several select workgroups per unit
    small = wl.get("llama8b_32k", n_tokens=5003)             # another shape, smaller: the array holds the first call's leftovers
    for w, seed in ((big, 31), (small, 32), (big, 33)):
        print(f"[case] static scratch {w}", flush=True)
        p = build_problem(w, seed=seed)
        (ia, oa), (ib, ob) = _both(pqc, p)
        np.testing.assert_array_equal(ib, ia)
        np.testing.assert_array_equal(ob.view(np.uint32), oa.view(np.uint32))
        assert check_indices(p, ib) == 0
        assert attn_error(p, ib, ob) <= ATTN_TOL[w.dtype]


def test_static_scratch_rejects_what_does_not_fit(pqc):
    lib = pqc.load()
    limit = lib.pqc_static_scratch_bytes()
    w = wl.get("llama70b_128k")  # 32 units of 131072 tokens: far more workspace than the array holds
    cfg = pqc.make_config(w)
    assert lib.pqc_workspace_bytes(C.byref(cfg)) > limit
    # rejected before anything is read or enqueued: the pointers only have to be non-null and aligned
    buf = torch.zeros(4096, dtype=torch.uint8, device=DEV)
    ptr = buf.data_ptr()
    rc = lib.pqc_decode_static(C.byref(cfg), ptr, ptr, ptr, ptr, ptr, ptr, ptr, None)
    assert rc == -5 and b"static scratch" in lib.pqc_strerror(rc)
    torch.cuda.synchronize()
    assert int(buf.sum().item()) == 0
