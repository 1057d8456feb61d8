"""GPU parity tests: the HIP decode path, called through the C ABI, against the CPU
oracle on the same seeded inputs.  Index sets must match exactly (near-ties within
1e-4 relative of the K-th score would be reported, none are expected because both
sides rank the same fp32 scores); attention outputs within 2e-3 (bf16 inputs) or
1e-5 (fp32 inputs) of the double-precision oracle, relative to the head's largest
output magnitude."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from paper_2407_12820_amd import workloads as wl

from parity_utils import ATTN_TOL, attn_error, build_problem, check_indices, check_structure, unit_slice

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def pqc():
    from paper_2407_12820_amd import binding
    binding.load()
    return binding


def upload(pqc, p):
    w = p.w
    return dict(q=pqc.to_device(p.q, w.dtype, DEV), k=pqc.to_device(p.k, w.dtype, DEV), v=pqc.to_device(p.v, w.dtype, DEV),
                centroids=torch.from_numpy(p.centroids).to(DEV), codes=torch.from_numpy(p.codes).to(DEV))


def run_decode(pqc, p, ctx=None, dev=None):
    ctx = ctx or pqc.PQCache(p.w, DEV)
    dev = dev or upload(pqc, p)
    idx, out = ctx.decode(dev["q"], dev["centroids"], dev["codes"], dev["k"], dev["v"])
    torch.cuda.synchronize()
    return idx.cpu().numpy(), out.cpu().numpy()


def full_check(p, idx, out):
    near = check_indices(p, idx)
    assert near == 0, f"{near} near-tie substitutions (allowed by the contract, but not expected)"
    err = attn_error(p, idx, out)
    assert err <= ATTN_TOL[p.w.dtype], f"attention error {err:.3e}"
    check_structure(p, idx, out)
    return err


SCALED = {
    "tiny_f32": {},
    "llama8b_32k": dict(n_tokens=10007),
    "llama8b_128k": dict(n_tokens=20011),
    "batch8_32k": dict(batch=2, n_tokens=6151),
    "llama70b_128k": dict(batch=1, n_tokens=9001),
}


@pytest.mark.parametrize("name", wl.CONFIG_ORDER)
def test_decode_matches_oracle_scaled(pqc, name):
    w = wl.get(name, **SCALED[name])
    print(f"[case] decode scaled {w}", flush=True)
    p = build_problem(w, seed=1)
    idx, out = run_decode(pqc, p)
    full_check(p, idx, out)


@pytest.mark.parametrize("name", ["tiny_f32", "llama8b_32k", "batch8_32k", "llama70b_128k"])
def test_stages_match_oracle(pqc, name):
    w = wl.get(name, **SCALED[name])
    print(f"[case] stages {w}", flush=True)
    p = build_problem(w, seed=2)
    dev = upload(pqc, p)
    ctx = pqc.PQCache(w, DEV)
    I, K, L, N = w.n_init, w.topk, w.n_local, w.n_tokens
    s32, _ = oracle.scores(p.q, w.dtype, p.centroids, p.codes)
    # table + scan: scores equal the oracle's fp32 scores bit for bit; windows hold -inf
    table = ctx.lut(dev["q"], dev["centroids"])
    scores = ctx.scan(table, dev["codes"])
    torch.cuda.synchronize()
    sg = scores.cpu().numpy()
    np.testing.assert_array_equal(sg[:, :, I:N - L].view(np.uint32), s32[:, :, I:N - L].view(np.uint32))
    assert np.all(np.isneginf(sg[:, :, :I])) and np.all(np.isneginf(sg[:, :, N - L:]))
    # table itself: entry = group query . centroid (double reference, tolerance of an fp32 dot product)
    qv = wl.to_f32(p.q, w.dtype).astype(np.float64).reshape(w.batch, w.n_kv_heads, w.group, w.pq_m, w.sub_dim).sum(2)
    ref = np.einsum("bgjd,bgjcd->bgjc", qv, p.centroids.astype(np.float64))
    np.testing.assert_allclose(table.cpu().numpy(), ref, rtol=0, atol=1e-4 * np.abs(ref).max())
    # top-k stage on the oracle's scores
    want = oracle.select(s32, K, I, L)
    idx = ctx.topk(torch.from_numpy(s32).to(DEV))
    torch.cuda.synchronize()
    ig = idx.cpu().numpy()
    np.testing.assert_array_equal(np.sort(ig, axis=-1), np.sort(want, axis=-1))
    # attention stage on the oracle's index list (best-first order: any order must do)
    out = ctx.gather_attn(dev["q"], dev["k"], dev["v"], torch.from_numpy(want).to(DEV))
    torch.cuda.synchronize()
    err = attn_error(p, want, out.cpu().numpy())
    assert err <= ATTN_TOL[w.dtype], f"attention error {err:.3e}"


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name", ["llama8b_32k", "llama8b_128k"])
def test_decode_matches_oracle_full_size(pqc, name):
    w = wl.get(name)
    print(f"[case] decode full size {w}", flush=True)
    p = build_problem(w, seed=0)
    dev, ctx = upload(pqc, p), pqc.PQCache(w, DEV)
    idx, out = run_decode(pqc, p, ctx, dev)
    err = full_check(p, idx, out)
    print(f"[result] {name}: attention error {err:.3e}", flush=True)
    # the code-pair path at the same size, in the launch shape the benchmark reports beside the general one
    counts = pqc.pair_counts(w, dev["codes"])
    idx2, out2 = ctx.decode_indexed(dev["q"], dev["centroids"], dev["codes"], counts, dev["k"], dev["v"])
    torch.cuda.synchronize()
    np.testing.assert_array_equal(np.sort(idx2.cpu().numpy(), -1), np.sort(idx, -1))
    assert attn_error(p, idx2.cpu().numpy(), out2.cpu().numpy()) <= ATTN_TOL[w.dtype]


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name,units", [("batch8_32k", [0, 37]), ("llama70b_128k", [5, 30])])
def test_decode_matches_oracle_full_size_every_unit(pqc, name, units):
    # The full launch shape.  Every unit is compared with the oracle: scores, full sort and
    # double-precision attention need only centroids and codes, so the units whose PQ structures
    # are not worth a CPU K-Means at this size (all but `units`) get centroids drawn from their
    # keys and random codes, which are inputs as valid as any other.
    w = wl.get(name)
    print(f"[case] decode full size, every unit (K-Means structures for {units}): {w}", flush=True)
    p = build_problem(w, seed=0, checked_units=units)
    idx, out = run_decode(pqc, p)
    every = range(w.batch * w.n_kv_heads)
    near = check_indices(p, idx, units=every)
    assert near == 0, f"{near} near-tie substitutions"
    err = attn_error(p, idx, out, units=every)
    assert err <= ATTN_TOL[w.dtype], f"attention error {err:.3e}"
    check_structure(p, idx, out)
    print(f"[result] {name}: {len(every)} units compared, attention error {err:.3e}", flush=True)


# ----------------------------------------------------------------------- edge cases
def _small(**kw):
    base = dict(name="edge", batch=1, n_q_heads=4, n_kv_heads=2, head_dim=128, n_tokens=3000, pq_m=2, pq_centroids=16,
                topk=300, n_init=4, n_local=64, dtype="bf16", kmeans_iters=2, recipe="plain")
    base.update(kw)
    return wl.Workload(**base)


@pytest.mark.parametrize("kw", [
    dict(topk=0),                                   # windows only
    dict(topk=3000 - 68),                           # every token attended: dense attention
    dict(n_tokens=70, topk=2),                      # two middle tokens
    dict(n_tokens=69, topk=1),                      # one middle token
    dict(n_init=0, n_local=0, topk=17),             # no windows
    dict(n_init=0, n_local=0, topk=1, n_tokens=1),  # a single cached token
    dict(pq_m=1, pq_centroids=2, topk=700),         # two distinct scores: huge tie classes
    dict(pq_m=8, pq_centroids=256, n_q_heads=2, n_kv_heads=2, topk=257),
    dict(pq_m=4, pq_centroids=7, n_q_heads=16, n_kv_heads=2, topk=999, n_tokens=4097),
    dict(dtype="f32", n_q_heads=8, n_kv_heads=1, topk=511, n_tokens=2500),
    dict(batch=3, n_tokens=2049, topk=100),
    dict(batch=3, n_q_heads=8, n_kv_heads=4, n_tokens=5000, topk=500),  # 12 units: 8 interleaved over the XCDs + 4
    # tie classes of different sizes at the threshold: about 90, 190, 380 and 1500 equal scores
    dict(pq_m=1, pq_centroids=32, topk=500),
    dict(pq_m=1, pq_centroids=16, topk=700),
    dict(pq_m=1, pq_centroids=8, topk=700),
    dict(dtype="f32", pq_m=1, pq_centroids=32, topk=500, n_q_heads=2, n_kv_heads=2),
    dict(dtype="f32", pq_m=1, pq_centroids=4, topk=900, n_q_heads=2, n_kv_heads=1),
    # windows far larger than usual: most of the cache, all of it as the local window, all of it as the initial one
    dict(n_tokens=5000, n_init=500, n_local=3000, topk=100),
    dict(n_tokens=2500, n_init=0, n_local=2500, topk=0),
    dict(n_tokens=2500, n_init=2500, n_local=0, topk=0),
    dict(n_tokens=4100, n_init=1, n_local=2047, topk=2052),
    # many units: more than the 256 compute units, a multiple of 8 and not (the last ones are not interleaved over the XCDs)
    dict(batch=40, n_q_heads=16, n_kv_heads=8, n_tokens=600, topk=60),
    dict(batch=37, n_q_heads=6, n_kv_heads=3, n_tokens=777, topk=99, pq_m=4),
    # more select workgroups per unit than the finalize kernel has threads
    dict(n_tokens=140001, topk=9000, n_q_heads=2, n_kv_heads=1, pq_centroids=64),
    dict(n_tokens=200003, topk=30000, n_q_heads=8, n_kv_heads=1, pq_centroids=64),
], ids=lambda kw: ",".join(f"{k}={v}" for k, v in kw.items()))
def test_edge_shapes(pqc, kw):
    w = _small(**kw)
    print(f"[case] edge {kw}", flush=True)
    p = build_problem(w, seed=3)
    idx, out = run_decode(pqc, p)
    full_check(p, idx, out)


@pytest.mark.timeout(600)
def test_maximum_context_length(pqc):
    # N = 2^22, the largest context the library accepts: 512 select workgroups of 8192 tokens
    w = _small(n_tokens=1 << 22, topk=150000, n_q_heads=1, n_kv_heads=1, pq_centroids=16, kmeans_iters=1)
    print(f"[case] maximum context {w}", flush=True)
    p = build_problem(w, seed=14)
    idx, out = run_decode(pqc, p)
    full_check(p, idx, out)


def _random_shapes(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        g = int(rng.choice([1, 2, 4, 8]))
        hkv = int(rng.choice([1, 2, 3]))
        m = int(rng.choice([1, 2, 4, 8]))
        c = int(rng.choice([2, 5, 16, 64, 200, 256]))
        n_tok = int(rng.integers(1, 7000))
        n_init = int(rng.integers(0, min(n_tok, 9) + 1))
        n_local = int(rng.integers(0, min(n_tok - n_init, 100) + 1))
        mid = n_tok - n_init - n_local
        topk = int(rng.integers(0, mid + 1)) if rng.random() < 0.8 else int(rng.choice([0, mid]))
        if n_init + topk + n_local == 0:
            topk, n_tok = 1, max(n_tok, 1)
            if mid < 1:
                n_init, n_local = 0, 0
        out.append(dict(batch=int(rng.choice([1, 2])), n_q_heads=g * hkv, n_kv_heads=hkv, n_tokens=n_tok, pq_m=m, pq_centroids=c,
                        topk=topk, n_init=n_init, n_local=n_local, dtype=str(rng.choice(["bf16", "bf16", "f32"])), kmeans_iters=1))
    return out


@pytest.mark.parametrize("kw", _random_shapes(24, seed=2024), ids=lambda kw: "-".join(str(v) for v in kw.values()))
def test_random_shapes(pqc, kw):
    # a seeded sweep over the supported shape space (group sizes, partitions, centroid counts, windows, dtypes)
    w = _small(**kw)
    print(f"[case] random shape {kw}", flush=True)
    p = build_problem(w, seed=21)
    idx, out = run_decode(pqc, p)
    full_check(p, idx, out)


def test_all_scores_equal_takes_lowest_indices(pqc):
    # A zero query ties every token: the K lowest middle indices win, attention is a plain mean.
    w = _small(topk=1500)
    p = build_problem(w, seed=4)
    p = type(p)(w, np.zeros_like(p.q), p.k, p.v, p.centroids, p.codes, p.checked_units)
    idx, out = run_decode(pqc, p)
    assert np.all(np.sort(idx[0, 0, 4:1504]) == np.arange(4, 1504))
    full_check(p, idx, out)


@pytest.mark.parametrize("batch", [1, 32], ids=["2units", "64units"])
@pytest.mark.parametrize("admitted", [1, 63, 64, 65, 96, 97, 150])
def test_any_number_of_a_tie_class_is_admitted(pqc, admitted, batch):
    # One partition of 16 centroids: 16 distinct scores, classes of about 190 tokens.  K is set so that unit 0 must
    # admit exactly `admitted` tokens of the class at the threshold (lowest indices first); the other units admit
    # whatever the same K means for them.  The counts bracket the sizes at which the finalize kernel changes the way
    # it fetches the admitted rows; 2 and 64 units give it four workgroups and one workgroup per query head.
    base = _small(pq_m=1, pq_centroids=16, batch=batch)
    p0 = build_problem(base, seed=6)
    q1, c1, cd1, _, _ = unit_slice(p0, 0)
    s32, _ = oracle.scores(q1, base.dtype, c1, cd1)
    mid = s32[0, 0, base.n_init:base.n_tokens - base.n_local]
    values, counts = np.unique(mid, return_counts=True)
    above = 0
    for val, cnt in zip(values[::-1], counts[::-1]):  # classes from the largest score down
        if cnt > admitted and above > 100:
            break
        above += int(cnt)
    else:
        pytest.skip("no tie class large enough")
    w = dataclasses.replace(base, topk=above + admitted)
    print(f"[case] tie class of {cnt}, {above} tokens above it, K={w.topk}, units={batch * 2}", flush=True)
    p = type(p0)(w, p0.q, p0.k, p0.v, p0.centroids, p0.codes, p0.checked_units)
    idx, out = run_decode(pqc, p)
    full_check(p, idx, out)
    klass = np.flatnonzero(s32[0, 0] == val)
    klass = klass[(klass >= w.n_init) & (klass < w.n_tokens - w.n_local)]
    got = np.sort(idx[0, 0, w.n_init:w.n_init + w.topk])
    assert np.intersect1d(got, klass).tolist() == klass[:admitted].tolist()


@pytest.mark.parametrize("sample_value", [-1.0, 10.0])
def test_topk_when_the_sample_misleads(pqc, sample_value):
    # The bin window is placed from 1024 evenly spaced tokens.  Give exactly those tokens one
    # extreme score: the window then misses the K-th largest score altogether (it falls into the
    # coarse bins above the window, or into the single bin below it, where every low token becomes
    # a candidate).  Only speed may suffer: the selection must still be the oracle's.
    w = _small(n_tokens=20068, topk=5000, n_q_heads=2, n_kv_heads=2)
    rng = np.random.default_rng(11)
    s32 = rng.random((1, 2, w.n_tokens), dtype=np.float32)
    nmid = w.n_tokens - w.n_init - w.n_local
    pos = w.n_init + (np.arange(1024, dtype=np.int64) * nmid) // 1024
    s32[:, :, pos] = sample_value
    ctx = pqc.PQCache(w, DEV)
    got = ctx.topk(torch.from_numpy(s32).to(DEV))
    torch.cuda.synchronize()
    want = oracle.select(s32, w.topk, w.n_init, w.n_local)
    np.testing.assert_array_equal(np.sort(got.cpu().numpy(), -1), np.sort(want, -1))


def test_context_reuse_and_two_contexts(pqc):
    # Calls on one context leave the workspace ready for the next call; contexts do not interfere.
    wa, wb = _small(topk=123), _small(n_tokens=5000, topk=900, pq_m=4)
    pa1, pa2, pb = build_problem(wa, 5), build_problem(wa, 6), build_problem(wb, 7)
    ca, cb = pqc.PQCache(wa, DEV), pqc.PQCache(wb, DEV)
    for _ in range(2):
        for p, c in ((pa1, ca), (pb, cb), (pa2, ca), (pa1, ca)):
            idx, out = run_decode(pqc, p, ctx=c)
            full_check(p, idx, out)
    # stage call between decode calls shares the same workspace
    s32, _ = oracle.scores(pa1.q, wa.dtype, pa1.centroids, pa1.codes)
    ig = ca.topk(torch.from_numpy(s32).to(DEV)).cpu().numpy()
    np.testing.assert_array_equal(np.sort(ig, -1), np.sort(oracle.select(s32, wa.topk, wa.n_init, wa.n_local), -1))
    idx, out = run_decode(pqc, pa2, ctx=ca)
    full_check(pa2, idx, out)


def test_decode_phase_by_phase_equals_decode(pqc):
    # the profiling entry point launches the same three kernels one at a time
    w = _small(n_tokens=9000, topk=1200, pq_m=4)
    p = build_problem(w, seed=9)
    dev, ctx = upload(pqc, p), pqc.PQCache(w, DEV)
    a = run_decode(pqc, p, ctx, dev)
    idx, out = ctx.empty_outputs()
    for _ in range(2):  # twice: a complete pass leaves the workspace ready for the next
        idx.zero_()
        out.zero_()
        for phase in range(3):
            ctx.decode_phase(phase, dev["q"], dev["centroids"], dev["codes"], dev["k"], dev["v"], idx, out)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(a[0], idx.cpu().numpy())
        np.testing.assert_array_equal(a[1].view(np.uint32), out.cpu().numpy().view(np.uint32))
    full_check(p, a[0], a[1])
    # a phase out of turn is refused, and a step left unfinished does not disturb the next full call
    args = (dev["q"], dev["centroids"], dev["codes"], dev["k"], dev["v"], idx, out)
    with pytest.raises(pqc.PQCacheError):
        ctx.decode_phase(1, *args)
    ctx.decode_phase(0, *args)
    with pytest.raises(pqc.PQCacheError):
        ctx.decode_phase(0, *args)
    with pytest.raises(pqc.PQCacheError):
        ctx.decode_phase(2, *args)
    b = run_decode(pqc, p, ctx, dev)
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_array_equal(a[1].view(np.uint32), b[1].view(np.uint32))


@pytest.mark.parametrize("kw", [
    dict(),                                                          # llama8b_128k scaled
    dict(n_tokens=4096, topk=512, n_q_heads=1, n_kv_heads=1, dtype="f32", pq_centroids=64),
    dict(topk=0),
    dict(n_tokens=3000 - 3000 % 8, topk=2000, pq_centroids=7),       # few pairs, big tie classes
    dict(n_tokens=72, topk=1),
    dict(n_tokens=2048, n_local=300, n_init=9, topk=100),            # more window tokens than threads
], ids=lambda kw: ",".join(f"{k}={v}" for k, v in kw.items()) or "scaled")
def test_indexed_decode_equals_decode(pqc, kw):
    # threshold from code-pair counts: same selection and attention as the general path, and as the oracle
    if kw:
        w = _small(**{**dict(pq_m=2, pq_centroids=16, n_tokens=3000 - 3000 % 8), **kw})
    else:
        w = wl.get("llama8b_128k", n_tokens=20008)
    p = build_problem(w, seed=12)
    dev, ctx = upload(pqc, p), pqc.PQCache(w, DEV)
    counts = pqc.pair_counts(w, dev["codes"])
    torch.cuda.synchronize()
    want_counts = np.zeros((w.batch, w.n_kv_heads, w.pq_centroids ** 2), np.int64)
    pair = p.codes[..., 0].astype(np.int64) + w.pq_centroids * p.codes[..., 1].astype(np.int64)
    for b in range(w.batch):
        for g in range(w.n_kv_heads):
            want_counts[b, g] = np.bincount(pair[b, g], minlength=w.pq_centroids ** 2)
    np.testing.assert_array_equal(counts.cpu().numpy(), want_counts)
    for _ in range(2):
        idx, out = ctx.decode_indexed(dev["q"], dev["centroids"], dev["codes"], counts, dev["k"], dev["v"])
        torch.cuda.synchronize()
        full_check(p, idx.cpu().numpy(), out.cpu().numpy())
    a = run_decode(pqc, p, ctx, dev)
    np.testing.assert_array_equal(np.sort(a[0], -1), np.sort(idx.cpu().numpy(), -1))


def test_indexed_decode_zero_query_and_unsupported(pqc):
    # all scores equal: one bin holds every pair (the radix branch of the threshold search)
    w = _small(pq_m=2, pq_centroids=64, n_tokens=3000 - 3000 % 8, topk=1500)
    p = build_problem(w, seed=13)
    p = type(p)(w, np.zeros_like(p.q), p.k, p.v, p.centroids, p.codes, p.checked_units)
    dev, ctx = upload(pqc, p), pqc.PQCache(w, DEV)
    counts = pqc.pair_counts(w, dev["codes"])
    idx, out = ctx.decode_indexed(dev["q"], dev["centroids"], dev["codes"], counts, dev["k"], dev["v"])
    torch.cuda.synchronize()
    assert np.all(np.sort(idx.cpu().numpy()[0, 0, 4:1504]) == np.arange(4, 1504))
    full_check(p, idx.cpu().numpy(), out.cpu().numpy())
    # four partitions: no pair counts
    w4 = _small(pq_m=4)
    with pytest.raises(pqc.PQCacheError):
        pqc.pair_counts(w4, torch.zeros((1, 2, 3000, 4), dtype=torch.uint8, device=DEV))


def test_pair_counts_follow_an_appended_code(pqc):
    w = _small(pq_m=2, pq_centroids=16, n_tokens=1000)
    rng = np.random.default_rng(3)
    codes = torch.from_numpy(rng.integers(0, 16, size=(1, 2, 1000, 2), dtype=np.uint8)).to(DEV)
    full = pqc.pair_counts(w, codes)
    # counts of the first 999 tokens, then token 999 appended
    codes2 = codes.clone()
    codes2[:, :, 999, :] = 255  # outside the code range: not counted
    part = pqc.pair_counts(w, codes2)
    pqc.pair_counts_add(w, codes, 999, part)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(full.cpu().numpy(), part.cpu().numpy())


def test_decode_is_deterministic(pqc):
    w = wl.get("llama8b_128k", n_tokens=20011)
    p = build_problem(w, seed=1)
    dev, ctx = upload(pqc, p), pqc.PQCache(w, DEV)
    a = run_decode(pqc, p, ctx, dev)
    b = run_decode(pqc, p, ctx, dev)
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_array_equal(a[1].view(np.uint32), b[1].view(np.uint32))


def test_runs_on_a_side_stream(pqc):
    w = _small(topk=200)
    p = build_problem(w, seed=8)
    dev, ctx = upload(pqc, p), pqc.PQCache(w, DEV)
    torch.cuda.synchronize()
    st = torch.cuda.Stream(device=DEV)
    idx, out = ctx.decode(dev["q"], dev["centroids"], dev["codes"], dev["k"], dev["v"], stream=st)
    st.synchronize()
    full_check(p, idx.cpu().numpy(), out.cpu().numpy())


@pytest.mark.parametrize("indexed", [False, True])
def test_layers_recorded_into_a_hip_graph_replay_correctly(pqc, indexed):
    # Algorithm 2 loops over the layers: one call per layer on a shared context, recorded once by stream
    # capture, replayed with eager calls on the same context in between.  Every replay must reproduce the
    # eager results bit for bit (a call leaves the workspace as it found it).
    w = _small(n_tokens=9000, topk=1100)
    layers = [build_problem(w, seed=40 + i) for i in range(3)]
    other = build_problem(w, seed=50)
    devs, dev_other, ctx = [upload(pqc, p) for p in layers], upload(pqc, other), pqc.PQCache(w, DEV)
    pcs = [pqc.pair_counts(w, d["codes"]) for d in devs] if indexed else [None] * len(layers)

    def call(d, pc, oi, oa):
        if indexed:
            ctx.decode_indexed(d["q"], d["centroids"], d["codes"], pc, d["k"], d["v"], oi, oa)
        else:
            ctx.decode(d["q"], d["centroids"], d["codes"], d["k"], d["v"], oi, oa)

    eager, bufs = [], []
    for d, pc in zip(devs, pcs):  # ordinary calls first: reference results, and the context's clearing launch is behind us
        oi, oa = ctx.empty_outputs()
        call(d, pc, oi, oa)
        eager.append((oi.cpu().numpy().copy(), oa.cpu().numpy().copy()))
        bufs.append(ctx.empty_outputs())
    torch.cuda.synchronize()
    graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream(device=DEV)
    with torch.cuda.graph(graph, stream=side):
        for d, pc, (oi, oa) in zip(devs, pcs, bufs):
            call(d, pc, oi, oa)
    for rep in range(3):
        for oi, oa in bufs:
            oi.fill_(-1)
            oa.fill_(float("nan"))
        ctx.decode(dev_other["q"], dev_other["centroids"], dev_other["codes"], dev_other["k"], dev_other["v"])  # eager, same context
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for (ei, ea), (oi, oa) in zip(eager, bufs):
            np.testing.assert_array_equal(oi.cpu().numpy(), ei, err_msg=f"replay {rep}")
            np.testing.assert_array_equal(oa.cpu().numpy().view(np.uint32), ea.view(np.uint32), err_msg=f"replay {rep}")
    full_check(layers[-1], bufs[-1][0].cpu().numpy(), bufs[-1][1].cpu().numpy())


def test_indexed_decode_with_counts_of_other_codes_stays_inside_its_outputs(pqc):
    # pair counts that do not belong to the codes (here: the counts of another code tensor, and counts that are all
    # zero but one) make the selection meaningless, but nothing may be written outside out_idx and out_attn: the
    # outputs are slices of larger buffers whose surroundings must stay as they were.  Codes 20..39 with 16 centroids
    # are out of range below 255 and name no pair either.
    w = _small(pq_m=2, pq_centroids=16, n_tokens=3000 - 3000 % 8, topk=300)
    p = build_problem(w, seed=17)
    dev, ctx = upload(pqc, p), pqc.PQCache(w, DEV)
    rng = np.random.default_rng(5)
    other = torch.from_numpy(rng.integers(0, 16, size=p.codes.shape, dtype=np.uint8)).to(DEV)
    skew = torch.zeros((w.batch, w.n_kv_heads, 256), dtype=torch.int32, device=DEV)
    skew[:, :, 7] = w.n_tokens
    for counts in (pqc.pair_counts(w, other), skew):
        pad = 4096
        big_i = torch.full((pad + w.batch * w.n_kv_heads * w.n_selected + pad,), -77, dtype=torch.int32, device=DEV)
        big_o = torch.full((pad + w.batch * w.n_q_heads * w.head_dim + pad,), 123.0, dtype=torch.float32, device=DEV)
        oi = big_i[pad:-pad].view(w.batch, w.n_kv_heads, w.n_selected)
        oo = big_o[pad:-pad].view(w.batch, w.n_q_heads, w.head_dim)
        ctx.decode_indexed(dev["q"], dev["centroids"], dev["codes"], counts, dev["k"], dev["v"], oi, oo)
        torch.cuda.synchronize()
        assert bool((big_i[:pad] == -77).all()) and bool((big_i[-pad:] == -77).all())
        assert bool((big_o[:pad] == 123.0).all()) and bool((big_o[-pad:] == 123.0).all())
        got = oi.cpu().numpy()
        written = got[got != -77]
        assert written.min() >= 0 and written.max() < w.n_tokens
    # and the context is none the worse for it
    idx, out = run_decode(pqc, p, ctx, dev)
    full_check(p, idx, out)


def test_pair_counts_skip_codes_that_name_no_centroid(pqc):
    # 16 centroids: a code byte of 20 in the first partition must not be counted as pair (4, 1)
    w = _small(pq_m=2, pq_centroids=16, n_tokens=1000)
    rng = np.random.default_rng(4)
    codes = rng.integers(0, 16, size=(1, 2, 1000, 2), dtype=np.uint8)
    codes[0, 0, 10] = (20, 0)
    codes[0, 1, 11] = (3, 16)
    codes[0, 1, 12] = (200, 200)
    counts = pqc.pair_counts(w, torch.from_numpy(codes).to(DEV))
    torch.cuda.synchronize()
    want = np.zeros((1, 2, 256), np.int64)
    for g in range(2):
        for c0, c1 in codes[0, g]:
            if c0 < 16 and c1 < 16:
                want[0, g, int(c0) + 16 * int(c1)] += 1
    np.testing.assert_array_equal(counts.cpu().numpy(), want)
    assert int(counts.sum().item()) == 2000 - 3
    # the single-token update applies the same rule
    cd = torch.from_numpy(codes).to(DEV)
    before = counts.clone()
    pqc.pair_counts_add(w, cd, 10, counts)   # unit 0: (20, 0) names no pair; unit 1: an ordinary code
    torch.cuda.synchronize()
    diff = (counts - before).cpu().numpy()
    assert diff[0, 0].sum() == 0 and diff[0, 1].sum() == 1
