#!/usr/bin/env python3
"""Benchmark of the PQ decode hot path on one MI355X.

A step is one pqc_decode call: look-up table, code scan, top-k selection, gather of the
selected K/V rows and attention, for one attention layer of the workload.  Inputs are
seeded synthetic tensors, resident in HBM before the timed region; several distinct
input sets are visited round-robin (as a model walks its layers) so that the K/V rows
are fetched from HBM, not from the 256 MB last-level cache.  PQ structures are built
on the GPU by the library's own K-Means (pqc_pq_build) before timing starts.

Prints ONE JSON line: the step time of the headline workload (us per layer: the median
of `--reps` repetitions of `--steps` back-to-back steps, with the spread beside it), the
achieved fraction of the HBM roofline for the whole path and for its dominant kernel
(timed live with HIP events through pqc_decode_phase), the same figures for the other
four benchmark shapes (`also`), and the CPU oracle's time for the same step as a
baseline, with a comparison of the GPU's results against the oracle's for every shape.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth
KERNELS = ("hist", "select_attn", "finalize")


def source_hash() -> str:
    """Hash of the kernel sources: profiles/*_traffic.json carry the hash they were measured at."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2407_12820_amd", "csrc")
    for name in sorted(os.listdir(d)):
        with open(os.path.join(d, name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--reps", type=int, default=5, help="repetitions of the timed loop of --steps steps (median reported)")
    ap.add_argument("--workload", default="llama8b_128k")
    ap.add_argument("--layers", type=int, default=8, help="distinct input sets visited round-robin")
    ap.add_argument("--profile-steps", type=int, default=24, help="rounds of the per-kernel timing (each launches every kernel once per input set)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip everything that runs the CPU oracle")
    ap.add_argument("--no-indexed", action="store_true", help="skip the pqc_decode_indexed measurement")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP graph replay measurement")
    ap.add_argument("--no-append", action="store_true", help="skip the encode-token + decode measurement")
    ap.add_argument("--no-copy-ceiling", action="store_true", help="skip the device-to-device copy measurement")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--also", default="tiny_f32,llama8b_32k,batch8_32k,llama70b_128k",
                    help="other workloads reported alongside, comma separated; '' to skip")
    ap.add_argument("--also-steps", type=int, default=100)
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="also run one plain device copy of this size (reference for scaling rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    ap.add_argument("--lib", default="", help="load this build of the library instead of the default one (comparison builds)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2407_12820_amd import binding, workloads as wl

    if args.lib:
        binding.LIB_PATH = os.path.abspath(args.lib)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    dev = "cuda:0"
    stream_handle = torch.cuda.current_stream(dev).cuda_stream
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with_cpu = not args.no_cpu_baseline
    if with_cpu:
        import oracle  # test infrastructure: used in this CPU-baseline leg only

    def make_sets(w, n_sets, seed0):
        sets, host0, build_ms = [], None, []
        for layer in range(n_sets):
            d = wl.generate(w, seed=seed0 + layer)
            q, k, v = (binding.to_device(d[n], w.dtype, dev) for n in ("q", "k", "v"))
            init = torch.from_numpy(wl.kmeans_init_indices(w, seed=seed0 + layer)).to(dev)
            torch.cuda.synchronize()
            tb = time.perf_counter()
            cent, codes = binding.pq_build(w, k, init)
            torch.cuda.synchronize()
            build_ms.append((time.perf_counter() - tb) * 1e3)
            sets.append((q, cent, codes, k, v))
            if layer == 0 and with_cpu:
                host0 = d
            else:
                del d
        return sets, host0, build_ms

    def time_steps(call, n_sets, steps, warmup, reps):
        """us per step of `reps` repetitions of `steps` back-to-back calls (each repetition between two events)."""
        for i in range(warmup):
            call(i % n_sets)
        torch.cuda.synchronize()
        out, issue_ms, wall_ms = [], 0.0, 0.0
        for _ in range(reps):
            t0 = time.perf_counter()
            ev0.record()
            for i in range(steps):
                call(i % n_sets)
            ev1.record()
            issue_ms += (time.perf_counter() - t0) * 1e3  # host time to enqueue the steps (the GPU must not wait for it)
            torch.cuda.synchronize()
            wall_ms += (time.perf_counter() - t0) * 1e3
            out.append(ev0.elapsed_time(ev1) / steps * 1e3)
        return np.array(out), issue_ms / (reps * steps), wall_ms / (reps * steps)

    def kernel_times(w, ctx, sets, margs, rounds):
        """Per-kernel durations: each kernel of the path is launched for every input set back to back (one
        context per set) between two HIP events on the launch stream, so that no event sits in front of a
        timed launch; duration = span / number of launches."""
        nk = len(KERNELS)
        kern_us = np.zeros(nk)
        if rounds <= 0:
            return kern_us
        ctxs = [ctx] + [binding.PQCache(w, dev) for _ in sets[1:]]
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(nk + 1)]
        for rnd in range(rounds + 2):  # two untimed rounds first
            for ph in range(nk):
                evs[ph].record()
                for c, a in zip(ctxs, margs):
                    c.decode_phase_marshalled(ph, a, stream_handle)
            evs[nk].record()
            torch.cuda.synchronize()
            if rnd >= 2:
                kern_us += np.array([evs[i].elapsed_time(evs[i + 1]) for i in range(nk)]) * 1e3 / len(sets)
        return kern_us / rounds

    def against_oracle(w, ctx, st, host, out_idx, out_attn):
        """The GPU's result for one input set against the oracle's: index sets equal, attention error."""
        cent_h, codes_h = st[1].cpu().numpy(), st[2].cpu().numpy()
        scale = wl.softmax_scale(w)
        t = time.perf_counter()
        idx_h, out_h, _ = oracle.decode(host["q"], cent_h, codes_h, host["k"], host["v"], w.dtype, w.topk, w.n_init,
                                        w.n_local, scale)
        t_cpu = time.perf_counter() - t
        ctx.decode(*st, out_idx, out_attn)
        torch.cuda.synchronize()
        same = bool(np.array_equal(np.sort(out_idx.cpu().numpy(), -1), np.sort(idx_h, -1)))
        err = float((np.abs(out_attn.cpu().numpy() - out_h).max(-1) / np.abs(out_h).max(-1)).max())
        return {"index_sets_equal": same, "attn_max_rel_err": err}, t_cpu, (cent_h, codes_h, scale)

    def sel_bytes_of(w):
        # dominant kernel (select + attention): the I+K+L attended K and V rows and the queries; the per-token
        # bins it reads instead of the codes are this implementation's own traffic and are not credited
        units = w.batch * w.n_kv_heads
        return units * w.n_selected * w.head_dim * 2 * w.elem_bytes + w.batch * w.n_q_heads * w.head_dim * w.elem_bytes

    # ------------------------------------------------------------------ the headline workload
    w = wl.get(args.workload)
    ctx = binding.PQCache(w, dev)
    sets, host0, build_ms = make_sets(w, args.layers, 100)
    out_idx, out_attn = ctx.empty_outputs()
    torch.cuda.synchronize()
    # argument checks and address look-ups done once per input set, outside the timed loops
    margs = [ctx.marshal_decode_args(*st, out_idx, out_attn) for st in sets]

    def step(i: int) -> None:
        ctx.decode_marshalled(margs[i], stream_handle)

    rep_us, issue_ms, wall_ms = time_steps(step, len(sets), args.steps, args.warmup, args.reps)
    us = float(np.median(rep_us))
    kern_us = kernel_times(w, ctx, sets, margs, args.profile_steps)

    if args.copy_calibration_mib:
        src = torch.empty(args.copy_calibration_mib << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)  # one elementwise copy kernel: reads and writes exactly this many bytes
        torch.cuda.synchronize()
        del src, dst

    path_bytes = w.algorithmic_bytes()
    sel_bytes = sel_bytes_of(w)
    sel_gbps = sel_bytes / (kern_us[1] * 1e-6) / 1e9 if kern_us[1] > 0 else 0.0
    path_gbps = path_bytes / (us * 1e-6) / 1e9

    # HBM bytes per launch of the dominant kernel measured with rocprofv3 --pmc (see the file for the commands);
    # the file carries the hash of the kernel sources it was measured at
    traffic, traffic_stale = None, None
    tpath = os.path.join(ROOT, "profiles", f"select_kernel_{w.name}_traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            tj = json.load(f)
        traffic = tj.get("hbm_bytes_per_launch")
        traffic_stale = tj.get("source_hash") != source_hash()

    result = {
        "metric": "decode µs per layer (PQ score+top-k+sparse attn) at 128K ctx",
        "value": round(us, 3), "unit": "us/layer", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(us * 1e-3, 6), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
                   "head_dim": w.head_dim, "n_tokens": w.n_tokens, "pq_m": w.pq_m, "pq_centroids": w.pq_centroids,
                   "topk": w.topk, "n_init": w.n_init, "n_local": w.n_local, "kv_dtype": w.dtype,
                   "kmeans_iters": w.kmeans_iters, "input_sets": len(sets), "accumulate": "f32"},
        "repetitions": {"count": args.reps, "steps_each": args.steps, "us_min": round(float(rep_us.min()), 3),
                        "us_median": round(us, 3), "us_max": round(float(rep_us.max()), 3)},
        "achieved_hbm_gbps": round(path_gbps, 1), "hbm_frac": round(path_gbps / HBM_PEAK_GBPS, 4),
        "algorithmic_bytes_per_step": path_bytes, "host_wall_ms_per_step": round(wall_ms, 6),
        "host_issue_ms_per_step": round(issue_ms, 6),
        "kernel_us": {n: round(float(x), 3) for n, x in zip(KERNELS, kern_us)},
        "roofline": {"kernel": "select_kernel", "bound": "hbm", "achieved": round(sel_gbps, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(sel_gbps / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "traffic_stale": traffic_stale, "bytes_per_launch": sel_bytes, "avg_us": round(float(kern_us[1]), 3)},
        "library": {"version": binding.load().pqc_version(), "source_hash": source_hash(),
                    "path": os.path.relpath(binding.LIB_PATH, ROOT)},
    }

    # the same step through pqc_decode_indexed (threshold from code-pair counts; two partitions only):
    # reported beside `value`, which stays the general path whose inputs are centroids and codes alone
    if not args.no_indexed and w.pq_m == 2 and w.pq_centroids <= 64 and w.n_tokens % 8 == 0:
        pcs = [binding.pair_counts(w, st[2]) for st in sets]
        pptr = [ctx._pair_ptr(pc) for pc in pcs]
        r_i, _, _ = time_steps(lambda i: ctx.decode_indexed_marshalled(margs[i], pptr[i], stream_handle), len(sets), args.steps,
                               args.warmup, max(1, args.reps // 2))
        us_i = float(np.median(r_i))
        result["indexed_path"] = {"entry_point": "pqc_decode_indexed", "us_per_layer": round(us_i, 3),
                                  "hbm_frac": round(path_bytes / (us_i * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                                  "extra_input": "tokens per code pair, [units][C*C] uint32, built once per code tensor"}

    # Algorithm 2 runs the step once per layer: the same `input_sets` calls recorded once into a HIP graph
    # (stream capture) and replayed, which takes the host's launch calls out of the loop
    if not args.no_graph:
        side = torch.cuda.Stream(device=dev)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for a in margs:
                ctx.decode_marshalled(a, torch.cuda.current_stream(dev).cuda_stream)
        reps = max(1, args.steps // len(sets))
        with torch.cuda.stream(side):
            for _ in range(max(1, args.warmup // len(sets))):
                graph.replay()
            side.synchronize()
            g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            tg = time.perf_counter()
            g0.record(side)
            for _ in range(reps):
                graph.replay()
            g1.record(side)
            issue_g = (time.perf_counter() - tg) * 1e3
            side.synchronize()
        result["graph_replay"] = {"layers_per_graph": len(sets), "replays": reps,
                                  "us_per_layer": round(g0.elapsed_time(g1) / (reps * len(sets)) * 1e3, 3),
                                  "host_issue_ms_per_layer": round(issue_g / (reps * len(sets)), 6)}
        del graph

    # the step as it runs inside a decode loop (Algorithm 2): the code of one more token per head is written
    # (pqc_pq_encode_token; here a token that already has that code, so the inputs stay as they are), then the step
    if not args.no_append:
        import ctypes as C

        pos = w.n_tokens - w.n_local - 1
        cfg = binding.make_config(w)
        lib = binding.load()
        keys1 = [st[3][:, :, pos].contiguous() for st in sets]

        def sep(i):
            a = margs[i]
            rc = lib.pqc_pq_encode_token(C.byref(cfg), keys1[i].data_ptr(), a[1], a[2], pos, stream_handle)
            assert rc == 0
            step(i)

        r_sep, _, _ = time_steps(sep, len(sets), args.steps, args.warmup, 1)
        # the same through pqc_decode_append, which writes the code from inside the step's own launches;
        # the position must be one whose code the step ignores: the last token of the local window
        last = w.n_tokens - 1
        keys2 = [st[3][:, :, last].contiguous() for st in sets]

        def fused(i):
            a = margs[i]
            rc = lib.pqc_decode_append(ctx.handle, a[0], a[1], a[2], a[3], a[4], keys2[i].data_ptr(), last, a[5], a[6], stream_handle)
            assert rc == 0

        r_app, _, _ = time_steps(fused, len(sets), args.steps, args.warmup, 1)
        result["decode_loop_step"] = {"us_per_layer": round(float(r_app[0]), 3),
                                      "calls": "pqc_decode_append (the appended token's code written inside the step)",
                                      "separate_calls_us_per_layer": round(float(r_sep[0]), 3)}

    # a plain device-to-device copy (reads and writes 1 GiB each way), as the ceiling a streaming kernel reaches here
    if not args.no_copy_ceiling:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(2):
            dst.copy_(src)
        torch.cuda.synchronize()
        ev0.record()
        for _ in range(5):
            dst.copy_(src)
        ev1.record()
        torch.cuda.synchronize()
        copy_gbps = 2 * src.numel() * 5 / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
        result["copy_ceiling"] = {"gbps": round(copy_gbps, 1), "path_frac_of_copy": round(path_gbps / copy_gbps, 4),
                                  "select_kernel_frac_of_copy": round(sel_gbps / copy_gbps, 4)}
        del src, dst

    # PQ construction on the GPU (not part of the decode step): K-Means over all cached keys of one layer
    # bytes a build must move: every round reads all keys twice (assignment, centroid sums) and writes and reads the
    # codes; one more assignment at the end; flops of the assignments (tokens x centroids x 128 multiply-adds)
    units = w.batch * w.n_kv_heads
    passes = 2 * w.kmeans_iters + 1
    build_bytes = units * passes * w.n_tokens * (w.head_dim * w.elem_bytes + w.pq_m)
    build_flops = units * (w.kmeans_iters + 1) * 2.0 * w.n_tokens * w.pq_centroids * w.head_dim
    build_s = float(np.median(build_ms)) * 1e-3
    result["pq_build"] = {"ms_per_layer": round(float(np.median(build_ms)), 3), "kmeans_iters": w.kmeans_iters,
                          "algorithmic_bytes": build_bytes, "hbm_frac": round(build_bytes / build_s / 1e9 / HBM_PEAK_GBPS, 4),
                          "assignment_tflops": round(build_flops / build_s / 1e12, 1),
                          "note": "host-timed pqc_pq_build (K-Means with kmeans_iters rounds), median over the input sets; "
                                  "not part of the decode step"}

    if with_cpu:
        check, t_first, (cent_h, codes_h, scale) = against_oracle(w, ctx, sets[0], host0, out_idx, out_attn)
        reps, t_cpu = 1, t_first
        while t_cpu < args.cpu_seconds and reps < 2000:
            t = time.perf_counter()
            oracle.decode(host0["q"], cent_h, codes_h, host0["k"], host0["v"], w.dtype, w.topk, w.n_init, w.n_local, scale)
            t_cpu += time.perf_counter() - t
            reps += 1
        result["cpu_baseline"] = {"value": round(t_cpu / reps * 1e6, 1), "unit": "us/layer", "cores": oracle.threads(),
                                  "kind": "oracle", "sample": f"{reps} full steps of the same workload (input set 0)",
                                  "gpu_matches_oracle": check}

    # ------------------------------------------------------------------ the other benchmark shapes
    del sets, margs, ctx, host0
    torch.cuda.empty_cache()
    also = []
    for name in [n for n in args.also.split(",") if n and n != w.name]:
        w2 = wl.get(name)
        # enough input sets for the attended rows of one round to exceed the last-level cache (at most 12 sets)
        n_sets = max(2, min(12, -(-300_000_000 // max(1, sel_bytes_of(w2)))))
        ctx2 = binding.PQCache(w2, dev)
        sets2, host2, _ = make_sets(w2, n_sets, 200)
        idx2, attn2 = ctx2.empty_outputs()
        margs2 = [ctx2.marshal_decode_args(*st, idx2, attn2) for st in sets2]
        r2, _, _ = time_steps(lambda i: ctx2.decode_marshalled(margs2[i], stream_handle), n_sets, args.also_steps,
                              min(args.warmup, 20), args.reps)
        us2 = float(np.median(r2))
        k2 = kernel_times(w2, ctx2, sets2, margs2, min(args.profile_steps, 12))
        b2, sb2 = w2.algorithmic_bytes(), sel_bytes_of(w2)
        entry = {"workload": w2.name, "us_per_layer": round(us2, 3), "us_min": round(float(r2.min()), 3),
                 "us_max": round(float(r2.max()), 3), "steps": args.also_steps, "repetitions": args.reps, "input_sets": n_sets,
                 "dtype": w2.dtype, "algorithmic_bytes_per_step": b2,
                 "hbm_frac": round(b2 / (us2 * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                 "kernel_us": {n: round(float(x), 3) for n, x in zip(KERNELS, k2)},
                 "select_kernel_hbm_frac": round(sb2 / (k2[1] * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4) if k2[1] > 0 else None}
        if with_cpu:
            entry["gpu_matches_oracle"], t_o, _ = against_oracle(w2, ctx2, sets2[0], host2, idx2, attn2)
            entry["oracle_us_per_layer"] = round(t_o * 1e6, 1)
        also.append(entry)
        del sets2, margs2, ctx2, host2, idx2, attn2
        torch.cuda.empty_cache()
    if also:
        result["also"] = also
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
