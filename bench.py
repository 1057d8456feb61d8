#!/usr/bin/env python3
"""Benchmark of the PQ decode hot path on one MI355X.

A step is one pqc_decode call: look-up table, code scan, top-k selection, gather of the
selected K/V rows and attention, for one attention layer of the workload.  Inputs are
seeded synthetic tensors, resident in HBM before the timed region; `--layers` distinct
input sets are visited round-robin (as a model walks its layers) so that the K/V rows
are fetched from HBM, not from the 256 MB last-level cache.  PQ structures are built
on the GPU by the library's own K-Means (pqc_pq_build) before timing starts.

Prints ONE JSON line: the step time (us per layer), the achieved fraction of the HBM
roofline for the whole path and for its dominant kernel (timed live with HIP events
through pqc_decode_phase), and the CPU oracle's time for the same step as a baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="llama8b_128k")
    ap.add_argument("--layers", type=int, default=8, help="distinct input sets visited round-robin")
    ap.add_argument("--profile-steps", type=int, default=24, help="rounds of the per-kernel timing (each launches every kernel once per input set)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-indexed", action="store_true", help="skip the pqc_decode_indexed measurement")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP graph replay measurement")
    ap.add_argument("--no-append", action="store_true", help="skip the encode-token + decode measurement")
    ap.add_argument("--no-copy-ceiling", action="store_true", help="skip the device-to-device copy measurement")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--also", default="llama70b_128k", help="second workload reported alongside (step time only); '' to skip")
    ap.add_argument("--also-layers", type=int, default=3)
    ap.add_argument("--also-steps", type=int, default=150)
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="also run one plain device copy of this size (reference for scaling rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2407_12820_amd import binding, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    dev = "cuda:0"
    w = wl.get(args.workload)
    ctx = binding.PQCache(w, dev)

    # ---- inputs: `layers` independent seeded sets, PQ structures from the GPU K-Means
    sets, host0 = [], None
    build_ms = []
    for layer in range(args.layers):
        d = wl.generate(w, seed=100 + layer)
        q, k, v = (binding.to_device(d[n], w.dtype, dev) for n in ("q", "k", "v"))
        init = torch.from_numpy(wl.kmeans_init_indices(w, seed=100 + layer)).to(dev)
        torch.cuda.synchronize()
        tb = time.perf_counter()
        cent, codes = binding.pq_build(w, k, init)
        torch.cuda.synchronize()
        build_ms.append((time.perf_counter() - tb) * 1e3)
        sets.append((q, cent, codes, k, v))
        if layer == 0:
            host0 = d
        else:
            del d
    out_idx, out_attn = ctx.empty_outputs()
    torch.cuda.synchronize()

    # argument checks and address look-ups done once per input set, outside the timed loops
    margs = [ctx.marshal_decode_args(*st, out_idx, out_attn) for st in sets]
    stream_handle = torch.cuda.current_stream(dev).cuda_stream

    def step(i: int) -> None:
        ctx.decode_marshalled(margs[i % len(sets)], stream_handle)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for i in range(args.steps):
        step(i)
    ev1.record()
    issue_ms = (time.perf_counter() - t0) * 1e3  # host time to enqueue the steps (the GPU must not wait for it)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = ev0.elapsed_time(ev1) / args.steps
    us = ms_per_step * 1e3

    # ---- per-kernel durations: each kernel of the path is launched for every input set back to
    # back (one context per set) between two HIP events on the launch stream, so that no event
    # sits in front of a timed launch; duration = span / number of launches
    kern_us = np.zeros(3)
    if args.profile_steps > 0:
        ctxs = [ctx] + [binding.PQCache(w, dev) for _ in sets[1:]]
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        for rnd in range(args.profile_steps + 2):  # two untimed rounds first
            for ph in range(3):
                evs[ph].record()
                for c, a in zip(ctxs, margs):
                    c.decode_phase_marshalled(ph, a, stream_handle)
            evs[3].record()
            torch.cuda.synchronize()
            if rnd >= 2:
                kern_us += np.array([evs[i].elapsed_time(evs[i + 1]) for i in range(3)]) * 1e3 / len(sets)
        kern_us /= args.profile_steps
        del ctxs

    if args.copy_calibration_mib:
        src = torch.empty(args.copy_calibration_mib << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)  # one elementwise copy kernel: reads and writes exactly this many bytes
        torch.cuda.synchronize()
        del src, dst

    units = w.batch * w.n_kv_heads
    path_bytes = w.algorithmic_bytes()
    # dominant kernel (select + attention): the I+K+L attended K and V rows and the queries; the per-token
    # bins it reads instead of the codes are this implementation's own traffic and are not credited
    sel_bytes = units * w.n_selected * w.head_dim * 2 * w.elem_bytes + w.batch * w.n_q_heads * w.head_dim * w.elem_bytes
    sel_gbps = sel_bytes / (kern_us[1] * 1e-6) / 1e9 if kern_us[1] > 0 else 0.0
    path_gbps = path_bytes / (us * 1e-6) / 1e9

    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"select_kernel_{w.name}_traffic.json")
    if os.path.exists(tpath):  # HBM bytes per launch measured with rocprofv3 --pmc (see the file for the commands)
        with open(tpath) as f:
            traffic = json.load(f).get("hbm_bytes_per_launch")

    result = {
        "metric": "decode \u00b5s per layer (PQ score+top-k+sparse attn) at 128K ctx",
        "value": round(us, 3), "unit": "us/layer", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
                   "head_dim": w.head_dim, "n_tokens": w.n_tokens, "pq_m": w.pq_m, "pq_centroids": w.pq_centroids,
                   "topk": w.topk, "n_init": w.n_init, "n_local": w.n_local, "kv_dtype": w.dtype,
                   "kmeans_iters": w.kmeans_iters, "input_sets": len(sets), "accumulate": "f32"},
        "achieved_hbm_gbps": round(path_gbps, 1), "hbm_frac": round(path_gbps / HBM_PEAK_GBPS, 4),
        "algorithmic_bytes_per_step": path_bytes, "host_wall_ms_per_step": round(wall_ms / args.steps, 6),
        "host_issue_ms_per_step": round(issue_ms / args.steps, 6),
        "kernel_us": {"hist": round(float(kern_us[0]), 3), "select_attn": round(float(kern_us[1]), 3),
                      "finalize": round(float(kern_us[2]), 3)},
        "roofline": {"kernel": "select_kernel", "bound": "hbm", "achieved": round(sel_gbps, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(sel_gbps / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "bytes_per_launch": sel_bytes, "avg_us": round(float(kern_us[1]), 3)},
    }

    # the same step through pqc_decode_indexed (threshold from code-pair counts; two partitions only):
    # reported beside `value`, which stays the general path whose inputs are centroids and codes alone
    if not args.no_indexed and w.pq_m == 2 and w.pq_centroids <= 64 and w.n_tokens % 8 == 0:
        pcs = [binding.pair_counts(w, st[2]) for st in sets]
        pptr = [ctx._pair_ptr(pc) for pc in pcs]
        for i in range(args.warmup):
            ctx.decode_indexed_marshalled(margs[i % len(sets)], pptr[i % len(sets)], stream_handle)
        torch.cuda.synchronize()
        ev0.record()
        for i in range(args.steps):
            ctx.decode_indexed_marshalled(margs[i % len(sets)], pptr[i % len(sets)], stream_handle)
        ev1.record()
        torch.cuda.synchronize()
        us_i = ev0.elapsed_time(ev1) / args.steps * 1e3
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
        pos = w.n_tokens - w.n_local - 1
        cfg = binding.make_config(w)
        lib = binding.load()
        import ctypes as C
        keys1 = [st[3][:, :, pos].contiguous() for st in sets]
        for i in range(args.warmup):
            lib.pqc_pq_encode_token(C.byref(cfg), keys1[i % len(sets)].data_ptr(), margs[i % len(sets)][1], margs[i % len(sets)][2],
                                    pos, stream_handle)
            step(i)
        torch.cuda.synchronize()
        ev0.record()
        for i in range(args.steps):
            a = margs[i % len(sets)]
            rc = lib.pqc_pq_encode_token(C.byref(cfg), keys1[i % len(sets)].data_ptr(), a[1], a[2], pos, stream_handle)
            step(i)
        ev1.record()
        torch.cuda.synchronize()
        assert rc == 0
        us_sep = ev0.elapsed_time(ev1) / args.steps * 1e3
        # the same through pqc_decode_append, which writes the code from inside the step's own launches;
        # the position must be one whose code the step ignores: the last token of the local window
        last = w.n_tokens - 1
        keys2 = [st[3][:, :, last].contiguous() for st in sets]
        for i in range(args.warmup + args.steps):
            if i == args.warmup:
                torch.cuda.synchronize()
                ev0.record()
            a = margs[i % len(sets)]
            rc = lib.pqc_decode_append(ctx.handle, a[0], a[1], a[2], a[3], a[4], keys2[i % len(sets)].data_ptr(), last, a[5], a[6],
                                       stream_handle)
        ev1.record()
        torch.cuda.synchronize()
        assert rc == 0
        result["decode_loop_step"] = {"us_per_layer": round(ev0.elapsed_time(ev1) / args.steps * 1e3, 3),
                                      "calls": "pqc_decode_append (the appended token's code written inside the step)",
                                      "separate_calls_us_per_layer": round(us_sep, 3)}

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
    result["pq_build"] = {"ms_per_layer": round(float(np.median(build_ms)), 3), "kmeans_iters": w.kmeans_iters,
                          "note": "host-timed pqc_pq_build, median over the input sets"}

    if not args.no_cpu_baseline:
        import oracle

        q0, cent0, codes0, _, _ = sets[0]
        cent_h, codes_h = cent0.cpu().numpy(), codes0.cpu().numpy()
        scale = wl.softmax_scale(w)
        reps, t_cpu = 0, 0.0
        while t_cpu < args.cpu_seconds and reps < 2000:
            t = time.perf_counter()
            idx_h, out_h, _ = oracle.decode(host0["q"], cent_h, codes_h, host0["k"], host0["v"], w.dtype, w.topk, w.n_init,
                                            w.n_local, scale)
            t_cpu += time.perf_counter() - t
            reps += 1
        # the GPU's result for the same set, as a last sanity check of what was timed
        ctx.decode(*sets[0], out_idx, out_attn)
        torch.cuda.synchronize()
        same = bool(np.array_equal(np.sort(out_idx.cpu().numpy(), -1), np.sort(idx_h, -1)))
        err = float((np.abs(out_attn.cpu().numpy() - out_h).max(-1) / np.abs(out_h).max(-1)).max())
        result["cpu_baseline"] = {"value": round(t_cpu / reps * 1e6, 1), "unit": "us/layer", "cores": oracle.threads(),
                                  "kind": "oracle", "sample": f"{reps} full steps of the same workload (input set 0)",
                                  "gpu_matches_oracle": {"index_sets_equal": same, "attn_max_rel_err": err}}
    # ---- the other 128K-token shape (Llama-3-70B-like, batch 4), step time only
    if args.also and args.also != w.name:
        del sets, margs, ctx
        torch.cuda.empty_cache()
        w2 = wl.get(args.also)
        ctx2 = binding.PQCache(w2, dev)
        idx2, attn2 = ctx2.empty_outputs()
        margs2, keep = [], []
        for layer in range(args.also_layers):
            d = wl.generate(w2, seed=200 + layer)
            q, k, v = (binding.to_device(d[n], w2.dtype, dev) for n in ("q", "k", "v"))
            del d
            cent, codes = binding.pq_build(w2, k, torch.from_numpy(wl.kmeans_init_indices(w2, seed=200 + layer)).to(dev))
            keep.append((q, cent, codes, k, v))
            margs2.append(ctx2.marshal_decode_args(q, cent, codes, k, v, idx2, attn2))
        for i in range(args.warmup):
            ctx2.decode_marshalled(margs2[i % len(margs2)], stream_handle)
        torch.cuda.synchronize()
        ev0.record()
        for i in range(args.also_steps):
            ctx2.decode_marshalled(margs2[i % len(margs2)], stream_handle)
        ev1.record()
        torch.cuda.synchronize()
        us2 = ev0.elapsed_time(ev1) / args.also_steps * 1e3
        b2 = w2.algorithmic_bytes()
        result["also"] = {"workload": w2.name, "us_per_layer": round(us2, 3), "steps": args.also_steps, "input_sets": len(margs2),
                          "algorithmic_bytes_per_step": b2, "hbm_frac": round(b2 / (us2 * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
