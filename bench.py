#!/usr/bin/env python3
"""Benchmark of the LoRANN query phase on one MI355X.

A "step" is one lorann_search call over one batch of synthetic queries (all stages: projection, routing,
int8 scoring, top-m, exact re-rank), with index, queries and outputs resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload embed-ip]
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

import numpy as np

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PEAK_BF16_MFMA_TFLOPS = 2500.0 # dense bf16 MFMA
PEAK_FP64_MFMA_TFLOPS = 78.6
PEAK_INT8_MFMA_TOPS = 5000.0
PEAK_VALU_LANE_TOPS = 256 * 64 * 2.4e9 / 1e12   # 256 CUs x 64 lanes x 2.4 GHz = 39.3 T lane-ops/s

# HBM bytes per launch (GB) measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by the copy-kernel
# calibration (profiles/hbm_traffic_embed-ip_pmc.txt).  Valid for the default workload only.
MEASURED_TRAFFIC_GB = {("embed-ip", 1.0, "rerank"): 3.26}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def recall_at_k(ids, dists, gt_dists):
    """Fraction of returned points that are true k-NN; a returned point counts when its exact distance does
    not exceed the k-th true distance (tolerance 1e-5 relative), so ties are not punished."""
    kth = gt_dists[:, -1:].astype(np.float64)
    ok = (dists.astype(np.float64) <= kth + 1e-5 * np.abs(kth)) & (ids >= 0)
    return float(ok.mean())


def kernel_models(wl, nq, touched_rows, npairs, column_scales=False, mixed=False):
    """Algorithmic work of one launch of each kernel: (bound, amount, unit-peak)."""
    d, dp, r, L, m = wl.d, wl.dp, wl.r, wl.L, wl.m
    b_bytes = touched_rows * (r + (4 if wl.metric == 1 else 0) + (4 if column_scales else 0) + (4 if mixed else 0)) + npairs * (r + 4 + (4 if mixed else 0))
    return {
        "project_f64": ("mfma", 2.0 * nq * d * dp / 1e12, PEAK_FP64_MFMA_TFLOPS, "TFLOP/s"),
        "centroid_dissim_f64": ("mfma", 2.0 * nq * dp * L / 1e12, PEAK_FP64_MFMA_TFLOPS, "TFLOP/s"),
        # approximate scores on the bf16 matrix cores; in practice bound by writing the nq x L float matrix
        "centroid_screen_bf16": ("mfma", 2.0 * nq * dp * L / 1e12, PEAK_BF16_MFMA_TFLOPS, "TFLOP/s"),
        "quantize_rows": ("hbm", nq * dp * 5 / 1e9, PEAK_HBM_GBS, "GB/s"),
        "select_clusters": ("hbm", nq * L * 4 / 1e9, PEAK_HBM_GBS, "GB/s"),
        "scatter_pairs": ("hbm", npairs * 12 / 1e9, PEAK_HBM_GBS, "GB/s"),
        "stage_a_i8": ("hbm", (L * dp * r + npairs * (dp + r + 4)) / 1e9, PEAK_HBM_GBS, "GB/s"),
        # B_c scoring (each of the two passes): every touched code once + the pairs' z / sigma (+ |c|^2 for Euclidean)
        "pair_max_i8": ("hbm", b_bytes / 1e9, PEAK_HBM_GBS, "GB/s"),
        "score_select_exact": ("hbm", b_bytes / 1e9, PEAK_HBM_GBS, "GB/s"),
        "rerank": ("hbm", nq * m * d * 4 / 1e9, PEAK_HBM_GBS, "GB/s"),
    }


def batch_sweep(torch, gix, wl, dev, batch_sizes, k, w, m, cluster_sizes, draw_queries):
    """Per-batch latency and throughput at several batch sizes, each batch a distinct query set; and the B_c
    scoring kernel (pair maxima) against the HBM roof: bytes = codes of the clusters the batch touches, once,
    plus the pairs' z and sigma."""
    rows = []
    for b in batch_sizes:
        iters = 200 if b <= 1024 else (40 if b <= 16384 else 10)
        n_sets = min(iters, max(1, (1 << 22) // b))               # distinct query sets held at once
        pool = draw_queries(wl, dev, b * n_sets, 100 + len(rows))
        out = (torch.empty((b, k), dtype=torch.int64, device=dev), torch.empty((b, k), dtype=torch.float32, device=dev))
        for i in range(3):
            gix.search(pool[(i % n_sets) * b:(i % n_sets + 1) * b], k, w, m, out=out)
        torch.cuda.synchronize()
        lat = []
        for i in range(iters):
            q = pool[(i % n_sets) * b:(i % n_sets + 1) * b]
            t0 = time.perf_counter()
            gix.search(q, k, w, m, out=out)
            torch.cuda.synchronize()
            lat.append((time.perf_counter() - t0) * 1e3)
        lat = np.sort(np.array(lat))
        # kernel table of this batch size (events on every kernel; separate pass)
        gix.profile_enable(1)
        n_ev = min(iters, 20)
        for i in range(n_ev):
            gix.search(pool[(i % n_sets) * b:(i % n_sets + 1) * b], k, w, m, out=out)
        torch.cuda.synchronize()
        prof = gix.profile_get()
        gix.profile_enable(0)
        sel = gix.search_stages(pool[:min(b, 20000)], k, w, m)[2]["sel"]
        touched = np.zeros(wl.L, bool)
        touched[np.unique(sel)] = True
        frac_seen = min(b, 20000) / b
        touched_rows = int(cluster_sizes[touched].sum()) if frac_seen == 1.0 else int(cluster_sizes.sum())
        b_bytes = touched_rows * (wl.r + (4 if wl.metric == 1 else 0)) + b * w * (wl.r + 4)
        row = {"batch": b, "iters": iters, "latency_ms_p50": round(float(np.percentile(lat, 50)), 4),
               "latency_ms_p99": round(float(np.percentile(lat, 99)), 4), "latency_ms_best": round(float(lat[0]), 4),
               "queries_per_s": round(b / (float(np.median(lat)) / 1e3), 1),
               "touched_clusters": int(touched.sum()) if frac_seen == 1.0 else None,
               "kernels_ms": {n: round(ms / max(1, c), 5) for n, (ms, c) in prof.items() if c}}
        pm = prof.get("pair_max_i8")
        if pm and pm[1]:
            avg_ms = pm[0] / pm[1] * (pm[1] / n_ev)               # per search call (large batches run in chunks)
            row["b_scoring"] = {"kernel": "pair_max_i8", "bytes": b_bytes, "ms_per_batch": round(avg_ms, 5),
                                "achieved_GBs": round(b_bytes / 1e9 / (avg_ms / 1e3), 1), "peak_GBs": PEAK_HBM_GBS,
                                "frac": round(b_bytes / 1e9 / (avg_ms / 1e3) / PEAK_HBM_GBS, 4)}
        log(f"[bench] sweep batch {b}: p50 {row['latency_ms_p50']} ms, p99 {row['latency_ms_p99']} ms, "
            f"{row['queries_per_s']:.0f} q/s, B scoring {row.get('b_scoring')}")
        rows.append(row)
        del pool, out
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="embed-ip")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (development only)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target duration of the oracle baseline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--random-index", action="store_true",
                    help="skip the index fit: random factors and codes of the workload's shapes (kernel timing and "
                         "profiling only; recall is not reported)")
    ap.add_argument("--batch", type=int, default=None, help="queries per step (default: the workload's batch)")
    ap.add_argument("--recall-queries", type=int, default=10000, help="recall is measured on this many queries of the batch")
    ap.add_argument("--batch-sweep", default="", help="comma-separated batch sizes: per-batch latency (p50/p99), "
                    "queries/s and the B_c scoring kernel's GB/s at each, reported under 'batch_sweep'")
    ap.add_argument("--rerank", choices=["f32", "f16", "none"], default="f32",
                    help="what the last step reads: the float corpus (the headline configuration), its half-precision "
                         "copy, or nothing (no re-ranking step)")
    ap.add_argument("--column-scales", action="store_true",
                    help="quantize every column of A_c and B_c with its own step size (Sec. 3.3 as printed) instead of "
                         "one step size per cluster (the configured format of the headline run)")
    ap.add_argument("--mixed-precision", action="store_true",
                    help="mixed-precision decomposition (paper Sec. 4.2): the first component of the projected query and the "
                         "first row of every A_c and B_c stay in float (implies --column-scales; a separate mode, not the headline)")
    ap.add_argument("--lanes", type=int, default=4,
                    help="batches in flight: the timed steps are enqueued round-robin on this many lanes of the index "
                         "(lorann_search_lane), each with its own workspace and stream; 1 = one batch at a time")
    ap.add_argument("--timed-only", action="store_true",
                    help="run the warm-up, the timed steps and one result pass only - no context loops, no per-kernel "
                         "event pass, no other modes - so that a profiler attached to the process sees the timed "
                         "configuration and little else")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 1 GiB elementwise copy (calibrates the HBM byte counters under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (query-sharded data parallelism would "
              "replicate the index and split the batch); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2410_18926_amd import binding
    from paper_2410_18926_amd.synth import get_workload, make_dataset, build_index, random_index, draw_queries
    from paper_2410_18926_amd.synth.data import brute_force_topk

    if not torch.cuda.is_available():
        print("bench.py needs the GPU (no CPU fallback exists for the search)", file=sys.stderr)
        sys.exit(2)
    binding.lib()
    dev = torch.device("cuda:0")
    wl = get_workload(args.workload)
    if args.scale != 1.0:
        wl = wl.scaled(args.scale)
    if args.batch:
        wl = dataclasses.replace(wl, nq=args.batch)
    K, W = args.steps, args.warmup

    t0 = time.time()
    nb = max(1, min(K + W, 8))
    corpus, queries, extra = make_dataset(wl, dev, extra_batches=nb - 1) if nb > 1 else (*make_dataset(wl, dev), [])
    batches = [queries] + list(extra)
    torch.cuda.synchronize()
    log(f"[bench] data {wl.name}: corpus {tuple(corpus.shape)}, {nb} batches of {wl.nq} queries in {time.time() - t0:.1f}s")
    t0 = time.time()
    if args.random_index:
        ix = random_index(corpus, wl)
    else:
        ix = build_index(corpus, wl, progress=lambda s: log(f"[bench]   index: {s}"), column_scales=args.column_scales or args.mixed_precision,
                         mixed_precision=args.mixed_precision)
    torch.cuda.synchronize()
    build_s = time.time() - t0
    log(f"[bench] index built in {build_s:.1f}s")
    n_rec = min(wl.nq, args.recall_queries if not args.random_index else 16)
    gt_ids, gt_d = brute_force_topk(corpus, queries[:n_rec], wl.metric, wl.k)
    gt_d = gt_d.cpu().numpy()
    del corpus
    log(f"[bench] ground truth for {n_rec} queries done")

    gix = binding.Index.from_arrays(ix)
    gix.use_torch_stream()
    rerank_modes = {"f32": binding.RERANK_F32, "f16": binding.RERANK_F16, "none": binding.RERANK_NONE}
    gix.set_rerank(rerank_modes[args.rerank])
    nq, k, w, m = wl.nq, wl.k, min(wl.w, wl.L), wl.m
    out = (torch.empty((nq, k), dtype=torch.int64, device=dev), torch.empty((nq, k), dtype=torch.float32, device=dev))
    n_lanes = max(1, min(args.lanes, binding.LANES))
    outs = [out] + [(torch.empty_like(out[0]), torch.empty_like(out[1])) for _ in range(n_lanes - 1)]

    def run_steps(n_steps, first):
        """Enqueue n_steps steps round-robin over the lanes and join the lanes onto the index's stream; no host wait."""
        for s in range(n_steps):
            gix.search(batches[(first + s) % nb], k, w, m, out=outs[s % n_lanes], lane=s % n_lanes)
        for l in range(n_lanes):
            gix.lane_join(l)

    run_steps(max(W, n_lanes), 0)          # warm-up (every lane sizes its workspace)
    torch.cuda.synchronize()
    # Timed region: K steps.  HIP events bracket the dominant kernel (the re-rank gather) only, so that timing
    # the kernels does not slow the step being timed.
    # The steps are enqueued without a host wait in between, round-robin on the index's lanes (lorann_search_lane),
    # as a serving loop would: up to n_lanes batches are in flight, each one passing through the whole path; the
    # timed region ends with the device synchronisation below.
    gix.profile_enable(2)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(K, W)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof_dom = gix.profile_get()
    fallback_queries = gix.profile_fallback_queries()
    # for context: the same loop with the gathers of different lanes allowed to overlap (each launch then takes
    # longer, so the kernel's own figures above are not taken from it)
    overlapped = None
    if n_lanes > 1 and not args.timed_only:
        gix.profile_enable(0)
        gix.set_gather_turns(False)
        run_steps(n_lanes, 0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_steps(K, W)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        gix.set_gather_turns(True)
        overlapped = {"queries_per_s": round(nq * K / dt, 1), "ms_per_step": round(dt / K * 1e3, 4)}
    elapsed_one_lane, elapsed_allev, prof_one, prof = float("nan"), float("nan"), {}, dict(prof_dom)
    if not args.timed_only:
        # for context: the same K steps one batch at a time (one lane)
        gix.profile_enable(2)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(K):
            gix.search(batches[(W + s) % nb], k, w, m, out=out, asynchronous=True)
        torch.cuda.synchronize()
        elapsed_one_lane = time.perf_counter() - t0
        prof_one = gix.profile_get()
        # The same loop again with events around every kernel, for the per-kernel table.
        gix.profile_enable(1)
        t0 = time.perf_counter()
        for s in range(K):
            gix.search(batches[(W + s) % nb], k, w, m, out=out)
        torch.cuda.synchronize()
        elapsed_allev = time.perf_counter() - t0
        prof = gix.profile_get()
    gix.profile_enable(0)

    ids, dists = gix.search(queries, k, w, m)
    ids_h, dists_h = ids.cpu().numpy(), dists.cpu().numpy()
    recall = recall_at_k(ids_h[:n_rec], dists_h[:n_rec], gt_d)
    # map returned ids (original corpus indices) check: true top-k ids overlap, as a second recall definition
    gt_ids_h = gt_ids.cpu().numpy()
    recall_ids = float(np.mean([len(set(ids_h[i]) & set(gt_ids_h[i])) / k for i in range(0, n_rec, max(1, n_rec // 2000))]))
    if args.rerank != "f32":
        recall = recall_ids          # the returned distances are not the exact ones: count by id only

    # per-kernel roofline figures from the events recorded over the timed region
    sizes = (ix.cluster_offsets[1:] - ix.cluster_offsets[:-1]).cpu().numpy()
    # clusters touched by the batch (their codes are what the scoring kernel has to read at least once)
    touched = np.ones(wl.L, bool)
    if not args.timed_only:
        sel_all = gix.search_stages(queries[:20000], k, w, m)[2]["sel"]
        touched[:] = False
        touched[np.unique(sel_all)] = True
    touched_rows = int(sizes[touched].sum())
    models = kernel_models(wl, nq, touched_rows, nq * w, args.column_scales or args.mixed_precision, args.mixed_precision)
    if args.rerank == "f16":
        bound, amount, peak, unit = models["rerank"]
        models["rerank"] = (bound, amount / 2, peak, unit)           # two bytes per gathered element
    kernels = []
    for name, (ms, launches) in prof.items():
        if launches == 0:
            continue
        avg_ms = ms / launches
        ent = {"kernel": name, "avg_ms": round(avg_ms, 5), "launches_per_step": launches / K}
        if name in models:
            # the models give the work of one STEP (a batch larger than 32768 queries runs in several launches)
            bound, amount, peak, unit = models[name]
            ach = amount / (ms / K / 1e3)
            ent.update({"bound": bound, "achieved": round(ach, 3), "peak": peak, "unit": unit, "frac": round(ach / peak, 4)})
        kernels.append(ent)
    kernels.sort(key=lambda e: -e["avg_ms"])
    dom = next((e for e in kernels if "bound" in e), None)
    roofline = None
    if dom:
        # the dominant kernel's figures come from the events of the timed region itself
        ms, launches = prof_dom.get(dom["kernel"], (0.0, 0))
        if launches:
            bound, amount, peak, unit = models[dom["kernel"]]
            ach = amount / (ms / K / 1e3)
            dom = dict(dom, avg_ms=round(ms / launches, 5), achieved=round(ach, 3), frac=round(ach / peak, 4))
        roofline = {"kernel": dom["kernel"], "bound": dom["bound"], "achieved": dom["achieved"], "peak": dom["peak"],
                    "unit": dom["unit"], "frac": dom["frac"], "avg_ms": dom["avg_ms"],
                    "traffic": MEASURED_TRAFFIC_GB.get((args.workload, args.scale, dom["kernel"])) if args.rerank == "f32" else None}
        if roofline["traffic"] and roofline["avg_ms"]:
            # the kernel shares row reads between neighbouring queries, so it moves fewer bytes than the algorithmic
            # count: the rate of the bytes it really moved is the figure to hold against the HBM peak
            roofline["traffic_rate"] = round(roofline["traffic"] / (roofline["avg_ms"] / 1e3), 1)
            roofline["traffic_frac"] = round(roofline["traffic_rate"] / PEAK_HBM_GBS, 4)

    # The other two modes of the last step, timed the same way (fewer steps), with recall by id against the true
    # neighbours: context for the headline figure, which is always the mode selected by --rerank.
    other_modes = {}
    for name, mode in rerank_modes.items():
        if name == args.rerank or args.timed_only:
            continue
        gix.set_rerank(mode)
        for s in range(2):
            gix.search(batches[s % nb], k, w, m, out=out)
        torch.cuda.synchronize()
        Km = max(1, min(K, 10))
        run_steps(n_lanes, 0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_steps(Km, 0)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        mi = gix.search(queries[:n_rec], k, w, m)[0].cpu().numpy()
        rec = float(np.mean([len(set(mi[i]) & set(gt_ids_h[i])) / k for i in range(n_rec)]))
        other_modes[name] = {"queries_per_s": round(nq * Km / dt, 1), "ms_per_step": round(dt / Km * 1e3, 4), "steps": Km,
                             "recall_at_10_by_id": None if args.random_index else round(rec, 4)}
        log(f"[bench] rerank mode {name}: {other_modes[name]}")
    gix.set_rerank(rerank_modes[args.rerank])

    sweep = None
    if args.batch_sweep:
        sweep = batch_sweep(torch, gix, wl, dev, [int(x) for x in args.batch_sweep.split(",")], k, w, m, sizes, draw_queries)

    cpu_baseline = None
    oracle_match = None
    if not args.no_cpu_baseline:
        from oracle import oracle as O
        t0 = time.time()
        a = ix.numpy()
        if args.rerank == "f16":
            a = O.with_half_precision_corpus(a)
        oix = O.OracleIndex(a)
        o_search = (lambda q: O.search_no_rerank(oix, q, k, w, threads=threads)) if args.rerank == "none" else \
                   (lambda q: O.search(oix, q, k, w, m, threads=threads))
        qh = torch.cat(batches, 0).cpu().numpy()      # the timed batches, in order (the first is the recall batch)
        threads = O.default_threads()
        o_search(qh[:threads * 2])            # warm pass
        t1 = time.perf_counter()
        n_cal = min(nq, threads * 8)
        o_search(qh[:n_cal])
        rate = n_cal / (time.perf_counter() - t1)
        n_s = int(max(n_cal, min(qh.shape[0], rate * args.cpu_seconds)))
        t1 = time.perf_counter()
        o_ids, o_d = o_search(qh[:n_s])
        dt = time.perf_counter() - t1
        cpu_baseline = {"value": round(n_s / dt, 1), "unit": "queries/s", "cores": threads, "kind": "oracle",
                        "sample": f"first {n_s} of the {qh.shape[0]} queries of the {nb} timed batches, same index, one pass of {dt:.1f}s"}
        n_m = min(n_s, nq)                 # the GPU results held on the host are those of the first batch
        oracle_match = {"queries": n_m, "id_lists_identical": float(np.mean(np.all(o_ids[:n_m] == ids_h[:n_m], axis=1))),
                        "ids_equal": float(np.mean(o_ids[:n_m] == ids_h[:n_m])),
                        "max_rel_dist_err": float(np.max(np.abs(o_d[:n_m] - dists_h[:n_m]) / np.maximum(np.abs(o_d[:n_m]), 1e-3)))}
        log(f"[bench] oracle baseline done in {time.time() - t0:.1f}s")

    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read + 1 GiB written per launch
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    metric_names = {0: "inner product", 1: "squared Euclidean", 2: "cosine"}
    res = {
        "metric": "queries/sec at recall@10>=0.9 (1 MI355X, batch 10k)",
        "value": round(nq * K / elapsed, 1),
        "unit": "queries/s",
        "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(elapsed / K * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"{wl.name}: corpus {wl.n}x{wl.d} fp32, {wl.G}-component anisotropic Gaussian mixture, "
                               f"{metric_names[wl.metric]}, L={wl.L} clusters, d'={wl.dp}, r={wl.r} int8, batch {nq}, "
                               f"w={w}, m={m}, k={k}",
                   "n": wl.n, "d": wl.d, "batch": nq, "L": wl.L, "dp": wl.dp, "r": wl.r, "w": w, "m": m, "k": k,
                   "quantization": "float first component of q' and first row of A_c and B_c; one step size per column of the rest" if args.mixed_precision else "one step size per column of A_c and of B_c" if args.column_scales else "one step size per cluster and matrix",
                   "rerank": {"f32": "float corpus", "f16": "half-precision copy of the corpus", "none": "no re-ranking step"}[args.rerank]},
        "recall_at_10": None if args.random_index else round(recall, 4),
        "recall_at_10_by_id": None if args.random_index else round(recall_ids, 4),
        "index": "random factors and codes (timing only)" if args.random_index else "fitted",
        "roofline": roofline, "cpu_baseline": cpu_baseline,
        "kernels": kernels, "oracle_match": oracle_match,
        "batches_in_flight": n_lanes,
        "with_overlapping_gathers": overlapped,
        "ms_per_step_one_batch_at_a_time": None if args.timed_only else round(elapsed_one_lane / K * 1e3, 4),
        "rerank_avg_ms_one_batch_at_a_time": round(prof_one["rerank"][0] / max(1, prof_one["rerank"][1]), 5) if "rerank" in prof_one else None,
        "ms_per_step_with_events_on_every_kernel": None if args.timed_only else round(elapsed_allev / K * 1e3, 4),
        "fallback_queries_per_step": fallback_queries / K,
        "index_build_s": round(build_s, 1),
        "other_rerank_modes": other_modes,
    }
    if sweep is not None:
        res["batch_sweep"] = sweep
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
