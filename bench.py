#!/usr/bin/env python3
"""Benchmark of the CAGRA search hot path on one MI355X.

A "step" is one pass of the whole hot path -- the single-workgroup search of the full
query batch, steps 0-3 of Sec. IV-A until convergence -- over the large-batch workload
(1M x 128 integer-valued fp32 rows, 10,000 queries, degree-64 graph, k = 10), with
dataset, graph and queries already resident in HBM.  The graph is built once, untimed,
by the library's own build; the exact neighbours for recall (Eq. 2) come from the
library's exhaustive search.  itopk is swept and the timed steps use the smallest itopk
whose recall@10 reaches the target (0.95).

Prints ONE JSON line (see the keys below).  `roofline` prices the search kernel against
the HBM peak with the bytes the algorithm has to move (dataset rows of first-time
candidates, graph rows of parents, queries, results), counted inside the kernel.
`cpu_baseline` times the CPU oracle on a sample of the same queries with the same graph.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published
TARGET_RECALL = 0.95


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def recall_at_k(found: np.ndarray, truth: np.ndarray) -> float:
    hit = 0
    for f, t in zip(found, truth):
        hit += len(np.intersect1d(f, t, assume_unique=False))
    return hit / float(truth.size)


def algorithmic_bytes(stats: np.ndarray, dim: int, degree: int, k: int) -> dict:
    n_dist = int(stats[:, 2].astype(np.int64).sum())
    n_parent = int(stats[:, 1].astype(np.int64).sum())
    B = stats.shape[0]
    vec = n_dist * dim * 4
    total = vec + n_parent * degree * 4 + B * dim * 4 + B * k * 8
    return {"vector_bytes": vec, "total_bytes": total, "n_dist": n_dist, "n_parent": n_parent,
            "iterations_mean": float(stats[:, 0].mean()), "hit_cap": int((stats[:, 3] & 1).sum())}


def kernel_sources_sha16() -> str:
    """Hash of the files the search kernels are compiled from; a counter summary under profiles/
    names the hash of the sources it was measured with.  Blocks under `#ifdef CAGRA_PHASE_CLOCKS`
    (the phase timers, which the product build does not compile) are left out."""
    import glob
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2308_15136_amd", "csrc")
    names = ("search_kernels_impl.h", "search_device.h", "team_distance.h", "device_util.h", "search_params.h")
    for path in sorted(glob.glob(os.path.join(csrc, "search_kernels_*.hip")) + [os.path.join(csrc, n) for n in names]):
        h.update(os.path.basename(path).encode())
        skip = False
        for line in open(path, "rb").read().splitlines(keepends=True):
            word = line.strip()
            if word == b"#ifdef CAGRA_PHASE_CLOCKS":
                skip = True
            elif skip and word in (b"#else", b"#endif"):
                skip = False
            elif not skip:
                h.update(line)
    return h.hexdigest()[:16]


def measured_traffic(workload: str, width: int, itopk: int):
    """HBM bytes per launch of the search kernel from the committed rocprofv3 counter summary
    (FETCH_SIZE and WRITE_SIZE runs of this same script), if it covers this configuration AND was
    measured with the kernel sources as they are now.  Returns (bytes or None, where it came from)."""
    import re
    rel = os.path.join("profiles", f"search_single_{workload}_pmc.md")
    try:
        text = open(os.path.join(ROOT, rel)).read()
    except OSError:
        return None, None
    m = re.search(r"kernel_sources_sha16:\s*([0-9a-f]{16})", text)
    src = {"file": rel, "kernel_sources_sha16_of_profile": m.group(1) if m else None,
           "kernel_sources_sha16_now": kernel_sources_sha16()}
    src["stale"] = src["kernel_sources_sha16_of_profile"] != src["kernel_sources_sha16_now"]
    if src["stale"]:
        return None, src          # the kernels changed since the counters were read: no figure rather than an old one
    for m in re.finditer(r"traffic_bytes_per_launch:\s*(\d+)\s*\(search_width (\d+), itopk (\d+)", text):
        if int(m.group(2)) == width and int(m.group(3)) == itopk:
            return float(m.group(1)), src
    return None, src


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="sift1m")
    ap.add_argument("--n", type=int, default=0, help="shrink the base set (debugging only)")
    ap.add_argument("--queries", type=int, default=0)
    ap.add_argument("--k", type=int, default=0, help="neighbours per query (default: the workload's)")
    ap.add_argument("--print-kernel-hash", action="store_true", help="print the hash of the kernel sources and exit")
    ap.add_argument("--itopk", type=int, default=0, help="skip the itopk sweep and time this itopk")
    ap.add_argument("--width", type=int, default=0, help="skip the search_width sweep and use this width")
    ap.add_argument("--full-sweep", action="store_true",
                    help="per search_width go on beyond the first itopk that reaches the recall target")
    ap.add_argument("--cpu-sample", type=int, default=10000, help="queries given to the CPU oracle")
    ap.add_argument("--exact-algo", choices=("auto", "plain", "filtered"), default="auto",
                    help="arithmetic of the exhaustive search behind the exact initial graph (same graph either way)")
    ap.add_argument("--no-short", action="store_true", help="skip the sweep of lists shorter than the named itopk range")
    ap.add_argument("--no-latency", action="store_true", help="skip the small-batch (multi mode) latency part")
    ap.add_argument("--latency-workers", type=int, default=8, help="workgroups per query in the latency part")
    ap.add_argument("--latency-itopk", type=int, default=128)
    ap.add_argument("--traffic-bytes", type=float, default=None,
                    help="HBM bytes per launch from rocprofv3 counters for roofline.traffic (default: the value "
                         "in profiles/search_single_<workload>_pmc.md if it is for the timed configuration)")
    ap.add_argument("--initial-graph", choices=("exact", "nn-descent"), default="exact",
                    help="initial k-NN graph of the build (Sec. III-B.1): exhaustive search or NN-descent")
    ap.add_argument("--reorder", choices=("rank", "distance"), default="rank",
                    help="edge reordering of the graph optimisation (Sec. III-B.2); rank is CAGRA's")
    ap.add_argument("--no-graph-report", action="store_true", help="skip the 2-hop / connected-component report")
    ap.add_argument("--no-graph", action="store_true", help="skip the captured-graph replay of the batch-1 call")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--ablations", action="store_true",
                    help="also time the alternatives to the automatic choices (team size, visited table, mode)")
    ap.add_argument("--no-scaling", action="store_true", help="skip the larger-batch runs")
    ap.add_argument("--no-storage", action="store_true", help="skip the fp16 / uint8 storage part")
    ap.add_argument("--no-reference", action="store_true", help="skip the stream / row-gather bandwidth references")
    ap.add_argument("--timeline", action="store_true",
                    help="per-query start / end times of one launch at the timed point, for 1, 2 and 4 wavefronts per query; "
                         "needs a library built with -DCAGRA_PHASE_CLOCKS (python -m paper_2308_15136_amd.buildlib --define "
                         "CAGRA_PHASE_CLOCKS --out <file>, then CAGRA_HIP_LIB=<file>)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reference dispatch for rocprofv3 counters)")
    args = ap.parse_args()
    if args.print_kernel_hash:
        print(kernel_sources_sha16())
        return 0
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU; queries are independent, so more GPUs would "
            "each take a slice of the batch, but no multi-GPU path is part of it.")
        return 2

    import torch
    import paper_2308_15136_amd as cagra
    from paper_2308_15136_amd import datagen

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible; the search has no CPU fallback")
        return 1
    cagra.load_library()
    dev = torch.device("cuda:0")

    t0 = time.time()
    w = datagen.workload(args.workload, n=args.n or None, n_queries=args.queries or None)
    if args.k:
        import dataclasses
        w = dataclasses.replace(w, k=args.k, itopk=tuple(m for m in w.itopk if m >= args.k) or (args.k,))
    N, dim = w.base.shape
    B = w.queries.shape[0]
    log(f"[bench] workload {w.name}: base {N}x{dim}, {B} queries, degree {w.degree}, "
        f"generated in {time.time() - t0:.1f}s")
    base = torch.from_numpy(w.base).to(dev)
    queries = torch.from_numpy(w.queries).to(dev)

    exact_algo = {"auto": cagra.EXACT_AUTO, "plain": cagra.EXACT_PLAIN, "filtered": cagra.EXACT_FILTERED}[args.exact_algo]
    t0 = time.time()
    if N <= 2_000_000 or args.initial_graph == "nn-descent":
        graph = cagra.build(base, w.degree, w.init_degree, w.metric,
                            reorder=cagra.REORDER_DISTANCE if args.reorder == "distance" else cagra.REORDER_RANK,
                            nn_descent=args.initial_graph == "nn-descent", exact_algo=exact_algo)
        torch.cuda.synchronize()
    else:
        # the same two stages as cagra_build, the first in slices of rows so that a long build
        # reports its progress
        knn = torch.empty((N, w.init_degree), dtype=torch.int32, device=dev)
        knn_d = torch.empty((N, w.init_degree), dtype=torch.float32, device=dev) if args.reorder == "distance" else None
        step = 250_000
        for lo in range(0, N, step):
            hi = min(N, lo + step)
            part = cagra.exact_search(base, base[lo:hi], w.init_degree, w.metric, exclude_self=True,
                                      self_offset=lo, return_dists=knn_d is not None, algo=exact_algo)
            if knn_d is not None:
                knn[lo:hi], knn_d[lo:hi] = part
            else:
                knn[lo:hi] = part
            torch.cuda.synchronize()
            log(f"[bench] k-NN graph rows {hi}/{N} after {time.time() - t0:.0f}s")
        graph = cagra.optimize(knn, w.degree, knn_dists=knn_d)
        torch.cuda.synchronize()
        del knn, knn_d
    build_s = time.time() - t0
    log(f"[bench] graph built on the GPU in {build_s:.1f}s")

    # reachability of the graph as the paper measures it (Sec. III-A)
    graph_quality = None
    if not args.no_graph_report and w.degree <= 64:
        t0 = time.time()
        two_hop = cagra.two_hop_counts(graph).to(torch.float64)
        strong, weak = cagra.count_components(graph)
        graph_quality = {"mean_two_hop_count": round(float(two_hop.mean().item()), 1),
                         "max_possible": w.degree + w.degree * w.degree,
                         "strong_components": strong, "weak_components": weak}
        log(f"[bench] graph: mean 2-hop count {graph_quality['mean_two_hop_count']} of {graph_quality['max_possible']}, "
            f"{strong} strong / {weak} weak components ({time.time() - t0:.1f}s)")

    t0 = time.time()
    gt = cagra.exact_search(base, queries, w.k, w.metric, return_dists=False)
    torch.cuda.synchronize()
    gt_np = gt.cpu().numpy().view(np.uint32)
    log(f"[bench] exact neighbours in {time.time() - t0:.1f}s")

    opts = cagra.SearchOptions(seed=20230815, mode=1)
    ws = torch.empty(4096, dtype=torch.uint8, device=dev)
    ids = torch.empty((B, w.k), dtype=torch.int32, device=dev)
    dists = torch.empty((B, w.k), dtype=torch.float32, device=dev)
    stats = torch.zeros((B, 4), dtype=torch.int32, device=dev)

    def run(itopk, width):
        # every launch also writes its per-query counters (16 bytes per query), so the algorithmic
        # bytes below are those of the timed launches themselves
        return cagra.search(graph, base, queries, w.k, itopk, width, w.metric, opts,
                            out=(ids, dists), workspace=ws, stats=stats)

    def timed(itopk, width, steps, warmup):
        for _ in range(warmup):
            run(itopk, width)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t_start = time.perf_counter()
        e0.record()
        for _ in range(steps):
            run(itopk, width)
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t_start) * 1e3 / steps
        return wall_ms, e0.elapsed_time(e1) / steps

    # ---- sweep (search_width, itopk): (recall, QPS) pairs; per width up to the first itopk that
    #      reaches the target (QPS only falls beyond it) -------------------------------------------
    sweep = []
    widths = (args.width,) if args.width else w.search_widths
    sweep_list = (args.itopk,) if args.itopk else w.itopk
    best = None
    interpolated = []

    def sweep_point(M, p):
        wall_ms, dev_ms = timed(M, p, 5, 2)
        rec = recall_at_k(ids.cpu().numpy().view(np.uint32), gt_np)
        ab = algorithmic_bytes(stats.cpu().numpy().view(np.uint32), dim, w.degree, w.k)
        pt = {"search_width": p, "itopk": M, "recall": round(rec, 5), "qps": round(B / (wall_ms * 1e-3), 1),
              "kernel_ms": round(dev_ms, 4),
              "vector_GBs": round(ab["vector_bytes"] / (dev_ms * 1e-3) / 1e9, 1),
              "iterations": round(ab["iterations_mean"], 2),
              "n_dist_per_query": round(ab["n_dist"] / B, 1)}
        log(f"[bench] width {p} itopk {M}: recall@{w.k} {rec:.4f}  {pt['qps']:.0f} QPS  "
            f"{pt['vector_GBs']:.0f} GB/s gathered")
        return pt

    for p in widths:
        prev = None
        for M in sweep_list:
            if M < w.k or p * w.degree > 2048:
                continue
            pt = sweep_point(M, p)
            rec = pt["recall"]
            sweep.append(pt)
            if rec >= TARGET_RECALL:
                if best is None or pt["qps"] > best["qps"]:
                    best = pt
                if prev is not None and prev["recall"] < TARGET_RECALL:
                    f = (TARGET_RECALL - prev["recall"]) / (rec - prev["recall"])
                    interpolated.append(prev["qps"] + f * (pt["qps"] - prev["qps"]))
                if not args.full_sweep:
                    break
            prev = pt
    chosen = best if best is not None else sweep[-1]
    M, P_WIDTH = chosen["itopk"], chosen["search_width"]
    qps_at_target = max(interpolated) if interpolated else None

    # ---- the timed region ---------------------------------------------------------------------
    wall_ms, dev_ms = timed(M, P_WIDTH, args.steps, args.warmup)
    st_np = stats.cpu().numpy().view(np.uint32)
    ab = algorithmic_bytes(st_np, dim, w.degree, w.k)
    gpu_ids = ids.cpu().numpy().view(np.uint32).copy()
    gpu_d = dists.cpu().numpy().copy()
    rec = recall_at_k(gpu_ids, gt_np)
    value = B / (wall_ms * 1e-3)
    achieved = ab["total_bytes"] / (dev_ms * 1e-3) / 1e9
    if args.traffic_bytes is not None:
        traffic, traffic_source = args.traffic_bytes, {"file": None, "note": "given on the command line"}
    else:
        traffic, traffic_source = measured_traffic(w.name, P_WIDTH, M)
    # the one-parent-per-pass search (search_width 1, the paper's basic form) at its own crossing of the target
    p1 = [pt for pt in sweep if pt["search_width"] == 1 and pt["recall"] >= TARGET_RECALL]
    p1_reference = min(p1, key=lambda pt: pt["itopk"]) if p1 else None

    out = {
        "metric": "QPS at recall@10>=0.95 (1Mx128, batch 10k)" if (w.name == "sift1m" and N == 1_000_000 and B == 10_000)
        else f"QPS at recall@{w.k}>={TARGET_RECALL} ({N}x{dim}, batch {B})", "value": round(value, 1), "unit": "queries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(wall_ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: N={N} dim={dim} fp32{' integer-valued 0..255' if w.name == 'sift1m' else ''}, B={B}, "
                               f"degree={w.degree} (init {w.init_degree}), k={w.k}, itopk={M}, "
                               f"search_width={P_WIDTH}, single-workgroup mode",
                   "itopk": M, "search_width": P_WIDTH, "recall_at_k": round(rec, 5), "target_recall": TARGET_RECALL,
                   "qps_interpolated_at_target": None if qps_at_target is None else round(qps_at_target, 1),
                   "graph_build_s": round(build_s, 2), "reorder": args.reorder, "initial_graph": args.initial_graph,
                   "exact_algo": args.exact_algo,
                   "p1_reference": p1_reference,
                   "graph_quality": graph_quality},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": traffic, "traffic_source": traffic_source,
                     "what": "algorithmic bytes (rows of first-time candidates, graph rows of parents, queries, results; "
                             "counted in the kernel) over the kernel's time, against the published HBM peak; the "
                             f"{N * dim * 4 / 1e6:.0f} MB dataset partly fits the 256 MB Infinity Cache, whose hits the "
                             "HBM counters do not see, so on datasets of this size the figure is a gather rate, not pure HBM",
                     "kernel": "search_single_wide_kernel" if P_WIDTH * w.degree > 256 else "search_single_kernel",
                     "kernel_ms": round(dev_ms, 4),
                     "algorithmic_bytes_per_launch": ab["total_bytes"],
                     "gathered_vector_GBs": round(ab["vector_bytes"] / (dev_ms * 1e-3) / 1e9, 1),
                     "n_dist_per_query": round(ab["n_dist"] / B, 1),
                     "iterations_per_query": round(ab["iterations_mean"], 2),
                     "queries_stopped_by_cap": ab["hit_cap"]},
        "sweep": sweep,
    }

    # ---- lists shorter than the itopk range the benchmark configuration names, with wider passes: reported
    #      beside the headline, never as `value` ------------------------------------------------------
    short = w.extra.get("short_itopk") if not (args.itopk or args.width or args.no_short) else None
    if short:
        pts, best_short = [], None
        for p in (5, 6, 7, 8, 10, 12):
            for M_s in short:
                if M_s < w.k or p * w.degree > 2048:
                    continue
                pt = sweep_point(M_s, p)
                pts.append(pt)
                if pt["recall"] >= TARGET_RECALL:
                    if best_short is None or pt["qps"] > best_short["qps"]:
                        best_short = pt
                    break
        run(M, P_WIDTH)                      # the shared result buffers hold the timed configuration again
        torch.cuda.synchronize()
        out["short_lists"] = {"note": f"itopk below {min(w.itopk)} (outside the sweep range of the benchmark configuration), "
                                      "search_width 5..12; 5 timed launches per point",
                              "best_at_target_recall": best_short, "sweep": pts}

    # ---- the same search on larger batches (the queries repeated; a query's seeds depend on its index
    #      in the batch, so the copies walk different paths): how much of the 10,000-query time is the
    #      start and the drain of the batch, during which the device is not full ----------------------
    if not args.no_scaling:
        scaling = []
        for rep in (2, 4, 8):
            qq = queries.repeat(rep, 1).contiguous()
            Bq = qq.shape[0]
            s_ids = torch.empty((Bq, w.k), dtype=torch.int32, device=dev)
            s_d = torch.empty((Bq, w.k), dtype=torch.float32, device=dev)
            s_st = torch.zeros((Bq, 4), dtype=torch.int32, device=dev)

            def run_s():
                return cagra.search(graph, base, qq, w.k, M, P_WIDTH, w.metric, opts, out=(s_ids, s_d),
                                    workspace=ws, stats=s_st)
            for _ in range(2):
                run_s()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(5):
                run_s()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 5
            ab_s = algorithmic_bytes(s_st.cpu().numpy().view(np.uint32), dim, w.degree, w.k)
            scaling.append({"batch": Bq, "kernel_ms": round(ms, 4), "qps_kernel": round(Bq / (ms * 1e-3), 1),
                            "achieved_GBs": round(ab_s["total_bytes"] / (ms * 1e-3) / 1e9, 1),
                            "frac_of_hbm_peak": round(ab_s["total_bytes"] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)})
            log(f"[bench] batch {Bq}: {ms:.3f} ms  {scaling[-1]['qps_kernel']:.0f} QPS  {scaling[-1]['achieved_GBs']:.0f} GB/s")
            del qq, s_ids, s_d, s_st
        out["batch_scaling"] = {"note": "same index and parameters, the query set repeated 2, 4 and 8 times",
                                "results": scaling}

    # ---- successive batches on two streams: the drain of one launch (a few long queries finishing on
    #      an emptying device) overlaps the start of the next, as a server with two batches in flight
    #      would run them.  Reported next to `value`, which stays the one-launch-after-the-other figure.
    if not args.no_scaling:
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        bufs = [(torch.empty((B, w.k), dtype=torch.int32, device=dev), torch.empty((B, w.k), dtype=torch.float32, device=dev),
                 torch.empty(4096, dtype=torch.uint8, device=dev)) for _ in range(2)]
        torch.cuda.synchronize()

        def run_two(n):
            for i in range(n):
                with torch.cuda.stream(streams[i & 1]):
                    cagra.search(graph, base, queries, w.k, M, P_WIDTH, w.metric, opts,
                                 out=(bufs[i & 1][0], bufs[i & 1][1]), workspace=bufs[i & 1][2])
        run_two(4)
        torch.cuda.synchronize()
        t_p = time.perf_counter()
        run_two(args.steps)
        torch.cuda.synchronize()
        ms_p = (time.perf_counter() - t_p) * 1e3 / args.steps
        same_p = bool(torch.equal(bufs[0][0], ids) and torch.equal(bufs[1][0], ids))
        out["two_streams"] = {"ms_per_step": round(ms_p, 4), "qps": round(B / (ms_p * 1e-3), 1),
                              "achieved_GBs": round(ab["total_bytes"] / (ms_p * 1e-3) / 1e9, 1),
                              "same_ids_as_single_stream": same_p}
        log(f"[bench] batches alternating on two streams: {ms_p:.3f} ms per batch, {out['two_streams']['qps']:.0f} QPS, "
            f"ids equal: {same_p}")

    # ---- the same search over narrower storage of the same rows (Sec. IV-C.1, last paragraph) ----
    if not args.no_storage:
        narrow = []
        for name, code, width_b in (("f16", cagra.F16, 2), ("u8", cagra.U8, 1)):
            if dim % (16 // width_b) != 0 or (code == cagra.U8 and w.name != "sift1m"):
                continue            # uint8 only where the values are integers 0..255
            conv = cagra.convert_dataset(base, code)
            n_ids = torch.empty((B, w.k), dtype=torch.int32, device=dev)
            n_d = torch.empty((B, w.k), dtype=torch.float32, device=dev)

            st_n = torch.zeros((B, 4), dtype=torch.int32, device=dev)

            def run_n():
                return cagra.search(graph, conv, queries, w.k, M, P_WIDTH, w.metric, opts,
                                    out=(n_ids, n_d), workspace=ws, stats=st_n)
            run_n()
            torch.cuda.synchronize()
            rec_n = recall_at_k(n_ids.cpu().numpy().view(np.uint32), gt_np)
            for _ in range(2):
                run_n()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                run_n()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 10
            nd = int(st_n.cpu().numpy().view(np.uint32)[:, 2].astype(np.int64).sum())
            narrow.append({"storage": name, "itopk": M, "search_width": P_WIDTH, "recall_at_k": round(rec_n, 5), "kernel_ms": round(ms, 4),
                           "qps_kernel": round(B / (ms * 1e-3), 1),
                           "gathered_vector_GBs": round(nd * dim * width_b / (ms * 1e-3) / 1e9, 1),
                           "same_ids_as_fp32": bool(torch.equal(n_ids, ids))})
            log(f"[bench] storage {name}: recall {rec_n:.4f}  {ms:.3f} ms  {narrow[-1]['qps_kernel']:.0f} QPS")
            del conv
        out["narrow_storage"] = narrow

    # ---- what the device delivers for the access patterns alone (no method arithmetic) ---------
    if not args.no_reference:
        sink = torch.zeros(1, dtype=torch.int32, device=dev)

        def time_probe(reps, **kw):
            cagra.probe_bandwidth(base, sink=sink, **kw)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for r in range(reps):
                cagra.probe_bandwidth(base, sink=sink, seed=r, **kw)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps
        n_read = ab["n_dist"]
        ms_stream = time_probe(10, pattern=0)
        ref = {"dataset_stream_read_GBs": round(N * dim * 4 / (ms_stream * 1e-3) / 1e9, 1), "row_bytes": dim * 4,
               "rows_gathered": n_read, "row_gather": []}
        best = 0.0
        for rif in (4, 8):
            for wpc in (8, 16):
                ms_g = time_probe(5, pattern=1, n_read=n_read, rows_in_flight=rif, waves_per_cu=wpc)
                gbs = n_read * dim * 4 / (ms_g * 1e-3) / 1e9
                best = max(best, gbs)
                ref["row_gather"].append({"rows_in_flight": rif, "waves_per_cu": wpc, "GBs": round(gbs, 1)})
        ref["best_row_gather_GBs"] = round(best, 1)
        ref["search_vs_best_row_gather"] = round(out["roofline"]["gathered_vector_GBs"] / best, 4)
        # The same two patterns over a buffer far beyond the 256 MB Infinity Cache (8 GiB, several ms per launch):
        # what the HBM alone delivers.  The stream figure is the achievable peak for reads; the gather figure is the
        # ceiling for a search over a dataset that no cache holds.
        row_b = dim * 4
        big_rows = (8 << 30) // row_b
        big = torch.empty((big_rows, row_b), dtype=torch.uint8, device=dev)
        big.view(-1)[: big_rows * row_b].view(torch.int32).fill_(0x3F800000)

        def time_big(reps, **kw):
            cagra.probe_bandwidth(big, sink=sink, **kw)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for r in range(reps):
                cagra.probe_bandwidth(big, sink=sink, seed=100 + r, **kw)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps
        big_stream = []
        for wpc in (8, 16, 32):
            ms_b = time_big(5, pattern=0, waves_per_cu=wpc)
            big_stream.append({"waves_per_cu": wpc, "ms": round(ms_b, 3), "GBs": round(big_rows * row_b / (ms_b * 1e-3) / 1e9, 1)})
        n_big = max(n_read, 40_000_000)
        big_gather = []
        for rif, wpc in ((4, 16), (8, 8), (8, 16)):
            ms_b = time_big(3, pattern=1, n_read=n_big, rows_in_flight=rif, waves_per_cu=wpc)
            big_gather.append({"rows_in_flight": rif, "waves_per_cu": wpc, "ms": round(ms_b, 3),
                               "GBs": round(n_big * row_b / (ms_b * 1e-3) / 1e9, 1)})
        del big
        ref["hbm_only"] = {"buffer_bytes": big_rows * row_b, "stream_read": big_stream,
                           "stream_read_GBs": max(x["GBs"] for x in big_stream),
                           "row_gather": big_gather, "row_gather_GBs": max(x["GBs"] for x in big_gather),
                           "rows_gathered": n_big}
        ref["search_vs_hbm_stream_read"] = round(out["roofline"]["achieved"] / ref["hbm_only"]["stream_read_GBs"], 4)
        out["hbm_reference"] = ref
        log(f"[bench] reference: dataset stream read {ref['dataset_stream_read_GBs']} GB/s, random {dim * 4}-byte rows of the "
            f"dataset {ref['best_row_gather_GBs']} GB/s; 8 GiB buffer: stream {ref['hbm_only']['stream_read_GBs']} GB/s, "
            f"random rows {ref['hbm_only']['row_gather_GBs']} GB/s")

    # ---- the choices the library makes by itself, each against its alternatives (the paper's own
    #      studies of team size, Sec. V-B, of the visited-table management, Sec. IV-B.3, and of the two
    #      modes over the batch size, Sec. IV-C.3) -----------------------------------------------------
    if args.ablations:
        def time_opts(o, p_w, m_itopk, qs, reps=5):
            nq = qs.shape[0]
            a_ids = torch.empty((nq, w.k), dtype=torch.int32, device=dev)
            a_d = torch.empty((nq, w.k), dtype=torch.float32, device=dev)
            a_st = torch.zeros((nq, 4), dtype=torch.int32, device=dev)
            a_ws = torch.empty(max(4096, cagra.search_workspace_bytes(N, w.degree, nq, w.k, m_itopk, p_w, o)),
                               dtype=torch.uint8, device=dev)
            for _ in range(2):
                cagra.search(graph, base, qs, w.k, m_itopk, p_w, w.metric, o, out=(a_ids, a_d), workspace=a_ws, stats=a_st)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                cagra.search(graph, base, qs, w.k, m_itopk, p_w, w.metric, o, out=(a_ids, a_d), workspace=a_ws, stats=a_st)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps
            rec_a = recall_at_k(a_ids.cpu().numpy().view(np.uint32), gt_np[:nq])
            nd = float(a_st.cpu().numpy().view(np.uint32)[:, 2].astype(np.int64).mean())
            return ms, rec_a, nd, a_ids
        abl = {"configuration": {"search_width": P_WIDTH, "itopk": M}}
        auto_plan = cagra.describe(w.degree, dim, B, w.k, M, P_WIDTH, opts)
        abl["automatic"] = {k2: auto_plan[k2] for k2 in ("team_size", "table_entries", "table_policy", "workgroups")}
        rows = []
        for team in (4, 8, 16, 32):
            ms, rec_a, nd, a_ids = time_opts(cagra.SearchOptions(seed=opts.seed, mode=1, team_size=team), P_WIDTH, M, queries)
            rows.append({"team_size": team, "kernel_ms": round(ms, 4), "qps": round(B / ms * 1e3, 1),
                         "same_ids": bool(torch.equal(a_ids, ids))})
            log(f"[bench] team size {team}: {ms:.3f} ms")
        abl["team_size"] = rows
        rows = []
        for pol, entries in ((2, 1024), (2, 2048), (2, 3072), (2, 4096), (2, 8192), (1, 2048), (1, 4096), (1, 8192)):
            try:
                ms, rec_a, nd, a_ids = time_opts(cagra.SearchOptions(seed=opts.seed, mode=1, table_policy=pol,
                                                                     table_entries=entries), P_WIDTH, M, queries)
            except cagra.CagraError as exc:
                rows.append({"table_policy": pol, "table_entries": entries, "rejected": str(exc)})
                continue
            rows.append({"table_policy": "replacement" if pol == 2 else "periodic reset", "table_entries": entries,
                         "kernel_ms": round(ms, 4), "qps": round(B / ms * 1e3, 1),
                         "distances_per_query": round(nd, 1), "same_ids": bool(torch.equal(a_ids, ids))})
            log(f"[bench] table policy {pol} entries {entries}: {ms:.3f} ms, {nd:.0f} distances per query")
        abl["visited_table"] = rows
        rows = []
        for nb in (1, 16, 64, 256, 1024, 4096, B):
            qs = queries[:nb]
            ms1, rec1, _, _ = time_opts(cagra.SearchOptions(seed=opts.seed, mode=1), P_WIDTH, M, qs, reps=10)
            ms2, rec2, _, _ = time_opts(cagra.SearchOptions(seed=opts.seed, mode=2, wg_per_query=8, max_iterations=16),
                                        1, 256, qs, reps=10)
            rows.append({"batch": nb, "single_ms": round(ms1, 4), "single_recall": round(rec1, 4),
                         "multi_ms": round(ms2, 4), "multi_recall": round(rec2, 4),
                         "automatic_mode": cagra.auto_mode(nb, M)})
            log(f"[bench] batch {nb}: single {ms1:.3f} ms (recall {rec1:.3f}), multi W=8 I_max=16 {ms2:.3f} ms (recall {rec2:.3f})")
        abl["mode_over_batch_size"] = rows
        out["ablations"] = abl

    # ---- small batches in multi-workgroup mode: host-side latency per call (Sec. IV-C.2) -------
    # Workers per query W and the pass limit I_max are swept (itopk = 32 W, so every worker keeps
    # the minimum list of 32); recall is measured on the first 1000 queries in one call (the seed of
    # a query depends on its index in the call, so that is a separate, untimed launch).
    if not args.no_latency:
        lat_configs = [(args.latency_workers, 0)] + [(W, i) for W in (8, 16, 32, 64) for i in (3, 4, 5, 6, 8, 10, 12, 16)]
        nq_rec = min(1000, B)
        small = []
        for W, imax in lat_configs:
            mopts = cagra.SearchOptions(seed=20230815, mode=2, wg_per_query=W, max_iterations=imax)
            m_itopk = 32 * W
            r_ids, _ = cagra.search(graph, base, queries[:nq_rec], w.k, m_itopk, 1, w.metric, mopts)
            rec_m = recall_at_k(r_ids.cpu().numpy().view(np.uint32), gt_np[:nq_rec])
            entry = {"workers": W, "itopk": m_itopk, "max_iterations": imax or "auto",
                     f"recall_at_k_b{nq_rec}": round(rec_m, 5)}
            for nb in (1, 10, 100):
                # a prepared call (arguments marshalled once), as a serving loop would hold it; each call: point it
                # at the next queries (already in device memory), enqueue, wait
                q_buf = queries[:nb].clone()
                call = cagra.PreparedSearch(graph, base, q_buf, w.k, m_itopk, 1, w.metric, mopts)
                n_calls = 200
                lat = np.empty(n_calls)
                for c in range(-10, n_calls):
                    lo = (max(c, 0) * nb) % (B - nb + 1)
                    t_c = time.perf_counter()
                    call(queries[lo:lo + nb])
                    torch.cuda.synchronize()
                    if c >= 0:
                        lat[c] = (time.perf_counter() - t_c) * 1e6
                entry[f"b{nb}"] = {"p50_us": round(float(np.percentile(lat, 50)), 1),
                                   "p99_us": round(float(np.percentile(lat, 99)), 1),
                                   "qps": round(nb / (float(np.mean(lat)) * 1e-6), 1)}
            small.append(entry)
            log(f"[bench] multi mode W={W} I_max={imax or 'auto'}: recall {rec_m:.4f}  batch 1 p50 "
                f"{entry['b1']['p50_us']} us  batch 10 {entry['b10']['p50_us']} us  batch 100 {entry['b100']['p50_us']} us")
        good = [e for e in small if e[f"recall_at_k_b{nq_rec}"] >= TARGET_RECALL]
        best_lat = min(good, key=lambda e: e["b1"]["p50_us"]) if good else None
        if best_lat is not None and not args.no_graph:
            # the same batch-1 call replayed from a captured HIP graph (copy of the query into a fixed
            # buffer + the two kernels of the search): what a serving loop would do
            W = best_lat["workers"]
            imax = 0 if best_lat["max_iterations"] == "auto" else best_lat["max_iterations"]
            mopts = cagra.SearchOptions(seed=20230815, mode=2, wg_per_query=W, max_iterations=imax)
            mws = torch.empty(cagra.search_workspace_bytes(N, w.degree, 1, w.k, 32 * W, 1, mopts),
                              dtype=torch.uint8, device=dev)
            # cleaned once; every search hands the workspace back clean, so the captured call is one kernel
            cagra.search_workspace_init(mws, N, w.degree, dim, 1, w.k, 32 * W, 1, mopts)
            import dataclasses
            mopts = dataclasses.replace(mopts, workspace_clean=1)
            q_fix = queries[:1].clone()
            g_ids = torch.empty((1, w.k), dtype=torch.int32, device=dev)
            g_d = torch.empty((1, w.k), dtype=torch.float32, device=dev)
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                cagra.search(graph, base, q_fix, w.k, 32 * W, 1, w.metric, mopts, out=(g_ids, g_d), workspace=mws)
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            hg = torch.cuda.CUDAGraph()
            with torch.cuda.graph(hg):
                cagra.search(graph, base, q_fix, w.k, 32 * W, 1, w.metric, mopts, out=(g_ids, g_d), workspace=mws)
            lat = np.empty(200)
            hit_graph = hit_eager = 0
            for c in range(-10, 200):
                qi_r = max(c, 0) % B
                src = queries[qi_r:qi_r + 1]
                t_c = time.perf_counter()
                q_fix.copy_(src)
                hg.replay()
                torch.cuda.synchronize()
                if c >= 0:
                    lat[c] = (time.perf_counter() - t_c) * 1e6
                if c >= 0:
                    # several workers interleave differently from run to run, so replay and eager call are
                    # compared by their recall over the same 200 queries, not id by id
                    hit_graph += len(np.intersect1d(g_ids.cpu().numpy().view(np.uint32)[0], gt_np[qi_r]))
                    e_ids, _ = cagra.search(graph, base, src, w.k, 32 * W, 1, w.metric, dataclasses.replace(mopts, workspace_clean=0))
                    hit_eager += len(np.intersect1d(e_ids.cpu().numpy().view(np.uint32)[0], gt_np[qi_r]))
            best_lat["graph_replay"] = {"p50_us": round(float(np.percentile(lat, 50)), 1),
                                        "p99_us": round(float(np.percentile(lat, 99)), 1),
                                        "recall_replayed": round(hit_graph / (200.0 * w.k), 4),
                                        "recall_eager_same_queries": round(hit_eager / (200.0 * w.k), 4)}
            log(f"[bench] batch 1 from a captured graph (W={W}, I_max={imax}): p50 {best_lat['graph_replay']['p50_us']} us, "
                f"recall {best_lat['graph_replay']['recall_replayed']} (eager {best_lat['graph_replay']['recall_eager_same_queries']})")
        out["small_batch"] = {"mode": "multi-workgroup, host wall-clock per call: launch through a prepared call on queries "
                                      "resident in device memory, stream sync",
                              "dataset": w.name, "best_batch1_at_target_recall": best_lat, "results": small}

    # ---- CPU oracle on a sample of the same queries (rank 0, N = 1 only) -----------------------
    if not args.no_cpu:
        import oracle
        ns = min(args.cpu_sample, B)
        g_np = graph.cpu().numpy().view(np.uint32)
        oracle.search(g_np, w.base, w.queries[:64], w.k, M, P_WIDTH, w.metric, seed=opts.seed)  # warm-up
        reps = 0
        t0 = time.perf_counter()
        while reps == 0 or (time.perf_counter() - t0 < 1.5 and reps < 20):     # >= 1.5 s of wall clock on all cores
            o_ids, o_d, o_st = oracle.search(g_np, w.base, w.queries[:ns], w.k, M, P_WIDTH, w.metric,
                                             seed=opts.seed, return_stats=True)
            reps += 1
        cpu_s = (time.perf_counter() - t0) / reps
        inter = sum(len(np.intersect1d(a, b)) for a, b in zip(gpu_ids[:ns], o_ids))
        same = gpu_ids[:ns] == o_ids
        rel = float(np.max(np.abs(gpu_d[:ns] - o_d)[same] / np.maximum(np.abs(o_d[same]), 1e-30))) if same.any() else 0.0
        cpu_model = "unknown"
        try:
            with open("/proc/cpuinfo") as f:
                cpu_model = next((ln.split(":", 1)[1].strip() for ln in f if ln.startswith("model name")), "unknown")
        except OSError:
            pass
        out["cpu_baseline"] = {"value": round(ns / cpu_s, 1), "unit": "queries/s", "cores": oracle.num_threads(),
                               "kind": "oracle", "cpu_model": cpu_model, "host_cpus": os.cpu_count(), "sample": f"first {ns} of the {B} queries, same graph, "
                               f"itopk={M}, search_width={P_WIDTH}, OpenMP over queries, "
                               f"{cpu_s:.2f}s per pass over the sample, {reps} passes"}
        if ns == B:
            # the oracle's visited set never forgets: its distance count is what the method has to compute; the
            # kernel's LDS table forgets and measures some rows twice (counted in n_dist_per_query above)
            nd_o = int(o_st[:, 2].astype(np.int64).sum())
            strict = nd_o * dim * 4 + ab["n_parent"] * w.degree * 4 + B * dim * 4 + B * w.k * 8
            out["roofline"]["n_dist_oracle_per_query"] = round(nd_o / B, 1)
            out["roofline"]["achieved_strict"] = round(strict / (dev_ms * 1e-3) / 1e9, 1)
            out["roofline"]["frac_strict"] = round(strict / (dev_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
        out["parity_at_full_size"] = {"sample": ns, "id_agreement": round(inter / float(ns * w.k), 6),
                                      "positionwise_equal": round(float(same.mean()), 6),
                                      "max_rel_dist_err": rel,
                                      "oracle_recall": round(recall_at_k(o_ids, gt_np[:ns]), 5),
                                      "gpu_recall_same_sample": round(recall_at_k(gpu_ids[:ns], gt_np[:ns]), 5)}
    if args.timeline:
        import ctypes
        lib = cagra.load_library()
        if not hasattr(lib, "cagra_debug_query_times_f32"):
            log("bench.py: --timeline needs a library built with -DCAGRA_PHASE_CLOCKS")
            return 1
        rows = []
        for nw in (1, 2, 4):
            o = cagra.SearchOptions(seed=opts.seed, mode=1, waves_per_query=nw)
            for _ in range(3):
                cagra.search(graph, base, queries, w.k, M, P_WIDTH, w.metric, o, out=(ids, dists), workspace=ws)
            _, _, st_t = cagra.search(graph, base, queries, w.k, M, P_WIDTH, w.metric, o, out=(ids, dists), workspace=ws,
                                      return_stats=True)
            torch.cuda.synchronize()
            buf = (ctypes.c_ulonglong * (2 * B))()
            lib.cagra_debug_query_times_f32(buf, B)
            t = np.array(list(buf), dtype=np.int64).reshape(B, 2)
            t0 = t[:, 0].min()
            s_us, e_us = (t[:, 0] - t0) / 100.0, (t[:, 1] - t0) / 100.0      # the wall clock counts at 100 MHz
            total, dur = float(e_us.max()), e_us - s_us
            edges = np.linspace(0.0, total, 21)
            mids = (edges[:-1] + edges[1:]) / 2
            rows.append({"waves_per_query": nw, "launch_us": round(total, 1), "last_query_started_us": round(float(s_us.max()), 1),
                         "duration_us": {"mean": round(float(dur.mean()), 1), "p50": round(float(np.percentile(dur, 50)), 1),
                                         "p99": round(float(np.percentile(dur, 99)), 1), "max": round(float(dur.max()), 1)},
                         "passes_mean": round(float(st_t[:, 0].float().mean().item()), 2),
                         "queries_in_flight_in_20_slices": [int(((s_us <= x) & (e_us > x)).sum()) for x in mids],
                         "queries_finished_by_slice_end": [int((e_us <= x).sum()) for x in edges[1:]]})
            log(f"[bench] timeline {nw} wavefront(s) per query: launch {total:.0f} us, last start {s_us.max():.0f} us, "
                f"duration mean {dur.mean():.0f} p99 {np.percentile(dur, 99):.0f} max {dur.max():.0f} us")
        out["timeline"] = {"note": "one launch at the timed point, phase-clock build (slower than the product build by the "
                                   "time stamps); times in microseconds from the first query's start", "results": rows}
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)   # 1 GiB read, 1 GiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
