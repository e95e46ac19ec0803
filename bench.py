#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

A step = one pass of the whole path over BASELINE config 1 ("skewed medium": A and B
10,000 x 20,000 CSR): spd_pairwise with L1 (union family), spd_pairwise with cosine
(dot-product family) and spd_knn with cosine, k = 32 (fused top-k).  Every call plans
(degree binning), repacks B with its row norms, stages A in LDS, scans, finishes and
writes.  Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

For profiling:  --only {l1,cosine,knn}  restricts the step to one call, and
--copy-calibration adds a plain device-to-device copy of known size per step, against which
the FETCH_SIZE / WRITE_SIZE counters of rocprofv3 are scaled.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
ALU_LANE_OPS = 78.6e12 / 2.0      # fp64 vector peak in FMAs = lane-instructions per second (256 CUs, 2.4 GHz)
COPY_BYTES = 256 << 20


def algorithmic_bytes(a_rows, nnz_b, n_b):
    """Bytes the method moves for `a_rows` rows of A against all of B: each row pair streams
    the stored entries of the B row (4-byte column + 4-byte value) and writes one fp32."""
    return a_rows * (8.0 * nnz_b + 4.0 * n_b)


def selfjoin(args):
    """k-NN of a matrix against itself, batch by batch: every call is a whole spd_knn (planning
    and repacking of the index included), the query rows a slice of the index's own arrays."""
    import torch

    import paper_2104_06357_amd as spd
    from gen import synth

    if not torch.cuda.is_available():
        sys.exit("bench.py needs an MI355X: no GPU is visible")
    torch.cuda.set_device(0)
    _, B = synth.workload(args.selfjoin)
    n, k = B["n_rows"], 32
    dB = spd.DeviceCsr.from_host(B, keep_host_indptr=not args.device_row_pointers)
    h = spd.Handle()
    idx = torch.empty((args.batch, k), dtype=torch.int64, device="cuda")
    dist = torch.empty((args.batch, k), dtype=torch.float32, device="cuda")
    starts = list(range(0, n, args.batch))
    if args.max_batches > 0:
        starts = starts[:args.max_batches]
    tiles = []
    for r0 in starts:                       # the slices are made before the clock starts
        r1 = min(n, r0 + args.batch)
        lo, hi = int(B["indptr"][r0]), int(B["indptr"][r1])
        tiles.append(spd.DeviceCsr(r1 - r0, B["n_cols"], (dB.indptr[r0:r1 + 1] - lo).contiguous(),
                                   dB.indices[lo:hi], dB.values[lo:hi],
                                   host_indptr=None if args.device_row_pointers else B["indptr"][r0:r1 + 1] - lo))
    h.knn(tiles[0], dB, args.metric, k, out_idx=idx[:tiles[0].n_rows], out_dist=dist[:tiles[0].n_rows])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    if args.index:
        ix = h.index_create(dB, args.metric)
        for q in tiles:
            ix.knn(q, k, out_idx=idx[:q.n_rows], out_dist=dist[:q.n_rows])
    else:
        for q in tiles:
            h.knn(q, dB, args.metric, k, out_idx=idx[:q.n_rows], out_dist=dist[:q.n_rows])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    rows = sum(q.n_rows for q in tiles)
    print(json.dumps({
        "metric": "self-join brute-force k-NN, row-pairs/s", "value": rows * float(n) / elapsed, "unit": "row-pairs/s",
        "n_gpus": 1, "dtype": "f32", "data": "synthetic", "k": k, "distance": args.metric,
        "config": {"workload": "shape %d self-join" % args.selfjoin, "rows": n, "n_cols": B["n_cols"],
                   "nnz": int(B["indptr"][-1]), "batch": args.batch,
                   "calls": "spd_index_create + spd_index_knn" if args.index else "spd_knn"},
        "query_rows_timed": rows, "calls": len(tiles), "seconds": elapsed, "ms_per_call": 1e3 * elapsed / len(tiles),
        "seconds_for_all_rows": elapsed * n / rows}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--only", choices=("l1", "cosine", "knn", "tropical", "l1_semiring"), default=None,
                    help="time one call instead of the step; the last two are semiring calls, "
                         "(min,+) over the intersection and (+,|x-y|) over the union, which are not part of the step")
    ap.add_argument("--copy-calibration", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--device-row-pointers", action="store_true",
                    help="give the library no host copy of the row pointers: every call then reads them "
                         "back and waits for the stream, so calls no longer overlap")
    ap.add_argument("--serial", action="store_true",
                    help="keep every launch on one stream in the timed region too (for kernel traces)")
    ap.add_argument("--selfjoin", type=int, choices=(2, 3, 4, 5, 6), default=None,
                    help="instead of the step: brute-force k-NN (k = 32) of every row of a dataset-shaped "
                         "synthetic matrix against the whole matrix, in batches of query rows (the protocol of "
                         "the paper's Table 3); prints a JSON line of its own")
    ap.add_argument("--metric", default="cosine", help="--selfjoin: the distance")
    ap.add_argument("--batch", type=int, default=4096, help="--selfjoin: query rows per call")
    ap.add_argument("--max-batches", type=int, default=0, help="--selfjoin: stop after this many calls (0: all rows)")
    ap.add_argument("--index", action="store_true",
                    help="--selfjoin: prepare the matrix once with spd_index_create (timed too) and query that")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (use --gpus 1)")
    if args.selfjoin is not None:
        return selfjoin(args)

    import numpy as np
    import torch

    import paper_2104_06357_amd as spd
    from gen import synth

    if not torch.cuda.is_available():
        sys.exit("bench.py needs an MI355X: no GPU is visible")
    torch.cuda.set_device(0)
    A, B = synth.workload(1)
    m, n = A["n_rows"], B["n_rows"]
    nnz_b = int(B["indptr"][-1])
    keep = not args.device_row_pointers
    dA, dB = spd.DeviceCsr.from_host(A, keep_host_indptr=keep), spd.DeviceCsr.from_host(B, keep_host_indptr=keep)
    h = spd.Handle()
    if args.serial:
        h.set_option("side_streams", 0)
    out = torch.empty((m, n), dtype=torch.float32, device="cuda")
    idx = torch.empty((m, 32), dtype=torch.int64, device="cuda")
    dist = torch.empty((m, 32), dtype=torch.float32, device="cuda")
    copy_src = copy_dst = None
    if args.copy_calibration:
        copy_src = torch.ones(COPY_BYTES // 4, dtype=torch.float32, device="cuda")
        copy_dst = torch.empty_like(copy_src)

    calls = {
        "l1": lambda: h.pairwise(dA, dB, "l1", out=out),
        "cosine": lambda: h.pairwise(dA, dB, "cosine", out=out),
        "knn": lambda: h.knn(dA, dB, "cosine", 32, out_idx=idx, out_dist=dist),
        "tropical": lambda: h.semiring_pairwise(dA, dB, "plus", "min", False, out=out),
        "l1_semiring": lambda: h.semiring_pairwise(dA, dB, "abs_diff", "plus", True, out=out),
    }
    names = [args.only] if args.only else ["l1", "cosine", "knn"]

    def step():
        for name in names:
            calls[name]()
        if copy_dst is not None:
            copy_dst.copy_(copy_src)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    pairs_per_step = float(len(names)) * m * n

    # per-kernel HIP-event timings (events recorded by the library around every launch, on the
    # stream of that launch), averaged over as many steps again.  The small launches of a call
    # normally overlap with the large one on side streams; here they are serialised so that a
    # launch's duration is its own.
    h.set_option("profile", 1)
    h.set_option("side_streams", 0)
    records = {name: [] for name in names}
    wall = {name: 0.0 for name in names}
    for _ in range(args.steps):
        for name in names:
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            calls[name]()
            records[name].append(h.profile_read())
            torch.cuda.synchronize()
            wall[name] += time.perf_counter() - t1
    h.set_option("profile", 0)

    def roofline(name):
        per_step = records[name]
        first = per_step[0]
        scans = [i for i, r in enumerate(first) if r["name"] == "scan"]
        big = max(scans, key=lambda i: first[i]["a_rows"])
        rec = first[big]
        ms = float(np.mean([recs[big]["ms"] for recs in per_step]))
        scan_ms = float(np.mean([sum(r["ms"] for r in recs if r["name"] == "scan") for recs in per_step]))
        all_ms = float(np.mean([sum(r["ms"] for r in recs) for recs in per_step]))
        alg = algorithmic_bytes(rec["a_rows"], nnz_b, n)
        achieved = alg / (ms * 1e-3) / 1e9
        # the same launch against the vector ALU: a visit (row of A x stored entry of B) cannot
        # cost less than the product's own instructions (L1: median, conversion, fp64 add;
        # dot: conversion, fp64 FMA), and the chip issues 78.6e12 / 2 fp64 lane-instructions/s
        # (semirings: compare, sign-flipped sum, select, max; the union sum: two masked conversions,
        # three fp64 terms and their adds, the count)
        per_visit = {"l1": 3, "tropical": 4, "l1_semiring": 9}.get(name, 2)
        visits = float(rec["a_rows"]) * nnz_b / (ms * 1e-3)
        alu_peak = ALU_LANE_OPS / per_visit
        alu = {"bound": "alu", "achieved": visits, "peak": alu_peak, "unit": "visits/s",
               "frac": round(visits / alu_peak, 4), "vector_instructions_per_visit": per_visit}
        return {
            "bound": "hbm", "kernel": "spd_scan_kernel (%s, R=%d rows of A per workgroup, staging kind %d)"
                                      % (name, rec["rows_per_group"], rec["staging_kind"]),
            "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
            "algorithmic_bytes_per_launch": alg, "launch_ms": round(ms, 4),
            "a_rows_in_launch": rec["a_rows"], "workgroups": rec["workgroups"], "block": rec["block"],
            "lds_bytes": rec["lds_bytes"], "scan_launches_per_call": len(scans),
            "all_scan_launches_ms": round(scan_ms, 4), "all_kernels_ms": round(all_ms, 4),
            "serialised_call_wall_ms": round(1e3 * wall[name] / args.steps, 4),
            "alu": alu,
            "note": "effective rate: the R rows staged together share every entry of B that is loaded and B "
                    "stays resident in L2, so the HBM stream is far below the algorithmic bytes (see traffic)",
        }

    line = {
        "metric": "distance row-pairs/sec + achieved HBM GB/s (% of peak), L1 & cosine",
        "value": pairs_per_step * args.steps / elapsed, "unit": "row-pairs/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "configs[1] skewed medium: A,B 10000x20000 CSR, Zipf degrees, |N(0,1)| values; "
                               "step = " + " + ".join({"l1": "pairwise L1", "cosine": "pairwise cosine",
                                                       "knn": "k-NN cosine k=32",
                                                       "tropical": "semiring {plus, min} over the intersection",
                                                       "l1_semiring": "semiring {abs_diff, plus} over the union"}[x]
                                                      for x in names),
                   "a_rows": m, "b_rows": n, "n_cols": A["n_cols"], "nnz_a": int(A["indptr"][-1]), "nnz_b": nnz_b,
                   "row_pointers": "device arrays only: read back by every call" if args.device_row_pointers
                                   else "device arrays, with the host copies the generator holds passed beside them"},
    }
    keys = {"l1": "roofline", "cosine": "roofline_cosine", "knn": "roofline_knn_cosine"}
    for name in names:
        line[keys.get(name, "roofline_" + name)] = roofline(name)
    if "roofline" not in line:
        line["roofline"] = line[keys.get(names[0], "roofline_" + names[0])]
    traffic_file = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(traffic_file):
        with open(traffic_file) as f:
            measured = json.load(f)
        for name in names:
            key = keys.get(name, "roofline_" + name)
            if key in measured:
                line[key]["traffic"] = measured[key]

    if not args.no_cpu_baseline:
        import oracle
        t1 = time.perf_counter()
        used = 1
        for metric in ("manhattan", "cosine", "euclidean", "chebyshev", "minkowski"):
            _, used = oracle.pairwise(A, B, metric, 3.0, return_threads=True)
        cpu_s = time.perf_counter() - t1
        # the same five metrics on one thread, over the first 200 rows of A
        one_rows = np.arange(min(200, m))
        t1 = time.perf_counter()
        for metric in ("manhattan", "cosine", "euclidean", "chebyshev", "minkowski"):
            oracle.pairwise(A, B, metric, 3.0, rows_a=one_rows, threads=1)
        one_s = time.perf_counter() - t1
        line["cpu_baseline"] = {
            "value": 5.0 * m * n / cpu_s, "unit": "row-pairs/s", "cores": int(used), "kind": "oracle",
            "sample": "all 10000 x 10000 row pairs of configs[1] for its five metrics (L1, cosine, L2, Chebyshev, "
                      "Minkowski p=3), support-restricted fp64 oracle, %.1f s of wall time" % cpu_s,
            "one_thread": {"value": 5.0 * one_rows.size * n / one_s, "unit": "row-pairs/s", "cores": 1,
                           "sample": "the first %d rows of A against all of B, the same five metrics, %.1f s"
                                     % (one_rows.size, one_s)}}
    print(json.dumps(line))


if __name__ == "__main__":
    main()
