#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

A step = one pass of the whole path over one batch of each BASELINE config that measures
throughput (configs 1 to 4; config 0 is the parity case):

  c1_l1, c1_cosine, c1_knn   config 1 (10,000 x 10,000 rows): spd_pairwise L1 and cosine, spd_knn cosine k=32
  c2_cosine                  config 2: spd_pairwise cosine, a tile of 1,024 queries against the 300,000-row index
  c3_l1, c3_js               config 3: spd_pairwise L1 and Jensen-Shannon, a 4,096-row tile of the 65,536-row self-join
  c4_jaccard                 config 4: spd_knn Jaccard, fused top-32, 4,096 queries against 500,000 rows

Every call plans (degree binning), repacks B with its row norms, stages A in LDS, scans,
finishes and writes.  Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

For profiling:  --only NAME[,NAME...]  restricts the step to the named calls (only their
configs are generated), and --copy-calibration adds a plain device-to-device copy of known
size per step, against which the FETCH_SIZE / WRITE_SIZE counters of rocprofv3 are scaled.
"""
import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# Vector ALU: 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz lane-instructions per second (one
# fp64 FMA or one fp32 instruction per lane and clock; the packed fp32 forms are compiled off).
ALU_LANE_OPS = 256 * 4 * 16 * 2.4e9
# LDS: 256 bytes per clock and compute unit, the rate of the 128-bit reads that fetch a column's staged
# values (a conflict-free stream of them measures 208 on this chip; 64-bit reads 163, 32-bit reads 83).
LDS_PEAK_BYTES = 256 * 256 * 2.4e9
COPY_BYTES = 256 << 20

# What one visit (a staged row of A meeting a stored entry of B) cannot cost less than in vector
# instructions, counted from the product's source (csrc/spd_ops.h): the conversion and the fp64
# FMA of the dot product; median, conversion and fp64 add of L1; the two logarithms, the refined
# quotient, the selects and the two fp64 sums of Jensen-Shannon; a quarter of a 32-bit add for
# the set metrics, whose byte counters take four rows to the word.
PRODUCT_INSTRUCTIONS = {"l1": 3.0, "cosine": 2.0, "jensen_shannon": 24.0, "jaccard": 0.25,
                        "tropical": 4.0, "sq_diff_semiring": 4.0}
# LDS bytes one lane reads per step for the column lookup, by staging kind (dense strip: none;
# column-slot strip: a 16-bit slot; hash: two buckets of 16 bytes; Bloom: two filter words;
# bitmap with ranks: one 8-byte word), and per staged row for the value (4, or 1 for the set metrics).
LOOKUP_BYTES = {1: 0, 2: 2, 3: 32, 4: 8, 5: 8}

CALLS = {
    # name: (config, kind of call, metric, label)
    "c1_l1": (1, "pairwise", "l1", "config 1 pairwise L1"),
    "c1_cosine": (1, "pairwise", "cosine", "config 1 pairwise cosine"),
    "c1_knn": (1, "knn", "cosine", "config 1 k-NN cosine k=32"),
    "c2_cosine": (2, "pairwise", "cosine", "config 2 pairwise cosine, 1,024-query tile"),
    "c3_l1": (3, "pairwise", "l1", "config 3 pairwise L1, 4,096-row tile"),
    "c3_js": (3, "pairwise", "jensen_shannon", "config 3 pairwise Jensen-Shannon, 4,096-row tile"),
    "c4_jaccard": (4, "knn", "jaccard", "config 4 k-NN Jaccard k=32"),
    # semiring calls, not part of the step
    "c1_tropical": (1, "semiring", "tropical", "config 1 semiring {plus, min} over the intersection"),
    "c1_sq_diff_semiring": (1, "semiring", "sq_diff_semiring", "config 1 semiring {sq_diff, plus} over the union"),
}
STEP = ["c1_l1", "c1_cosine", "c1_knn", "c2_cosine", "c3_l1", "c3_js", "c4_jaccard"]
ROOFLINE_KEYS = {"c1_l1": "roofline_config1_l1", "c1_cosine": "roofline_config1_cosine",
                 "c1_knn": "roofline_config1_knn_cosine", "c2_cosine": "roofline_config2",
                 "c3_l1": "roofline_config3", "c3_js": "roofline_config3_jensen_shannon",
                 "c4_jaccard": "roofline_config4"}
HEADLINE = "c3_l1"       # the largest single-GPU configuration (4.9e11 visits per call), union family
TILE_ROWS = {2: 1024, 3: 4096}
KNN_K = 32


def algorithmic_bytes(a_rows, nnz_b, n_b, writes_matrix):
    """Bytes the method moves for `a_rows` rows of A against all of B: each row pair streams
    the stored entries of the B row (4-byte column + 4-byte value) and, for spd_pairwise, writes
    one fp32."""
    return a_rows * (8.0 * nnz_b + (4.0 * n_b if writes_matrix else 0.0))


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
    n, k = B["n_rows"], KNN_K
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
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--only", default=None,
                    help="comma-separated calls to time instead of the whole step: " + ", ".join(CALLS))
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
    names = args.only.split(",") if args.only else list(STEP)
    for name in names:
        if name not in CALLS:
            sys.exit("unknown call %r (known: %s)" % (name, ", ".join(CALLS)))
    configs = sorted({CALLS[name][0] for name in names})

    # ---- inputs: generated on the host (the larger configs side by side), then copied to HBM
    t_gen = time.perf_counter()
    with ThreadPoolExecutor(max_workers=len(configs)) as pool:
        futures = {c: pool.submit(synth.workload, c) for c in sorted(configs, reverse=True)}
        host = {c: f.result() for c, f in futures.items()}
    for c, rows in TILE_ROWS.items():
        if c in host:                      # the query tile: the first rows of the query matrix
            host[c] = (synth.slice_rows(host[c][0], 0, rows), host[c][1])
    gen_s = time.perf_counter() - t_gen
    keep = not args.device_row_pointers
    dev = {c: (spd.DeviceCsr.from_host(a, keep_host_indptr=keep), spd.DeviceCsr.from_host(b, keep_host_indptr=keep))
           for c, (a, b) in host.items()}
    shape = {c: (a["n_rows"], b["n_rows"], int(b["indptr"][-1])) for c, (a, b) in host.items()}
    h = spd.Handle()
    if args.serial:
        h.set_option("side_streams", 0)
    biggest = max(shape[CALLS[name][0]][0] * shape[CALLS[name][0]][1] for name in names if CALLS[name][1] != "knn") \
        if any(CALLS[name][1] != "knn" for name in names) else 0
    out_flat = torch.empty(biggest, dtype=torch.float32, device="cuda")      # one buffer serves every pairwise call
    m_max = max(shape[c][0] for c in configs)
    idx = torch.empty((m_max, KNN_K), dtype=torch.int64, device="cuda")
    dist = torch.empty((m_max, KNN_K), dtype=torch.float32, device="cuda")
    copy_src = copy_dst = None
    if args.copy_calibration:
        copy_src = torch.ones(COPY_BYTES // 4, dtype=torch.float32, device="cuda")
        copy_dst = torch.empty_like(copy_src)

    def make_call(name):
        config, kind, metric, _ = CALLS[name]
        dA, dB = dev[config]
        m, n, _ = shape[config]
        if kind == "pairwise":
            out = out_flat[:m * n].view(m, n)
            return lambda: h.pairwise(dA, dB, metric, out=out)
        if kind == "knn":
            return lambda: h.knn(dA, dB, metric, KNN_K, out_idx=idx[:m], out_dist=dist[:m])
        out = out_flat[:m * n].view(m, n)
        if metric == "tropical":
            return lambda: h.semiring_pairwise(dA, dB, "plus", "min", False, out=out)
        # (no distance of the library is spelled this way, so the call runs on the run-time-product kernels)
        return lambda: h.semiring_pairwise(dA, dB, "sq_diff", "plus", True, out=out)

    calls = {name: make_call(name) for name in names}

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
    pairs_per_step = float(sum(shape[CALLS[name][0]][0] * shape[CALLS[name][0]][1] for name in names))

    # per-kernel HIP-event timings (events recorded by the library around every launch, on the
    # stream of that launch), over a few steps more.  The small launches of a call normally
    # overlap with the large one on side streams; here they are serialised so that a launch's
    # duration is its own.
    h.set_option("profile", 1)
    h.set_option("side_streams", 0)
    profile_steps = max(1, min(args.steps, 5))
    records = {name: [] for name in names}
    wall = {name: 0.0 for name in names}
    for _ in range(profile_steps):
        for name in names:
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            calls[name]()
            records[name].append(h.profile_read())
            torch.cuda.synchronize()
            wall[name] += time.perf_counter() - t1
    h.set_option("profile", 0)

    traffic_file = os.path.join(ROOT, "profiles", "traffic.json")
    stored_traffic = {}
    if os.path.exists(traffic_file):
        with open(traffic_file) as f:
            stored_traffic = json.load(f)

    def roofline(name):
        config, kind, metric, label = CALLS[name]
        m, n, nnz_b = shape[config]
        per_step = records[name]
        first = per_step[0]
        scans = [i for i, r in enumerate(first) if r["name"] == "scan"]
        mean_ms = lambda i: float(np.mean([recs[i]["ms"] for recs in per_step]))
        big = max(scans, key=mean_ms)                     # the dominant launch: the longest one
        rec = first[big]
        ms = mean_ms(big)
        scan_ms = float(np.mean([sum(r["ms"] for r in recs if r["name"] == "scan") for recs in per_step]))
        all_ms = float(np.mean([sum(r["ms"] for r in recs) for recs in per_step]))
        alg = algorithmic_bytes(rec["a_rows"], nnz_b, n, kind != "knn")
        visits = float(rec["a_rows"]) * nnz_b / (ms * 1e-3)
        R, staging = rec["rows_per_group"], rec["staging_kind"]
        # vector ALU: the product's own instructions, nothing else counted
        per_visit = PRODUCT_INSTRUCTIONS[metric]
        alu = {"achieved": visits * per_visit, "peak": ALU_LANE_OPS, "unit": "lane-instructions/s",
               "frac": round(visits * per_visit / ALU_LANE_OPS, 4), "vector_instructions_per_visit": per_visit}
        # LDS: what a lane must read per step (the column's map entry, the R staged values)
        value_bytes = 1.0 if metric == "jaccard" else 4.0
        lds_per_visit = LOOKUP_BYTES.get(staging, 0) / float(R) + value_bytes
        lds = {"achieved": visits * lds_per_visit, "peak": LDS_PEAK_BYTES, "unit": "B/s",
               "frac": round(visits * lds_per_visit / LDS_PEAK_BYTES, 4), "lds_bytes_per_visit": round(lds_per_visit, 3)}
        bound = "alu" if alu["frac"] >= lds["frac"] else "lds"
        binding = alu if bound == "alu" else lds
        all_visits = float(sum(r["a_rows"] for r in first if r["name"] == "scan")) * nnz_b / (scan_ms * 1e-3)
        out = {
            "bound": bound, "achieved": binding["achieved"], "peak": binding["peak"], "unit": binding["unit"],
            "frac": binding["frac"], "traffic": None, "traffic_source": None,
            "call": label,
            "kernel": "spd_scan_kernel (%s, R=%d rows of A per workgroup, staging kind %d%s)"
                      % (metric, R, staging, ", fused top-%d" % KNN_K if kind == "knn" else ""),
            "launch_ms": round(ms, 4), "visits_per_s": visits, "a_rows_in_launch": rec["a_rows"],
            "rows_per_group": R, "staging_kind": staging, "workgroups": rec["workgroups"], "block": rec["block"],
            "lds_bytes": rec["lds_bytes"],
            "alu": alu, "lds": lds,
            "effective_hbm": {"achieved": round(alg / (ms * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                              "frac": round(alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                              "algorithmic_bytes_per_launch": alg,
                              "note": "algorithmic bytes (8 per visit, 4 per distance written) over the launch time: "
                                      "an effective rate, above the HBM peak because the R staged rows share every "
                                      "entry of B that is loaded and workgroups share B through L2"},
            "scan_launches_per_call": len(scans), "all_scan_launches_ms": round(scan_ms, 4),
            "all_scan_launches_visits_per_s": all_visits, "all_kernels_ms": round(all_ms, 4),
            "serialised_call_wall_ms": round(1e3 * wall[name] / profile_steps, 4),
            "row_pairs_per_s_of_call": m * float(n) / (wall[name] / profile_steps),
        }
        key = ROOFLINE_KEYS.get(name, "roofline_" + name)
        if key in stored_traffic:
            st = stored_traffic[key]
            out["traffic"] = st["bytes_per_launch"]
            out["traffic_source"] = "stored, not measured in this run: " + st["source"]
            # what the counters said of the same launch (of the build that was profiled): how busy
            # the vector ALUs and the LDS units really were, beside the instruction and byte models above
            out["counters_of_the_profiled_run"] = {k: st[k] for k in ("valu_busy", "lds_busy", "l2_hit_rate",
                                                                         "valu_instructions_per_wavefront_step",
                                                                         "fetch_bytes", "write_bytes") if k in st}
        return out

    described = [CALLS[name][3] for name in names]
    line = {
        "metric": "distance row-pairs/sec + achieved HBM GB/s (% of peak), L1 & cosine",
        "value": pairs_per_step * args.steps / elapsed, "unit": "row-pairs/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "configs[1]-[4], one batch of each per step (headline roofline: configs[3], 4,096 x 65,536 "
                               "rows, pairwise L1): " + "; ".join(described),
                   "shapes": {"config%d" % c: {"a_rows": shape[c][0], "b_rows": shape[c][1], "nnz_b": shape[c][2],
                                               "n_cols": host[c][0]["n_cols"], "nnz_a": int(host[c][0]["indptr"][-1])}
                              for c in configs},
                   "row_pairs_per_step": pairs_per_step,
                   "row_pointers": "device arrays only: read back by every call" if args.device_row_pointers
                                   else "device arrays, with the host copies the generator holds passed beside them",
                   "input_generation_s": round(gen_s, 1)},
    }
    for name in names:
        line[ROOFLINE_KEYS.get(name, "roofline_" + name)] = roofline(name)
    head = HEADLINE if HEADLINE in names else names[0]
    line["roofline"] = dict(line[ROOFLINE_KEYS.get(head, "roofline_" + head)])

    if not args.no_cpu_baseline:
        import oracle
        # a bounded sample of the same workload: every pair of config 1 for L1 and cosine, and a
        # few query rows of each larger config against a sample of its index rows
        samples = {1: (None, None), 2: (128, 65536), 3: (128, 16384), 4: (32, 131072)}
        oracle_name = {"l1": "manhattan", "cosine": "cosine", "jensen_shannon": "jensen_shannon", "jaccard": "jaccard"}
        rng = np.random.default_rng(0)
        pairs, used, parts = 0.0, 1, []
        t1 = time.perf_counter()
        for name in names:
            config, kind, metric, label = CALLS[name]
            if metric not in oracle_name or name == "c1_knn":
                continue
            A, B = host[config]
            na, nb = samples[config]
            ra = None if na is None else np.sort(rng.choice(A["n_rows"], size=min(na, A["n_rows"]), replace=False))
            rb = None if nb is None else np.sort(rng.choice(B["n_rows"], size=min(nb, B["n_rows"]), replace=False))
            t2 = time.perf_counter()
            got, used = oracle.pairwise(A, B, oracle_name[metric], 2.0, rows_a=ra, rows_b=rb, return_threads=True)
            parts.append("%s: %d x %d pairs in %.1f s" % (name, got.shape[0], got.shape[1], time.perf_counter() - t2))
            pairs += float(got.shape[0]) * got.shape[1]
        cpu_s = time.perf_counter() - t1
        line["cpu_baseline"] = {
            "value": pairs / cpu_s, "unit": "row-pairs/s", "cores": int(used), "kind": "oracle",
            "sample": "support-restricted fp64 oracle on a sample of each call's row pairs (%s), %.1f s of wall time"
                      % ("; ".join(parts), cpu_s)}
    print(json.dumps(line))


if __name__ == "__main__":
    main()
