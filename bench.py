#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

A step = one pass of the whole path over BASELINE config 1 ("skewed medium": A and B
10,000 x 20,000 CSR): spd_pairwise with L1 (union family), spd_pairwise with cosine
(dot-product family) and spd_knn with cosine, k = 32 (fused top-k).  Inputs are resident in
HBM before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def algorithmic_bytes(a_rows, nnz_b, n_b):
    """Bytes the method moves for `a_rows` rows of A against all of B: each row pair streams
    the stored entries of the B row (4-byte column + 4-byte value) and writes one fp32."""
    return a_rows * (8.0 * nnz_b + 4.0 * n_b)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (use --gpus 1)")

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
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    h = spd.Handle()
    out = torch.empty((m, n), dtype=torch.float32, device="cuda")
    idx = torch.empty((m, 32), dtype=torch.int64, device="cuda")
    dist = torch.empty((m, 32), dtype=torch.float32, device="cuda")

    def step():
        h.pairwise(dA, dB, "l1", out=out)
        h.pairwise(dA, dB, "cosine", out=out)
        h.knn(dA, dB, "cosine", 32, out_idx=idx, out_dist=dist)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    pairs_per_step = 3.0 * m * n

    # per-kernel HIP-event timings over the same region, averaged over the timed steps
    h.set_option("profile", 1)
    per_call = {"l1": [], "cosine": [], "knn_cosine": []}
    wall = {"l1": 0.0, "cosine": 0.0, "knn_cosine": 0.0}
    for _ in range(args.steps):
        for name, fn in (("l1", lambda: h.pairwise(dA, dB, "l1", out=out)),
                         ("cosine", lambda: h.pairwise(dA, dB, "cosine", out=out)),
                         ("knn_cosine", lambda: h.knn(dA, dB, "cosine", 32, out_idx=idx, out_dist=dist))):
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            fn()
            per_call[name].append(h.profile_read())
            torch.cuda.synchronize()
            wall[name] += time.perf_counter() - t1
    h.set_option("profile", 0)

    def dominant_scan(records_per_step):
        """Average duration of the scan launch that covers the most rows of A."""
        first = records_per_step[0]
        scans = [i for i, r in enumerate(first) if r["name"] == "scan"]
        big = max(scans, key=lambda i: first[i]["a_rows"])
        ms = float(np.mean([recs[big]["ms"] for recs in records_per_step]))
        total_scan = float(np.mean([sum(r["ms"] for r in recs if r["name"] == "scan") for recs in records_per_step]))
        total_all = float(np.mean([sum(r["ms"] for r in recs) for recs in records_per_step]))
        return first[big], ms, total_scan, total_all

    def roofline(name):
        rec, ms, total_scan, total_all = dominant_scan(per_call[name])
        alg = algorithmic_bytes(rec["a_rows"], nnz_b, n)
        achieved = alg / (ms * 1e-3) / 1e9
        return {"bound": "hbm", "kernel": "spd_scan_kernel<%s, R=%d>" % (name, rec["rows_per_group"]),
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                "algorithmic_bytes_per_launch": alg, "launch_ms": round(ms, 4),
                "a_rows_in_launch": rec["a_rows"], "rows_staged_together": rec["rows_per_group"],
                "block": rec["block"], "lds_bytes": rec["lds_bytes"],
                "all_scan_launches_ms": round(total_scan, 4), "all_kernels_ms": round(total_all, 4),
                "call_wall_ms": round(1e3 * wall[name] / args.steps, 4),
                "note": "effective rate: R rows of A share each entry of B loaded, so the HBM stream is 1/R of the algorithmic bytes"}

    line = {
        "metric": "distance row-pairs/sec + achieved HBM GB/s (% of peak), L1 & cosine",
        "value": pairs_per_step * args.steps / elapsed, "unit": "row-pairs/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "configs[1] skewed medium: A,B 10000x20000 CSR, Zipf degrees, |N(0,1)| values; "
                               "step = pairwise L1 + pairwise cosine + k-NN cosine k=32",
                   "a_rows": m, "b_rows": n, "n_cols": A["n_cols"], "nnz_a": int(A["indptr"][-1]), "nnz_b": nnz_b},
        "roofline": roofline("l1"),
        "roofline_cosine": roofline("cosine"),
        "roofline_knn_cosine": roofline("knn_cosine"),
    }
    traffic_file = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(traffic_file):
        with open(traffic_file) as f:
            t = json.load(f)
        for key in ("roofline", "roofline_cosine"):
            if key in t:
                line[key]["traffic"] = t[key]

    if not args.no_cpu_baseline:
        import oracle
        rng = np.random.default_rng(0)
        rows = np.sort(rng.choice(m, size=192, replace=False))
        t1 = time.perf_counter()
        _, used = oracle.pairwise(A, B, "manhattan", rows_a=rows, return_threads=True)
        oracle.pairwise(A, B, "cosine", rows_a=rows)
        cpu_s = time.perf_counter() - t1
        line["cpu_baseline"] = {"value": 2.0 * rows.size * n / cpu_s, "unit": "row-pairs/s", "cores": int(used),
                                "kind": "oracle",
                                "sample": "192 seeded query rows of configs[1] x all 10000 index rows, L1 and cosine, "
                                          "support-restricted fp64 oracle, %.1f s" % cpu_s}
    print(json.dumps(line))


if __name__ == "__main__":
    main()
