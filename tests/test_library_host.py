"""The C-ABI library without a GPU: it loads, exports what include/*.h declares, rejects
bad arguments, and its host logic (planner; shared per-visit arithmetic) is consistent."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2104_06357_amd as spd
from gen import synth
from util import ALL_METRICS, NONNEGATIVE_ONLY, ORACLE_NAME, assert_distances_close, quotient_cases

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    names = set()
    for header in os.listdir(os.path.join(ROOT, "include")):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names.update(re.findall(r"\b(spd_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_library_loads_and_exports_every_declared_symbol():
    L = spd.lib()
    declared = _declared_functions()
    assert {"spd_create", "spd_destroy", "spd_pairwise", "spd_knn", "spd_workspace_bytes", "spd_set_workspace",
            "spd_csr_validate", "spd_set_option", "spd_last_error", "spd_metric_name", "spd_version",
            "spd_host_pair_value", "spd_host_plan_summary"} <= set(declared)
    for name in declared:
        assert hasattr(L, name), name
    assert b"gfx950" in L.spd_version()
    for i, name in enumerate(spd.METRICS):
        assert L.spd_metric_name(i).decode() == name


def test_null_handle_and_missing_gpu_fail_loudly():
    L = spd.lib()
    assert L.spd_pairwise(None, None, None, 0, 2.0, None) == 1          # SPD_ERR_NULL
    assert L.spd_knn(None, None, None, 0, 2.0, 1, None, None) == 1
    assert L.spd_destroy(None) == 1
    import torch
    if not torch.cuda.is_available():
        h = ctypes.c_void_p()
        assert L.spd_create(ctypes.byref(h), None) == 8                   # SPD_ERR_HIP: no CPU fallback
        assert not h
        with pytest.raises(RuntimeError):
            spd.Handle()


def test_host_pair_value_argument_checks():
    c = np.array([1], dtype=np.int32); v = np.array([1.0], dtype=np.float32)
    with pytest.raises(spd.SpdError) as e:
        spd.testing.host_pair_value("minkowski", 0.0, 4, c, v, c, v)
    assert e.value.status_name == "SPD_ERR_BAD_P"
    with pytest.raises(spd.SpdError) as e:
        spd.testing.host_pair_value(99, 2.0, 4, c, v, c, v)
    assert e.value.status_name == "SPD_ERR_BAD_METRIC"


@pytest.mark.parametrize("metric", ALL_METRICS)
def test_single_sweep_arithmetic_matches_the_oracle(metric):
    """The products g(a, b), norms and expansion functions the kernels run, evaluated on
    the host for single pairs: the union family's one-sweep form (norms plus corrections on
    the intersection) and the expanded forms equal the oracle's plain definitions."""
    A, B = synth.workload(0)
    ra, rb = np.arange(0, 256, 7), np.arange(0, 256, 5)
    for p in ((0.5, 1.0, 3.0) if metric == "minkowski" else (2.0,)):
        want = oracle.pairwise(A, B, ORACLE_NAME[metric], p, rows_a=ra, rows_b=rb)
        got = np.empty_like(want)
        for x, i in enumerate(ra):
            a0, a1 = A["indptr"][i], A["indptr"][i + 1]
            for y, j in enumerate(rb):
                b0, b1 = B["indptr"][j], B["indptr"][j + 1]
                got[x, y] = spd.testing.host_pair_value(metric, p, A["n_cols"], A["indices"][a0:a1], A["values"][a0:a1],
                                                B["indices"][b0:b1], B["values"][b0:b1])
        assert_distances_close(got, want, "%s p=%g" % (metric, p))


@pytest.mark.parametrize("metric", ALL_METRICS)
def test_single_sweep_arithmetic_identical_and_signed_rows(metric):
    rng = np.random.default_rng(5)
    signed = metric not in NONNEGATIVE_ONLY
    k = 300
    rows = []
    for _ in range(6):
        cols = np.sort(rng.choice(k, size=rng.integers(1, 120), replace=False)).astype(np.int32)
        vals = (rng.standard_normal(cols.size) if signed else rng.random(cols.size) + 0.01) * 40.0
        rows.append((cols, vals.astype(np.float32)))
    rows.append((np.empty(0, np.int32), np.empty(0, np.float32)))            # an empty row
    rows.append((rows[0][0].copy(), rows[0][1].copy()))                      # a duplicate of row 0
    half = rows[1][1].copy(); half[::2] = rows[1][1][::2] * np.float32(1.0000001)
    rows.append((rows[1][0].copy(), half))                                   # a near duplicate of row 1
    dense = np.zeros((len(rows), k))
    for r, (c, v) in enumerate(rows):
        dense[r, c] = v
    M = synth.from_dense(dense)
    want = oracle.pairwise(M, M, ORACLE_NAME[metric], 3.0)
    got = np.array([[spd.testing.host_pair_value(metric, 3.0, k, ca, va, cb, vb) for cb, vb in rows] for ca, va in rows])
    assert_distances_close(got, want, metric)


def test_planner_paths_and_thresholds():
    A, B = synth.workload(1, 0.2)
    auto = spd.testing.host_plan_summary(A["indptr"], B["indptr"], A["n_cols"], "cosine")
    assert all(c["kind"] == 2 for c in auto["classes"])                      # 20,000 columns: slot strip
    assert auto["packed_entries"] == B["indptr"][-1] and auto["spilled_rows"] == 0
    for kind in (1, 3, 5):
        s = spd.testing.host_plan_summary(A["indptr"], B["indptr"], A["n_cols"], "cosine", force_kind=kind)
        assert all(c["kind"] == kind for c in s["classes"])
    small, _ = synth.workload(0)
    s = spd.testing.host_plan_summary(small["indptr"], small["indptr"], small["n_cols"], "l1")
    assert [c["kind"] for c in s["classes"]] == [1] and s["classes"][0]["R"] == 8
    # a tight LDS budget forces slices (partitions) of the long rows
    s = spd.testing.host_plan_summary(A["indptr"], B["indptr"], A["n_cols"], "l1", force_kind=3, lds_budget=16384)
    assert s["spilled_rows"] > 0 and s["partial_slots"] >= 2 * s["spilled_rows"]
    assert all(c["lds_bytes"] + 4096 <= 16384 for c in s["classes"])
    # rows at the split threshold (256 for a small B, or the option): one below stays whole
    for length, split in ((255, 0), (256, 1), (257, 1)):
        ip = np.array([0, length], dtype=np.int64)
        s = spd.testing.host_plan_summary(ip, ip, 4096, "l1", force_kind=3)
        assert s["split_rows"] == split, (length, s)
    for length, split in ((127, 0), (128, 1), (129, 1)):
        ip = np.array([0, length], dtype=np.int64)
        s = spd.testing.host_plan_summary(ip, ip, 4096, "l1", force_kind=3, split_len=128)
        assert s["split_rows"] == split, (length, s)
    # a B of 2^22 stored entries or more is cut at 512
    ip = np.arange(0, 511 * 8300, 511, dtype=np.int64)
    assert spd.testing.host_plan_summary(ip[:2], ip, 4096, "l1", force_kind=3)["split_rows"] == 0
    ip = np.arange(0, 512 * 8300, 512, dtype=np.int64)
    assert spd.testing.host_plan_summary(ip[:2], ip, 4096, "l1", force_kind=3)["split_rows"] == 8299
    # Jensen-Shannon keeps at most 8 rows per group
    s = spd.testing.host_plan_summary(small["indptr"], small["indptr"], small["n_cols"], "jensen_shannon")
    assert max(c["R"] for c in s["classes"]) == 8
    # the fused k-NN keeps a list and a queue of 64 keys per staged row beside the tables
    s = spd.testing.host_plan_summary(A["indptr"], B["indptr"], A["n_cols"], "cosine", k_neighbors=64)
    p = spd.testing.host_plan_summary(A["indptr"], B["indptr"], A["n_cols"], "cosine")
    assert max(c["lds_bytes"] for c in s["classes"]) <= 160 * 1024 - 4096
    light = [c for c in s["classes"] if c["R"] == 8 and c["groups"] > 100]
    assert light and all(c["lds_bytes"] >= 20001 * 2 + 8 * 1024 for c in light)
    assert sum(c["R"] * c["groups"] for c in s["classes"]) >= A["n_rows"] and p["classes"]


def test_planner_rejects_bad_row_pointers():
    good = np.array([0, 2, 5], dtype=np.int64)
    bad = np.array([0, 3, 2], dtype=np.int64)
    with pytest.raises(spd.SpdError):
        spd.testing.host_plan_summary(bad, good, 16, "l1")
    with pytest.raises(spd.SpdError):
        spd.testing.host_plan_summary(good, bad, 16, "l1")
    with pytest.raises(spd.SpdError):
        spd.testing.host_plan_summary(np.array([0, 40], dtype=np.int64), good, 16, "l1")   # row longer than k


@pytest.mark.parametrize("config,scale", [(2, 0.02), (3, 0.01), (4, 0.02)])
def test_planner_on_the_large_shapes(config, scale):
    A, B = synth.workload(config, scale)
    metric = {2: "cosine", 3: "jensen_shannon", 4: "jaccard"}[config]
    s = spd.testing.host_plan_summary(A["indptr"], B["indptr"], A["n_cols"], metric, k_neighbors=32 if config == 4 else 0)
    assert s["packed_entries"] == B["indptr"][-1]
    expected_kind = {2: 5, 3: 2, 4: 3}[config]                               # bitmap / slot strip / hash
    assert all(c["kind"] == expected_kind for c in s["classes"]), s
    if config == 3:
        # the 16-bit column-slot strip leaves room for a whole 12,000-entry row; a hash table does not
        assert s["spilled_rows"] == 0
        h = spd.testing.host_plan_summary(A["indptr"], B["indptr"], A["n_cols"], metric, force_kind=3)
        assert h["spilled_rows"] >= 1 and h["partial_slots"] >= 2


def test_planner_sort_key_small_classes_and_bloom_rows():
    A, B = synth.workload(1)
    # sorting B's rows by whole blocks of four steps costs no step, and keeps equal rows in row order
    exact = spd.testing.host_plan_summary(A["indptr"], B["indptr"], A["n_cols"], "cosine", sort_slack=0)
    blocks = spd.testing.host_plan_summary(A["indptr"], B["indptr"], A["n_cols"], "cosine", sort_slack=1)
    assert blocks["total_slab_steps"] == exact["total_slab_steps"] and blocks["slabs"] == exact["slabs"]
    # a class of a few groups joins the class of the same R that needs more LDS, and the longest rows go
    # three to a group of four rather than two to a group of two: three launches, not five
    assert sorted((c["R"], c["groups"]) for c in blocks["classes"]) == [(4, 43), (8, 29), (8, 1202)]
    halved = spd.testing.host_plan_summary(A["indptr"], B["indptr"], A["n_cols"], "cosine", partial_groups=0)
    assert sorted((c["R"], c["groups"]) for c in halved["classes"]) == [(2, 28), (4, 24), (8, 29), (8, 1202)]
    # Chebyshev keeps full groups: an idle place there still ranks its column
    ch = spd.testing.host_plan_summary(A["indptr"], B["indptr"], A["n_cols"], "chebyshev")
    ch0 = spd.testing.host_plan_summary(A["indptr"], B["indptr"], A["n_cols"], "chebyshev", partial_groups=0)
    assert [(c["R"], c["groups"]) for c in ch["classes"]] == [(c["R"], c["groups"]) for c in ch0["classes"]]
    js = spd.testing.host_plan_summary(A["indptr"], B["indptr"], A["n_cols"], "jensen_shannon")
    js0 = spd.testing.host_plan_summary(A["indptr"], B["indptr"], A["n_cols"], "jensen_shannon", partial_groups=0)
    assert sum(c["groups"] for c in js["classes"]) < sum(c["groups"] for c in js0["classes"])
    assert sum(c["R"] * c["groups"] for c in blocks["classes"]) >= A["n_rows"]
    # the cost model's estimates: the large launch far above the small ones, a few groups of long rows get 2 chunks
    by_groups = sorted(blocks["classes"], key=lambda c: c["groups"])
    assert by_groups[-1]["cost"] > 3 * max(c["cost"] for c in by_groups[:-1]) > 0
    assert all(c["chunks"] <= 2 for c in by_groups[:-1])
    # Bloom staging: every row alone, or only the rows that would have been cut into slices
    s = spd.testing.host_plan_summary(A["indptr"], B["indptr"], A["n_cols"], "l1", force_kind=4)
    assert [(c["kind"], c["R"], c["groups"]) for c in s["classes"]] == [(4, 1, A["n_rows"])]
    assert all(c["lds_bytes"] <= 65536 for c in s["classes"])
    with pytest.raises(spd.SpdError):
        spd.testing.host_plan_summary(A["indptr"], B["indptr"], A["n_cols"], "chebyshev", force_kind=4)
    tight = dict(force_kind=3, lds_budget=8192 + 65536)
    long_rows = int((np.diff(A["indptr"]) > 2048).sum())
    sliced = spd.testing.host_plan_summary(A["indptr"], B["indptr"], A["n_cols"], "l1", **tight)
    assert sliced["spilled_rows"] == long_rows == 0 or sliced["spilled_rows"] == long_rows
    ip = np.array([0, 5, 3005, 3010, 9010], dtype=np.int64)                  # rows of 5, 3000, 5, 6000 entries
    sliced = spd.testing.host_plan_summary(ip, ip, 10000, "l1", **tight)
    filtered = spd.testing.host_plan_summary(ip, ip, 10000, "l1", bloom_long_rows=1, **tight)
    assert sliced["spilled_rows"] == 2 and filtered["spilled_rows"] == 0
    assert sorted(c["kind"] for c in filtered["classes"]) == [3, 4]


@pytest.mark.parametrize("metric", ["jensen_shannon", "kl_divergence", "kl_divergence_strict"])
def test_quotients_inside_the_logarithms_on_the_host(metric):
    """A quotient that rounds to 1, or underflows, must not leave log(0) behind: a column whose
    two entries differ by a factor of 1e8 adds what the formula says, not minus infinity."""
    for a, b in quotient_cases():
        A, B = synth.from_dense(a[None, :]), synth.from_dense(b[None, :])
        want = oracle.pairwise(A, B, ORACLE_NAME[metric], mode="full")
        got = spd.testing.host_pair_value(metric, 2.0, 16, A["indices"], A["values"], B["indices"], B["values"])
        assert_distances_close(np.array([[got]]), want, "%s on %s" % (metric, (a[3], b[3])))
    # the case the advisor gave: a = {1, 0.5}, b = {1e-8, 0.5}
    A = synth.from_dense(np.array([[1.0, 0.5]])); B = synth.from_dense(np.array([[1e-8, 0.5]]))
    got = spd.testing.host_pair_value("jensen_shannon", 2.0, 2, A["indices"], A["values"], B["indices"], B["values"])
    assert abs(got - 0.5887) < 1e-4
