"""The Bloom-filter staging (Section 3.3.2's alternative to the hash table): a row of A alone in
its workgroup, its columns in a Bloom filter in LDS, its values looked up by binary search in
global memory.  Parity with the CPU oracle through the C-ABI (needs an MI355X)."""
import numpy as np
import pytest

import oracle
from gen import synth
from test_gpu_parity import _edge_matrices, _p_of, _wide_pair
from util import ALL_METRICS, NONNEGATIVE_ONLY, ORACLE_NAME, assert_distances_close, assert_knn_matches

pytestmark = pytest.mark.gpu

SERVED = [m for m in ALL_METRICS if m != "chebyshev"]


@pytest.fixture(scope="module")
def spd():
    import paper_2104_06357_amd as lib
    return lib


@pytest.fixture()
def handle(spd):
    h = spd.Handle()
    h.set_option("check_plan", 1)
    yield h
    h.close()


def _np(t):
    import torch
    torch.cuda.synchronize()
    return t.cpu().numpy()


@pytest.mark.parametrize("metric", SERVED)
def test_config0_every_pair(handle, spd, metric):
    A, B = synth.workload(0)
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    print("bloom config0", metric, flush=True)
    p = _p_of(metric)
    handle.set_option("force_kind", 4)
    want = oracle.pairwise(A, B, ORACLE_NAME[metric], p)
    assert_distances_close(_np(handle.pairwise(dA, dB, metric, p)), want, metric)
    kinds = {r["staging_kind"] for r in _profile(handle, lambda: handle.pairwise(dA, dB, metric, p))}
    assert kinds == {4}
    idx, dist = handle.knn(dA, dB, metric, 9, p)
    assert_knn_matches(_np(idx), _np(dist), want, 9, metric, metric)


def _profile(handle, call):
    handle.set_option("profile", 1)
    call()
    recs = [r for r in handle.profile_read() if r["name"] == "scan"]
    handle.set_option("profile", 0)
    return recs


@pytest.mark.parametrize("metric", SERVED)
def test_rows_of_every_length_split_rows_and_edge_rows(handle, spd, metric):
    signed = metric not in NONNEGATIVE_ONLY
    p = _p_of(metric)
    handle.set_option("force_kind", 4)
    handle.set_option("split_len", 4)
    handle.set_option("window", 64)
    for name, (A, B) in (("wide", _wide_pair(signed)), ("edge", (_edge_matrices(signed),) * 2)):
        print("bloom", name, metric, flush=True)
        dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
        want = oracle.pairwise(A, B, ORACLE_NAME[metric], p, mode="full")
        assert_distances_close(_np(handle.pairwise(dA, dB, metric, p)), want, "%s %s" % (name, metric))


def _long_pair(signed):
    rng = np.random.default_rng(31)
    k = 8000
    out = []
    for rows, lens in ((21, (0, 5, 300, 2048, 2049, 3000, 6000)), (60, (0, 1, 40, 700, 4000, 8000))):
        d = np.zeros((rows, k))
        for r in range(rows):
            n = lens[r % len(lens)]
            d[r, rng.choice(k, size=n, replace=False)] = rng.standard_normal(n) if signed else rng.random(n) + 0.01
        out.append(synth.from_dense(np.asarray(d.astype(np.float32), dtype=np.float64)))
    return out


@pytest.mark.parametrize("metric", ["cosine", "l1", "minkowski", "jensen_shannon", "kl_divergence_strict", "hamming"])
def test_long_rows_get_a_filter_instead_of_slices(handle, spd, metric):
    """Option bloom_long_rows: with a 72 KB LDS budget a hash table holds 2,048 entries; the longer
    rows of A go behind a Bloom filter, whole, the shorter ones are staged as ever."""
    A, B = _long_pair(metric not in NONNEGATIVE_ONLY)
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    p = _p_of(metric)
    options = dict(force_kind=3, lds_budget=8192 + 65536, bloom_long_rows=1)
    for name, value in options.items():
        handle.set_option(name, value)
    plan = spd.testing.host_plan_summary(A["indptr"], B["indptr"], 8000, metric, **options)
    assert plan["spilled_rows"] == 0 and {c["kind"] for c in plan["classes"]} == {3, 4}
    without = spd.testing.host_plan_summary(A["indptr"], B["indptr"], 8000, metric, force_kind=3, lds_budget=8192 + 65536)
    assert without["spilled_rows"] == 9
    want = oracle.pairwise(A, B, ORACLE_NAME[metric], p, mode="full")
    assert_distances_close(_np(handle.pairwise(dA, dB, metric, p)), want, metric)
    idx, dist = handle.knn(dA, dB, metric, 7, p)
    assert_knn_matches(_np(idx), _np(dist), want, 7, metric, metric)


def test_a_row_longer_than_the_largest_filter_serves(handle, spd):
    """40,000 entries in one row: the filter is capped at 2^19 bits, the search takes 16 steps."""
    rng = np.random.default_rng(12)
    k = 50_000
    d = np.zeros((3, k))
    for r, n in enumerate((40_000, 33_000, 5)):
        d[r, rng.choice(k, size=n, replace=False)] = rng.random(n) + 0.01
    e = np.zeros((130, k))
    for r in range(130):
        n = [0, 1, 7, 300, 2500, 20_000][r % 6]
        e[r, rng.choice(k, size=n, replace=False)] = rng.random(n) + 0.01
    A = synth.from_dense(np.asarray(d.astype(np.float32), dtype=np.float64))
    B = synth.from_dense(np.asarray(e.astype(np.float32), dtype=np.float64))
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    for options in (dict(force_kind=4), dict(bloom_long_rows=1)):
        h = spd.Handle()
        h.set_option("check_plan", 1)
        for name, value in options.items():
            h.set_option(name, value)
        for metric in ("cosine", "l1", "jensen_shannon"):
            want = oracle.pairwise(A, B, ORACLE_NAME[metric])
            assert_distances_close(_np(h.pairwise(dA, dB, metric)), want, "%s %s" % (metric, options))
        if "bloom_long_rows" in options:
            plan = spd.testing.host_plan_summary(A["indptr"], B["indptr"], k, "cosine", **options)
            assert plan["spilled_rows"] == 0 and 4 in {c["kind"] for c in plan["classes"]}
        h.close()


def test_semirings_and_what_the_filter_does_not_serve(handle, spd):
    A, B = _wide_pair(True)
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    handle.set_option("force_kind", 4)
    for sr in (("times", "plus", False), ("abs_diff", "plus", True), ("max", "plus", True), ("min", "plus", False)):
        want = oracle.semiring_pairwise(A, B, *sr, mode="full")
        assert_distances_close(_np(handle.semiring_pairwise(dA, dB, *sr)), want, str(sr))
    for call in (lambda: handle.pairwise(dA, dB, "chebyshev"), lambda: handle.semiring_pairwise(dA, dB, "plus", "min", False)):
        with pytest.raises(spd.SpdError) as e:
            call()
        assert e.value.status_name == "SPD_ERR_UNSUPPORTED"
    # with the option, the products it does not serve keep their slices
    A, B = _long_pair(True)
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    options = dict(force_kind=3, lds_budget=8192 + 65536, bloom_long_rows=1)
    for name, value in options.items():
        handle.set_option(name, value)
    assert spd.testing.host_plan_summary(A["indptr"], B["indptr"], 8000, "chebyshev", **options)["spilled_rows"] > 0
    want = oracle.pairwise(A, B, "chebyshev", mode="full")
    assert_distances_close(_np(handle.pairwise(dA, dB, "chebyshev")), want, "chebyshev keeps its slices")
