"""Parity of the semiring entry points (spd_semiring_pairwise / spd_semiring_knn) with the CPU
oracle's semiring products, element by element, through the C-ABI (needs an MI355X)."""
import itertools

import numpy as np
import pytest

import oracle
from gen import synth
from test_gpu_parity import _edge_matrices, _sample_rows, _wide_pair
from util import (ALL_METRICS, NONNEGATIVE_ONLY, ORACLE_NAME, TABLE1_SEMIRINGS, assert_distances_close,
                  assert_knn_matches)

pytestmark = pytest.mark.gpu

SEMIRINGS = [(p, s, u) for p in oracle.PRODUCTS for s in oracle.SUMS for u in (False, True)]
# one of each kind of kernel work: the tropical semiring, a sum over the union, a maximum and a
# minimum over the union (one-sided columns completed from the ranked entries), a bottleneck
SELECTED = [("plus", "min", False), ("sq_diff", "plus", True), ("abs_diff", "max", True), ("max", "min", True),
            ("min", "max", False), ("times", "plus", False)]


def _name(sr):
    return "%s/%s/%s" % (sr[0], sr[1], "union" if sr[2] else "intersection")


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


@pytest.fixture(scope="module")
def config0(spd):
    A, B = synth.workload(0)
    return A, B, spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)


@pytest.fixture(scope="module")
def signed0(spd):
    """Configuration 0 with a random sign on every value."""
    A, B = synth.workload(0)
    rng = np.random.default_rng(5)
    for M in (A, B):
        M["values"] = (M["values"] * rng.choice([-1.0, 1.0], size=M["values"].size)).astype(np.float32)
    return A, B, spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)


def _run(handle, dA, dB, sr):
    import torch
    out = handle.semiring_pairwise(dA, dB, *sr)
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("sr", SEMIRINGS, ids=_name)
def test_config0_every_pair(handle, config0, signed0, sr):
    for tag, (A, B, dA, dB) in (("config0", config0), ("signed", signed0)):
        print("semiring", tag, _name(sr), flush=True)
        got = _run(handle, dA, dB, sr)
        want = oracle.semiring_pairwise(A, B, *sr)
        assert_distances_close(got, want, "%s %s" % (tag, _name(sr)))


@pytest.mark.parametrize("kind", [1, 2, 3, 5])
@pytest.mark.parametrize("max_rows", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("sr", SELECTED, ids=_name)
def test_every_staging_path(handle, signed0, sr, kind, max_rows):
    A, B, dA, dB = signed0
    print("semiring staging", _name(sr), kind, max_rows, flush=True)
    handle.set_option("force_kind", kind)
    handle.set_option("max_rows", max_rows)
    want = oracle.semiring_pairwise(A, B, *sr)
    assert_distances_close(_run(handle, dA, dB, sr), want, "%s kind=%d R=%d" % (_name(sr), kind, max_rows))


@pytest.mark.parametrize("sr", SEMIRINGS, ids=_name)
def test_split_rows_and_sliced_rows(handle, spd, sr):
    """Rows of B cut over several lanes and rows of A cut into slices: the slices' sums add up,
    their maxima are joined by max, and each slice answers only for its own range of columns."""
    A, B = _wide_pair(True)
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    print("semiring split+slices", _name(sr), flush=True)
    for name, value in (("split_len", 4), ("window", 64), ("force_kind", 3), ("lds_budget", 8192), ("chunks", 3)):
        handle.set_option(name, value)
    want = oracle.semiring_pairwise(A, B, *sr, mode="full")
    assert_distances_close(_run(handle, dA, dB, sr), want, _name(sr))


@pytest.mark.parametrize("sr", SEMIRINGS, ids=_name)
def test_edge_rows_and_self_join(handle, spd, sr):
    """Empty rows, single entries, a full row, duplicates, a stored zero; A and B the same matrix."""
    M = _edge_matrices(True)
    dM = spd.DeviceCsr.from_host(M)
    print("semiring edge rows", _name(sr), flush=True)
    got = _run(handle, dM, dM, sr)
    want = oracle.semiring_pairwise(M, M, *sr, mode="full")
    assert_distances_close(got, want, _name(sr))
    finite = np.isfinite(want)
    np.testing.assert_allclose(np.where(finite, got, 0), np.where(finite, got.T, 0), rtol=2e-4, atol=2e-5)
    one = synth.slice_rows(M, 6, 7)
    d1 = spd.DeviceCsr.from_host(one)
    assert_distances_close(_run(handle, d1, dM, sr), want[6:7], _name(sr) + " m=1")
    assert_distances_close(_run(handle, dM, d1, sr), want[:, 6:7], _name(sr) + " n=1")
    E = synth.from_dense(np.zeros((3, 130)))
    dE = spd.DeviceCsr.from_host(E)
    assert_distances_close(_run(handle, dE, dM, sr), oracle.semiring_pairwise(E, M, *sr), _name(sr) + " empty A")


def test_rows_with_more_entries_than_are_ranked(handle, spd):
    """sum() = max over the union with staged rows of several hundred entries: when every ranked
    entry of a row meets a column of the other row, the rest is found by walking the two rows."""
    rng = np.random.default_rng(41)
    k = 600
    d = np.zeros((24, k))
    for r in range(24):
        n = [600, 599, 400, 300, 64, 33, 32, 31][r % 8]
        d[r, rng.choice(k, size=n, replace=False)] = rng.standard_normal(n)
    e = np.zeros((90, k))
    for r in range(90):
        n = [600, 598, 500, 200, 50, 1, 0][r % 7]
        e[r, rng.choice(k, size=n, replace=False)] = rng.standard_normal(n)
    A = synth.from_dense(np.asarray(d.astype(np.float32), dtype=np.float64))
    B = synth.from_dense(np.asarray(e.astype(np.float32), dtype=np.float64))
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    for sr in (("abs_diff", "max", True), ("plus", "min", True), ("sq_diff", "max", True), ("min", "min", True),
               ("max", "max", True), ("times", "min", True)):
        for kind in (1, 2, 3, 5):
            handle.set_option("force_kind", kind)
            want = oracle.semiring_pairwise(A, B, *sr, mode="full")
            assert_distances_close(_run(handle, dA, dB, sr), want, "%s kind %d" % (_name(sr), kind))


@pytest.mark.parametrize("k", [1, 10, 64])
@pytest.mark.parametrize("sr", SELECTED, ids=_name)
def test_config0_knn(handle, signed0, sr, k):
    import torch
    A, B, dA, dB = signed0
    print("semiring knn", _name(sr), k, flush=True)
    idx, val = handle.semiring_knn(dA, dB, *sr, k)
    torch.cuda.synchronize()
    rows = oracle.semiring_pairwise(A, B, *sr)
    assert_knn_matches(idx.cpu().numpy(), val.cpu().numpy(), rows, k, "semiring", _name(sr))


def test_knn_with_sliced_rows_and_split_rows(handle, spd):
    import torch
    A, B = _wide_pair(True)
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    for name, value in (("split_len", 4), ("window", 64), ("force_kind", 3), ("lds_budget", 8192), ("chunks", 3)):
        handle.set_option(name, value)
    for sr in SELECTED:
        idx, val = handle.semiring_knn(dA, dB, *sr, 9)
        torch.cuda.synchronize()
        rows = oracle.semiring_pairwise(A, B, *sr, mode="full")
        assert_knn_matches(idx.cpu().numpy(), val.cpu().numpy(), rows, 9, "semiring", _name(sr))


def _call(handle, dA, dB, sr, p=3.0):
    """spd_semiring_pairwise for a dict {product, sum, over_union[, transform][, epilogue][, p]}."""
    import torch
    out = handle.semiring_pairwise(dA, dB, sr["product"], sr["sum"], sr["over_union"], p=sr.get("p", p),
                                   transform=sr.get("transform", "none"), epilogue=sr.get("epilogue", "none"))
    torch.cuda.synchronize()
    return out.cpu().numpy()


def _oracle_call(A, B, sr, p=3.0, **kw):
    return oracle.semiring_pairwise(A, B, sr["product"], sr["sum"], sr["over_union"], p=sr.get("p", p),
                                    transform=sr.get("transform", "none"), epilogue=sr.get("epilogue", "none"), **kw)


@pytest.mark.parametrize("metric", ALL_METRICS)
def test_semirings_reproduce_the_metrics(handle, spd, config0, metric):
    """Every distance of Table 1 (and the library's variants of them) through spd_semiring_pairwise
    and spd_semiring_knn: transform, product, sum, domain and epilogue as Section 2.2 and Table 1
    give them, against the oracle's semiring evaluator, the oracle's plain formula, and the
    library's own spd_pairwise."""
    import torch
    sr = TABLE1_SEMIRINGS[metric]
    p = sr.get("p", 3.0)
    cases = [("config0",) + tuple(config0)]
    M = _edge_matrices(metric not in NONNEGATIVE_ONLY)
    dM = spd.DeviceCsr.from_host(M)
    cases.append(("edge rows", M, M, dM, dM))
    for tag, A, B, dA, dB in cases:
        print("table 1 as a semiring", metric, tag, flush=True)
        got = _call(handle, dA, dB, sr)
        assert_distances_close(got, _oracle_call(A, B, sr, mode="full"), "%s as a semiring, %s" % (metric, tag))
        want = oracle.pairwise(A, B, ORACLE_NAME[metric], p, mode="full")
        lib = handle.pairwise(dA, dB, metric, p)
        torch.cuda.synchronize()
        lib = lib.cpu().numpy()
        if metric == "chebyshev":      # the identity of max between two empty rows, where the distance says 0
            both_empty = (np.diff(A["indptr"]) == 0)[:, None] & (np.diff(B["indptr"]) == 0)[None, :]
            assert np.all(got[both_empty] == -np.inf)
            got = np.where(both_empty, 0.0, got)
        assert_distances_close(got, want, "%s as a semiring against the formula, %s" % (metric, tag))
        if metric != "chebyshev":
            assert np.array_equal(got, lib, equal_nan=True), metric     # the same kernels ran
    A, B, dA, dB = config0
    if metric != "inner_product":          # (spd_knn returns the largest inner products)
        idx, val = handle.semiring_knn(dA, dB, sr["product"], sr["sum"], sr["over_union"], 9, p=p,
                                       transform=sr.get("transform", "none"), epilogue=sr.get("epilogue", "none"))
        torch.cuda.synchronize()
        rows = _oracle_call(A, B, sr)
        assert_knn_matches(idx.cpu().numpy(), val.cpu().numpy(), rows, 9, "semiring", metric + " knn")


# combinations that spell none of Table 1's distances: they run on the kernels that take the
# product as a run-time choice
OTHER_SEMIRINGS = [
    dict(product="abs_diff_pow", sum="max", over_union=True, p=2.5),
    dict(product="abs_diff_pow", sum="plus", over_union=True, p=3.0),                       # no root
    dict(product="abs_diff_pow", sum="plus", over_union=False, p=0.5, epilogue="root_p"),
    dict(product="canberra", sum="plus", over_union=False),
    dict(product="canberra", sum="max", over_union=True),
    dict(product="canberra", sum="plus", over_union=True, epilogue="div_k"),
    dict(product="not_equal", sum="plus", over_union=False),
    dict(product="not_equal", sum="min", over_union=True),
    dict(product="x_log_x_over_y", sum="max", over_union=False),
    dict(product="x_log_x_over_y", sum="min", over_union=False),
    dict(product="x_log_x_over_y", sum="plus", over_union=False, transform="sqrt"),
    dict(product="js_term", sum="plus", over_union=False),
    dict(product="js_term", sum="max", over_union=True),
    dict(product="js_term", sum="plus", over_union=True),                                    # the divergence, no root
    dict(product="times", sum="plus", over_union=False, transform="sqrt"),                   # the Bhattacharyya coefficient
    dict(product="abs_diff", sum="plus", over_union=True, transform="nonzero", epilogue="div_k"),
    dict(product="sq_diff", sum="plus", over_union=True, epilogue="sqrt_half"),
    dict(product="min", sum="plus", over_union=False, transform="sqrt", epilogue="root_p", p=2.0),
    dict(product="max", sum="max", over_union=True, epilogue="div_k"),
]


def _sr_name(sr):
    return "/".join(str(sr[k]) for k in ("product", "sum", "over_union", "transform", "epilogue", "p") if k in sr)


@pytest.mark.parametrize("sr", OTHER_SEMIRINGS, ids=_sr_name)
def test_other_combinations_of_the_menu(handle, spd, config0, sr):
    """Pairwise on config 0 through every staging kind, on rows cut into slices with the operands'
    roles exchanged, on the edge rows, and fused k-NN."""
    import torch
    A, B, dA, dB = config0
    print("semiring", _sr_name(sr), flush=True)
    want = _oracle_call(A, B, sr, mode="full")
    for kind, max_rows in ((1, 8), (2, 4), (3, 8), (5, 2)):
        handle.set_option("force_kind", kind)
        handle.set_option("max_rows", max_rows)
        assert_distances_close(_call(handle, dA, dB, sr), want, "%s kind %d" % (_sr_name(sr), kind))
    idx, val = handle.semiring_knn(dA, dB, sr["product"], sr["sum"], sr["over_union"], 10, p=sr.get("p", 3.0),
                                   transform=sr.get("transform", "none"), epilogue=sr.get("epilogue", "none"))
    torch.cuda.synchronize()
    assert_knn_matches(idx.cpu().numpy(), val.cpu().numpy(), _oracle_call(A, B, sr), 10, "semiring", _sr_name(sr) + " knn")
    handle.set_option("force_kind", 0)
    handle.set_option("max_rows", 8)
    M = _edge_matrices(False)
    dM = spd.DeviceCsr.from_host(M)
    assert_distances_close(_call(handle, dM, dM, sr), _oracle_call(M, M, sr, mode="full"), _sr_name(sr) + " edge rows")
    A, B = _wide_pair(False)
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    want = _oracle_call(A, B, sr, mode="full")
    for swap in (0, 2):
        for name, value in (("split_len", 4), ("window", 64), ("force_kind", 3), ("lds_budget", 8192), ("chunks", 3),
                            ("swap_operands", swap)):
            handle.set_option(name, value)
        assert_distances_close(_call(handle, dA, dB, sr), want, "%s slices, swap_operands %d" % (_sr_name(sr), swap))


@pytest.mark.parametrize("sr", [("plus", "min", False), ("abs_diff", "max", True), ("max", "plus", True)], ids=_name)
def test_config1_sampled_pairs(handle, spd, sr):
    A, B = synth.workload(1)
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    print("semiring config1", _name(sr), flush=True)
    rng = np.random.default_rng(1)
    ra, rb = _sample_rows(A, 64, rng), _sample_rows(B, 2048, rng)
    got = _run(handle, dA, dB, sr)
    want = oracle.semiring_pairwise(A, B, *sr, rows_a=ra, rows_b=rb)
    assert_distances_close(got[np.ix_(ra, rb)], want, _name(sr))


def test_error_statuses(handle, spd, config0):
    A, B, dA, dB = config0
    with pytest.raises(spd.SpdError) as e:
        handle.semiring_pairwise(dA, dB, 17, 0, False)
    assert e.value.status_name == "SPD_ERR_BAD_METRIC"
    with pytest.raises(spd.SpdError) as e:
        handle.semiring_pairwise(dA, dB, 0, 3, False)
    assert e.value.status_name == "SPD_ERR_BAD_METRIC"
    with pytest.raises(spd.SpdError) as e:
        handle.semiring_knn(dA, dB, "plus", "min", False, 65)
    assert e.value.status_name == "SPD_ERR_BAD_K"
    for bad in (dict(product="x_log_x_over_y", sum="plus", over_union=True),             # no value where y is absent
                dict(product="abs_diff", sum="plus", over_union=True, epilogue="cosine"),   # an expansion outside its distance
                dict(product="times", sum="max", over_union=False, epilogue="l2"),
                dict(product="times", sum="plus", over_union=False, transform="sqrt", epilogue="jaccard"),
                dict(product="times", sum="plus", over_union=False, transform=7),
                dict(product="times", sum="plus", over_union=False, epilogue=40)):
        with pytest.raises(spd.SpdError) as e:
            handle.semiring_pairwise(dA, dB, bad["product"], bad["sum"], bad["over_union"],
                                     transform=bad.get("transform", "none"), epilogue=bad.get("epilogue", "none"))
        assert e.value.status_name == "SPD_ERR_BAD_METRIC", bad
    for p in (0.0, -1.0, float("nan"), float("inf")):
        with pytest.raises(spd.SpdError) as e:
            handle.semiring_pairwise(dA, dB, "abs_diff_pow", "plus", True, p=p)
        assert e.value.status_name == "SPD_ERR_BAD_P"
        with pytest.raises(spd.SpdError) as e:
            handle.semiring_knn(dA, dB, "abs_diff", "plus", True, 3, p=p, epilogue="root_p")
        assert e.value.status_name == "SPD_ERR_BAD_P"


@pytest.mark.parametrize("sr", SEMIRINGS, ids=_name)
def test_operands_swapped(handle, spd, signed0, sr):
    """Every product offered is commutative, so spd_semiring_pairwise may stage B and stream A
    like spd_pairwise: forced here, on the signed config 0 and on rows cut into slices."""
    A, B, dA, dB = signed0
    print("semiring swapped", _name(sr), flush=True)
    handle.set_option("swap_operands", 2)
    assert_distances_close(_run(handle, dA, dB, sr), oracle.semiring_pairwise(A, B, *sr), "swapped " + _name(sr))
    A, B = _wide_pair(True)
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    for name, value in (("split_len", 4), ("window", 64), ("force_kind", 3), ("lds_budget", 8192), ("chunks", 3)):
        handle.set_option(name, value)
    want = oracle.semiring_pairwise(A, B, *sr, mode="full")
    assert_distances_close(_run(handle, dA, dB, sr), want, "swapped slices " + _name(sr))
