"""Parity of the HIP path with the CPU oracle, element by element, through the C-ABI
(needs an MI355X; run with -m gpu)."""
import numpy as np
import pytest

import oracle
from gen import synth
from util import (ALL_METRICS, NONNEGATIVE_ONLY, ORACLE_NAME, assert_distances_close, assert_knn_matches,
                  quotient_cases)

pytestmark = pytest.mark.gpu


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


def _run_pairwise(handle, dA, dB, metric, p=2.0):
    import torch
    out = handle.pairwise(dA, dB, metric, p)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def _p_of(metric):
    return 3.0 if metric == "minkowski" else 2.0


# ------------------------------------------------------------------ config 0: every pair
@pytest.mark.parametrize("metric", ALL_METRICS)
def test_config0_every_pair(handle, config0, metric):
    A, B, dA, dB = config0
    print("config0 pairwise", metric, flush=True)
    got = _run_pairwise(handle, dA, dB, metric, _p_of(metric))
    want = oracle.pairwise(A, B, ORACLE_NAME[metric], _p_of(metric), mode="full")
    assert_distances_close(got, want, metric)


@pytest.mark.parametrize("kind", [1, 2, 3, 5])
@pytest.mark.parametrize("max_rows", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("metric", ["cosine", "l1", "chebyshev", "jensen_shannon", "minkowski", "hamming",
                                    "jaccard", "russell_rao"])
def test_config0_every_staging_path(handle, config0, metric, kind, max_rows):
    """Dense strip, column-slot strip, hash and bitmap staging, with 1..16 rows of A per workgroup
    (4..32 for the set metrics, which stage a byte per row)."""
    A, B, dA, dB = config0
    print("config0 staging", metric, kind, max_rows, flush=True)
    handle.set_option("force_kind", kind)
    handle.set_option("max_rows", max_rows)
    got = _run_pairwise(handle, dA, dB, metric, _p_of(metric))
    want = oracle.pairwise(A, B, ORACLE_NAME[metric], _p_of(metric))
    assert_distances_close(got, want, "%s kind=%d R=%d" % (metric, kind, max_rows))


@pytest.mark.parametrize("p", [0.5, 1.0, 1.5, 2.0, 2.5, 3.0, 4.0, 7.0])
def test_minkowski_degrees(handle, spd, config0, p):
    """Every class of degree the kernel specialises (1 runs as the Manhattan distance, 2 to 4 as
    plain products, the rest through exp2/log2), on config 0 and on signed rows with slices."""
    A, B, dA, dB = config0
    print("minkowski p", p, flush=True)
    assert_distances_close(_run_pairwise(handle, dA, dB, "minkowski", p),
                           oracle.pairwise(A, B, "minkowski", p), "minkowski p=%g" % p)
    A, B = _wide_pair(True)
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    for name, value in (("split_len", 4), ("window", 64), ("force_kind", 3), ("lds_budget", 8192)):
        handle.set_option(name, value)
    assert_distances_close(_run_pairwise(handle, dA, dB, "minkowski", p),
                           oracle.pairwise(A, B, "minkowski", p, mode="full"), "minkowski p=%g, slices" % p)


def _wide_pair(signed):
    """Two small matrices over 400 columns whose rows have 0..400 entries."""
    rng = np.random.default_rng(77)
    out = []
    for rows in (37, 75):
        d = np.zeros((rows, 400))
        for r in range(rows):
            n = int(rng.choice([0, 3, 40, 129, 150, 280, 300, 400]))
            cols = rng.choice(400, size=n, replace=False)
            d[r, cols] = rng.standard_normal(n) if signed else rng.random(n) + 0.01
        out.append(synth.from_dense(np.asarray(d.astype(np.float32), dtype=np.float64)))
    return out


@pytest.mark.parametrize("metric", ALL_METRICS)
def test_split_rows_and_sliced_rows(handle, spd, metric):
    """B rows cut over several lanes (split_len 4) and A rows cut into slices whose partial
    results are summed afterwards (an 8 KB LDS budget with hash staging holds 128 entries)."""
    A, B = _wide_pair(metric not in NONNEGATIVE_ONLY)
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    print("split+slices", metric, flush=True)
    plan = spd.testing.host_plan_summary(A["indptr"], B["indptr"], 400, metric, split_len=4, window=64, force_kind=3,
                                 lds_budget=8192, chunks=3)
    assert plan["spilled_rows"] > 0 and plan["split_rows"] > 0
    handle.set_option("split_len", 4)
    handle.set_option("window", 64)
    handle.set_option("force_kind", 3)
    handle.set_option("lds_budget", 8192)
    handle.set_option("chunks", 3)
    got = _run_pairwise(handle, dA, dB, metric, _p_of(metric))
    want = oracle.pairwise(A, B, ORACLE_NAME[metric], _p_of(metric), mode="full")
    assert_distances_close(got, want, metric)


def _long_rows_pair():
    """Rows of up to 900 entries over 1,000 columns: with splitting switched off a slab has
    far more than 255 steps, so the byte counters of the set metrics are folded on the way."""
    rng = np.random.default_rng(78)
    out = []
    for rows in (21, 70):
        d = np.zeros((rows, 1000))
        for r in range(rows):
            n = int(rng.choice([0, 3, 250, 256, 300, 700, 900]))
            cols = rng.choice(1000, size=n, replace=False)
            d[r, cols] = rng.random(n) + 0.01
        out.append(synth.from_dense(np.asarray(d.astype(np.float32), dtype=np.float64)))
    return out


@pytest.mark.parametrize("byte_counters", [1, 0])
@pytest.mark.parametrize("metric", ["jaccard", "dice", "russell_rao"])
def test_set_metrics_both_routes_and_long_slabs(handle, spd, metric, byte_counters):
    """Jaccard, Dice and Russell-Rao through the byte counters and through the dot product of
    0/1 values, on slabs of up to 900 steps, pairwise and fused k-NN."""
    import torch
    A, B = _long_rows_pair()
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    print("set metric", metric, "byte_counters", byte_counters, flush=True)
    handle.set_option("byte_counters", byte_counters)
    handle.set_option("split_len", 1 << 20)
    plan = spd.testing.host_plan_summary(A["indptr"], B["indptr"], 1000, metric, split_len=1 << 20)
    assert plan["split_rows"] == 0 and plan["max_slab_steps"] >= 900
    want = oracle.pairwise(A, B, ORACLE_NAME[metric], mode="full")
    for kind in (2, 3, 5):
        handle.set_option("force_kind", kind)
        assert_distances_close(_run_pairwise(handle, dA, dB, metric), want, "%s kind %d" % (metric, kind))
        idx, dist = handle.knn(dA, dB, metric, 8)
        torch.cuda.synchronize()
        assert_knn_matches(idx.cpu().numpy(), dist.cpu().numpy(), want, 8, metric, "%s kind %d" % (metric, kind))
    # and with rows of B cut over lanes again
    handle.set_option("split_len", 64)
    assert_distances_close(_run_pairwise(handle, dA, dB, metric), want, metric + " split")


def _edge_matrices(signed):
    """Empty rows, single-entry rows, a dense row, duplicates, stored zeros, 130 columns."""
    rng = np.random.default_rng(99)
    k = 130
    d = np.zeros((70, k))
    for r in range(70):
        n = [0, 1, 1, 2, 5, 17, 64, 65, 129, 130][r % 10]
        cols = rng.choice(k, size=n, replace=False)
        vals = rng.standard_normal(n) if signed else rng.random(n) + 0.01
        d[r, cols] = vals
    d[33] = d[4]                       # duplicates
    d[34] = d[9]
    d[35] = d[8] * 1.0
    M = synth.from_dense(np.asarray(d.astype(np.float32), dtype=np.float64))
    # turn one stored value of row 5 into an explicit zero
    s = int(M["indptr"][5])
    M["values"] = M["values"].copy()
    M["values"][s] = 0.0
    return M


@pytest.mark.parametrize("metric", ALL_METRICS)
def test_edge_rows_and_self_join(handle, spd, metric):
    signed = metric not in NONNEGATIVE_ONLY
    M = _edge_matrices(signed)
    dM = spd.DeviceCsr.from_host(M)
    print("edge rows", metric, flush=True)
    got = _run_pairwise(handle, dM, dM, metric, _p_of(metric))          # A and B alias
    want = oracle.pairwise(M, M, ORACLE_NAME[metric], _p_of(metric), mode="full")
    assert_distances_close(got, want, metric)
    if metric not in ("inner_product", "russell_rao", "jaccard_literal"):
        defined = np.abs(np.diag(want)) < 1e-9   # a row without variance has correlation distance 1
        assert defined.sum() >= 55 and np.abs(np.diag(got)[defined]).max() <= 1e-5, "d(x, x) must vanish"
    if metric not in ("kl_divergence", "kl_divergence_strict"):
        np.testing.assert_allclose(got, got.T, rtol=2e-4, atol=2e-5)
    # single rows on either side
    one = synth.slice_rows(M, 6, 7)
    d1 = spd.DeviceCsr.from_host(one)
    assert_distances_close(_run_pairwise(handle, d1, dM, metric, _p_of(metric)), want[6:7], metric + " m=1")
    assert_distances_close(_run_pairwise(handle, dM, d1, metric, _p_of(metric)), want[:, 6:7], metric + " n=1")


def test_all_rows_empty(handle, spd):
    E = synth.from_dense(np.zeros((3, 40)))
    dE = spd.DeviceCsr.from_host(E)
    for metric in ALL_METRICS:
        got = _run_pairwise(handle, dE, dE, metric, 2.0)
        want = oracle.pairwise(E, E, ORACLE_NAME[metric], 2.0, mode="full")
        assert_distances_close(got, want, metric)


def test_results_are_bitwise_reproducible(handle, config0):
    A, B, dA, dB = config0
    for metric in ("l1", "cosine", "jensen_shannon"):
        a = _run_pairwise(handle, dA, dB, metric)
        b = _run_pairwise(handle, dA, dB, metric)
        assert np.array_equal(a, b), metric


def test_row_pointers_from_the_host_or_read_back(handle, spd, config0):
    """The same results, bit for bit, whether the library reads the row pointers back or takes
    the caller's host copies (of either operand, of both, of one matrix on both sides)."""
    A, B, _, _ = config0
    variants = {}
    for ka in (True, False):
        for kb in (True, False):
            dA = spd.DeviceCsr.from_host(A, keep_host_indptr=ka)
            dB = spd.DeviceCsr.from_host(B, keep_host_indptr=kb)
            variants[(ka, kb)] = (_run_pairwise(handle, dA, dB, "l1"), handle.knn(dA, dB, "cosine", 5))
    ref = variants[(False, False)]
    for key, (d, (idx, dist)) in variants.items():
        assert np.array_equal(d, ref[0]), key
        assert np.array_equal(idx.cpu().numpy(), ref[1][0].cpu().numpy()), key
    assert_distances_close(ref[0], oracle.pairwise(A, B, "manhattan"), "l1")
    for keep in (True, False):
        dM = spd.DeviceCsr.from_host(A, keep_host_indptr=keep)
        assert_distances_close(_run_pairwise(handle, dM, dM, "l1"), oracle.pairwise(A, A, "manhattan"), "self-join")
    # a host copy whose end does not match nnz is refused
    bad = spd.DeviceCsr.from_host(A)
    bad.host_indptr = bad.host_indptr.copy()
    bad.host_indptr[-1] += 1
    with pytest.raises(spd.SpdError) as e:
        handle.pairwise(bad, bad, "l1")
    assert e.value.status_name == "SPD_ERR_BAD_CSR"


def test_calls_in_flight_behind_one_another(spd):
    """With host copies of the row pointers a call returns without waiting for the stream: twelve
    calls with different operands, metrics and sizes are enqueued back to back (more than the
    handle has staging buffers) before any result is looked at."""
    import torch
    h = spd.Handle()
    c0a, c0b = synth.workload(0)
    wa, wb = _wide_pair(False)
    edge = _edge_matrices(False)
    c1a, c1b = synth.workload(1, scale=0.05)
    mats = [c0a, c0b, wa, wb, edge, c1a, c1b]
    dev = [spd.DeviceCsr.from_host(m) for m in mats]
    pairs = [(0, 1), (2, 3), (4, 4), (5, 6), (1, 0), (3, 2), (6, 5), (0, 0), (5, 5), (2, 2), (1, 1), (6, 6)]
    jobs = []
    for t, (i, j) in enumerate(pairs):
        metric = ("l1", "cosine", "jensen_shannon", "jaccard")[t % 4]
        if t % 3 == 2:
            jobs.append((i, j, metric, "knn", h.knn(dev[i], dev[j], metric, 3)))
        else:
            jobs.append((i, j, metric, "pairwise", h.pairwise(dev[i], dev[j], metric)))
    torch.cuda.synchronize()
    for i, j, metric, kind, got in jobs:
        want = oracle.pairwise(mats[i], mats[j], ORACLE_NAME[metric])
        if kind == "knn":
            assert_knn_matches(got[0].cpu().numpy(), got[1].cpu().numpy(), want, 3, metric, "queued %s" % metric)
        else:
            assert_distances_close(got.cpu().numpy(), want, "queued %s" % metric)
    h.close()


# ------------------------------------------------------------------ config 1: sampled pairs
def _sample_rows(csr, n, rng):
    deg = np.diff(csr["indptr"])
    order = np.argsort(deg, kind="stable")
    forced = [order[0], order[-1], order[len(order) // 2]]
    rest = rng.choice(csr["n_rows"], size=min(n, csr["n_rows"]) - len(forced), replace=False)
    return np.unique(np.concatenate([forced, rest]))


@pytest.fixture(scope="module")
def config1(spd):
    A, B = synth.workload(1)
    return A, B, spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)


@pytest.mark.parametrize("metric", ["l1", "l2_expanded", "cosine", "chebyshev", "minkowski",
                                    "canberra", "jaccard", "correlation", "hamming"])
def test_config1_sampled_pairs(handle, config1, metric):
    A, B, dA, dB = config1
    print("config1 pairwise", metric, flush=True)
    rng = np.random.default_rng(1)
    ra, rb = _sample_rows(A, 64, rng), _sample_rows(B, 2048, rng)
    got = _run_pairwise(handle, dA, dB, metric, _p_of(metric))
    want = oracle.pairwise(A, B, ORACLE_NAME[metric], _p_of(metric), rows_a=ra, rows_b=rb)
    assert_distances_close(got[np.ix_(ra, rb)], want, metric)


@pytest.mark.parametrize("kind", [1, 3, 5])
def test_config1_other_staging_kinds(handle, config1, kind):
    A, B, dA, dB = config1
    print("config1 kind", kind, flush=True)
    rng = np.random.default_rng(2)
    ra, rb = _sample_rows(A, 64, rng), _sample_rows(B, 1024, rng)
    handle.set_option("force_kind", kind)
    for metric in ("l1", "cosine"):
        got = _run_pairwise(handle, dA, dB, metric)
        want = oracle.pairwise(A, B, ORACLE_NAME[metric], rows_a=ra, rows_b=rb)
        assert_distances_close(got[np.ix_(ra, rb)], want, "%s kind %d" % (metric, kind))


# ------------------------------------------------------------------ k-NN
@pytest.mark.parametrize("metric", ALL_METRICS)
@pytest.mark.parametrize("k", [1, 5, 32, 64])
def test_config0_knn(handle, config0, metric, k):
    import torch
    A, B, dA, dB = config0
    print("config0 knn", metric, k, flush=True)
    idx, dist = handle.knn(dA, dB, metric, k, _p_of(metric))
    torch.cuda.synchronize()
    rows = oracle.pairwise(A, B, ORACLE_NAME[metric], _p_of(metric))
    assert_knn_matches(idx.cpu().numpy(), dist.cpu().numpy(), rows, k, metric, metric)


def test_knn_ties_go_to_the_lower_index(handle, spd):
    import torch
    rng = np.random.default_rng(3)
    base = (rng.random((40, 96)) < 0.1).astype(np.float64)
    dense = np.concatenate([base, base, base])             # every row three times
    I = synth.from_dense(dense)
    Q = synth.from_dense(base)
    dI, dQ = spd.DeviceCsr.from_host(I), spd.DeviceCsr.from_host(Q)
    for metric in ("jaccard", "hamming", "dice", "l1"):
        idx, dist = handle.knn(dQ, dI, metric, 6)
        torch.cuda.synchronize()
        want_idx, want_dist = oracle.knn(Q, I, ORACLE_NAME[metric], 6)
        assert np.array_equal(idx.cpu().numpy(), want_idx), metric
        assert_distances_close(dist.cpu().numpy(), want_dist, metric)


@pytest.mark.parametrize("k", [6, 32, 64])
def test_knn_first_bound_from_the_first_slabs(spd, k):
    """A chunk of eight slabs or more per wavefront: the wavefronts agree on a bound of the k-th key from
    their first slabs before any candidate is queued (option knn_seed).  Every row of the index 250
    times over, so that the bound itself is a distance many rows tie at: same lists with and without
    it, and the oracle's (ties to the lower index)."""
    import torch
    rng = np.random.default_rng(31)
    base = (rng.random((40, 96)) < 0.1) * rng.integers(1, 4, size=(40, 96)).astype(np.float64)
    base[7] = 0.0                                          # an empty row among them
    I = synth.from_dense(np.concatenate([base] * 250))     # 10,000 rows: 157 slabs
    Q = synth.from_dense(base[:24])
    dI, dQ = spd.DeviceCsr.from_host(I), spd.DeviceCsr.from_host(Q)
    for metric in ("l1", "hamming", "chebyshev", "l2_unexpanded", "canberra", "jensen_shannon", "l2_expanded", "hellinger",
                   "cosine", "jaccard"):
        print("knn first bound", metric, k, flush=True)
        results = []
        for seed in (1, 0):
            h = spd.Handle()
            h.set_option("check_plan", 1)
            h.set_option("chunks", 1)
            h.set_option("knn_seed", seed)
            idx, dist = h.knn(dQ, dI, metric, k)
            torch.cuda.synchronize()
            results.append((idx.cpu().numpy(), dist.cpu().numpy()))
            h.close()
        assert np.array_equal(results[0][0], results[1][0]), metric
        assert np.array_equal(results[0][1], results[1][1], equal_nan=True), metric
        want_idx, want_dist = oracle.knn(Q, I, ORACLE_NAME[metric], k)
        if metric in ("jaccard", "l1", "chebyshev", "hamming"):       # (exact in fp32 on these small integers: ties are ties)
            assert np.array_equal(results[0][0], want_idx), metric
        else:
            rows = oracle.pairwise(Q, I, ORACLE_NAME[metric])
            assert_knn_matches(results[0][0], results[0][1], rows, k, metric, metric)
        assert_distances_close(results[0][1], want_dist, metric)


def test_knn_first_bound_with_sliced_rows(spd):
    """The same exchange while some staged rows are slices of a row that does not fit the table whole (their
    partial sums go to memory and take no part in it) and rows of the index are split over lanes."""
    import torch
    rng = np.random.default_rng(32)
    base = (rng.random((40, 400)) < 0.05) * rng.integers(1, 4, size=(40, 400)).astype(np.float64)
    I = synth.from_dense(np.concatenate([base] * 250))
    queries = base[:12].copy()
    queries[3] = rng.integers(1, 4, size=400)              # a full row: cut into slices
    queries[8, ::2] = 2.0                                  # and a half-full one
    Q = synth.from_dense(queries)
    dI, dQ = spd.DeviceCsr.from_host(I), spd.DeviceCsr.from_host(Q)
    options = dict(split_len=4, force_kind=3, lds_budget=12288, chunks=1)
    for metric in ("l1", "l2_expanded", "hamming"):
        print("knn first bound, slices", metric, flush=True)
        plan = spd.testing.host_plan_summary(Q["indptr"], I["indptr"], 400, metric, k_neighbors=32, **options)
        assert plan["spilled_rows"] >= 1 and plan["split_rows"] > 0 and plan["slabs"] >= 128
        results = []
        for seed in (1, 0):
            h = spd.Handle()
            h.set_option("check_plan", 1)
            for name, value in options.items():
                h.set_option(name, value)
            h.set_option("knn_seed", seed)
            idx, dist = h.knn(dQ, dI, metric, 32)
            torch.cuda.synchronize()
            results.append((idx.cpu().numpy(), dist.cpu().numpy()))
            h.close()
        assert np.array_equal(results[0][0], results[1][0]), metric
        assert np.array_equal(results[0][1], results[1][1]), metric
        rows = oracle.pairwise(Q, I, ORACLE_NAME[metric])
        assert_knn_matches(results[0][0], results[0][1], rows, 32, metric, metric)


def test_knn_with_sliced_rows_and_split_rows(handle, spd):
    import torch
    A, B = _wide_pair(False)
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    handle.set_option("split_len", 4)
    handle.set_option("force_kind", 3)
    handle.set_option("lds_budget", 12288)       # (a kilobyte per staged row goes to the k-NN lists)
    for metric in ("l1", "cosine", "inner_product", "jensen_shannon", "minkowski", "chebyshev", "jaccard"):
        print("knn slices", metric, flush=True)
        plan = spd.testing.host_plan_summary(A["indptr"], B["indptr"], 400, metric, k_neighbors=16, split_len=4, force_kind=3,
                                     lds_budget=12288)
        assert plan["spilled_rows"] > 0 and plan["split_rows"] > 0
        idx, dist = handle.knn(dA, dB, metric, 16, _p_of(metric))
        torch.cuda.synchronize()
        rows = oracle.pairwise(A, B, ORACLE_NAME[metric], _p_of(metric))
        assert_knn_matches(idx.cpu().numpy(), dist.cpu().numpy(), rows, 16, metric, metric)


def test_config1_knn(handle, config1):
    import torch
    A, B, dA, dB = config1
    rng = np.random.default_rng(4)
    rq = _sample_rows(A, 24, rng)
    for metric in ("cosine", "l1"):
        print("config1 knn", metric, flush=True)
        idx, dist = handle.knn(dA, dB, metric, 32)
        torch.cuda.synchronize()
        rows = oracle.pairwise(A, B, ORACLE_NAME[metric], rows_a=rq)
        assert_knn_matches(idx.cpu().numpy()[rq], dist.cpu().numpy()[rq], rows, 32, metric, metric)


def test_config1_self_join_knn(handle, config1):
    """The paper's benchmark protocol (Section 4.2): the queries are the indexed rows themselves,
    so every row's nearest neighbour is itself, at distance 0 (not excluded)."""
    import torch
    A, _, dA, _ = config1
    rng = np.random.default_rng(5)
    rq = _sample_rows(A, 16, rng)
    for metric in ("l1", "l2_unexpanded", "jaccard"):
        print("config1 self-join knn", metric, flush=True)
        idx, dist = handle.knn(dA, dA, metric, 8)
        torch.cuda.synchronize()
        idx, dist = idx.cpu().numpy(), dist.cpu().numpy()
        rows = oracle.pairwise(A, A, ORACLE_NAME[metric], rows_a=rq)
        assert_knn_matches(idx[rq], dist[rq], rows, 8, metric, "self-join " + metric)
        assert np.all(dist[:, 0] <= 1e-5), metric
        if metric != "jaccard":                   # rows with the same support tie at Jaccard distance 0
            assert np.array_equal(idx[:, 0], np.arange(A["n_rows"])), metric


def test_knn_in_a_caller_workspace_of_the_documented_size(spd, config1):
    """spd_workspace_bytes bounds what a k-NN call carves (candidate lists of every chunk included), whatever
    the planner's options make of the chunks: the call runs inside exactly that many bytes and returns what it
    returns with the handle's own scratch."""
    import torch
    A, B, dA, dB = config1
    for options in ({}, {"chunk_scale": 4}, {"chunks": 7}, {"split_len": 16, "window": 64}, {"max_rows": 2}):
        for metric, k in (("cosine", 32), ("jaccard", 64), ("l1", 5)):
            print("knn workspace", options, metric, k, flush=True)
            own = spd.Handle()
            lent = spd.Handle()
            for h in (own, lent):
                h.set_option("check_plan", 1)
                for name, value in options.items():
                    h.set_option(name, value)
            need = lent.workspace_bytes(dA, dB, metric, k)
            lent.set_workspace(torch.empty(need, dtype=torch.uint8, device="cuda"))
            want_idx, want_dist = own.knn(dA, dB, metric, k)
            idx, dist = lent.knn(dA, dB, metric, k)
            torch.cuda.synchronize()
            assert torch.equal(idx, want_idx) and torch.equal(dist, want_dist), (options, metric, k)
            own.close(); lent.close()


# ------------------------------------------------------------------ the boundary's error paths
def test_error_statuses(handle, spd, config0):
    import torch
    A, B, dA, dB = config0
    other = spd.DeviceCsr.from_host(synth.from_dense(np.eye(4)))
    with pytest.raises(spd.SpdError) as e:
        handle.pairwise(dA, other, "l1", out=torch.empty((256, 4), dtype=torch.float32, device="cuda"))
    assert e.value.status_name == "SPD_ERR_DIM_MISMATCH"
    with pytest.raises(spd.SpdError) as e:
        handle.pairwise(dA, dB, "minkowski", p=0.0)
    assert e.value.status_name == "SPD_ERR_BAD_P"
    with pytest.raises(spd.SpdError) as e:
        handle.pairwise(dA, dB, "minkowski", p=float("nan"))
    assert e.value.status_name == "SPD_ERR_BAD_P"
    with pytest.raises(spd.SpdError) as e:
        handle.pairwise(dA, dB, 99)
    assert e.value.status_name == "SPD_ERR_BAD_METRIC"
    for k in (0, 65, 257):
        with pytest.raises(spd.SpdError) as e:
            handle.knn(dA, dB, "l1", k)
        assert e.value.status_name == "SPD_ERR_BAD_K"
    with pytest.raises(spd.SpdError) as e:
        handle.set_option("no_such_option", 1)
    assert e.value.status_name == "SPD_ERR_UNSUPPORTED"
    for name, value in (("window", 63), ("window", 1 << 25), ("chunk_scale", 9), ("chunk_scale", -1), ("knn_seed", 2),
                        ("swap_operands", 3), ("cuckoo_attempts", 4), ("chunks", 4097), ("force_kind", 6), ("side_streams", 4)):
        with pytest.raises(spd.SpdError) as e:
            handle.set_option(name, value)
        assert e.value.status_name == "SPD_ERR_UNSUPPORTED", (name, value)
    # a caller workspace that is too small is reported, a large enough one is used
    need = handle.workspace_bytes(dA, dB, "l1")
    handle.set_workspace(torch.empty(256, dtype=torch.uint8, device="cuda"))
    with pytest.raises(spd.SpdError) as e:
        handle.pairwise(dA, dB, "l1")
    assert e.value.status_name == "SPD_ERR_WORKSPACE"
    handle.set_workspace(torch.empty(need, dtype=torch.uint8, device="cuda"))
    got = handle.pairwise(dA, dB, "l1")
    torch.cuda.synchronize()
    assert_distances_close(got.cpu().numpy(), oracle.pairwise(A, B, "manhattan"), "caller workspace")
    handle.set_workspace(None)


def test_csr_validate(handle, spd, config0):
    import torch
    A, B, dA, dB = config0
    handle.csr_validate(dA)
    handle.csr_validate(dA, require_nonnegative=True)
    bad = spd.DeviceCsr(dA.n_rows, dA.n_cols, dA.indptr.clone(), dA.indices.clone(), dA.values.clone())
    bad.indices[1] = bad.indices[0]                          # columns no longer ascend strictly
    with pytest.raises(spd.SpdError) as e:
        handle.csr_validate(bad)
    assert e.value.status_name == "SPD_ERR_BAD_CSR"
    bad = spd.DeviceCsr(dA.n_rows, dA.n_cols, dA.indptr.clone(), dA.indices.clone(), dA.values.clone())
    bad.values[7] = float("inf")
    with pytest.raises(spd.SpdError):
        handle.csr_validate(bad)
    bad = spd.DeviceCsr(dA.n_rows, dA.n_cols, dA.indptr.clone(), dA.indices.clone(), -dA.values)
    handle.csr_validate(bad)
    with pytest.raises(spd.SpdError):
        handle.csr_validate(bad, require_nonnegative=True)
    bad = spd.DeviceCsr(dA.n_rows, dA.n_cols, dA.indptr.clone(), dA.indices.clone(), dA.values.clone())
    bad.indptr[5] = bad.indptr[4] - 1
    with pytest.raises(spd.SpdError):
        handle.csr_validate(bad)
    torch.cuda.synchronize()


@pytest.mark.parametrize("kind", [1, 3])
@pytest.mark.parametrize("metric", ["jensen_shannon", "kl_divergence", "kl_divergence_strict", "canberra"])
def test_device_quotients_on_crafted_pairs(handle, spd, metric, kind):
    """The kernels' quotients (reciprocal, estimate, residual, correction) and logarithms on the
    pairs that stress them: equal entries, one entry twice the other, ratios of 1e8 and 1e12
    either way, entries near both ends of the fp32 range.  Every row of the first set meets
    every row of the second."""
    cases = quotient_cases()
    A = synth.from_dense(np.stack([a for a, _ in cases]))
    B = synth.from_dense(np.stack([b for _, b in cases]))
    print("device quotients", metric, kind, flush=True)
    handle.set_option("force_kind", kind)
    got = _run_pairwise(handle, spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B), metric)
    want = oracle.pairwise(A, B, ORACLE_NAME[metric], mode="full")
    if metric == "kl_divergence":
        # (the library documents a quotient of two entries beyond the fp32 range as undefined)
        ratio = np.array([[a[3] / b[3] for _, b in cases] for a, _ in cases])
        ok = (ratio > 1e-36) & (ratio < 1e36)
        got, want = np.where(ok, got, 0.0), np.where(ok, want, 0.0)
    assert_distances_close(got, want, metric)
    # the same rows against themselves: equal entries everywhere give exactly 0
    self_d = _run_pairwise(handle, spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(A), metric)
    assert np.all(np.diag(self_d) == 0.0)


# ------------------------------------------------------------------ operands with their roles exchanged
SWAPPABLE = tuple(m for m in ALL_METRICS if not m.startswith("kl_divergence"))


@pytest.mark.parametrize("metric", SWAPPABLE)
def test_operands_swapped_config0_and_edge_rows(handle, spd, config0, metric):
    """spd_pairwise with B staged (groups of consecutive rows) and A streamed, which the library
    does by itself only for large operands with short rows: forced here, on config 0 through every
    staging kind and group size, and on the matrix of edge rows against itself and single rows."""
    A, B, dA, dB = config0
    print("swapped config0", metric, flush=True)
    p = _p_of(metric)
    handle.set_option("swap_operands", 2)
    want = oracle.pairwise(A, B, ORACLE_NAME[metric], p)
    for kind, max_rows in ((1, 8), (2, 8), (3, 8), (5, 8), (2, 1), (3, 4), (5, 2), (2, 16)):
        handle.set_option("force_kind", kind)
        handle.set_option("max_rows", max_rows)
        assert_distances_close(_run_pairwise(handle, dA, dB, metric, p), want, "%s kind=%d R=%d" % (metric, kind, max_rows))
    handle.set_option("force_kind", 0)
    handle.set_option("max_rows", 8)
    M = _edge_matrices(metric not in NONNEGATIVE_ONLY)
    dM = spd.DeviceCsr.from_host(M)
    want = oracle.pairwise(M, M, ORACLE_NAME[metric], p, mode="full")
    assert_distances_close(_run_pairwise(handle, dM, dM, metric, p), want, metric + " edge rows")
    d1 = spd.DeviceCsr.from_host(synth.slice_rows(M, 6, 7))
    assert_distances_close(_run_pairwise(handle, d1, dM, metric, p), want[6:7], metric + " m=1")
    assert_distances_close(_run_pairwise(handle, dM, d1, metric, p), want[:, 6:7], metric + " n=1")


@pytest.mark.parametrize("metric", SWAPPABLE)
def test_operands_swapped_split_rows_and_sliced_rows(handle, spd, metric):
    """The same with the streamed rows (now A's) cut over lanes and the staged rows (now B's) cut
    into slices: a sliced row leaves an empty place in its group of consecutive rows."""
    A, B = _wide_pair(metric not in NONNEGATIVE_ONLY)
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    print("swapped split+slices", metric, flush=True)
    plan = spd.testing.host_plan_summary(B["indptr"], A["indptr"], 400, metric, split_len=4, window=64, force_kind=3,
                                 lds_budget=8192, chunks=3, consecutive_groups=1)
    assert plan["spilled_rows"] > 0 and plan["split_rows"] > 0
    for name, value in (("split_len", 4), ("window", 64), ("force_kind", 3), ("lds_budget", 8192), ("chunks", 3),
                        ("swap_operands", 2)):
        handle.set_option(name, value)
    got = _run_pairwise(handle, dA, dB, metric, _p_of(metric))
    want = oracle.pairwise(A, B, ORACLE_NAME[metric], _p_of(metric), mode="full")
    assert_distances_close(got, want, metric)


def test_config1_both_orientations(handle, config1):
    """Config 1 is large enough, and its rows short enough, for the library to exchange the
    operands' roles by itself: the same sampled pairs with the exchange switched off, left to
    the library, and forced."""
    A, B, dA, dB = config1
    rng = np.random.default_rng(3)
    ra, rb = _sample_rows(A, 64, rng), _sample_rows(B, 2048, rng)
    for metric in ("cosine", "l1", "jaccard", "jensen_shannon"):
        want = oracle.pairwise(A, B, ORACLE_NAME[metric], rows_a=ra, rows_b=rb)
        for mode in (0, 1, 2):
            print("config1 orientation", metric, mode, flush=True)
            handle.set_option("swap_operands", mode)
            got = _run_pairwise(handle, dA, dB, metric)
            assert_distances_close(got[np.ix_(ra, rb)], want, "%s swap_operands=%d" % (metric, mode))
            assert np.all(np.isfinite(got))


# ------------------------------------------------------------------ branches that ordinary inputs do not reach
@pytest.mark.parametrize("attempts", [0, 1, 3])
def test_hash_staging_falls_back_to_linear_probing(handle, spd, attempts):
    """A half-full hash table is filled by cuckoo hashing with up to three pairs of hash functions
    and, should all fail, by linear probing with as many probes as the fullest run needs.  No input
    has made them fail: the option limits the attempts (0: linear probing at once)."""
    A, B = _wide_pair(True)
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    options = dict(split_len=4, window=64, force_kind=3, lds_budget=8192)
    plan = spd.testing.host_plan_summary(A["indptr"], B["indptr"], 400, "l1", **options)
    assert any(c["hscale"] == 1 for c in plan["classes"])          # tables as full as they get
    for name, value in options.items():
        handle.set_option(name, value)
    handle.set_option("cuckoo_attempts", attempts)
    for metric in ("l1", "cosine", "chebyshev", "jaccard", "hamming"):
        print("hash fall-back", attempts, metric, flush=True)
        got = _run_pairwise(handle, dA, dB, metric)
        assert_distances_close(got, oracle.pairwise(A, B, ORACLE_NAME[metric], mode="full"), "%s attempts=%d" % (metric, attempts))
    idx, dist = handle.knn(dA, dB, "l1", 9)
    import torch
    torch.cuda.synchronize()
    assert_knn_matches(idx.cpu().numpy(), dist.cpu().numpy(), oracle.pairwise(A, B, "manhattan"), 9, "l1", "fall-back knn")


def _threshold(lo, hi, pred):
    """Largest v in [lo, hi] with pred(v), pred being true up to some point and false after it."""
    assert pred(lo) and not pred(hi)
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if pred(mid):
            lo = mid
        else:
            hi = mid
    return lo


def _rows_of_lengths(lengths, k, rng):
    d = np.zeros((len(lengths), k))
    for r, n in enumerate(lengths):
        d[r, rng.choice(k, size=n, replace=False)] = rng.random(n) + 0.05
    return synth.from_dense(np.asarray(d.astype(np.float32), dtype=np.float64))


def test_rows_and_column_counts_at_the_planner_thresholds(handle, spd):
    """One below, at and one above each point where the planner changes its mind: the column
    count where the dense strip gives way to the column-slot strip, that to the bitmap and that
    to the hash table; the row length from which a row is cut into slices; the row length from
    which a row of B is split over lanes.  The thresholds are read off the planner itself."""
    rng = np.random.default_rng(314)
    ip = np.array([0, 3, 5], dtype=np.int64)
    kind_at = lambda k: spd.testing.host_plan_summary(ip, ip, k, "l1")["classes"][0]["kind"]
    k_strip = _threshold(16, 1 << 22, lambda k: kind_at(k) == 1)
    k_slot = _threshold(k_strip + 1, 1 << 22, lambda k: kind_at(k) == 2)
    k_bitmap = _threshold(k_slot + 1, 1 << 22, lambda k: kind_at(k) == 5)
    assert kind_at(k_bitmap + 1) == 3
    for k_edge in (k_strip, k_slot, k_bitmap):
        for k in (k_edge - 1, k_edge, k_edge + 1):
            A = _rows_of_lengths([0, 1, 7, 40, 300], k, rng)
            B = _rows_of_lengths([2, 0, 9, 64, 65, 257], k, rng)
            # the last column is stored too: the map has to reach it
            for M in (A, B):
                M["indices"] = M["indices"].copy()
                last = int(M["indptr"][-1]) - 1
                M["indices"][last] = k - 1
            print("threshold k", k, "kind", kind_at(k), flush=True)
            dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
            handle.csr_validate(dA)
            handle.csr_validate(dB)
            for metric in ("l1", "cosine", "chebyshev", "jaccard"):
                assert_distances_close(_run_pairwise(handle, dA, dB, metric), oracle.pairwise(A, B, ORACLE_NAME[metric]),
                                       "%s at k=%d" % (metric, k))
    # the longest row that is staged whole (hash staging under a 16 KB budget), and one more entry
    opts = dict(force_kind=3, lds_budget=16384)
    one = lambda n: np.array([0, n], dtype=np.int64)
    spilled = lambda n: spd.testing.host_plan_summary(one(n), ip, 4000, "l1", **opts)["spilled_rows"]
    d_whole = _threshold(1, 3999, lambda n: spilled(n) == 0)
    # the shortest row of B that is split over lanes
    split = lambda n: spd.testing.host_plan_summary(ip, one(n), 4000, "l1", **opts)["split_rows"]
    b_unsplit = _threshold(1, 3999, lambda n: split(n) == 0)
    A = _rows_of_lengths([d_whole - 1, d_whole, d_whole + 1, 2 * d_whole, 2 * d_whole + 1, 3], 4000, rng)
    B = _rows_of_lengths([b_unsplit - 1, b_unsplit, b_unsplit + 1, b_unsplit + 2, 1, 0], 4000, rng)
    plan = spd.testing.host_plan_summary(A["indptr"], B["indptr"], 4000, "l1", **opts)
    assert plan["spilled_rows"] == 3 and plan["split_rows"] == 2, plan
    for name, value in opts.items():
        handle.set_option(name, value)
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    for metric in ("l1", "cosine", "chebyshev", "jaccard", "minkowski", "jensen_shannon"):
        print("threshold rows", metric, d_whole, b_unsplit, flush=True)
        assert_distances_close(_run_pairwise(handle, dA, dB, metric, 3.0), oracle.pairwise(A, B, ORACLE_NAME[metric], 3.0),
                               "%s at the row thresholds" % metric)
    idx, dist = handle.knn(dA, dB, "l1", 4)
    import torch
    torch.cuda.synchronize()
    assert_knn_matches(idx.cpu().numpy(), dist.cpu().numpy(), oracle.pairwise(A, B, "manhattan"), 4, "l1", "threshold knn")


def test_set_metrics_beyond_2_to_23_columns_and_2_to_24_entries(handle, spd):
    """Jaccard and Dice take an exact fp32 quotient of their integer counts while those are
    exact in fp32, and an fp64 one beyond: more than 2^22 / 2^23 columns, and two rows whose
    union holds more than 2^24 entries (9 million each, a million shared; the staged one is cut
    into some nine hundred slices)."""
    import torch
    rng = np.random.default_rng(2718)
    for k in ((1 << 22) + 1, (1 << 23) + 1):
        A = _rows_of_lengths([0, 5, 60], 2000, rng)
        B = _rows_of_lengths([3, 0, 61, 400], 2000, rng)
        for M in (A, B):                     # spread the columns over all k, the last one included
            M["n_cols"] = k
            M["indices"] = (M["indices"].astype(np.int64) * ((k - 1) // 1999)).astype(np.int32)
        dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
        handle.csr_validate(dA)
        handle.csr_validate(dB)
        for metric in ("jaccard", "dice", "russell_rao", "hamming", "cosine", "correlation"):
            print("wide k", k, metric, flush=True)
            want = oracle.pairwise(A, B, ORACLE_NAME[metric], threads=2)
            assert_distances_close(_run_pairwise(handle, dA, dB, metric), want, "%s at k=%d" % (metric, k))
    k = 17_000_001
    x = np.arange(0, 9_000_000, dtype=np.int32)
    y = np.arange(8_000_000, 17_000_000, dtype=np.int32)
    small = np.array([5, 8_500_000, 16_999_999], dtype=np.int32)

    def csr(rows):
        ip = np.zeros(len(rows) + 1, dtype=np.int64)
        np.cumsum([r.size for r in rows], out=ip[1:])
        cols = np.concatenate(rows)
        return {"n_rows": len(rows), "n_cols": k, "indptr": ip, "indices": cols, "values": np.ones(cols.size, dtype=np.float32)}

    A, B = csr([x, small]), csr([y, small, x])
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    for metric in ("jaccard", "dice"):
        print("2^24 entries", metric, flush=True)
        got = _run_pairwise(handle, dA, dB, metric)
        want = oracle.pairwise(A, B, ORACLE_NAME[metric], threads=1)
        assert_distances_close(got, want, metric + " beyond 2^24 entries")
        exact = {"jaccard": 1.0 - 1_000_000 / 17_000_000, "dice": 1.0 - 2_000_000 / 18_000_000}[metric]
        assert abs(got[0, 0] - exact) <= 1e-6 and got[0, 2] == 0.0
    idx, dist = handle.knn(dA, dB, "jaccard", 2)
    torch.cuda.synchronize()
    assert idx.cpu().numpy().tolist() == [[2, 0], [1, 0]]
