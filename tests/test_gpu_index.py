"""The prepared index (spd_index_create / spd_index_pairwise / spd_index_knn): the same results as
spd_pairwise / spd_knn, bit for bit, and parity with the CPU oracle (needs an MI355X)."""
import numpy as np
import pytest

import oracle
from gen import synth
from test_gpu_parity import _edge_matrices, _p_of, _sample_rows, _wide_pair
from util import ALL_METRICS, NONNEGATIVE_ONLY, ORACLE_NAME, assert_distances_close, assert_knn_matches

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


def _np(t):
    import torch
    torch.cuda.synchronize()
    return t.cpu().numpy()


@pytest.mark.parametrize("metric", ALL_METRICS)
def test_config0_same_as_the_plain_calls(handle, config0, metric):
    A, B, dA, dB = config0
    print("index config0", metric, flush=True)
    p = _p_of(metric)
    ix = handle.index_create(dB, metric, p)
    got = _np(ix.pairwise(dA))
    assert np.array_equal(got, _np(handle.pairwise(dA, dB, metric, p)), equal_nan=True)
    assert_distances_close(got, oracle.pairwise(A, B, ORACLE_NAME[metric], p), metric)
    for k in (1, 32):
        idx, dist = ix.knn(dA, k)
        ridx, rdist = handle.knn(dA, dB, metric, k, p)
        assert np.array_equal(_np(idx), _np(ridx)) and np.array_equal(_np(dist), _np(rdist))
    # the index serves any number of calls, with other query matrices too
    again = _np(ix.pairwise(dB))
    assert np.array_equal(again, _np(handle.pairwise(dB, dB, metric, p)), equal_nan=True)
    ix.close()


@pytest.mark.parametrize("metric", ["cosine", "l1", "chebyshev", "minkowski", "jaccard", "jensen_shannon"])
def test_split_rows_sliced_rows_and_every_staging_kind(handle, spd, metric):
    A, B = _wide_pair(metric not in NONNEGATIVE_ONLY)
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    print("index split+slices", metric, flush=True)
    p = _p_of(metric)
    handle.set_option("split_len", 4)
    handle.set_option("window", 64)
    ix = handle.index_create(dB, metric, p)            # the index keeps this cut of B's rows
    want = oracle.pairwise(A, B, ORACLE_NAME[metric], p, mode="full")
    for kind, budget in ((1, 163840), (2, 163840), (3, 163840), (5, 163840), (3, 12288)):
        handle.set_option("force_kind", kind)
        handle.set_option("lds_budget", budget)
        assert_distances_close(_np(ix.pairwise(dA)), want, "%s kind %d budget %d" % (metric, kind, budget))
        idx, dist = ix.knn(dA, 7)
        assert_knn_matches(_np(idx), _np(dist), want, 7, metric, "%s kind %d" % (metric, kind))
    ix.close()


def test_edge_rows_minkowski_degree_one_and_empty_operands(handle, spd):
    M = _edge_matrices(True)
    dM = spd.DeviceCsr.from_host(M)
    for metric, p in (("minkowski", 1.0), ("minkowski", 2.5), ("inner_product", 2.0), ("hamming", 2.0)):
        ix = handle.index_create(dM, metric, p)
        want = oracle.pairwise(M, M, ORACLE_NAME[metric], p, mode="full")
        assert_distances_close(_np(ix.pairwise(dM)), want, "%s p=%g" % (metric, p))
        idx, dist = ix.knn(dM, 5)
        assert_knn_matches(_np(idx), _np(dist), want, 5, metric, metric)
        ix.close()
    E = spd.DeviceCsr.from_host(synth.from_dense(np.zeros((0, 130))))
    ix = handle.index_create(E, "cosine")
    assert tuple(ix.pairwise(dM).shape) == (70, 0)
    ix.close()
    ix = handle.index_create(dM, "cosine")
    assert tuple(ix.pairwise(E).shape) == (0, 70)
    ix.close()


def test_config1_batches_against_one_index(handle, spd):
    """The protocol of Section 4.2: the index once, the queries batch by batch."""
    A, B = synth.workload(1)
    dB = spd.DeviceCsr.from_host(B)
    ix = handle.index_create(dB, "cosine")
    rng = np.random.default_rng(9)
    for r0, r1 in ((0, 2048), (2048, 2500), (9000, 10000)):
        Q = synth.slice_rows(A, r0, r1)
        dQ = spd.DeviceCsr.from_host(Q)
        idx, dist = ix.knn(dQ, 32)
        ridx, rdist = handle.knn(dQ, dB, "cosine", 32)
        assert np.array_equal(_np(idx), _np(ridx)) and np.array_equal(_np(dist), _np(rdist))
        rows = _sample_rows(Q, 24, rng)
        want = oracle.pairwise(Q, B, "cosine", rows_a=rows)
        assert_knn_matches(_np(idx)[rows], _np(dist)[rows], want, 32, "cosine", "batch %d" % r0)
    ix.close()


def test_error_statuses(handle, spd, config0):
    A, B, dA, dB = config0
    with pytest.raises(spd.SpdError) as e:
        handle.index_create(dB, 99)
    assert e.value.status_name == "SPD_ERR_BAD_METRIC"
    with pytest.raises(spd.SpdError) as e:
        handle.index_create(dB, "minkowski", 0.0)
    assert e.value.status_name == "SPD_ERR_BAD_P"
    ix = handle.index_create(dB, "l1")
    with pytest.raises(spd.SpdError) as e:
        ix.knn(dA, 257)
    assert e.value.status_name == "SPD_ERR_BAD_K"
    other = spd.DeviceCsr.from_host(synth.from_dense(np.ones((3, 7))))
    with pytest.raises(spd.SpdError) as e:
        ix.pairwise(other)
    assert e.value.status_name == "SPD_ERR_DIM_MISMATCH"
    ix.close()
    ix.close()                                            # closing twice is harmless
