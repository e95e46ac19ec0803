"""The synthetic generators: valid CSR, seeded, shaped as the recipe says (no GPU needed)."""
import numpy as np
import pytest

from gen import synth


def _check_csr(m):
    ip, ix, v = m["indptr"], m["indices"], m["values"]
    assert ip.dtype == np.int64 and ix.dtype == np.int32 and v.dtype == np.float32
    assert ip[0] == 0 and ip[-1] == ix.size == v.size and np.all(np.diff(ip) >= 0)
    assert ix.min() >= 0 and ix.max() < m["n_cols"]
    step = np.diff(ix.astype(np.int64))
    inner = np.ones(ix.size - 1, dtype=bool)
    ends = ip[1:-1] - 1
    inner[ends[(ends >= 0) & (ends < inner.size)]] = False
    assert np.all(step[inner] > 0), "columns must ascend strictly inside a row"
    assert np.all(v != 0.0) and np.all(np.isfinite(v))


@pytest.mark.parametrize("config,scale", [(0, 1.0), (1, 0.2), (2, 0.01), (3, 0.004), (4, 0.01)])
def test_workloads_are_valid_and_seeded(config, scale):
    A, B = synth.workload(config, scale)
    _check_csr(A); _check_csr(B)
    assert A["n_cols"] == B["n_cols"]
    A2, B2 = synth.workload(config, scale)
    for k in ("indptr", "indices", "values"):
        assert np.array_equal(A[k], A2[k]) and np.array_equal(B[k], B2[k])
    assert np.diff(A["indptr"]).min() >= 1 and np.diff(B["indptr"]).min() >= 1


def test_shapes_follow_the_recipe():
    A, B = synth.workload(0)
    assert (A["n_rows"], A["n_cols"]) == (256, 512) and 0.0 < A["values"].min() and A["values"].max() <= 1.0
    A, _ = synth.workload(1, 0.3)
    deg = np.diff(A["indptr"])
    assert deg.min() >= 1 and deg.max() <= 2000 and np.median(deg) == 4
    Q, I = synth.workload(2, 0.01)
    for M in (Q, I):
        sq = np.bincount(synth._row_ids(M["indptr"]), weights=M["values"].astype(np.float64) ** 2)
        np.testing.assert_allclose(sq, 1.0, atol=1e-5)
    C, _ = synth.workload(3, 0.004)
    deg = np.diff(C["indptr"])
    assert deg.min() >= 500 and deg.max() <= 12_000 and (deg > 10_240).sum() >= 8
    s = np.bincount(synth._row_ids(C["indptr"]), weights=C["values"].astype(np.float64))
    np.testing.assert_allclose(s, 1.0, atol=1e-5)
    Q, I = synth.workload(4, 0.01)
    assert I["n_cols"] == 1 << 20 and np.all(I["values"] == 1.0)


def test_row_helpers():
    A, _ = synth.workload(0)
    D = synth.to_dense(A)
    assert np.array_equal(synth.to_dense(synth.slice_rows(A, 10, 40)), D[10:40])
    assert np.array_equal(synth.to_dense(synth.take_rows(A, [7, 7, 0, 255])), D[[7, 7, 0, 255]])
    assert np.array_equal(synth.to_dense(synth.from_dense(D)), D)
