"""Parity at the full sizes of BASELINE configs 2-4 and of two more shapes (the ultra-short rows
of an n-gram matrix, the extreme skew of a ratings matrix); needs an MI355X, run with -m gpu.

The library runs a whole query tile against the whole index, exactly as a user would call
it; the oracle then recomputes a seeded sample of the outputs one by one (always including
the rows of smallest, median and largest degree), or, for k-NN, the full distance rows of
a sample of queries.
"""
import time

import numpy as np
import pytest

import oracle
from gen import synth
from util import ORACLE_NAME, assert_distances_close, assert_knn_matches, progress

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def spd():
    import paper_2104_06357_amd as lib
    return lib


def _extremes_and_sample(csr, n, rng, extra=()):
    deg = np.diff(csr["indptr"])
    order = np.argsort(deg, kind="stable")
    forced = [order[0], order[-1], order[len(order) // 2], *extra]
    rest = rng.choice(csr["n_rows"], size=max(0, n - len(forced)), replace=False)
    return np.unique(np.concatenate([np.asarray(forced, dtype=np.int64), rest]))


def _gather(out, rows, cols):
    import torch
    r = torch.as_tensor(rows, device=out.device)
    c = torch.as_tensor(cols, device=out.device)
    return out.index_select(0, r).index_select(1, c).cpu().numpy()


def _timed(capsys, label, fn):
    import torch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    out = fn()
    torch.cuda.synchronize()
    progress(capsys, "%s: %.1f ms" % (label, 1e3 * (time.perf_counter() - t0)))
    return out


def test_config2_bag_of_words_tile(spd, capsys):
    """1,024 queries (one output tile of 1.2 GB) against the 300,000-row index."""
    import torch
    Q, I = synth.workload(2)
    progress(capsys, "config2 generated")
    rng = np.random.default_rng(2)
    tile_rows = _extremes_and_sample(Q, 1024, rng)
    tile = synth.take_rows(Q, tile_rows)
    dQ, dI = spd.DeviceCsr.from_host(tile), spd.DeviceCsr.from_host(I)
    h = spd.Handle()
    h.set_option("check_plan", 1)
    out = torch.empty((tile["n_rows"], I["n_rows"]), dtype=torch.float32, device="cuda")
    ra = _extremes_and_sample(tile, 64, rng)
    rb = _extremes_and_sample(I, 2048, rng)
    for metric in ("cosine", "inner_product", "hellinger"):
        _timed(capsys, "config2 " + metric, lambda: h.pairwise(dQ, dI, metric, out=out))
        want = oracle.pairwise(tile, I, ORACLE_NAME[metric], rows_a=ra, rows_b=rb)
        assert_distances_close(_gather(out, ra, rb), want, "config2 " + metric)
        progress(capsys, "config2 %s checked against the oracle" % metric)
    # rows are L2-normalised: cosine distance = 1 - inner product (a property at any size)
    cos = h.pairwise(dQ, dI, "cosine", out=out).index_select(0, torch.as_tensor(ra, device="cuda")).clone()
    ip = h.pairwise(dQ, dI, "inner_product", out=out).index_select(0, torch.as_tensor(ra, device="cuda"))
    assert float((cos + ip - 1.0).abs().max()) < 2e-6
    # correlation (means over all 102,660 columns) on the same tile
    _timed(capsys, "config2 correlation", lambda: h.pairwise(dQ, dI, "correlation", out=out))
    want = oracle.pairwise(tile, I, "correlation", rows_a=ra, rows_b=rb)
    assert_distances_close(_gather(out, ra, rb), want, "config2 correlation")
    del out
    # the fused top-32 of the same tile: full distance rows of a sample of the queries
    rq = _extremes_and_sample(tile, 12, rng)
    idx, dist = _timed(capsys, "config2 knn cosine", lambda: h.knn(dQ, dI, "cosine", 32))
    rows = oracle.pairwise(tile, I, "cosine", rows_a=rq)
    assert_knn_matches(idx.cpu().numpy()[rq], dist.cpu().numpy()[rq], rows, 32, "cosine", "config2 knn cosine")
    progress(capsys, "config2 knn cosine checked against the oracle")
    h.close()


def test_config3_count_matrix_tile(spd, capsys):
    """A 4,096-row query tile of the 65,536-row self-join, union-family metrics."""
    import torch
    M, _ = synth.workload(3)
    progress(capsys, "config3 generated")
    deg = np.diff(M["indptr"])
    heavy = np.nonzero(deg > 10_240)[0]
    assert heavy.size >= 8
    rng = np.random.default_rng(3)
    tile_rows = _extremes_and_sample(M, 4096, rng, extra=heavy[:8])
    tile = synth.take_rows(M, tile_rows)
    dQ, dM = spd.DeviceCsr.from_host(tile), spd.DeviceCsr.from_host(M)
    h = spd.Handle()
    h.set_option("check_plan", 1)
    out = torch.empty((tile["n_rows"], M["n_rows"]), dtype=torch.float32, device="cuda")
    heavy_in_tile = np.nonzero(np.isin(tile_rows, heavy))[0]
    ra = _extremes_and_sample(tile, 64, rng, extra=heavy_in_tile)
    # index sample: extremes, the heavy rows, and the tile's own rows (the self-join diagonal)
    rb = _extremes_and_sample(M, 2048, rng, extra=list(heavy) + list(tile_rows[ra]))
    for metric in ("kl_divergence", "jensen_shannon", "canberra", "l1"):
        _timed(capsys, "config3 " + metric, lambda: h.pairwise(dQ, dM, metric, out=out))
        want = oracle.pairwise(tile, M, ORACLE_NAME[metric], rows_a=ra, rows_b=rb)
        assert_distances_close(_gather(out, ra, rb), want, "config3 " + metric)
        progress(capsys, "config3 %s checked against the oracle" % metric)
    # the protocol of Section 4.2 on the same tile (its rows are rows of the index): fused top-32
    rq = _extremes_and_sample(tile, 8, rng, extra=heavy_in_tile[:2])
    for metric in ("l1", "jensen_shannon"):
        idx, dist = _timed(capsys, "config3 knn " + metric, lambda: h.knn(dQ, dM, metric, 32))
        idx, dist = idx.cpu().numpy(), dist.cpu().numpy()
        rows = oracle.pairwise(tile, M, ORACLE_NAME[metric], rows_a=rq)
        assert_knn_matches(idx[rq], dist[rq], rows, 32, metric, "config3 knn " + metric)
        assert np.all(dist[:, 0] <= 1e-5), metric           # every query finds itself (or a copy) first
        progress(capsys, "config3 knn %s checked against the oracle" % metric)
    # the same rows through hash staging: the >10,240-entry rows are cut into slices
    h.set_option("force_kind", 3)
    plan = spd.testing.host_plan_summary(tile["indptr"], M["indptr"], M["n_cols"], "l1", force_kind=3)
    assert plan["spilled_rows"] >= 8
    _timed(capsys, "config3 l1 (hash staging)", lambda: h.pairwise(dQ, dM, "l1", out=out))
    want = oracle.pairwise(tile, M, "manhattan", rows_a=ra, rows_b=rb)
    assert_distances_close(_gather(out, ra, rb), want, "config3 l1 with slices")
    h.close()


def test_config4_binary_knn(spd, capsys):
    """4,096 binary queries against 500,000 index rows over 2^20 columns, fused top-32."""
    import torch
    Q, I = synth.workload(4)
    progress(capsys, "config4 generated")
    dQ, dI = spd.DeviceCsr.from_host(Q), spd.DeviceCsr.from_host(I)
    h = spd.Handle()
    h.set_option("check_plan", 1)
    rng = np.random.default_rng(4)
    rq = _extremes_and_sample(Q, 24, rng)
    plan = spd.testing.host_plan_summary(Q["indptr"], I["indptr"], Q["n_cols"], "jaccard", k_neighbors=32)
    progress(capsys, "config4 plan: spilled rows %d, slabs %d" % (plan["spilled_rows"], plan["slabs"]))
    for metric in ("jaccard", "dice", "hamming"):
        idx, dist = _timed(capsys, "config4 knn " + metric, lambda: h.knn(dQ, dI, metric, 32))
        # (the oracle takes 3 s per query row here: 24 rows for Jaccard, the extremes and 5 more for the others)
        rows_checked = rq if metric == "jaccard" else rq[:: 3]
        rows = oracle.pairwise(Q, I, ORACLE_NAME[metric], rows_a=rows_checked)
        assert_knn_matches(idx.cpu().numpy()[rows_checked], dist.cpu().numpy()[rows_checked], rows, 32, metric,
                           "config4 " + metric)
        progress(capsys, "config4 %s checked against the oracle" % metric)
    h.close()


def _knn_tile_against_oracle(spd, capsys, label, M, tile_rows, metrics, k, n_checked, options=()):
    """Self-join protocol: a tile of the matrix's own rows queries the whole matrix."""
    tile = synth.take_rows(M, tile_rows)
    dQ, dM = spd.DeviceCsr.from_host(tile), spd.DeviceCsr.from_host(M)
    h = spd.Handle()
    h.set_option("check_plan", 1)
    for name, value in options:
        h.set_option(name, value)
    rng = np.random.default_rng(len(tile_rows))
    rq = _extremes_and_sample(tile, n_checked, rng)
    for metric in metrics:
        idx, dist = _timed(capsys, "%s knn %s" % (label, metric), lambda: h.knn(dQ, dM, metric, k))
        idx, dist = idx.cpu().numpy(), dist.cpu().numpy()
        rows = oracle.pairwise(tile, M, ORACLE_NAME[metric], rows_a=rq)
        assert_knn_matches(idx[rq], dist[rq], rows, k, metric, "%s %s" % (label, metric))
        progress(capsys, "%s %s checked against the oracle" % (label, metric))
        # every query is in the index: it, or a row at the same distance, comes first
        assert np.all(dist[:, 0] <= 1e-5), metric
    h.close()
    return tile, dQ, dM


def test_shape5_ngram_like(spd, capsys):
    """663,000 x 858,000 with 2.2 entries per row on average (99.5 % of the rows under 10, none
    above 51): 4,096 of its rows against all of it, fused top-32, and a pairwise tile."""
    import torch
    M, _ = synth.workload(5)
    progress(capsys, "shape 5 generated: %d entries" % int(M["indptr"][-1]))
    rng = np.random.default_rng(5)
    tile_rows = _extremes_and_sample(M, 4096, rng)
    tile, dQ, dM = _knn_tile_against_oracle(spd, capsys, "shape5", M, tile_rows, ("cosine", "jaccard"), 32, 8)
    h = spd.Handle()
    small = synth.slice_rows(tile, 0, 256)
    dS = spd.DeviceCsr.from_host(small)
    out = torch.empty((256, M["n_rows"]), dtype=torch.float32, device="cuda")
    ra = _extremes_and_sample(small, 16, rng)
    rb = _extremes_and_sample(M, 4096, rng, extra=list(tile_rows[:256][ra]))
    for metric in ("l1", "hamming"):
        _timed(capsys, "shape5 pairwise " + metric, lambda: h.pairwise(dS, dM, metric, out=out))
        want = oracle.pairwise(small, M, ORACLE_NAME[metric], rows_a=ra, rows_b=rb)
        assert_distances_close(_gather(out, ra, rb), want, "shape5 " + metric)
    h.close()


def test_shape6_ratings_like(spd, capsys):
    """283,000 x 194,000 with power-law degrees up to 24,000 (46 M entries): 1,024 of its rows,
    the 24,000-entry one among them, against all of it, fused top-32."""
    M, _ = synth.workload(6)
    progress(capsys, "shape 6 generated: %d entries" % int(M["indptr"][-1]))
    rng = np.random.default_rng(6)
    tile_rows = _extremes_and_sample(M, 1024, rng)
    tile_ip = synth.take_rows(M, tile_rows)["indptr"]
    plan = spd.testing.host_plan_summary(tile_ip, M["indptr"], M["n_cols"], "cosine", k_neighbors=32)
    progress(capsys, "shape6 plan: spilled rows %d, slabs %d" % (plan["spilled_rows"], plan["slabs"]))
    # 194,000 columns: the bitmap of the columns leaves room for the 24,000-entry row as a whole
    assert all(c["kind"] == 5 for c in plan["classes"]) and plan["spilled_rows"] == 0
    _knn_tile_against_oracle(spd, capsys, "shape6", M, tile_rows, ("cosine", "l1"), 32, 8)
    # behind a hash table that row is cut into slices
    hashed = spd.testing.host_plan_summary(tile_ip, M["indptr"], M["n_cols"], "l1", k_neighbors=32, force_kind=3)
    assert hashed["spilled_rows"] >= 1
    _knn_tile_against_oracle(spd, capsys, "shape6 (hash staging)", M, tile_rows, ("l1",), 32, 8, options=(("force_kind", 3),))


def test_output_of_more_than_2_to_32_distances(spd, capsys):
    """70,000 x 70,000 rows of the config-1 kind: 4.9e9 distances (19.6 GB), so every product
    of a row number and a row length in the kernels' addressing has to be formed in 64 bits."""
    import torch
    A, B = synth.workload(1, scale=7.0)
    assert A["n_rows"] == 70_000 and B["n_rows"] == 70_000
    progress(capsys, "70,000-row pair generated")
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    h = spd.Handle()
    out = torch.empty((A["n_rows"], B["n_rows"]), dtype=torch.float32, device="cuda")
    rng = np.random.default_rng(7)
    ra = _extremes_and_sample(A, 48, rng, extra=(0, A["n_rows"] - 1, 61_357, 65_536))
    rb = _extremes_and_sample(B, 1024, rng, extra=(0, B["n_rows"] - 1, 61_356, 65_535))
    for metric in ("cosine", "l1"):
        out.fill_(float("nan"))
        _timed(capsys, "70,000 x 70,000 %s" % metric, lambda: h.pairwise(dA, dB, metric, out=out))
        want = oracle.pairwise(A, B, ORACLE_NAME[metric], rows_a=ra, rows_b=rb)
        assert_distances_close(_gather(out, ra, rb), want, metric)
        # nothing was left unwritten, nothing was written past the end
        assert not bool(torch.isnan(out[-1]).any()) and not bool(torch.isnan(out[::4099, ::13]).any())
    h.close()
    del out
