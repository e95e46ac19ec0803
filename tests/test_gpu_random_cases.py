"""Seeded random cases: shapes, degree mixes, values, metrics (and semirings), planner options and
k drawn at random, each compared with the CPU oracle through the C-ABI (needs an MI355X).  The
other parity files pick their cases on purpose; this one looks for interactions nobody thought of."""
import numpy as np
import pytest

import oracle
from gen import synth
from util import ALL_METRICS, NONNEGATIVE_ONLY, ORACLE_NAME, assert_distances_close, assert_knn_matches

pytestmark = pytest.mark.gpu

N_CASES = 200


@pytest.fixture(scope="module")
def spd():
    import paper_2104_06357_amd as lib
    return lib


def _matrix(rng, rows, k, signed, binary):
    """Rows whose lengths mix empty, single, short, long and full; a few duplicated rows; a
    few stored zeros; columns uniform or crowded into a popular head."""
    lens_menu = [0, 1, 2, rng.integers(3, 20), rng.integers(20, max(21, k // 4)), rng.integers(k // 4, k // 2 + 2), k]
    weights = np.array([1, 2, 3, 8, 5, 2, 0.5])
    weights /= weights.sum()
    popular = rng.random() < 0.5
    col_p = None
    if popular:
        w = 1.0 / np.arange(1, k + 1) ** 0.9
        col_p = w[rng.permutation(k)] / w.sum()
    indptr, indices, values = [0], [], []
    for r in range(rows):
        n = int(min(k, lens_menu[rng.choice(len(lens_menu), p=weights)]))
        cols = np.sort(rng.choice(k, size=n, replace=False, p=col_p))
        if binary:
            v = np.ones(n)
        elif signed:
            v = rng.standard_normal(n)
        else:
            v = rng.random(n) + 0.01
        if n and rng.random() < 0.1:
            v[rng.integers(n)] = 0.0                      # a stored zero
        indices.append(cols); values.append(v); indptr.append(indptr[-1] + n)
    M = {"n_rows": rows, "n_cols": k, "indptr": np.asarray(indptr, dtype=np.int64),
         "indices": np.concatenate(indices).astype(np.int32) if indices else np.zeros(0, np.int32),
         "values": np.concatenate(values).astype(np.float32) if values else np.zeros(0, np.float32)}
    return M


def _case(seed):
    rng = np.random.default_rng(1000 + seed)
    semiring = rng.random() < 0.25
    if semiring:
        what = (oracle.PRODUCTS[rng.integers(len(oracle.PRODUCTS))], oracle.SUMS[rng.integers(len(oracle.SUMS))],
                bool(rng.integers(2)))
        signed = True
    else:
        what = ALL_METRICS[rng.integers(len(ALL_METRICS))]
        signed = what not in NONNEGATIVE_ONLY and rng.random() < 0.7
    k = int(rng.choice([7, 64, 65, 300, 1000, 3000]))
    m, n = int(rng.integers(1, 120)), int(rng.integers(1, 400))
    long_index = rng.random() < 0.12
    if long_index:
        # an index of many slabs (a chunk then has eight or more per wavefront), few query rows
        k = int(rng.choice([64, 300]))
        m, n = int(rng.integers(1, 24)), int(rng.integers(8200, 11000))
    binary = (not semiring) and rng.random() < 0.15
    A = _matrix(rng, m, k, signed, binary)
    B = A if (rng.random() < 0.15) else _matrix(rng, n, k, signed, binary)
    options = {}
    if rng.random() < 0.7:
        options["force_kind"] = int(rng.choice([1, 2, 3, 4, 5]))
    if rng.random() < 0.2:
        options["bloom_long_rows"] = 1
    if rng.random() < 0.6:
        options["max_rows"] = int(rng.choice([1, 2, 4, 8, 16]))
    if rng.random() < 0.6:
        options["split_len"] = int(rng.choice([2, 4, 16, 64, 256]))
    if rng.random() < 0.5:
        options["window"] = int(rng.choice([64, 128, 1024]))
    if rng.random() < 0.5:
        options["chunks"] = int(rng.choice([1, 2, 3, 7]))
    if rng.random() < 0.4 and options.get("force_kind") != 1:
        options["lds_budget"] = int(rng.choice([8192, 16384, 40000]))
    if rng.random() < 0.3:
        options["waves_per_cu"] = int(rng.choice([8, 16, 32]))
    if rng.random() < 0.2:
        options["byte_counters"] = 0
    if rng.random() < 0.2:
        options["side_streams"] = int(rng.choice([0, 1, 3]))
    if rng.random() < 0.2:
        options["sort_slack"] = 0
    if rng.random() < 0.3:
        options["partial_groups"] = int(rng.choice([0, 2]))
    if rng.random() < 0.4:
        options["swap_operands"] = int(rng.choice([0, 2]))       # never / wherever the distance allows it
    if rng.random() < 0.2:
        options["knn_seed"] = 0
    if rng.random() < 0.15:
        options["cuckoo_attempts"] = int(rng.choice([0, 1]))
    if long_index:
        options.pop("lds_budget", None)
        if options.get("force_kind") == 1:
            options.pop("force_kind")
        options["chunks"] = int(rng.choice([1, 2]))
    knn_k = int(rng.choice([1, 3, 17, 64]))
    p = float(rng.choice([0.5, 1.0, 2.0, 3.0, 3.5]))
    via_index = (not semiring) and rng.random() < 0.3
    return semiring, what, p, A, B, options, knn_k, via_index


@pytest.mark.parametrize("seed", range(N_CASES))
def test_random_case(spd, seed):
    semiring, what, p, A, B, options, knn_k, via_index = _case(seed)
    print("random case", seed, what, p, A["n_rows"], B["n_rows"], A["n_cols"], options, knn_k, via_index, flush=True)
    dA = spd.DeviceCsr.from_host(A)
    dB = dA if B is A else spd.DeviceCsr.from_host(B)
    h = spd.Handle()
    h.set_option("check_plan", 1)
    try:
        for name, value in options.items():
            h.set_option(name, value)
        import torch
        tag = "case %d %s %s" % (seed, what, options)
        try:
            if semiring:
                want = oracle.semiring_pairwise(A, B, *what, mode="full")
                got = h.semiring_pairwise(dA, dB, *what)
            else:
                want = oracle.pairwise(A, B, ORACLE_NAME[what], p, mode="full")
                index = h.index_create(dB, what, p) if via_index else None
                got = index.pairwise(dA) if via_index else h.pairwise(dA, dB, what, p)
        except spd.SpdError as e:
            # the refusals a random draw may meet: a forced staging kind that the LDS budget cannot
            # hold, a Bloom filter asked to serve a maximum
            forced = options.get("force_kind")
            ranked = what == "chebyshev" or (semiring and what[1] != "plus")
            assert e.status_name == "SPD_ERR_UNSUPPORTED" and forced is not None and \
                (forced == 1 or "lds_budget" in options or (forced == 4 and ranked)), (tag, str(e))
            print("refused:", e, flush=True)
            return
        torch.cuda.synchronize()
        assert_distances_close(got.cpu().numpy(), want, tag)
        kk = min(knn_k, B["n_rows"])
        try:
            if semiring:
                idx, dist = h.semiring_knn(dA, dB, *what, kk)
            else:
                idx, dist = index.knn(dA, kk) if via_index else h.knn(dA, dB, what, kk, p)
        except spd.SpdError as e:
            # the k-NN lists take a kilobyte of LDS per staged row: a tight budget may not hold them
            assert e.status_name == "SPD_ERR_UNSUPPORTED" and "lds_budget" in options, (tag, str(e))
            print("k-NN refused:", e, flush=True)
            return
        torch.cuda.synchronize()
        assert_knn_matches(idx.cpu().numpy(), dist.cpu().numpy(), want, kk, "semiring" if semiring else what, tag)
    finally:
        h.close()
