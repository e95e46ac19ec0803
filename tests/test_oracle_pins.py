"""Pins of the CPU oracle to things other than itself: the values the paper prints, scipy's
library routines on tiny dense inputs, closed forms and invariants (no GPU needed)."""
import os

import numpy as np
import pytest
import scipy.spatial.distance as ssd
from scipy.special import rel_entr

import oracle
from gen import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out.setdefault(key, []).append([float(v) for v in vals])
    return out


def _random_sparse_dense(rng, rows, cols, density, signed=True, zero_rows=True):
    d = rng.standard_normal((rows, cols)) if signed else rng.random((rows, cols)) + 0.05
    d *= rng.random((rows, cols)) < density
    if zero_rows:
        d[rows // 2] = 0.0
    return np.asarray(d.astype(np.float32), dtype=np.float64)


def _both(A, B, metric, p=2.0):
    """Oracle result in both modes; they must agree."""
    full = oracle.pairwise(A, B, metric, p, mode="full")
    sup = oracle.pairwise(A, B, metric, p, mode="support")
    np.testing.assert_allclose(sup, full, rtol=1e-12, atol=1e-13)
    return full


def _scipy_pairs(X, Y, fn):
    return np.array([[fn(x, y) for y in Y] for x in X])


# ---------------------------------------------------------------- values the paper prints
def test_paper_manhattan_worked_example():
    g = _golden("appendix_manhattan_example.txt")
    a, b = synth.from_dense([g["a"][0]]), synth.from_dense([g["b"][0]])
    assert _both(a, b, "manhattan")[0, 0] == g["manhattan"][0][0] == 3.0
    # the annihilating product of the same appendix: only the intersection contributes
    assert _both(a, b, "inner_product")[0, 0] == g["annihilating_sum"][0][0] == 0.0


def test_paper_namm_truth_table():
    rows = _golden("appendix_namm_truth_table.txt")
    for key, vals in rows.items():
        x, (y, want) = float(key), vals[0]
        got = _both(synth.from_dense([[x, 5.0]]), synth.from_dense([[y, 5.0]]), "manhattan")[0, 0]
        assert got == want


def test_paper_spmv_example_union_vs_intersection():
    g = _golden("appendix_spmv_example.txt")
    A, b = synth.from_dense([g["A"][0]]), synth.from_dense([g["b"][0]])
    assert _both(A, b, "manhattan")[0, 0] == g["manhattan_from_truth_table"][0][0] == 2.0
    # Russell-Rao counts the intersection: exactly one shared column out of k = 3
    inter = 3.0 * (1.0 - _both(A, b, "russell_rao")[0, 0])
    assert round(inter) == len(g["intersection_columns"][0]) == 1
    # Jaccard's denominator is the union: 1 - 1/3
    assert _both(A, b, "jaccard")[0, 0] == pytest.approx(1.0 - 1.0 / len(g["union_columns"][0]))


# ---------------------------------------------------------------- scipy on tiny dense inputs
SIGNED = [
    ("manhattan", ssd.cityblock, {}),
    ("euclidean", ssd.euclidean, {}),
    ("chebyshev", ssd.chebyshev, {}),
    ("canberra", ssd.canberra, {}),
    ("hamming", ssd.hamming, {}),
]


@pytest.mark.parametrize("metric,fn,kw", SIGNED)
def test_scipy_signed(metric, fn, kw):
    rng = np.random.default_rng(11)
    X = _random_sparse_dense(rng, 9, 37, 0.3)
    Y = _random_sparse_dense(rng, 7, 37, 0.3)
    Y[1] = X[2]                       # an identical pair
    Y[2, :5] = X[3, :5]               # equal values on some shared columns (Hamming)
    got = _both(synth.from_dense(X), synth.from_dense(Y), metric)
    np.testing.assert_allclose(got, _scipy_pairs(X, Y, fn), rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("p", [0.5, 1.0, 1.5, 2.0, 3.0, 4.5])
def test_scipy_minkowski(p):
    rng = np.random.default_rng(12)
    X = _random_sparse_dense(rng, 6, 29, 0.35)
    Y = _random_sparse_dense(rng, 8, 29, 0.35)
    got = _both(synth.from_dense(X), synth.from_dense(Y), "minkowski", p)
    want = _scipy_pairs(X, Y, lambda x, y: ssd.minkowski(x, y, p))
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-14)


def test_scipy_cosine_and_zero_rows():
    rng = np.random.default_rng(13)
    X = _random_sparse_dense(rng, 8, 31, 0.3)
    Y = _random_sparse_dense(rng, 6, 31, 0.3)
    got = _both(synth.from_dense(X), synth.from_dense(Y), "cosine")
    nzx, nzy = np.abs(X).sum(1) > 0, np.abs(Y).sum(1) > 0
    want = _scipy_pairs(X[nzx], Y[nzy], ssd.cosine)
    np.testing.assert_allclose(got[np.ix_(nzx, nzy)], want, rtol=1e-12, atol=1e-14)
    # a zero row: similarity 0 with a non-zero row, distance 0 to another zero row
    assert np.all(got[~nzx][:, nzy] == 1.0) and np.all(got[nzx][:, ~nzy] == 1.0)
    assert np.all(got[~nzx][:, ~nzy] == 0.0)
    assert got.min() >= 0.0 and got.max() <= 2.0


def test_scipy_correlation_and_its_invariance():
    rng = np.random.default_rng(14)
    X = _random_sparse_dense(rng, 7, 23, 0.4, zero_rows=False)
    Y = _random_sparse_dense(rng, 5, 23, 0.4, zero_rows=False)
    got = _both(synth.from_dense(X), synth.from_dense(Y), "correlation")
    np.testing.assert_allclose(got, _scipy_pairs(X, Y, ssd.correlation), rtol=1e-11, atol=1e-13)
    # unchanged under x -> alpha x + beta (alpha > 0): the means run over all k columns
    X2 = np.asarray((2.5 * X + 0.75).astype(np.float32), dtype=np.float64)
    got2 = _both(synth.from_dense(X2), synth.from_dense(Y), "correlation")
    np.testing.assert_allclose(got2, got, rtol=0, atol=5e-6)
    # equals the cosine distance of the mean-centred rows
    Xc, Yc = X - X.mean(1, keepdims=True), Y - Y.mean(1, keepdims=True)
    np.testing.assert_allclose(got, _scipy_pairs(Xc, Yc, ssd.cosine), rtol=1e-10, atol=1e-12)
    # a row without variance (all zero) has no correlation: distance 1
    Z = synth.from_dense(np.zeros((1, 23)))
    assert np.all(_both(Z, synth.from_dense(Y), "correlation") == 1.0)


def test_scipy_inner_product_is_matmul():
    rng = np.random.default_rng(15)
    X = _random_sparse_dense(rng, 9, 41, 0.3)
    Y = _random_sparse_dense(rng, 11, 41, 0.3)
    got = _both(synth.from_dense(X), synth.from_dense(Y), "inner_product")
    np.testing.assert_allclose(got, X @ Y.T, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("binary", [True, False])
def test_scipy_set_metrics(binary):
    rng = np.random.default_rng(16)
    X = _random_sparse_dense(rng, 8, 33, 0.35, zero_rows=False)
    Y = _random_sparse_dense(rng, 9, 33, 0.35, zero_rows=False)
    if binary:
        X, Y = (X != 0).astype(np.float64), (Y != 0).astype(np.float64)
    bx, by = X != 0, Y != 0
    A, B = synth.from_dense(X), synth.from_dense(Y)
    jac = _both(A, B, "jaccard")
    dice = _both(A, B, "dice")
    rr = _both(A, B, "russell_rao")
    np.testing.assert_allclose(jac, _scipy_pairs(bx, by, ssd.jaccard), rtol=1e-12)
    np.testing.assert_allclose(dice, _scipy_pairs(bx, by, ssd.dice), rtol=1e-12)
    np.testing.assert_allclose(rr, _scipy_pairs(bx, by, ssd.russellrao), rtol=1e-12)
    np.testing.assert_allclose(dice, jac / (2.0 - jac), rtol=1e-12)
    assert jac.min() >= 0.0 and jac.max() <= 1.0


def test_set_metrics_empty_rows_and_explicit_zeros():
    E = synth.from_dense(np.zeros((2, 6)))
    F = synth.from_dense([[0, 1, 0, 2, 0, 0]])
    for m in ("jaccard", "dice"):
        assert np.all(_both(E, E, m) == 0.0)
        assert np.all(_both(E, F, m) == 1.0)
    # a stored zero is not part of the support
    G = dict(F)
    G["indptr"] = np.array([0, 3], dtype=np.int64)
    G["indices"] = np.array([1, 3, 5], dtype=np.int32)
    G["values"] = np.array([1.0, 2.0, 0.0], dtype=np.float32)
    for m in ("jaccard", "dice", "hamming", "canberra", "manhattan"):
        assert _both(G, F, m)[0, 0] == 0.0


def test_hellinger_through_library_euclidean_and_bhattacharyya():
    rng = np.random.default_rng(17)
    X = _random_sparse_dense(rng, 7, 27, 0.4, signed=False)
    Y = _random_sparse_dense(rng, 6, 27, 0.4, signed=False)
    got = _both(synth.from_dense(X), synth.from_dense(Y), "hellinger")
    want = _scipy_pairs(np.sqrt(X), np.sqrt(Y), ssd.euclidean) / np.sqrt(2.0)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)
    # on probability vectors d^2 = 1 - sum sqrt(x y), and d lies in [0, 1]
    P = X.copy(); P[3, 0] = 1.0; P /= P.sum(1, keepdims=True)
    Q = Y.copy(); Q[3, 1] = 1.0; Q /= Q.sum(1, keepdims=True)
    P = np.asarray(P.astype(np.float32), dtype=np.float64)
    Q = np.asarray(Q.astype(np.float32), dtype=np.float64)
    d = _both(synth.from_dense(P), synth.from_dense(Q), "hellinger")
    bc = np.sqrt(P) @ np.sqrt(Q).T
    np.testing.assert_allclose(d * d, 0.5 * (P.sum(1)[:, None] + Q.sum(1)[None, :]) - bc, atol=1e-12)
    assert d.min() >= 0.0 and d.max() <= 1.0 + 1e-6


def test_scipy_jensen_shannon():
    rng = np.random.default_rng(18)
    X = _random_sparse_dense(rng, 7, 25, 0.4, signed=False, zero_rows=False)
    Y = _random_sparse_dense(rng, 6, 25, 0.4, signed=False, zero_rows=False)
    X[:, 0] += 0.1; Y[:, 1] += 0.1
    X /= X.sum(1, keepdims=True); Y /= Y.sum(1, keepdims=True)
    X = np.asarray(X.astype(np.float32), dtype=np.float64)
    Y = np.asarray(Y.astype(np.float32), dtype=np.float64)
    got = _both(synth.from_dense(X), synth.from_dense(Y), "jensen_shannon")
    # scipy renormalises its inputs: the float32 rounding of the sums is ~1e-7
    want = _scipy_pairs(X, Y, lambda x, y: ssd.jensenshannon(x, y))
    np.testing.assert_allclose(got, want, rtol=0, atol=2e-7)
    assert got.max() <= np.sqrt(np.log(2.0)) + 1e-6
    # disjoint supports, each summing to 1: sqrt(ln 2)
    a = synth.from_dense([[0.25, 0.75, 0, 0]]); b = synth.from_dense([[0, 0, 0.5, 0.5]])
    assert _both(a, b, "jensen_shannon")[0, 0] == pytest.approx(0.8325546111576977, abs=1e-15)


def test_kl_against_rel_entr():
    rng = np.random.default_rng(19)
    X = _random_sparse_dense(rng, 6, 21, 0.5, signed=False, zero_rows=False)
    Y = _random_sparse_dense(rng, 5, 21, 0.5, signed=False, zero_rows=False)
    got = _both(synth.from_dense(X), synth.from_dense(Y), "kl_divergence")
    want = np.array([[rel_entr(x, y)[(x > 0) & (y > 0)].sum() for y in Y] for x in X])
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)
    # support of x inside support of y and both sum to 1: the textbook divergence, >= 0
    Yf = Y + 0.01; Yf /= Yf.sum(1, keepdims=True)
    Xn = X / X.sum(1, keepdims=True)
    Xn = np.asarray(Xn.astype(np.float32), dtype=np.float64)
    Yf = np.asarray(Yf.astype(np.float32), dtype=np.float64)
    d = _both(synth.from_dense(Xn), synth.from_dense(Yf), "kl_divergence")
    np.testing.assert_allclose(d, _scipy_pairs(Xn, Yf, lambda x, y: rel_entr(x, y).sum()), atol=1e-13)
    assert d.min() > -1e-6
    # not symmetric
    dT = _both(synth.from_dense(Yf), synth.from_dense(Xn), "kl_divergence")
    assert np.abs(d - dT.T).max() > 1e-3


def test_strict_kl_is_the_textbook_divergence():
    """The strict variant is scipy's rel_entr sum (infinite where x has mass and y has none);
    where supp(x) lies inside supp(y) it is the paper-mode value, elsewhere +inf."""
    rng = np.random.default_rng(23)
    X = _random_sparse_dense(rng, 7, 19, 0.4, signed=False, zero_rows=True)
    Y = _random_sparse_dense(rng, 6, 19, 0.7, signed=False, zero_rows=True)
    Y[0] = X[1]                                   # same support: finite
    Y[1] = X[2] + 0.25                            # full support: finite
    Y = np.asarray(Y.astype(np.float32), dtype=np.float64)
    got = _both(synth.from_dense(X), synth.from_dense(Y), "kl_divergence_strict")
    want = _scipy_pairs(X, Y, lambda x, y: rel_entr(x, y).sum())
    assert np.array_equal(np.isinf(got), np.isinf(want)) and np.isinf(got).any() and np.isfinite(got).any()
    fin = np.isfinite(want)
    np.testing.assert_allclose(got[fin], want[fin], rtol=1e-12, atol=1e-14)
    paper = _both(synth.from_dense(X), synth.from_dense(Y), "kl_divergence")
    inside = np.array([[not np.any((x > 0) & ~(y > 0)) for y in Y] for x in X])
    assert np.array_equal(inside, fin)
    np.testing.assert_allclose(got[inside], paper[inside], rtol=0, atol=0)
    assert got[3].tolist() == [0.0] * 6           # the empty row is at divergence 0 from everything
    same = _both(synth.from_dense(X), synth.from_dense(X), "kl_divergence_strict")
    assert np.all(np.diag(same) == 0.0)


def test_literal_jaccard_reading():
    """Expansion column of Table 1 taken literally: 1 - <x,y>/(|x|_0 + |y|_0 - <x,y>).  On 0/1
    data it is the set reading (scipy's boolean jaccard); on other values a hand-computed case."""
    rng = np.random.default_rng(29)
    Xb = (rng.random((8, 23)) < 0.3).astype(np.float64); Xb[4] = 0.0
    Yb = (rng.random((5, 23)) < 0.4).astype(np.float64); Yb[0] = 0.0
    lit = _both(synth.from_dense(Xb), synth.from_dense(Yb), "jaccard_literal")
    sets = _both(synth.from_dense(Xb), synth.from_dense(Yb), "jaccard")
    np.testing.assert_allclose(lit, sets, rtol=0, atol=1e-15)
    for i, x in enumerate(Xb):
        for j, y in enumerate(Yb):
            if x.any() or y.any():
                assert lit[i, j] == pytest.approx(ssd.jaccard(x.astype(bool), y.astype(bool)), abs=1e-15)
            else:
                assert lit[i, j] == 0.0
    x = np.array([[0.5, 0.5, 0.0, 2.0]]); y = np.array([[0.5, 0.0, 3.0, 1.0]])
    # <x,y> = 0.25 + 2 = 2.25; |x|_0 = 3, |y|_0 = 3: 1 - 2.25 / (6 - 2.25) = 0.4
    assert _both(synth.from_dense(x), synth.from_dense(y), "jaccard_literal")[0, 0] == pytest.approx(0.4, abs=1e-15)
    # not a metric on general values: d(x, x) = 1 - 5.25/(6 - 5.25) is negative here
    assert _both(synth.from_dense(x), synth.from_dense(x), "jaccard_literal")[0, 0] == pytest.approx(1 - 4.5 / 1.5, abs=1e-14)


# ---------------------------------------------------------------- closed forms and invariants
def test_self_distance_symmetry_triangle():
    A, _ = synth.workload(0)
    for m in ("manhattan", "euclidean", "chebyshev", "minkowski", "canberra", "hamming", "hellinger",
              "jensen_shannon", "cosine", "jaccard", "dice", "kl_divergence", "correlation"):
        d = oracle.pairwise(A, A, m, 3.0, rows_a=np.arange(48), rows_b=np.arange(48))
        assert np.abs(np.diag(d)).max() < 1e-7, m
        if m != "kl_divergence":
            np.testing.assert_allclose(d, d.T, rtol=1e-12, atol=1e-14, err_msg=m)
        if m in ("manhattan", "euclidean", "chebyshev", "minkowski", "canberra", "hamming",
                 "hellinger", "jensen_shannon", "jaccard"):
            viol = d[:, None, :] - (d[:, :, None] + d[None, :, :])   # d(a,c) - d(a,b) - d(b,c)
            assert viol.max() < 1e-9, m


def test_minkowski_family_closed_forms():
    A, B = synth.workload(0)
    ra, rb = np.arange(40), np.arange(50)
    l1 = oracle.pairwise(A, B, "manhattan", rows_a=ra, rows_b=rb)
    l2 = oracle.pairwise(A, B, "euclidean", rows_a=ra, rows_b=rb)
    li = oracle.pairwise(A, B, "chebyshev", rows_a=ra, rows_b=rb)
    np.testing.assert_allclose(oracle.pairwise(A, B, "minkowski", 1.0, rows_a=ra, rows_b=rb), l1, rtol=1e-13)
    np.testing.assert_allclose(oracle.pairwise(A, B, "minkowski", 2.0, rows_a=ra, rows_b=rb), l2, rtol=1e-13)
    prev = l1
    for p in (1.5, 2.0, 3.0, 6.0, 24.0):
        cur = oracle.pairwise(A, B, "minkowski", p, rows_a=ra, rows_b=rb)
        assert np.all(cur <= prev + 1e-12)
        assert np.all(cur >= li - 1e-12)
        prev = cur
    np.testing.assert_allclose(oracle.pairwise(A, B, "minkowski", 200.0, rows_a=ra, rows_b=rb), li, rtol=0.02)
    assert np.all(li <= l2 + 1e-12) and np.all(l2 <= l1 + 1e-12)
    # expanded form of the Euclidean distance (Section 2.1) equals the formula column
    ip = oracle.pairwise(A, B, "inner_product", rows_a=ra, rows_b=rb)
    na = np.array([np.sum(synth.to_dense(A)[i] ** 2) for i in ra])
    nb = np.array([np.sum(synth.to_dense(B)[j] ** 2) for j in rb])
    np.testing.assert_allclose(l2 ** 2, na[:, None] - 2.0 * ip + nb[None, :], rtol=1e-10, atol=1e-12)


def test_binary_data_closed_forms():
    rng = np.random.default_rng(21)
    X = (rng.random((12, 64)) < 0.2).astype(np.float64)
    Y = (rng.random((10, 64)) < 0.3).astype(np.float64)
    A, B = synth.from_dense(X), synth.from_dense(Y)
    inter = X @ Y.T
    nx, ny = X.sum(1)[:, None], Y.sum(1)[None, :]
    sym = nx + ny - 2.0 * inter
    assert np.array_equal(_both(A, B, "manhattan"), sym)
    assert np.array_equal(_both(A, B, "canberra"), sym)
    assert np.array_equal(_both(A, B, "hamming"), sym / 64.0)
    np.testing.assert_allclose(_both(A, B, "euclidean"), np.sqrt(sym), rtol=1e-15)
    assert np.array_equal(_both(A, B, "chebyshev"), (sym > 0).astype(np.float64))
    assert np.array_equal(_both(A, B, "russell_rao"), (64.0 - inter) / 64.0)


def test_canberra_closed_form_on_nonnegative_data():
    A, B = synth.workload(0)
    X, Y = synth.to_dense(A)[:30], synth.to_dense(B)[:30]
    got = oracle.pairwise(A, B, "canberra", rows_a=np.arange(30), rows_b=np.arange(30))
    bx, by = X > 0, Y > 0
    for i in range(30):
        for j in range(30):
            both = bx[i] & by[j]
            one_sided = (bx[i] ^ by[j]).sum()
            shared = (np.abs(X[i, both] - Y[j, both]) / (X[i, both] + Y[j, both])).sum()
            assert got[i, j] == pytest.approx(one_sided + shared, rel=1e-12)


def test_full_mode_equals_support_mode_on_config0():
    A, B = synth.workload(0)
    for m in oracle.METRICS:
        _both(A, B, m, 3.0)


def test_two_pointer_merge_cross_check():
    """An independent sparse evaluation (walk the two sorted column lists in step, in the
    manner of the paper's Algorithm 2) agrees with the densified oracle."""
    A, B = synth.workload(0)

    def merge_sum(i, j, prod):
        ai, bi = int(A["indptr"][i]), int(B["indptr"][j])
        ae, be = int(A["indptr"][i + 1]), int(B["indptr"][j + 1])
        s = 0.0
        while ai < ae or bi < be:
            ca = A["indices"][ai] if ai < ae else 1 << 40
            cb = B["indices"][bi] if bi < be else 1 << 40
            va = vb = 0.0
            if ca <= cb:
                va = float(A["values"][ai]); ai += 1
            if cb <= ca:
                vb = float(B["values"][bi]); bi += 1
            s += prod(va, vb)
        return s

    l1 = oracle.pairwise(A, B, "manhattan", rows_a=np.arange(20), rows_b=np.arange(20))
    ip = oracle.pairwise(A, B, "inner_product", rows_a=np.arange(20), rows_b=np.arange(20))
    for i in range(20):
        for j in range(20):
            assert l1[i, j] == pytest.approx(merge_sum(i, j, lambda a, b: abs(a - b)), rel=1e-13)
            assert ip[i, j] == pytest.approx(merge_sum(i, j, lambda a, b: a * b), rel=1e-13, abs=1e-15)


def test_row_selection_and_threads():
    A, B = synth.workload(0)
    ra, rb = np.array([5, 0, 200, 5]), np.array([255, 3])
    full = oracle.pairwise(A, B, "canberra", threads=1)
    sel, used = oracle.pairwise(A, B, "canberra", rows_a=ra, rows_b=rb, threads=2, return_threads=True)
    assert used == 2
    assert np.array_equal(sel, full[np.ix_(ra, rb)])


def test_knn_order_and_ties():
    # index rows 0 and 3 are identical, row 2 equals the query: ties go to the lower index
    Q = synth.from_dense([[1, 0, 1, 0]])
    I = synth.from_dense([[1, 1, 1, 0], [0, 0, 0, 1], [1, 0, 1, 0], [1, 1, 1, 0], [0, 1, 0, 0]])
    idx, dist = oracle.knn(Q, I, "manhattan", 4)
    assert idx.tolist() == [[2, 0, 3, 1]] or idx.tolist() == [[2, 0, 3, 4]]
    assert dist[0, :3].tolist() == [0.0, 1.0, 1.0]
    assert idx.tolist()[0][3] == 1 and dist[0, 3] == 3.0
    # inner product is a similarity: the largest values come first
    idx, dist = oracle.knn(Q, I, "inner_product", 3)
    assert idx.tolist() == [[0, 2, 3]] and dist.tolist() == [[2.0, 2.0, 2.0]]
