"""Pins of the oracle's semiring products (Section 2.2) to things other than itself: the worked
examples of the paper's appendix, dense numpy formulations (a matrix product, tensors filled with
the identity of sum() where a row stores nothing), scipy's distances, and algebraic identities."""
import itertools
import os

import numpy as np
import pytest
import scipy.spatial.distance as ssd

import oracle
from gen import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _dense_pair(seed, rows_a=9, rows_b=11, cols=23, density=0.35, signed=True):
    rng = np.random.default_rng(seed)

    def one(rows):
        d = rng.standard_normal((rows, cols)) if signed else rng.random((rows, cols)) + 0.05
        d *= rng.random((rows, cols)) < density
        d[rows // 2] = 0.0                                   # an empty row
        return np.asarray(d.astype(np.float32), dtype=np.float64)

    X, Y = one(rows_a), one(rows_b)
    Y[0] = X[0]                                              # a pair with equal supports
    return X, Y


def _both_modes(A, B, product, sum_, union):
    full = oracle.semiring_pairwise(A, B, product, sum_, union, mode="full")
    sup = oracle.semiring_pairwise(A, B, product, sum_, union, mode="support")
    np.testing.assert_allclose(sup, full, rtol=1e-12, atol=1e-13)   # the two modes add in different orders
    return full


PRODUCT_FN = {
    "times": lambda a, b: a * b, "plus": lambda a, b: a + b, "min": np.minimum, "max": np.maximum,
    "abs_diff": lambda a, b: np.abs(a - b), "sq_diff": lambda a, b: (a - b) ** 2,
}
FOLD = {"plus": (np.sum, 0.0), "min": (np.min, np.inf), "max": (np.max, -np.inf)}


def _masked_tensor(X, Y, product, sum_, union):
    """The definition written a second way: the m x n x k tensor of products with the columns
    outside the domain replaced by the identity of sum(), folded along k by numpy."""
    fold, ident = FOLD[sum_]
    px, py = X[:, None, :] != 0.0, Y[None, :, :] != 0.0
    domain = (px | py) if union else (px & py)
    t = PRODUCT_FN[product](X[:, None, :], Y[None, :, :])
    return fold(np.where(domain, t, ident), axis=2)


@pytest.mark.parametrize("union", [False, True])
@pytest.mark.parametrize("sum_", oracle.SUMS)
@pytest.mark.parametrize("product", oracle.PRODUCTS)
def test_against_masked_dense_tensor(product, sum_, union):
    X, Y = _dense_pair(7)
    got = _both_modes(synth.from_dense(X), synth.from_dense(Y), product, sum_, union)
    want = _masked_tensor(X, Y, product, sum_, union)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_paper_appendix_examples():
    # first worked example: the non-annihilating |a - b| summed over the union is the Manhattan
    # distance the paper prints, the annihilating product over the intersection is what it prints too
    g = {}
    with open(os.path.join(GOLDEN, "appendix_manhattan_example.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                key, *vals = line.split()
                g[key] = [float(v) for v in vals]
    a, b = synth.from_dense([g["a"]]), synth.from_dense([g["b"]])
    assert _both_modes(a, b, "abs_diff", "plus", True)[0, 0] == g["manhattan"][0] == 3.0
    assert _both_modes(a, b, "times", "plus", False)[0, 0] == g["annihilating_sum"][0] == 0.0
    # second example: A = [1, 0, 1], b = [0, 1, 1]: one shared column, three in the union
    A, y = synth.from_dense([[1.0, 0.0, 1.0]]), synth.from_dense([[0.0, 1.0, 1.0]])
    assert _both_modes(A, y, "times", "plus", False)[0, 0] == 1.0          # |intersection|
    assert _both_modes(A, y, "max", "plus", True)[0, 0] == 3.0             # |union|
    assert _both_modes(A, y, "abs_diff", "plus", True)[0, 0] == 2.0


def test_dot_product_semiring_is_the_matrix_product():
    X, Y = _dense_pair(11)
    got = _both_modes(synth.from_dense(X), synth.from_dense(Y), "times", "plus", False)
    np.testing.assert_allclose(got, X @ Y.T, rtol=1e-12, atol=1e-13)
    # 0 annihilates: the union adds nothing
    np.testing.assert_array_equal(got, _both_modes(synth.from_dense(X), synth.from_dense(Y), "times", "plus", True))


def test_namm_semirings_are_the_library_distances():
    X, Y = _dense_pair(13)
    A, B = synth.from_dense(X), synth.from_dense(Y)
    np.testing.assert_allclose(_both_modes(A, B, "abs_diff", "plus", True), ssd.cdist(X, Y, "cityblock"), rtol=1e-12)
    np.testing.assert_allclose(_both_modes(A, B, "sq_diff", "plus", True), ssd.cdist(X, Y, "sqeuclidean"), rtol=1e-12)
    cheb = _both_modes(A, B, "abs_diff", "max", True)
    lib = ssd.cdist(X, Y, "chebyshev")
    nonempty = (np.abs(X).sum(1)[:, None] + np.abs(Y).sum(1)[None, :]) > 0
    np.testing.assert_allclose(cheb[nonempty], lib[nonempty], rtol=1e-12)
    assert np.all(cheb[~nonempty] == -np.inf) and (~nonempty).sum() == 1    # empty union: identity of max


def test_tropical_semiring_is_the_min_plus_matrix_product():
    # Eq. 1: (min, +) over R with +infinity, the additive identity, standing for an absent entry
    X, Y = _dense_pair(17)
    Xi, Yi = np.where(X != 0, X, np.inf), np.where(Y != 0, Y, np.inf)
    want = np.min(Xi[:, None, :] + Yi[None, :, :], axis=2)
    got = _both_modes(synth.from_dense(X), synth.from_dense(Y), "plus", "min", False)
    np.testing.assert_array_equal(got, want)
    assert np.isinf(got).any() and np.isfinite(got).any()
    # and (max, +) with -infinity
    Xm, Ym = np.where(X != 0, X, -np.inf), np.where(Y != 0, Y, -np.inf)
    np.testing.assert_array_equal(_both_modes(synth.from_dense(X), synth.from_dense(Y), "plus", "max", False),
                                  np.max(Xm[:, None, :] + Ym[None, :, :], axis=2))


def test_identities_on_nonnegative_data():
    X, Y = _dense_pair(19, signed=False)
    A, B = synth.from_dense(X), synth.from_dense(Y)
    smin = _both_modes(A, B, "min", "plus", False)           # histogram intersection
    smax = _both_modes(A, B, "max", "plus", True)
    np.testing.assert_allclose(smin, np.minimum(X[:, None, :], Y[None, :, :]).sum(2), rtol=1e-12)
    np.testing.assert_allclose(smax, np.maximum(X[:, None, :], Y[None, :, :]).sum(2), rtol=1e-12)
    # min + max = x + y column by column; |x - y| = max - min
    np.testing.assert_allclose(smin + smax, X.sum(1)[:, None] + Y.sum(1)[None, :], rtol=1e-12)
    np.testing.assert_allclose(smax - smin, _both_modes(A, B, "abs_diff", "plus", True), rtol=1e-10, atol=1e-12)
    # plus over the union with sum() = plus is separable
    np.testing.assert_allclose(_both_modes(A, B, "plus", "plus", True), X.sum(1)[:, None] + Y.sum(1)[None, :], rtol=1e-12)
    # bottleneck (max, min) on the intersection, by brute force over columns
    want = np.full((X.shape[0], Y.shape[0]), -np.inf)
    for i, j, c in itertools.product(range(X.shape[0]), range(Y.shape[0]), range(X.shape[1])):
        if X[i, c] != 0 and Y[j, c] != 0:
            want[i, j] = max(want[i, j], min(X[i, c], Y[j, c]))
    np.testing.assert_array_equal(_both_modes(A, B, "min", "max", False), want)


def test_symmetry_stored_zeros_and_transposition():
    X, Y = _dense_pair(23)
    A, B = synth.from_dense(X), synth.from_dense(Y)
    for product, sum_, union in itertools.product(oracle.PRODUCTS, oracle.SUMS, (False, True)):
        ab = oracle.semiring_pairwise(A, B, product, sum_, union)
        ba = oracle.semiring_pairwise(B, A, product, sum_, union)
        # every product offered is commutative (sums are taken in a different order)
        np.testing.assert_allclose(ab, ba.T, rtol=1e-12, atol=1e-13) if sum_ == "plus" else np.testing.assert_array_equal(ab, ba.T)
    # a stored zero is an absent entry: (min, plus over the union) would otherwise see a 0
    a = {"n_rows": 1, "n_cols": 4, "indptr": [0, 3], "indices": [0, 1, 3], "values": [2.0, 0.0, 5.0]}
    b = {"n_rows": 1, "n_cols": 4, "indptr": [0, 2], "indices": [1, 3], "values": [0.0, 1.0]}
    assert oracle.semiring_pairwise(a, b, "plus", "min", True)[0, 0] == 2.0
    assert oracle.semiring_pairwise(a, b, "plus", "min", False)[0, 0] == 6.0
    assert oracle.semiring_pairwise(a, b, "max", "plus", True)[0, 0] == 7.0


def test_semiring_knn_orders_by_value_then_index():
    X, Y = _dense_pair(29, rows_a=5, rows_b=40)
    A, B = synth.from_dense(X), synth.from_dense(Y)
    idx, val = oracle.semiring_knn(A, B, "plus", "min", False, 7)
    full = oracle.semiring_pairwise(A, B, "plus", "min", False)
    for r in range(5):
        order = sorted(range(40), key=lambda j: (full[r, j], j))[:7]
        assert list(idx[r]) == order
        np.testing.assert_array_equal(val[r], full[r, order])


# ---------------------------------------------------------------- Table 1 through the semiring evaluator
MORE_PRODUCT_FN = {
    "abs_diff_pow": lambda a, b, p: np.abs(a - b) ** p,
    "canberra": lambda a, b, p: np.where(np.abs(a) + np.abs(b) != 0, np.abs(a - b) / np.where(np.abs(a) + np.abs(b) != 0, np.abs(a) + np.abs(b), 1.0), 0.0),
    "not_equal": lambda a, b, p: (a != b).astype(np.float64),
}


@pytest.mark.parametrize("union", [False, True])
@pytest.mark.parametrize("sum_", oracle.SUMS)
@pytest.mark.parametrize("product", sorted(MORE_PRODUCT_FN))
def test_more_products_against_masked_dense_tensor(product, sum_, union):
    X, Y = _dense_pair(23)
    fold, ident = FOLD[sum_]
    px, py = X[:, None, :] != 0.0, Y[None, :, :] != 0.0
    domain = (px | py) if union else (px & py)
    t = MORE_PRODUCT_FN[product](X[:, None, :], Y[None, :, :], 2.5)
    want = fold(np.where(domain, t, ident), axis=2)
    for mode in ("full", "support"):
        got = oracle.semiring_pairwise(synth.from_dense(X), synth.from_dense(Y), product, sum_, union, mode=mode, p=2.5)
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_log_products_against_scipy_special():
    from scipy.special import rel_entr
    X, Y = _dense_pair(29, signed=False)
    A, B = synth.from_dense(X), synth.from_dense(Y)
    both = (X[:, None, :] > 0) & (Y[None, :, :] > 0)
    kl = np.where(both, rel_entr(np.where(both, X[:, None, :], 1.0), np.where(both, Y[None, :, :], 1.0)), 0.0).sum(axis=2)
    np.testing.assert_allclose(oracle.semiring_pairwise(A, B, "x_log_x_over_y", "plus", False, mode="full"), kl,
                               rtol=1e-12, atol=1e-13)
    mu = 0.5 * (X[:, None, :] + Y[None, :, :])
    js = (rel_entr(X[:, None, :] + 0 * mu, mu) + rel_entr(Y[None, :, :] + 0 * mu, mu)).sum(axis=2)   # rel_entr(0, m) = 0
    np.testing.assert_allclose(oracle.semiring_pairwise(A, B, "js_term", "plus", True, mode="full"), js,
                               rtol=1e-12, atol=1e-13)
    # the same product over the intersection leaves the one-sided columns (a log 2 each) out
    inter = oracle.semiring_pairwise(A, B, "js_term", "plus", False, mode="full")
    one_sided = np.log(2.0) * (np.where(Y[None, :, :] == 0, X[:, None, :], 0.0) + np.where(X[:, None, :] == 0, Y[None, :, :], 0.0)).sum(axis=2)
    np.testing.assert_allclose(inter + one_sided, js, rtol=1e-12, atol=1e-13)


def test_transforms_and_epilogues_against_scipy():
    X, Y = _dense_pair(31, signed=False)
    keep = np.ones(X.shape[0], bool); keep[X.shape[0] // 2] = False          # scipy has no convention for zero rows
    keepy = np.ones(Y.shape[0], bool); keepy[Y.shape[0] // 2] = False
    Xs, Ys = X[keep], Y[keepy]
    A, B = synth.from_dense(Xs), synth.from_dense(Ys)
    k = Xs.shape[1]

    def run(**kw):
        kw.setdefault("over_union", False)
        product, sum_, union = kw.pop("product"), kw.pop("sum"), kw.pop("over_union")
        full = oracle.semiring_pairwise(A, B, product, sum_, union, mode="full", **kw)
        np.testing.assert_allclose(oracle.semiring_pairwise(A, B, product, sum_, union, mode="support", **kw), full,
                                   rtol=1e-12, atol=1e-13)
        return full

    close = lambda got, want: np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)
    close(run(product="times", sum="plus", epilogue="cosine"), ssd.cdist(Xs, Ys, "cosine"))
    close(run(product="times", sum="plus", epilogue="l2"), ssd.cdist(Xs, Ys, "euclidean"))
    close(run(product="times", sum="plus", epilogue="correlation"), ssd.cdist(Xs, Ys, "correlation"))
    close(run(product="times", sum="plus", transform="nonzero", epilogue="jaccard"), ssd.cdist(Xs != 0, Ys != 0, "jaccard"))
    close(run(product="times", sum="plus", transform="nonzero", epilogue="dice"), ssd.cdist(Xs != 0, Ys != 0, "dice"))
    close(run(product="times", sum="plus", transform="nonzero", epilogue="russell_rao"), ssd.cdist(Xs != 0, Ys != 0, "russellrao"))
    close(run(product="times", sum="plus", transform="sqrt", epilogue="hellinger"),
          ssd.cdist(np.sqrt(Xs), np.sqrt(Ys), "euclidean") / np.sqrt(2.0))
    close(run(product="abs_diff_pow", sum="plus", over_union=True, epilogue="root_p", p=3.0), ssd.cdist(Xs, Ys, "minkowski", p=3.0))
    close(run(product="sq_diff", sum="plus", over_union=True, epilogue="root_p", p=2.0), ssd.cdist(Xs, Ys, "euclidean"))
    close(run(product="canberra", sum="plus", over_union=True), ssd.cdist(Xs, Ys, "canberra"))
    close(run(product="not_equal", sum="plus", over_union=True, epilogue="div_k"), ssd.cdist(Xs, Ys, "hamming"))
    P, Q = Xs / Xs.sum(1, keepdims=True), Ys / Ys.sum(1, keepdims=True)
    Ap, Bq = synth.from_dense(P), synth.from_dense(Q)
    js = oracle.semiring_pairwise(Ap, Bq, "js_term", "plus", True, mode="full", epilogue="sqrt_half")
    # the arrays went through fp32 on their way into the CSR: compare on what the oracle saw
    P32, Q32 = synth.to_dense(Ap), synth.to_dense(Bq)
    want = np.array([[ssd.jensenshannon(p / p.sum(), q / q.sum()) for q in Q32] for p in P32])
    scale = np.sqrt(0.5 * (P32.sum(1)[:, None] + Q32.sum(1)[None, :]))       # rows sum to 1 up to fp32 rounding
    np.testing.assert_allclose(js, want * scale, rtol=1e-6)
    # strict: infinite exactly where x holds mass that y does not cover
    strict = oracle.semiring_pairwise(A, B, "x_log_x_over_y", "plus", False, mode="full", epilogue="strict")
    uncovered = ((Xs[:, None, :] > 0) & ~(Ys[None, :, :] > 0)).any(axis=2)
    assert np.array_equal(np.isinf(strict), uncovered) and uncovered.any() and (~uncovered).any()
    assert k == 23


def test_every_distance_of_table_1_is_a_semiring_call():
    """The composition (transform, product, sum, domain, epilogue) against the plain formula the
    metric oracle evaluates: Table 1's expansion column equals its formula column."""
    import sys
    sys.path.insert(0, os.path.dirname(__file__))
    from util import NONNEGATIVE_ONLY, ORACLE_NAME, TABLE1_SEMIRINGS
    assert set(TABLE1_SEMIRINGS) == set(ORACLE_NAME)
    for signed in (True, False):
        X, Y = _dense_pair(37 + signed, rows_a=13, rows_b=17, signed=signed)
        Y[3] = X[3] * 2.0                      # proportional rows, equal supports
        A, B = synth.from_dense(X), synth.from_dense(Y)
        for metric, sr in TABLE1_SEMIRINGS.items():
            if signed and metric in NONNEGATIVE_ONLY:
                continue
            sr = dict(sr)
            p = sr.pop("p", 3.0)
            for mode in ("full", "support"):
                got = oracle.semiring_pairwise(A, B, sr["product"], sr["sum"], sr["over_union"],
                                               mode=mode, p=p, transform=sr.get("transform", "none"),
                                               epilogue=sr.get("epilogue", "none"))
                want = oracle.pairwise(A, B, ORACLE_NAME[metric], p, mode=mode)
                if metric == "chebyshev":      # two empty rows: the identity of max, where the distance says 0
                    empty = (np.abs(X).sum(1)[:, None] + np.abs(Y).sum(1)[None, :]) == 0
                    assert np.all(got[empty] == -np.inf) and empty.sum() == 1
                    got = np.where(empty, 0.0, got)
                inf = np.isinf(want)
                assert np.array_equal(np.isinf(got), inf), metric
                np.testing.assert_allclose(np.where(inf, 0, got), np.where(inf, 0, want), rtol=1e-9, atol=1e-11, err_msg=metric)
