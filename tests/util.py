"""Helpers shared by the tests: metric naming on the two sides and the tolerance rule."""
import numpy as np

# library metric name -> oracle metric name (the two sides keep their own vocabularies)
ORACLE_NAME = {
    "inner_product": "inner_product", "cosine": "cosine", "l2_expanded": "euclidean",
    "correlation": "correlation", "jaccard": "jaccard", "dice": "dice", "hellinger": "hellinger",
    "l1": "manhattan", "chebyshev": "chebyshev", "minkowski": "minkowski", "canberra": "canberra",
    "hamming": "hamming", "kl_divergence": "kl_divergence", "jensen_shannon": "jensen_shannon",
    "russell_rao": "russell_rao",
    "l2_unexpanded": "euclidean", "kl_divergence_strict": "kl_divergence_strict", "jaccard_literal": "jaccard_literal",
}
ALL_METRICS = tuple(ORACLE_NAME)
NONNEGATIVE_ONLY = ("hellinger", "kl_divergence", "jensen_shannon", "kl_divergence_strict")

REL_TOL = 1e-4      # max relative error of an fp32 distance
ABS_TOL = 1e-5      # absolute error allowed near zero


def tolerance(oracle_values):
    return np.maximum(REL_TOL * np.abs(oracle_values), ABS_TOL)


def assert_distances_close(got, want, what=""):
    """|got - want| <= max(1e-4 |want|, 1e-5) element by element (got fp32, want fp64)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    # an infinite oracle value (the strict KL divergence) must be met by the same infinity
    infinite = np.isinf(want)
    assert np.array_equal(got[infinite], want[infinite]), what + ": infinite values differ"
    assert np.all(np.isfinite(got[~infinite])), what + ": non-finite result"
    got = np.where(infinite, 0.0, got)
    want = np.where(infinite, 0.0, want)
    excess = np.abs(got - want) / tolerance(want)
    worst = np.unravel_index(np.argmax(excess), excess.shape) if excess.size else None
    assert excess.size == 0 or excess.max() <= 1.0, (
        "%s: worst error %.3g x tolerance at %s (got %.9g, want %.9g)"
        % (what, excess.max(), worst, got[worst], want[worst]))


def assert_knn_matches(idx, dist, oracle_rows, k, metric, what=""):
    """Exact index parity except at ties within tolerance.

    `oracle_rows` is the full fp64 distance row of every query (m, n).  The returned
    distances must match the oracle's at the returned indices; the list must be ordered
    by (distance, index); and wherever the index differs from the oracle's choice, the
    two candidates' oracle distances must be within tolerance of each other (a tie)."""
    idx = np.asarray(idx); dist = np.asarray(dist, dtype=np.float64)
    m, n = oracle_rows.shape
    key = -oracle_rows if metric == "inner_product" else oracle_rows
    for r in range(m):
        order = np.lexsort((np.arange(n), key[r]))[:k]
        assert len(set(idx[r].tolist())) == k, "%s: duplicate neighbours in row %d" % (what, r)
        assert idx[r].min() >= 0 and idx[r].max() < n
        assert_distances_close(dist[r], oracle_rows[r, idx[r]], "%s row %d distances" % (what, r))
        gk = -dist[r] if metric == "inner_product" else dist[r]
        for t in range(k - 1):
            assert gk[t] < gk[t + 1] or (gk[t] == gk[t + 1] and idx[r, t] < idx[r, t + 1]), \
                "%s: row %d not ordered at %d" % (what, r, t)
        diff = np.nonzero(idx[r] != order)[0]
        for t in diff:
            a, b = oracle_rows[r, idx[r, t]], oracle_rows[r, order[t]]
            assert a == b or abs(a - b) <= 2.0 * max(REL_TOL * abs(b), ABS_TOL), \
                "%s: row %d position %d: index %d (%.9g) instead of %d (%.9g)" % (
                    what, r, t, idx[r, t], a, order[t], b)


def progress(capsys, message):
    """A line on stderr past pytest's capture (`capsys` is the test's fixture): the steps of the
    long tests, so that they stay visibly alive."""
    import sys
    import time
    with capsys.disabled():
        sys.stderr.write("[step %s] %s\n" % (time.strftime("%H:%M:%S"), message))
        sys.stderr.flush()


def quotient_cases():
    """Row pairs (over 16 columns) that stress the quotients inside the logarithms of KL and
    Jensen-Shannon: equal entries, one entry twice the other, ratios of 1e8 and 1e12 either
    way, entries near the ends of the fp32 range, and a plain pair beside each so that the
    result is not dominated by the extreme column alone."""
    cases = []
    for x, y in ((1.0, 1.0), (0.25, 0.5), (0.5, 0.25), (1.0, 1e-8), (1e-8, 1.0), (1.0, 1e-12), (1e-12, 1.0),
                 (3e-31, 2e-31), (2e29, 5e28), (7e-31, 7e-31), (1e-37, 1.0), (1.0, 1e-37), (1.5e-38, 1.5e-38)):
        a = np.zeros(16); b = np.zeros(16)
        a[3], b[3] = x, y
        a[5], b[5] = 0.5, 0.5
        a[9], b[11] = 0.125, 0.375            # one-sided columns
        cases.append((a, b))
    return cases


# Every distance of Table 1 as a semiring call: product(), sum(), domain, the transform of the
# stored values and the epilogue (Section 2.2; Table 1's expansion column).  `p` where it matters.
TABLE1_SEMIRINGS = {
    "inner_product": dict(product="times", sum="plus", over_union=False),
    "cosine": dict(product="times", sum="plus", over_union=False, epilogue="cosine"),
    "l2_expanded": dict(product="times", sum="plus", over_union=False, epilogue="l2"),
    "correlation": dict(product="times", sum="plus", over_union=False, epilogue="correlation"),
    "jaccard": dict(product="times", sum="plus", over_union=False, transform="nonzero", epilogue="jaccard"),
    "dice": dict(product="times", sum="plus", over_union=False, transform="nonzero", epilogue="dice"),
    "hellinger": dict(product="times", sum="plus", over_union=False, transform="sqrt", epilogue="hellinger"),
    "l1": dict(product="abs_diff", sum="plus", over_union=True),
    "chebyshev": dict(product="abs_diff", sum="max", over_union=True),      # (-infinity, not 0, between two empty rows)
    "minkowski": dict(product="abs_diff_pow", sum="plus", over_union=True, epilogue="root_p"),
    "canberra": dict(product="canberra", sum="plus", over_union=True),
    "hamming": dict(product="not_equal", sum="plus", over_union=True, epilogue="div_k"),
    "kl_divergence": dict(product="x_log_x_over_y", sum="plus", over_union=False),
    "jensen_shannon": dict(product="js_term", sum="plus", over_union=True, epilogue="sqrt_half"),
    "russell_rao": dict(product="times", sum="plus", over_union=False, transform="nonzero", epilogue="russell_rao"),
    "l2_unexpanded": dict(product="sq_diff", sum="plus", over_union=True, epilogue="root_p", p=2.0),
    "kl_divergence_strict": dict(product="x_log_x_over_y", sum="plus", over_union=False, epilogue="strict"),
    "jaccard_literal": dict(product="times", sum="plus", over_union=False, epilogue="jaccard"),
}
