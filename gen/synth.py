"""Seeded synthetic CSR workloads shaped like the paper's datasets (Table "Datasets used
in experiments" and the degree-CDF figure of the Experiments section).

This module only draws random sparse matrices.  It contains none of the distance
arithmetic: it serves the CPU oracle and the HIP library alike and imports neither.

Every matrix is returned as a dict
    {"n_rows", "n_cols", "indptr" (int64, n_rows+1), "indices" (int32, nnz, strictly
     ascending inside a row), "values" (float32, nnz, never an explicit zero)}.

Seeds: ``SEED0 + 1000*config + role`` with role 0 = A / queries, 1 = B / index.
"""
from __future__ import annotations

import numpy as np

SEED0 = 210406357


def seed_for(config: int, role: int) -> int:
    return SEED0 + 1000 * config + role


# --------------------------------------------------------------------------------------
# column laws
# --------------------------------------------------------------------------------------
class UniformColumns:
    """Every column equally likely."""

    def __init__(self, n_cols: int):
        self.n_cols = int(n_cols)

    def draw(self, rng: np.random.Generator, size: int) -> np.ndarray:
        return rng.integers(0, self.n_cols, size=size, dtype=np.int64)


class ZipfColumns:
    """Column popularity follows a continuous power law over ranks.

    Rank r in [1, K] is drawn with probability proportional to the integral of
    x**(-s) over [r, r+1) (closed-form inverse transform, no tables), and ranks are
    mapped to column ids through a seeded permutation so that popular columns are
    spread over the whole id range.
    """

    def __init__(self, n_cols: int, exponent: float, perm_seed: int):
        self.n_cols = int(n_cols)
        self.s = float(exponent)
        self.perm = np.random.Generator(np.random.PCG64(perm_seed)).permutation(self.n_cols)
        one_minus_s = 1.0 - self.s
        self._e = one_minus_s
        self._span = (self.n_cols + 1.0) ** one_minus_s - 1.0

    def draw(self, rng: np.random.Generator, size: int) -> np.ndarray:
        u = rng.random(size)
        x = (1.0 + u * self._span) ** (1.0 / self._e)
        r = np.minimum(x.astype(np.int64), self.n_cols) - 1
        np.maximum(r, 0, out=r)
        return self.perm[r].astype(np.int64)


# --------------------------------------------------------------------------------------
# rows of distinct columns with prescribed degrees
# --------------------------------------------------------------------------------------
def _isin_sorted(sorted_arr: np.ndarray, q: np.ndarray) -> np.ndarray:
    if sorted_arr.size == 0:
        return np.zeros(q.shape, dtype=bool)
    pos = np.searchsorted(sorted_arr, q)
    pos[pos == sorted_arr.size] = sorted_arr.size - 1
    return sorted_arr[pos] == q


def _distinct_columns_chunk(rng, deg: np.ndarray, law) -> np.ndarray:
    """Sorted int64 keys (local_row << 32 | col): row r gets exactly deg[r] distinct columns.

    Columns are drawn from the law with replacement; duplicates are dropped and the
    shortfall redrawn, keeping draws in the order they were made (sequential sampling
    without replacement).
    """
    nr = deg.size
    short = deg.astype(np.int64).copy()
    base = np.empty(0, dtype=np.int64)
    extra = np.empty(0, dtype=np.int64)
    over = 1.0
    while True:
        rows = np.nonzero(short)[0]
        if rows.size == 0:
            break
        cnt = np.ceil(short[rows] * over).astype(np.int64)
        rr = np.repeat(rows, cnt)
        cols = law.draw(rng, rr.size)
        keys = (rr.astype(np.int64) << 32) | cols
        if over == 1.0:
            # nothing can exceed the shortfall: every distinct fresh key is accepted
            uniq = np.sort(keys)
            if uniq.size > 1:
                uniq = uniq[np.concatenate(([True], uniq[1:] != uniq[:-1]))]
            if base.size or extra.size:
                uniq = uniq[~(_isin_sorted(base, uniq) | _isin_sorted(extra, uniq))]
            accepted = uniq
        else:
            uniq, first = np.unique(keys, return_index=True)
            fresh = ~(_isin_sorted(base, uniq) | _isin_sorted(extra, uniq))
            uniq = uniq[fresh]
            first = first[fresh]
            order = np.argsort(first, kind="stable")   # draw order (rows stay grouped)
            uniq = uniq[order]
            urow = uniq >> 32
            row_start = np.searchsorted(urow, np.arange(nr))
            rank = np.arange(uniq.size) - row_start[urow]
            accepted = uniq[rank < short[urow]]
            accepted.sort()
        short -= np.bincount(accepted >> 32, minlength=nr)
        if base.size == 0:
            base = accepted
        else:
            extra = np.sort(np.concatenate([extra, accepted]))
        rate = accepted.size / max(keys.size, 1)
        over = float(min(16.0, max(1.0, 1.0 / max(rate, 1e-3))))
    out = np.concatenate([base, extra])
    out.sort()
    return out


def rows_with_degrees(rng, deg: np.ndarray, law, chunk_nnz: int = 1 << 22):
    """indptr (int64) and indices (int32, ascending in each row) for the given degrees."""
    deg = np.asarray(deg, dtype=np.int64)
    if np.any(deg > law.n_cols):
        raise ValueError("degree exceeds number of columns")
    n = deg.size
    indptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(deg, out=indptr[1:])
    indices = np.empty(int(indptr[-1]), dtype=np.int32)
    r0 = 0
    while r0 < n:
        r1 = int(np.searchsorted(indptr, indptr[r0] + chunk_nnz, side="right")) - 1
        r1 = min(max(r1, r0 + 1), n)
        keys = _distinct_columns_chunk(rng, deg[r0:r1], law)
        indices[indptr[r0]:indptr[r1]] = (keys & 0xFFFFFFFF).astype(np.int32)
        r0 = r1
    return indptr, indices


def _row_ids(indptr: np.ndarray) -> np.ndarray:
    return np.repeat(np.arange(indptr.size - 1, dtype=np.int64), np.diff(indptr))


def _row_sums(indptr, v64):
    return np.bincount(_row_ids(indptr), weights=v64, minlength=indptr.size - 1)


def _csr(n_rows, n_cols, indptr, indices, values):
    return {
        "n_rows": int(n_rows),
        "n_cols": int(n_cols),
        "indptr": np.ascontiguousarray(indptr, dtype=np.int64),
        "indices": np.ascontiguousarray(indices, dtype=np.int32),
        "values": np.ascontiguousarray(values, dtype=np.float32),
    }


def stats(csr) -> dict:
    deg = np.diff(csr["indptr"])
    return {
        "rows": csr["n_rows"], "cols": csr["n_cols"], "nnz": int(csr["indptr"][-1]),
        "deg_mean": float(deg.mean()) if deg.size else 0.0,
        "deg_min": int(deg.min()) if deg.size else 0,
        "deg_p50": float(np.percentile(deg, 50)) if deg.size else 0.0,
        "deg_p99": float(np.percentile(deg, 99)) if deg.size else 0.0,
        "deg_max": int(deg.max()) if deg.size else 0,
    }


# --------------------------------------------------------------------------------------
# config 0: tiny uniform
# --------------------------------------------------------------------------------------
def tiny(role: int, n_rows: int = 256, n_cols: int = 512, density: float = 0.02, config: int = 0):
    rng = np.random.Generator(np.random.PCG64(seed_for(config, role)))
    mask = rng.random((n_rows, n_cols)) < density
    empty = ~mask.any(axis=1)
    mask[empty, rng.integers(0, n_cols, size=int(empty.sum()))] = True
    rows, cols = np.nonzero(mask)
    indptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(np.bincount(rows, minlength=n_rows), out=indptr[1:])
    values = (1.0 - rng.random(cols.size)).astype(np.float32)      # (0, 1]
    return _csr(n_rows, n_cols, indptr, cols, values)


# --------------------------------------------------------------------------------------
# config 1: skewed medium
# --------------------------------------------------------------------------------------
def skewed_medium(role: int, n_rows: int = 10_000, n_cols: int = 20_000, config: int = 1):
    rng = np.random.Generator(np.random.PCG64(seed_for(config, role)))
    z = rng.zipf(1.8, size=n_rows).astype(np.float64)
    deg = np.clip(4.0 * z, 1, min(2000, n_cols)).astype(np.int64)
    law = ZipfColumns(n_cols, 1.1, perm_seed=seed_for(config, 7))
    indptr, indices = rows_with_degrees(rng, deg, law)
    v = np.abs(rng.standard_normal(indices.size))
    while True:
        bad = np.nonzero(v.astype(np.float32) == 0.0)[0]
        if bad.size == 0:
            break
        v[bad] = np.abs(rng.standard_normal(bad.size))
    return _csr(n_rows, n_cols, indptr, indices, v)


# --------------------------------------------------------------------------------------
# config 2: bag-of-words-like (queries vs index share the column law and the idf vector)
# --------------------------------------------------------------------------------------
def _bow_structure(rng, n_rows, n_cols, law):
    sigma = 0.8
    mu = np.log(230.0) - 0.5 * sigma * sigma
    deg = np.clip(np.rint(rng.lognormal(mu, sigma, size=n_rows)), 1, min(2000, n_cols)).astype(np.int64)
    indptr, indices = rows_with_degrees(rng, deg, law)
    counts = np.ceil(rng.lognormal(0.0, 1.0, size=indices.size))
    return indptr, indices, counts


def bag_of_words(n_queries: int = 8192, n_index: int = 300_000, n_cols: int = 102_660, config: int = 2):
    """Returns (queries, index)."""
    law = ZipfColumns(n_cols, 1.1, perm_seed=seed_for(config, 7))
    rng_b = np.random.Generator(np.random.PCG64(seed_for(config, 1)))
    ip_b, ix_b, cnt_b = _bow_structure(rng_b, n_index, n_cols, law)
    df = np.bincount(ix_b, minlength=n_cols).astype(np.float64)
    idf = np.log((1.0 + n_index) / (1.0 + df)) + 1.0
    rng_a = np.random.Generator(np.random.PCG64(seed_for(config, 0)))
    ip_a, ix_a, cnt_a = _bow_structure(rng_a, n_queries, n_cols, law)

    def finish(n_rows, indptr, indices, counts):
        v = counts * idf[indices]
        nrm = np.sqrt(_row_sums(indptr, v * v))
        v = v / nrm[_row_ids(indptr)]
        return _csr(n_rows, n_cols, indptr, indices, v)

    return finish(n_queries, ip_a, ix_a, cnt_a), finish(n_index, ip_b, ix_b, cnt_b)


# --------------------------------------------------------------------------------------
# config 3: count-matrix-like, rows are probability vectors; self-join
# --------------------------------------------------------------------------------------
def count_matrix(n_rows: int = 65_536, n_cols: int = 26_000, config: int = 3, n_heavy: int = 8):
    rng = np.random.Generator(np.random.PCG64(seed_for(config, 1)))
    sigma = 0.5
    mean_deg = 0.07 * n_cols
    mu = np.log(mean_deg) - 0.5 * sigma * sigma
    hi = min(12_000, n_cols)
    lo = min(500, hi)
    deg = np.clip(np.rint(rng.lognormal(mu, sigma, size=n_rows)), lo, hi).astype(np.int64)
    if n_heavy and hi > 10_240:
        n_heavy = min(n_heavy, n_rows)
        heavy_rows = rng.choice(n_rows, size=n_heavy, replace=False)
        deg[heavy_rows] = rng.integers(10_300, hi + 1, size=n_heavy)
    indptr, indices = rows_with_degrees(rng, deg, UniformColumns(n_cols))
    v = rng.negative_binomial(2.0, 0.4, size=indices.size).astype(np.float64)
    while True:
        bad = np.nonzero(v == 0.0)[0]
        if bad.size == 0:
            break
        v[bad] = rng.negative_binomial(2.0, 0.4, size=bad.size)
    v = v / _row_sums(indptr, v)[_row_ids(indptr)]
    return _csr(n_rows, n_cols, indptr, indices, v)


# --------------------------------------------------------------------------------------
# config 4: binary, very high dimensional, power-law degrees
# --------------------------------------------------------------------------------------
def _powerlaw_degrees(rng, n_rows, alpha, d_max):
    d = np.arange(1, d_max + 1, dtype=np.float64)
    cdf = np.cumsum(d ** (-alpha))
    cdf /= cdf[-1]
    return (np.searchsorted(cdf, rng.random(n_rows), side="left") + 1).astype(np.int64)


def binary_highdim(role: int, n_rows: int, n_cols: int = 1 << 20, d_max: int = 50_000, config: int = 4):
    rng = np.random.Generator(np.random.PCG64(seed_for(config, role)))
    deg = np.minimum(_powerlaw_degrees(rng, n_rows, 1.5, d_max), n_cols)
    law = ZipfColumns(n_cols, 1.1, perm_seed=seed_for(config, 7))
    indptr, indices = rows_with_degrees(rng, deg, law)
    return _csr(n_rows, n_cols, indptr, indices, np.ones(indices.size, dtype=np.float32))


# --------------------------------------------------------------------------------------
# two more shapes, at the ends the five configs leave out (the shapes of two of the paper's
# datasets, Section 4.1 / Table 2; the data itself is drawn here, not reconstructed)
#   5: n-gram-like   - 663,000 x 858,000, almost every row under 10 entries, none above 51
#   6: ratings-like  - 283,000 x 194,000, power-law degrees up to 24,000 (mean ~100)
# --------------------------------------------------------------------------------------
def ngram_like(n_rows: int = 663_000, n_cols: int = 858_000, config: int = 5):
    rng = np.random.Generator(np.random.PCG64(seed_for(config, 0)))
    deg = np.minimum(rng.geometric(0.45, size=n_rows), 51).astype(np.int64)      # P(deg >= 10) = 0.5 %
    deg[rng.integers(0, n_rows, size=4)] = 51                                    # the longest rows are always there
    law = ZipfColumns(n_cols, 1.05, perm_seed=seed_for(config, 7))
    indptr, indices = rows_with_degrees(rng, deg, law)
    v = 1.0 + rng.poisson(0.3, size=indices.size)                                # small counts
    return _csr(n_rows, n_cols, indptr, indices, v.astype(np.float32))


def ratings_like(n_rows: int = 283_000, n_cols: int = 194_000, d_max: int = 24_000, config: int = 6):
    rng = np.random.Generator(np.random.PCG64(seed_for(config, 0)))
    deg = np.minimum(_powerlaw_degrees(rng, n_rows, 1.45, d_max), n_cols)
    deg[rng.integers(0, n_rows)] = min(d_max, n_cols)                           # the extreme row is always there
    law = ZipfColumns(n_cols, 1.02, perm_seed=seed_for(config, 7))
    indptr, indices = rows_with_degrees(rng, deg, law)
    v = 0.5 * rng.integers(1, 11, size=indices.size)                             # 0.5 .. 5.0 in steps of 0.5
    return _csr(n_rows, n_cols, indptr, indices, v.astype(np.float32))


# --------------------------------------------------------------------------------------
# named workloads
# --------------------------------------------------------------------------------------
def workload(config: int, scale: float = 1.0):
    """(A, B) for BASELINE config 0..4, and the two extra shapes 5 and 6.  ``scale`` < 1 shrinks row counts only (the
    column count, degree law, column law and value law stay those of the full size)."""
    s = float(scale)

    def rows(n):
        return max(8, int(round(n * s)))

    if config == 0:
        return tiny(0), tiny(1)
    if config == 1:
        return skewed_medium(0, rows(10_000)), skewed_medium(1, rows(10_000))
    if config == 2:
        return bag_of_words(rows(8192), rows(300_000))
    if config == 3:
        b = count_matrix(rows(65_536))
        return b, b                                   # self-join; callers slice query tiles
    if config == 4:
        return binary_highdim(0, rows(4096)), binary_highdim(1, rows(500_000))
    if config == 5:
        b = ngram_like(rows(663_000))
        return b, b                                   # self-join; callers slice query tiles
    if config == 6:
        b = ratings_like(rows(283_000))
        return b, b
    raise ValueError("config must be 0..6")


def slice_rows(csr, r0: int, r1: int):
    """Rows [r0, r1) as a CSR of its own (copies the three arrays)."""
    ip = csr["indptr"]
    lo, hi = int(ip[r0]), int(ip[r1])
    return _csr(r1 - r0, csr["n_cols"], ip[r0:r1 + 1] - lo, csr["indices"][lo:hi], csr["values"][lo:hi])


def take_rows(csr, rows):
    """The listed rows, in the given order, as a CSR of its own."""
    rows = np.asarray(rows, dtype=np.int64)
    ip = csr["indptr"]
    deg = ip[rows + 1] - ip[rows]
    indptr = np.zeros(rows.size + 1, dtype=np.int64)
    np.cumsum(deg, out=indptr[1:])
    src = np.repeat(ip[rows] - indptr[:-1], deg) + np.arange(int(indptr[-1]), dtype=np.int64)
    return _csr(rows.size, csr["n_cols"], indptr, csr["indices"][src], csr["values"][src])


def from_dense(dense) -> dict:
    """CSR of a small dense array (zeros are not stored)."""
    d = np.asarray(dense, dtype=np.float64)
    rows, cols = np.nonzero(d)
    indptr = np.zeros(d.shape[0] + 1, dtype=np.int64)
    np.cumsum(np.bincount(rows, minlength=d.shape[0]), out=indptr[1:])
    return _csr(d.shape[0], d.shape[1], indptr, cols, d[rows, cols])


def to_dense(csr) -> np.ndarray:
    out = np.zeros((csr["n_rows"], csr["n_cols"]), dtype=np.float64)
    out[_row_ids(csr["indptr"]), csr["indices"]] = csr["values"]
    return out
