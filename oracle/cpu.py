"""ctypes front end of the fp64 CPU oracle in ``spd_oracle.c``.

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's
CPU-baseline leg.  It never touches the HIP library and the HIP library never touches it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spd_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

METRICS = (
    "inner_product", "cosine", "euclidean", "correlation", "jaccard", "dice", "hellinger",
    "manhattan", "chebyshev", "minkowski", "canberra", "hamming", "kl_divergence",
    "jensen_shannon", "russell_rao", "kl_divergence_strict", "jaccard_literal",
)

PRODUCTS = ("times", "plus", "min", "max", "abs_diff", "sq_diff")          # the commutative menu, any sum(), any domain
MORE_PRODUCTS = ("abs_diff_pow", "canberra", "not_equal", "x_log_x_over_y", "js_term")   # Table 1's other products
ALL_PRODUCTS = PRODUCTS + MORE_PRODUCTS
SUMS = ("plus", "min", "max")
TRANSFORMS = ("none", "sqrt", "nonzero")
EPILOGUES = ("none", "root_p", "div_k", "sqrt_half", "cosine", "l2", "correlation", "jaccard", "dice", "hellinger",
             "russell_rao", "strict")

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, -O2, OpenMP over query rows)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-shared", "-fPIC",
             _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.oracle_metric_id.argtypes = [ctypes.c_char_p]
        lib.oracle_metric_id.restype = ctypes.c_int
        lib.oracle_max_threads.restype = ctypes.c_int
        P = ctypes.c_void_p
        lib.oracle_pairwise.argtypes = [
            ctypes.c_int64, ctypes.c_int64, P, P, P, ctypes.c_int64, P, P, P, ctypes.c_int,
            ctypes.c_double, P, ctypes.c_int64, P, ctypes.c_int64, ctypes.c_int, ctypes.c_int, P]
        lib.oracle_pairwise.restype = ctypes.c_int
        lib.oracle_semiring_pairwise.argtypes = [
            ctypes.c_int64, ctypes.c_int64, P, P, P, ctypes.c_int64, P, P, P, ctypes.c_int, ctypes.c_int,
            ctypes.c_int, ctypes.c_double, ctypes.c_int, ctypes.c_int, P, ctypes.c_int64, P, ctypes.c_int64,
            ctypes.c_int, ctypes.c_int, P]
        lib.oracle_semiring_pairwise.restype = ctypes.c_int
        _lib = lib
    return _lib


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def _csr_arrays(m):
    return (np.ascontiguousarray(m["indptr"], dtype=np.int64),
            np.ascontiguousarray(m["indices"], dtype=np.int32),
            np.ascontiguousarray(m["values"], dtype=np.float32))


def pairwise(A, B, metric: str, p: float = 2.0, rows_a=None, rows_b=None, mode: str = "support",
             threads: int = 0, return_threads: bool = False):
    """fp64 distances d(A[rows_a[a]], B[rows_b[b]]) as an array (len(rows_a), len(rows_b)).

    mode "full" visits every column of every pair; "support" visits only the union of
    the two supports (proven equal by the tests)."""
    lib = _load()
    mid = lib.oracle_metric_id(metric.encode())
    if mid < 0:
        raise ValueError("unknown metric %r" % metric)
    if A["n_cols"] != B["n_cols"]:
        raise ValueError("column counts differ")
    aip, aix, av = _csr_arrays(A)
    bip, bix, bv = _csr_arrays(B)
    ra = None if rows_a is None else np.ascontiguousarray(rows_a, dtype=np.int64)
    rb = None if rows_b is None else np.ascontiguousarray(rows_b, dtype=np.int64)
    na = A["n_rows"] if ra is None else ra.size
    nb = B["n_rows"] if rb is None else rb.size
    out = np.empty((na, nb), dtype=np.float64)
    used = lib.oracle_pairwise(
        A["n_rows"], A["n_cols"], _ptr(aip), _ptr(aix), _ptr(av), B["n_rows"], _ptr(bip), _ptr(bix),
        _ptr(bv), mid, float(p), _ptr(ra), na, _ptr(rb), nb, {"full": 0, "support": 1}[mode],
        int(threads), _ptr(out))
    if used < 0:
        raise RuntimeError("oracle failed (%d)" % used)
    return (out, used) if return_threads else out


def semiring_pairwise(A, B, product: str, sum: str, over_union: bool, rows_a=None, rows_b=None,
                      mode: str = "support", threads: int = 0, p: float = 2.0, transform: str = "none",
                      epilogue: str = "none"):
    """fp64 semiring products between rows (Section 2.2): the `sum` fold of `product` over the
    columns stored in both rows (over_union False) or in either row, the missing side read as 0
    (over_union True); the identity of `sum` where that set is empty.  `transform` is applied to
    every stored value first, `epilogue` (Table 1's expansion functions and closing steps) to the
    folded value; `p` is the degree of "abs_diff_pow" and "root_p"."""
    lib = _load()
    if A["n_cols"] != B["n_cols"]:
        raise ValueError("column counts differ")
    aip, aix, av = _csr_arrays(A)
    bip, bix, bv = _csr_arrays(B)
    ra = None if rows_a is None else np.ascontiguousarray(rows_a, dtype=np.int64)
    rb = None if rows_b is None else np.ascontiguousarray(rows_b, dtype=np.int64)
    na = A["n_rows"] if ra is None else ra.size
    nb = B["n_rows"] if rb is None else rb.size
    out = np.empty((na, nb), dtype=np.float64)
    used = lib.oracle_semiring_pairwise(
        A["n_rows"], A["n_cols"], _ptr(aip), _ptr(aix), _ptr(av), B["n_rows"], _ptr(bip), _ptr(bix),
        _ptr(bv), ALL_PRODUCTS.index(product), SUMS.index(sum), int(bool(over_union)), float(p),
        TRANSFORMS.index(transform), EPILOGUES.index(epilogue), _ptr(ra), na, _ptr(rb), nb,
        {"full": 0, "support": 1}[mode], int(threads), _ptr(out))
    if used < 0:
        raise RuntimeError("oracle failed (%d)" % used)
    return out


def semiring_knn(Q, Index, product: str, sum: str, over_union: bool, k: int, rows_q=None, threads: int = 0,
                 p: float = 2.0, transform: str = "none", epilogue: str = "none"):
    """The k index rows with the smallest semiring value for each query row, by (value, index)."""
    d = semiring_pairwise(Q, Index, product, sum, over_union, rows_a=rows_q, threads=threads, p=p,
                          transform=transform, epilogue=epilogue)
    n = d.shape[1]
    idx = np.empty((d.shape[0], k), dtype=np.int64)
    for r in range(d.shape[0]):
        idx[r] = np.lexsort((np.arange(n), d[r]))[:k]
    return idx, np.take_along_axis(d, idx, axis=1)


def knn(Q, Index, metric: str, k: int, p: float = 2.0, rows_q=None, threads: int = 0):
    """Brute-force k nearest index rows of each query row (the benchmark protocol of the
    Experiments section: full distance row, then select).

    Returns (idx int64 [m, k], dist fp64 [m, k]) ordered by (distance, index) ascending;
    for the inner product, which is a similarity, by (-value, index)."""
    d = pairwise(Q, Index, metric, p, rows_a=rows_q, threads=threads)
    key = -d if metric == "inner_product" else d
    n = d.shape[1]
    idx = np.empty((d.shape[0], k), dtype=np.int64)
    for r in range(d.shape[0]):
        order = np.lexsort((np.arange(n), key[r]))     # last key is the primary one
        idx[r] = order[:k]
    return idx, np.take_along_axis(d, idx, axis=1)
