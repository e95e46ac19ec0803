"""fp64 CPU oracle (test infrastructure only; never imported by the product path)."""
from .cpu import (METRICS, PRODUCTS, SUMS, build, knn, max_threads, pairwise,  # noqa: F401
                  semiring_knn, semiring_pairwise)
