"""fp64 CPU oracle (test infrastructure only; never imported by the product path)."""
from .cpu import (ALL_PRODUCTS, EPILOGUES, METRICS, MORE_PRODUCTS, PRODUCTS, SUMS, TRANSFORMS, build, knn,  # noqa: F401
                  max_threads, pairwise, semiring_knn, semiring_pairwise)
