"""fp64 CPU oracle (test infrastructure only; never imported by the product path)."""
from .cpu import METRICS, build, knn, max_threads, pairwise  # noqa: F401
