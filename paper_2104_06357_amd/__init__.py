"""spd: sparse all-pairs distances as a semiring product on one MI355X (gfx950).

The package is a thin binding over ``libspd.so`` (built from ``csrc/`` by ``build.py``).
"""
from .binding import (KNN_MAX_K, METRICS, PRODUCTS, SUMS, DeviceCsr, Handle, SpdError, host_pair_value,  # noqa: F401
                      host_plan_summary, lib)
