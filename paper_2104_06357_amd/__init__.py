"""spd: sparse all-pairs distances as a semiring product on one MI355X (gfx950).

The package is a thin binding over ``libspd.so`` (built from ``csrc/`` by ``build.py``);
``paper_2104_06357_amd.testing`` holds the host-only hooks the tests use.
"""
from . import testing  # noqa: F401
from .binding import (EPILOGUES, KNN_MAX_K, METRICS, PRODUCTS, SUMS, TRANSFORMS, DeviceCsr, Handle, SpdError,  # noqa: F401
                      lib)
