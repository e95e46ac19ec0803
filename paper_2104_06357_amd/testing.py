"""Host-only test hooks of libspd.so (include/spd_testing.h): the planner's summary of a call and
one distance evaluated on the host with the kernels' arithmetic.  For tests; no product call
reaches them, and they touch no GPU."""
from __future__ import annotations

import ctypes

from .binding import SpdError, lib, metric_id


def host_pair_value(metric, p, n_cols, a_cols, a_vals, b_cols, b_vals) -> float:
    import numpy as np
    a_cols = np.ascontiguousarray(a_cols, dtype=np.int32); a_vals = np.ascontiguousarray(a_vals, dtype=np.float32)
    b_cols = np.ascontiguousarray(b_cols, dtype=np.int32); b_vals = np.ascontiguousarray(b_vals, dtype=np.float32)
    out = ctypes.c_float()
    st = lib().spd_host_pair_value(metric_id(metric), float(p), int(n_cols), a_cols.ctypes.data, a_vals.ctypes.data,
                                   a_cols.size, b_cols.ctypes.data, b_vals.ctypes.data, b_cols.size, ctypes.byref(out))
    if st != 0:
        raise SpdError(st, "spd_host_pair_value")
    return float(out.value)


def host_plan_summary(a_indptr, b_indptr, n_cols, metric, k_neighbors=0, **options) -> dict:
    import json

    import numpy as np
    a_indptr = np.ascontiguousarray(a_indptr, dtype=np.int64)
    b_indptr = np.ascontiguousarray(b_indptr, dtype=np.int64)
    names = (ctypes.c_char_p * max(1, len(options)))(*[k.encode() for k in options])
    vals = (ctypes.c_int64 * max(1, len(options)))(*[int(v) for v in options.values()])
    buf = ctypes.create_string_buffer(1 << 16)
    st = lib().spd_host_plan_summary(a_indptr.ctypes.data, a_indptr.size - 1, b_indptr.ctypes.data, b_indptr.size - 1,
                                     int(n_cols), metric_id(metric), int(k_neighbors), names, vals, len(options),
                                     buf, len(buf))
    text = buf.value.decode()
    if st != 0:
        raise SpdError(st, text)
    return json.loads(text)
