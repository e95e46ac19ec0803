"""Thin ctypes binding of libspd.so: argument marshalling only.

Every step of the hot path runs inside the library's HIP kernels; PyTorch is used for
device memory and streams.  The names mirror include/spd.h.
"""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libspd.so")

METRICS = (
    "inner_product", "cosine", "l2_expanded", "correlation", "jaccard", "dice", "hellinger", "l1",
    "chebyshev", "minkowski", "canberra", "hamming", "kl_divergence", "jensen_shannon", "russell_rao",
    "l2_unexpanded", "kl_divergence_strict", "jaccard_literal",
)
METRIC_ID = {name: i for i, name in enumerate(METRICS)}
PRODUCTS = ("times", "plus", "min", "max", "abs_diff", "sq_diff", "abs_diff_pow", "canberra", "not_equal",
            "x_log_x_over_y", "js_term")                                 # spd_product
SUMS = ("plus", "min", "max")                                            # spd_sum
TRANSFORMS = ("none", "sqrt", "nonzero")                                 # spd_transform
EPILOGUES = ("none", "root_p", "div_k", "sqrt_half", "cosine", "l2", "correlation", "jaccard", "dice", "hellinger",
             "russell_rao", "strict")                                    # spd_epilogue
STATUS = ("SPD_OK", "SPD_ERR_NULL", "SPD_ERR_DIM_MISMATCH", "SPD_ERR_BAD_CSR", "SPD_ERR_BAD_METRIC",
          "SPD_ERR_BAD_P", "SPD_ERR_BAD_K", "SPD_ERR_WORKSPACE", "SPD_ERR_HIP", "SPD_ERR_UNSUPPORTED")
KNN_MAX_K = 64


class SpdError(RuntimeError):
    def __init__(self, status: int, message: str):
        self.status = status
        self.status_name = STATUS[status] if 0 <= status < len(STATUS) else str(status)
        super().__init__("%s: %s" % (self.status_name, message))


class CsrStruct(ctypes.Structure):
    _fields_ = [("n_rows", ctypes.c_int64), ("n_cols", ctypes.c_int64), ("nnz", ctypes.c_int64),
                ("indptr", ctypes.c_void_p), ("indices", ctypes.c_void_p), ("values", ctypes.c_void_p),
                ("host_indptr", ctypes.c_void_p)]


class SemiringStruct(ctypes.Structure):
    _fields_ = [("product", ctypes.c_int), ("sum", ctypes.c_int), ("over_union", ctypes.c_int), ("p", ctypes.c_float),
                ("transform", ctypes.c_int), ("epilogue", ctypes.c_int)]


class KernelTime(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 24), ("rows_per_group", ctypes.c_int32), ("staging_kind", ctypes.c_int32),
                ("block", ctypes.c_int32), ("lds_bytes", ctypes.c_int32), ("a_rows", ctypes.c_int64),
                ("workgroups", ctypes.c_int64), ("ms", ctypes.c_double)]


_lib = None


def lib():
    """Loads libspd.so; there is no fallback when it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                "%s is missing: build it with `python -m paper_2104_06357_amd.build`" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, i32, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float
        csr_p = ctypes.POINTER(CsrStruct)
        L.spd_create.argtypes = [ctypes.POINTER(vp), vp]
        L.spd_destroy.argtypes = [vp]
        L.spd_workspace_bytes.argtypes = [vp, csr_p, csr_p, i32, i32, ctypes.POINTER(ctypes.c_size_t)]
        L.spd_set_workspace.argtypes = [vp, vp, ctypes.c_size_t]
        L.spd_pairwise.argtypes = [vp, csr_p, csr_p, i32, f32, vp]
        L.spd_pairwise_static.argtypes = [vp, csr_p, csr_p, i32, f32, vp]
        L.spd_knn.argtypes = [vp, csr_p, csr_p, i32, f32, i32, vp, vp]
        L.spd_semiring_pairwise.argtypes = [vp, csr_p, csr_p, ctypes.POINTER(SemiringStruct), vp]
        L.spd_semiring_knn.argtypes = [vp, csr_p, csr_p, ctypes.POINTER(SemiringStruct), i32, vp, vp]
        L.spd_index_create.argtypes = [vp, csr_p, i32, f32, ctypes.POINTER(vp)]
        L.spd_index_destroy.argtypes = [vp, vp]
        L.spd_index_pairwise.argtypes = [vp, csr_p, vp, vp]
        L.spd_index_knn.argtypes = [vp, csr_p, vp, i32, vp, vp]
        L.spd_csr_validate.argtypes = [vp, csr_p, i32]
        L.spd_set_option.argtypes = [vp, ctypes.c_char_p, i64]
        L.spd_last_error.argtypes = [vp]
        L.spd_last_error.restype = ctypes.c_char_p
        L.spd_metric_name.argtypes = [i32]
        L.spd_metric_name.restype = ctypes.c_char_p
        L.spd_version.restype = ctypes.c_char_p
        L.spd_profile_read.argtypes = [vp, ctypes.POINTER(KernelTime), i32]
        L.spd_profile_read.restype = ctypes.c_int
        L.spd_host_pair_value.argtypes = [i32, f32, i64, vp, vp, i64, vp, vp, i64, ctypes.POINTER(f32)]
        L.spd_host_plan_summary.argtypes = [vp, i64, vp, i64, i64, i32, i32, ctypes.POINTER(ctypes.c_char_p),
                                            ctypes.POINTER(i64), i32, ctypes.c_char_p, ctypes.c_size_t]
        for fn in ("spd_create", "spd_destroy", "spd_workspace_bytes", "spd_set_workspace", "spd_pairwise",
                   "spd_pairwise_static",
                   "spd_knn", "spd_semiring_pairwise", "spd_semiring_knn", "spd_index_create", "spd_index_destroy",
                   "spd_index_pairwise", "spd_index_knn", "spd_csr_validate", "spd_set_option", "spd_host_pair_value",
                   "spd_host_plan_summary"):
            getattr(L, fn).restype = ctypes.c_int
        _lib = L
    return _lib


def metric_id(metric) -> int:
    if isinstance(metric, str):
        if metric not in METRIC_ID:
            raise ValueError("unknown metric %r" % metric)
        return METRIC_ID[metric]
    return int(metric)


class DeviceCsr:
    """A CSR matrix whose three arrays are torch tensors on the GPU; `host_indptr`, if given, is
    a host copy of the row pointers (a contiguous int64 numpy array) that spares the library
    reading them back."""

    def __init__(self, n_rows, n_cols, indptr, indices, values, host_indptr=None):
        import torch
        assert indptr.dtype == torch.int64 and indices.dtype == torch.int32 and values.dtype == torch.float32
        assert indptr.is_cuda and indices.is_cuda and values.is_cuda
        self.n_rows, self.n_cols = int(n_rows), int(n_cols)
        self.indptr, self.indices, self.values = indptr.contiguous(), indices.contiguous(), values.contiguous()
        self.nnz = int(self.indices.numel())
        self.host_indptr = None
        if host_indptr is not None:
            import numpy as np
            self.host_indptr = np.ascontiguousarray(host_indptr, dtype=np.int64)
            assert self.host_indptr.shape == (self.n_rows + 1,)

    @classmethod
    def from_host(cls, csr: dict, device="cuda:0", keep_host_indptr=True):
        import torch
        return cls(csr["n_rows"], csr["n_cols"],
                   torch.from_numpy(csr["indptr"]).to(device),
                   torch.from_numpy(csr["indices"]).to(device),
                   torch.from_numpy(csr["values"]).to(device),
                   host_indptr=csr["indptr"] if keep_host_indptr else None)

    def struct(self) -> CsrStruct:
        return CsrStruct(self.n_rows, self.n_cols, self.nnz, self.indptr.data_ptr(),
                         self.indices.data_ptr() if self.nnz else None,
                         self.values.data_ptr() if self.nnz else None,
                         self.host_indptr.ctypes.data if self.host_indptr is not None else None)


class Handle:
    """spd_handle bound to torch's current stream at creation (or to `stream`)."""

    def __init__(self, stream=None):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("spd needs a GPU: torch.cuda.is_available() is False")
        self._lib = lib()
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        self._h = ctypes.c_void_p()
        st = self._lib.spd_create(ctypes.byref(self._h), ctypes.c_void_p(self.stream.cuda_stream))
        if st != 0:
            raise SpdError(st, "spd_create failed")

    def close(self):
        if self._h:
            self._lib.spd_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st):
        if st != 0:
            raise SpdError(st, (self._lib.spd_last_error(self._h) or b"").decode())

    def set_option(self, name: str, value: int):
        self._check(self._lib.spd_set_option(self._h, name.encode(), int(value)))

    def profile_read(self):
        """Kernel timings of the last call (option "profile" = 1): a list of dicts."""
        buf = (KernelTime * 64)()
        n = self._lib.spd_profile_read(self._h, buf, 64)
        if n < 0:
            raise SpdError(8, "spd_profile_read failed (%d)" % n)
        return [{f[0]: (getattr(buf[i], f[0]).decode() if f[0] == "name" else getattr(buf[i], f[0]))
                 for f in KernelTime._fields_} for i in range(min(n, 64))]

    def workspace_bytes(self, A: DeviceCsr, B: DeviceCsr, metric, k_neighbors: int = 0) -> int:
        out = ctypes.c_size_t()
        sa, sb = A.struct(), B.struct()
        self._check(self._lib.spd_workspace_bytes(self._h, ctypes.byref(sa), ctypes.byref(sb), metric_id(metric),
                                                  int(k_neighbors), ctypes.byref(out)))
        return int(out.value)

    def set_workspace(self, tensor):
        if tensor is None:
            self._check(self._lib.spd_set_workspace(self._h, None, 0))
        else:
            self._ws_keepalive = tensor
            self._check(self._lib.spd_set_workspace(self._h, tensor.data_ptr(), tensor.numel() * tensor.element_size()))

    def csr_validate(self, M: DeviceCsr, require_nonnegative: bool = False):
        s = M.struct()
        self._check(self._lib.spd_csr_validate(self._h, ctypes.byref(s), int(require_nonnegative)))

    def pairwise(self, A: DeviceCsr, B: DeviceCsr, metric, p: float = 2.0, out=None):
        """out[i, j] = d(A_i, B_j) as an fp32 torch tensor (m, n) on the GPU."""
        import torch
        if out is None:
            out = torch.empty((A.n_rows, B.n_rows), dtype=torch.float32, device=A.indptr.device)
        assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous()
        assert tuple(out.shape) == (A.n_rows, B.n_rows)
        sa, sb = A.struct(), B.struct()
        self._check(self._lib.spd_pairwise(self._h, ctypes.byref(sa), ctypes.byref(sb), metric_id(metric),
                                           float(p), out.data_ptr() if out.numel() else None))
        return out

    def pairwise_static(self, A: DeviceCsr, B: DeviceCsr, metric, out, p: float = 2.0):
        """spd_pairwise_static: the same distances into `out` (which the caller allocates), with the
        library's static scratch array; the call allocates nothing."""
        import torch
        assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous()
        assert tuple(out.shape) == (A.n_rows, B.n_rows)
        sa, sb = A.struct(), B.struct()
        self._check(self._lib.spd_pairwise_static(self._h, ctypes.byref(sa), ctypes.byref(sb), metric_id(metric),
                                                  float(p), out.data_ptr() if out.numel() else None))
        return out

    def knn(self, Q: DeviceCsr, Index: DeviceCsr, metric, k: int, p: float = 2.0, out_idx=None, out_dist=None):
        """(idx int64 [m, k], dist fp32 [m, k]) of the k nearest index rows per query row."""
        import torch
        if out_idx is None:
            out_idx = torch.empty((Q.n_rows, k), dtype=torch.int64, device=Q.indptr.device)
        if out_dist is None:
            out_dist = torch.empty((Q.n_rows, k), dtype=torch.float32, device=Q.indptr.device)
        sa, sb = Q.struct(), Index.struct()
        self._check(self._lib.spd_knn(self._h, ctypes.byref(sa), ctypes.byref(sb), metric_id(metric), float(p), int(k),
                                      out_idx.data_ptr() if out_idx.numel() else None,
                                      out_dist.data_ptr() if out_dist.numel() else None))
        return out_idx, out_dist


    def index_create(self, Index: DeviceCsr, metric, p: float = 2.0) -> "Index":
        """Prepares `Index` as the second operand of `metric` (spd_index_create)."""
        ptr = ctypes.c_void_p()
        s = Index.struct()
        self._check(self._lib.spd_index_create(self._h, ctypes.byref(s), metric_id(metric), float(p), ctypes.byref(ptr)))
        return Index_(self, ptr, Index)

    @staticmethod
    def _semiring(product, sum, over_union, p=2.0, transform="none", epilogue="none") -> SemiringStruct:
        prod = PRODUCTS.index(product) if isinstance(product, str) else int(product)
        sm = SUMS.index(sum) if isinstance(sum, str) else int(sum)
        tr = TRANSFORMS.index(transform) if isinstance(transform, str) else int(transform)
        ep = EPILOGUES.index(epilogue) if isinstance(epilogue, str) else int(epilogue)
        return SemiringStruct(prod, sm, int(bool(over_union)), float(p), tr, ep)

    def semiring_pairwise(self, A: DeviceCsr, B: DeviceCsr, product, sum, over_union: bool, out=None, p: float = 2.0,
                          transform="none", epilogue="none"):
        """out[i, j] = the semiring's value between A_i and B_j as an fp32 torch tensor (m, n)."""
        import torch
        if out is None:
            out = torch.empty((A.n_rows, B.n_rows), dtype=torch.float32, device=A.indptr.device)
        assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous()
        assert tuple(out.shape) == (A.n_rows, B.n_rows)
        sa, sb, sr = A.struct(), B.struct(), self._semiring(product, sum, over_union, p, transform, epilogue)
        self._check(self._lib.spd_semiring_pairwise(self._h, ctypes.byref(sa), ctypes.byref(sb), ctypes.byref(sr),
                                                    out.data_ptr() if out.numel() else None))
        return out

    def semiring_knn(self, Q: DeviceCsr, Index: DeviceCsr, product, sum, over_union: bool, k: int, p: float = 2.0,
                     transform="none", epilogue="none"):
        """(idx int64 [m, k], value fp32 [m, k]) of the k smallest semiring values per query row."""
        import torch
        out_idx = torch.empty((Q.n_rows, k), dtype=torch.int64, device=Q.indptr.device)
        out_dist = torch.empty((Q.n_rows, k), dtype=torch.float32, device=Q.indptr.device)
        sa, sb, sr = Q.struct(), Index.struct(), self._semiring(product, sum, over_union, p, transform, epilogue)
        self._check(self._lib.spd_semiring_knn(self._h, ctypes.byref(sa), ctypes.byref(sb), ctypes.byref(sr), int(k),
                                               out_idx.data_ptr() if out_idx.numel() else None,
                                               out_dist.data_ptr() if out_dist.numel() else None))
        return out_idx, out_dist


class Index_:
    """spd_index: owned by the handle that made it; keeps the matrix's tensors alive."""

    def __init__(self, handle: Handle, ptr, matrix: DeviceCsr):
        self._handle, self._ptr, self.matrix = handle, ptr, matrix

    def close(self):
        if self._ptr and self._handle._h:
            self._handle._lib.spd_index_destroy(self._handle._h, self._ptr)
        self._ptr = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def pairwise(self, A: DeviceCsr, out=None):
        import torch
        h = self._handle
        if out is None:
            out = torch.empty((A.n_rows, self.matrix.n_rows), dtype=torch.float32, device=A.indptr.device)
        assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous()
        assert tuple(out.shape) == (A.n_rows, self.matrix.n_rows)
        sa = A.struct()
        h._check(h._lib.spd_index_pairwise(h._h, ctypes.byref(sa), self._ptr, out.data_ptr() if out.numel() else None))
        return out

    def knn(self, Q: DeviceCsr, k: int, out_idx=None, out_dist=None):
        import torch
        h = self._handle
        if out_idx is None:
            out_idx = torch.empty((Q.n_rows, k), dtype=torch.int64, device=Q.indptr.device)
        if out_dist is None:
            out_dist = torch.empty((Q.n_rows, k), dtype=torch.float32, device=Q.indptr.device)
        sa = Q.struct()
        h._check(h._lib.spd_index_knn(h._h, ctypes.byref(sa), self._ptr, int(k),
                                      out_idx.data_ptr() if out_idx.numel() else None,
                                      out_dist.data_ptr() if out_dist.numel() else None))
        return out_idx, out_dist
