"""ctypes binding of libcbm.so: same names as the C ABI (include/cbm.h), argument
marshalling only.  PyTorch tensors supply device memory and the stream; every
step of the product runs in the library's HIP kernels.  There is no fallback:
a missing library raises."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libcbm.so")

CBM_FLAG_HOST_ONLY = 1
CBM_FLAG_EXACT_TREE = 2
CBM_FLAG_DEVICE_BUILD = 4
CBM_FLAG_TRANSPOSE = 8
CBM_FLAG_HOST_SEARCH = 16

EXPORTS = [
    "cbm_build", "cbm_spmm", "cbm_spmm_noalloc", "cbm_spmm_normalized", "cbm_spmm_normalized_relu", "cbm_spmm_mean", "cbm_spmm_gin",
    "cbm_dense_matmul", "cbm_reserve",
    "cbm_gcn2_forward", "cbm_gcn2_workspace_bytes", "cbm_stats", "cbm_get_tree", "cbm_decompress",
    "cbm_profile_enable", "cbm_profile_read", "cbm_free", "cbm_status_string", "cbm_last_error_detail",
]


class CbmError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = _lib().cbm_last_error_detail().decode() if status in (3, 4) else ""
        super().__init__(f"{where}: {_lib().cbm_status_string(status).decode()} (status {status})"
                         + (f" [{detail}]" if detail else ""))


class cbm_build_opts(C.Structure):
    _fields_ = [("alpha", C.c_int32), ("add_self_loops", C.c_int32), ("max_depth", C.c_int32),
                ("hub_cap", C.c_int32), ("max_candidates", C.c_int32), ("seed_roots", C.c_int32),
                ("num_threads", C.c_int32),
                ("device", C.c_int32), ("flags", C.c_uint32), ("column_blocks", C.c_int32)]


class cbm_stats_t(C.Structure):
    _fields_ = [("m", C.c_int64), ("n", C.c_int64), ("nnz", C.c_int64), ("num_delta_plus", C.c_int64),
                ("num_delta_minus", C.c_int64), ("num_roots", C.c_int64), ("num_internal", C.c_int64),
                ("scalar_ops", C.c_int64), ("num_tasks", C.c_int64), ("num_split_rows", C.c_int64),
                ("bytes_csr", C.c_int64), ("bytes_cbm", C.c_int64), ("depth", C.c_int32), ("alpha", C.c_int32),
                ("add_self_loops", C.c_int32), ("rounds", C.c_int32), ("build_seconds", C.c_double),
                ("column_blocks", C.c_int32), ("bundled_rounds", C.c_int32)]

    def as_dict(self) -> dict:
        return {f: getattr(self, f) for f, _ in self._fields_}


class cbm_launch_record(C.Structure):
    _fields_ = [("kind", C.c_int32), ("level", C.c_int32), ("tasks", C.c_int64), ("deltas", C.c_int64),
                ("algorithmic_bytes", C.c_int64), ("milliseconds", C.c_float), ("per_xcd", C.c_int32)]


_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built: run `python -m paper_2409_02208_amd.build`")
        # PyTorch ships its own HIP runtime.  It must be in the process before libcbm.so is loaded, so that
        # the library binds to that same runtime: device pointers and streams are only meaningful within one.
        import torch  # noqa: F401

        lib = C.CDLL(LIB_PATH)
        vp, i64, i32, f32p = C.c_void_p, C.c_int64, C.c_int32, C.c_void_p
        lib.cbm_build.argtypes = [i64, i64, vp, vp, C.POINTER(cbm_build_opts), C.POINTER(vp)]
        for name in ("cbm_spmm", "cbm_spmm_noalloc", "cbm_spmm_normalized", "cbm_spmm_normalized_relu", "cbm_spmm_mean"):
            getattr(lib, name).argtypes = [vp, f32p, i64, i32, f32p, i64, vp]
        lib.cbm_spmm_gin.argtypes = [vp, C.c_float, f32p, i64, i32, f32p, i64, vp]
        lib.cbm_reserve.argtypes = [vp, i32]
        lib.cbm_dense_matmul.argtypes = [i64, i32, i32, f32p, i64, f32p, i64, f32p, i64, vp]
        lib.cbm_gcn2_forward.argtypes = [vp, f32p, i32, f32p, i32, f32p, i32, f32p, vp, C.c_size_t, vp]
        lib.cbm_gcn2_workspace_bytes.argtypes = [vp, i32, i32, i32]
        lib.cbm_gcn2_workspace_bytes.restype = C.c_size_t
        lib.cbm_stats.argtypes = [vp, C.POINTER(cbm_stats_t)]
        lib.cbm_get_tree.argtypes = [vp, vp, vp, vp, vp]
        lib.cbm_decompress.argtypes = [vp, vp, vp]
        lib.cbm_profile_enable.argtypes = [vp, i32]
        lib.cbm_profile_read.argtypes = [vp, C.POINTER(cbm_launch_record), i32, C.POINTER(i32)]
        lib.cbm_free.argtypes = [vp]
        lib.cbm_free.restype = None
        lib.cbm_status_string.argtypes = [C.c_int]
        lib.cbm_status_string.restype = C.c_char_p
        lib.cbm_last_error_detail.argtypes = []
        lib.cbm_last_error_detail.restype = C.c_char_p
        _LIB = lib
    return _LIB


def _check(status: int, where: str):
    if status != 0:
        raise CbmError(status, where)


def _stream_ptr(stream):
    if stream is None:
        import torch

        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _dev_f32(t, name):
    if not (t.is_cuda and t.dtype.is_floating_point and t.element_size() == 4 and t.dim() == 2 and t.stride(1) == 1):
        raise ValueError(f"{name} must be a 2-D fp32 device tensor with unit column stride")
    return t.data_ptr(), t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])


class Handle:
    """Owner of one cbm_handle*."""

    def __init__(self, ptr):
        self._ptr = ptr

    @property
    def ptr(self):
        if not self._ptr:
            raise RuntimeError("handle already freed")
        return self._ptr

    def __del__(self):
        try:
            cbm_free(self)
        except Exception:
            pass


def cbm_build(m: int, n: int, rowptr: np.ndarray, colidx: np.ndarray, *, alpha: int = 0,
              add_self_loops: bool = False, max_depth: int = 0, hub_cap: int = 0, max_candidates: int = 0,
              seed_roots: int = 0, num_threads: int = 0, device: int = -1, host_only: bool = False, exact_tree: bool = False,
              device_build: bool = False, transpose: bool = False, host_search: bool = False,
              column_blocks: int = 0) -> Handle:
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    if rowptr.shape != (m + 1,):
        raise ValueError("rowptr must have m + 1 entries")
    if len(colidx) < int(rowptr[-1]):
        raise ValueError("colidx shorter than rowptr[m]")
    opts = cbm_build_opts(alpha, int(add_self_loops), max_depth, hub_cap, max_candidates, seed_roots, num_threads, device,
                          (CBM_FLAG_HOST_ONLY if host_only else 0) | (CBM_FLAG_EXACT_TREE if exact_tree else 0) |
                          (CBM_FLAG_DEVICE_BUILD if device_build else 0) | (CBM_FLAG_TRANSPOSE if transpose else 0) |
                          (CBM_FLAG_HOST_SEARCH if host_search else 0), column_blocks)
    out = C.c_void_p()
    _check(_lib().cbm_build(m, n, rowptr.ctypes.data, colidx.ctypes.data, C.byref(opts), C.byref(out)), "cbm_build")
    return Handle(out.value)


def _product(fn_name, h: Handle, X, Y, stream):
    xp, ldx = _dev_f32(X, "X")
    yp, ldy = _dev_f32(Y, "Y")
    if X.shape[1] != Y.shape[1]:
        raise ValueError("X and Y must have the same number of columns")
    _check(getattr(_lib(), fn_name)(h.ptr, xp, ldx, X.shape[1], yp, ldy, _stream_ptr(stream)), fn_name)
    return Y


def cbm_spmm(h: Handle, X, Y, stream=None):
    return _product("cbm_spmm", h, X, Y, stream)


def cbm_spmm_noalloc(h: Handle, X, Y, stream=None):
    return _product("cbm_spmm_noalloc", h, X, Y, stream)


def cbm_spmm_normalized(h: Handle, X, Y, stream=None):
    return _product("cbm_spmm_normalized", h, X, Y, stream)


def cbm_spmm_normalized_relu(h: Handle, X, Y, stream=None):
    return _product("cbm_spmm_normalized_relu", h, X, Y, stream)


def cbm_spmm_mean(h: Handle, X, Y, stream=None):
    return _product("cbm_spmm_mean", h, X, Y, stream)


def cbm_spmm_gin(h: Handle, eps: float, X, Y, stream=None):
    xp, ldx = _dev_f32(X, "X")
    yp, ldy = _dev_f32(Y, "Y")
    if X.shape[1] != Y.shape[1]:
        raise ValueError("X and Y must have the same number of columns")
    _check(_lib().cbm_spmm_gin(h.ptr, float(eps), xp, ldx, X.shape[1], yp, ldy, _stream_ptr(stream)), "cbm_spmm_gin")
    return Y


def cbm_reserve(h: Handle, max_k: int):
    _check(_lib().cbm_reserve(h.ptr, int(max_k)), "cbm_reserve")


def cbm_dense_matmul(A, B, Cout, stream=None):
    ap, lda = _dev_f32(A, "A")
    bp, ldb = _dev_f32(B, "B")
    cp, ldc = _dev_f32(Cout, "C")
    M, K = A.shape
    if B.shape[0] != K or Cout.shape != (M, B.shape[1]):
        raise ValueError("shape mismatch")
    _check(_lib().cbm_dense_matmul(M, B.shape[1], K, ap, lda, bp, ldb, cp, ldc, _stream_ptr(stream)),
           "cbm_dense_matmul")
    return Cout


def cbm_gcn2_workspace_bytes(h: Handle, f_in: int, hidden: int, f_out: int) -> int:
    return int(_lib().cbm_gcn2_workspace_bytes(h.ptr, f_in, hidden, f_out))


def cbm_gcn2_forward(h: Handle, X, W0, W1, out, workspace, stream=None):
    for t, name in ((X, "X"), (W0, "W0"), (W1, "W1"), (out, "out")):
        _dev_f32(t, name)
        if not t.is_contiguous():
            raise ValueError(f"{name} must be densely packed")
    f_in, hidden, f_out = X.shape[1], W0.shape[1], W1.shape[1]
    if W0.shape[0] != f_in or W1.shape[0] != hidden or out.shape != (X.shape[0], f_out):
        raise ValueError("shape mismatch")
    _check(_lib().cbm_gcn2_forward(h.ptr, X.data_ptr(), f_in, W0.data_ptr(), hidden, W1.data_ptr(), f_out,
                                   out.data_ptr(), workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                   _stream_ptr(stream)), "cbm_gcn2_forward")
    return out


def cbm_stats(h: Handle) -> dict:
    s = cbm_stats_t()
    _check(_lib().cbm_stats(h.ptr, C.byref(s)), "cbm_stats")
    return s.as_dict()


def cbm_get_tree(h: Handle):
    s = cbm_stats(h)
    m = s["m"] * max(1, s["column_blocks"])
    arrs = [np.empty(m, dtype=np.int32) for _ in range(4)]
    _check(_lib().cbm_get_tree(h.ptr, *[a.ctypes.data for a in arrs]), "cbm_get_tree")
    return dict(zip(("parent", "nplus", "nminus", "level"), arrs))


def cbm_decompress(h: Handle):
    s = cbm_stats(h)
    rowptr = np.empty(s["m"] + 1, dtype=np.int64)
    colidx = np.empty(max(1, s["nnz"]), dtype=np.int32)
    _check(_lib().cbm_decompress(h.ptr, rowptr.ctypes.data, colidx.ctypes.data), "cbm_decompress")
    return rowptr, colidx[:s["nnz"]]


def cbm_profile_enable(h: Handle, on: bool = True):
    _check(_lib().cbm_profile_enable(h.ptr, int(on)), "cbm_profile_enable")


def cbm_profile_read(h: Handle) -> list:
    cap = 4096
    recs = (cbm_launch_record * cap)()
    cnt = C.c_int32()
    _check(_lib().cbm_profile_read(h.ptr, recs, cap, C.byref(cnt)), "cbm_profile_read")
    return [dict(kind=r.kind, level=r.level, tasks=r.tasks, deltas=r.deltas,
                 algorithmic_bytes=r.algorithmic_bytes, milliseconds=r.milliseconds, per_xcd=r.per_xcd)
            for r in recs[:min(cap, cnt.value)]]


def cbm_free(h: Handle):
    if h is not None and getattr(h, "_ptr", None):
        _lib().cbm_free(h._ptr)
        h._ptr = None


def cbm_status_string(status: int) -> str:
    return _lib().cbm_status_string(status).decode()
